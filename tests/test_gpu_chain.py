"""The pieces in the order the method uses them (Sec. 3: monitoring -> freeze
ratios -> progressive freezing), on a small fp32 stage, library against oracle
at every hand-over: measured-style action times -> linear program -> expected
ratio of this stage's backward -> per step the actual ratio, a seeded draw of
row blocks, the backward that skips them, their element masks, the masked
AdamW step - and the updated parameters are the weights of the next step.
Bounds: fp32 path, relative Frobenius 1e-5 per tensor after four chained steps;
rows frozen in every step bit-identical."""
import numpy as np
import pytest
import torch

import oracle
from oracle import schedule as sc
import workloads as wl
import paper_2602_05754_amd as tf
from gpu_util import host64, rel_fro

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx():
    c = tf.Context(0)
    yield c
    c.close()


def test_monitoring_to_masked_update_chain(ctx):
    cfg = wl.scaled(wl.CONFIGS[1], blocks=1)
    shapes, L, T, br = cfg.shapes, cfg.n_layers, 96, 16
    numel = [k * n for k, n in shapes]
    hp = {k: float(np.float32(getattr(cfg, k))) for k in ("lr", "beta1", "beta2", "eps", "weight_decay")}

    # -- phase II: 2 stages x 2 microbatches under 1F1B, backward between 1.2 (all frozen) and 2.0 (none)
    S, M = 2, 2
    w_max = np.r_[np.full(S * M, 1.0), np.full(S * M, 2.0)]
    w_min = np.r_[np.full(S * M, 1.0), np.full(S * M, 1.2)]
    lib = tf.tf_freeze_ratio_lp(S, M, tf.TF_SCHEDULE_1F1B, w_min, w_max, 0.8, 1e-4)
    ref = sc.freeze_ratio_lp(S, M, sc.ONE_F_ONE_B, w_min, w_max, 0.8, 1e-4)
    assert lib["P_d"] == pytest.approx(ref["P_d"], rel=1e-7) and lib["P_d"] < lib["P_d_max"]
    # the backward action of stage 0 that the program shortens most
    r_star = max(float(lib["r"][sc.node_id(1, m, 0, M, S)]) for m in range(M))
    assert 0.0 < r_star <= 1.0

    # -- phase III: four steps, ratio ramping up over the first three
    rs = np.random.default_rng(2026)
    f32 = lambda a: np.ascontiguousarray(a, dtype=np.float32)
    p0 = [f32(rs.standard_normal(s) * 0.02) for s in shapes]
    dp = [torch.from_numpy(a.copy()).cuda() for a in p0]
    dm = [torch.zeros(s, device="cuda") for s in shapes]
    dv = [torch.zeros(s, device="cuda") for s in shapes]
    dW = [torch.zeros(s, device="cuda") for s in shapes]
    bits = [torch.zeros((n + 31) // 32, dtype=torch.int32, device="cuda") for n in numel]
    op = [np.asarray(a, dtype=np.float64) for a in p0]
    om = [np.zeros(n) for n in numel]
    ov = [np.zeros(n) for n in numel]
    steps = [1] * L
    ever_unfrozen = [np.zeros(k // br, bool) for k, n in shapes]
    for t in range(1, 5):
        afr = tf.tf_actual_freeze_ratio(r_star, t, 0, 3)
        assert afr == pytest.approx(sc.actual_freeze_ratio(r_star, t, 0, 3), abs=1e-15)
        masks, frozen = tf.tf_select_row_blocks(shapes, br, afr, 1000 + t)
        ref_masks, ref_frozen = oracle.select_row_blocks(shapes, br, afr, 1000 + t)
        assert frozen == ref_frozen and all(np.array_equal(a, b) for a, b in zip(masks, ref_masks))
        for l in range(L):
            ever_unfrozen[l] |= masks[l] == 0
        X = [f32(rs.standard_normal((T, k))) for k, n in shapes]
        dY = [f32(rs.standard_normal((T, n)) * 1e-3) for k, n in shapes]
        # library: the fp32 master weights are the weights of this step
        gdX = [torch.empty((T, k), device="cuda") for k, n in shapes]
        tf.tf_stage_backward_blocks(ctx, shapes, T, tf.TF_F32, dp, [torch.from_numpy(a).cuda() for a in X],
                                    [torch.from_numpy(a).cuda() for a in dY], None, masks, br, gdX, dW, tf.TF_F32)
        tf.tf_row_blocks_to_bits(ctx, shapes, masks, br, bits)
        tmask = np.array([int(m.all()) for m in masks], dtype=np.uint8)
        tf.tf_masked_adamw(ctx, numel, dp, dm, dv, dW, tf.TF_F32, steps, hp["lr"], hp["beta1"], hp["beta2"], hp["eps"],
                           hp["weight_decay"], tensor_freeze_mask=tmask, elem_freeze_bits=bits)
        # oracle: the same chain in fp64
        oW = [a.reshape(s) for a, s in zip(op, shapes)]
        odX = [np.zeros((T, k)) for k, n in shapes]
        odW = [np.zeros(s) for s in shapes]
        oracle.stage_backward_blocks(shapes, T, oW, [np.asarray(a, np.float64) for a in X], [np.asarray(a, np.float64) for a in dY],
                                     None, masks, br, odX, odW)
        for l in range(L):
            if tmask[l]:
                continue
            em = oracle.row_blocks_to_elem_mask(shapes[l], br, masks[l])
            flat = op[l].reshape(-1)
            oracle.masked_adamw(flat, om[l], ov[l], odW[l].reshape(-1), step=steps[l], elem_frozen=em, **hp)
            steps[l] += 1
        torch.cuda.synchronize()
        for l in range(L):
            assert rel_fro(host64(gdX[l]), odX[l]) <= 1e-5, (t, l)
    for l, (k, n) in enumerate(shapes):
        assert rel_fro(host64(dp[l]), op[l].reshape(shapes[l])) <= 1e-5, l
        assert rel_fro(host64(dm[l]).ravel(), om[l]) <= 1e-5 and rel_fro(host64(dv[l]).ravel(), ov[l]) <= 1e-5, l
        never = np.repeat(~ever_unfrozen[l], br)
        if never.any():                                   # rows frozen in all four steps: not a bit of p moved
            assert np.array_equal(dp[l].cpu().numpy()[never], p0[l][never])
