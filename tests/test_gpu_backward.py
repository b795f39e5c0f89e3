"""GPU parity of tf_stage_backward against the fp64 oracle, through the C ABI.
Bounds: relative Frobenius error per output tensor <= 1e-5 (fp32) / 1e-2 (bf16);
frozen dW buffers bit-identical; dX independent of the mask (Sec. 3.2.1)."""
import numpy as np
import pytest
import torch

import oracle
import workloads as wl
import paper_2602_05754_amd as tf
from gpu_util import CODE, TDT, TOL, assert_elementwise, canary, dev, host64, raw_bytes, rel_fro

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx():
    c = tf.Context(0)
    yield c
    c.close()


def _inputs(cfg, T, microbatch=0):
    W, X, dY = [], [], []
    for l in range(cfg.n_layers):
        w, x, dy = wl.gen_layer(cfg, l, T=T, microbatch=microbatch)
        W.append(w); X.append(x); dY.append(dy)
    return W, X, dY


def _oracle_backward(cfg, T, W, X, dY, mask, dW0=None, accumulate=False):
    sh = cfg.shapes
    W64 = [w.astype(np.float64) for w in W]
    X64 = [x.astype(np.float64) for x in X]
    dY64 = [d.astype(np.float64) for d in dY]
    dX = [np.empty((T, k)) for k, n in sh]
    dW = [None if mask[l] else (np.zeros((k, n)) if dW0 is None else dW0[l]) for l, (k, n) in enumerate(sh)]
    oracle.stage_backward(sh, T, W64, X64, dY64, mask, dX, dW, accumulate=accumulate)
    return dX, dW


def _run_case(ctx, cfg, T, mask, tol):
    sh = cfg.shapes
    W, X, dY = _inputs(cfg, T)
    dXo, dWo = _oracle_backward(cfg, T, W, X, dY, mask)
    dW_t = TDT[cfg.dw_dtype]
    gW = [dev(w, cfg.dtype) for w in W]
    gX = [dev(x, cfg.dtype) for x in X]
    gdY = [dev(d, cfg.dtype) for d in dY]
    gdX = [canary((T, k), TDT[cfg.dtype]) for k, n in sh]
    gdW = [canary((k, n), dW_t) for k, n in sh]
    before = [raw_bytes(t) for t in gdW]
    tf.tf_stage_backward(ctx, sh, T, CODE[cfg.dtype], gW, gX, gdY, mask, gdX, gdW, CODE[cfg.dw_dtype])
    torch.cuda.synchronize()
    worst = 0.0
    for l in range(len(sh)):
        e = rel_fro(host64(gdX[l]), dXo[l]); worst = max(worst, e)
        assert e <= tol, f"dX[{l}] {sh[l]} rel_fro {e:.3e}"
        assert_elementwise(host64(gdX[l]), dXo[l], cfg.dtype, f"dX[{l}] {sh[l]}")
        if mask[l]:
            assert raw_bytes(gdW[l]) == before[l], f"frozen dW[{l}] was touched"
        else:
            e = rel_fro(host64(gdW[l]), dWo[l]); worst = max(worst, e)
            assert e <= tol, f"dW[{l}] {sh[l]} rel_fro {e:.3e}"
            assert_elementwise(host64(gdW[l]), dWo[l], cfg.dw_dtype, f"dW[{l}] {sh[l]}")
    return [raw_bytes(t) for t in gdX], worst


def test_cfg1_tiny_fp32_r_half(ctx):
    cfg = wl.CONFIGS[1]
    mask = wl.permutation_mask(cfg, 0.5)
    assert mask.sum() == 7
    dx_half, worst = _run_case(ctx, cfg, cfg.T, mask, TOL["f32"])
    # r = 0 is the full backward, r = 1 leaves every dW untouched; dX never depends on the mask
    dx0, _ = _run_case(ctx, cfg, cfg.T, np.zeros(14, np.uint8), TOL["f32"])
    dx1, _ = _run_case(ctx, cfg, cfg.T, np.ones(14, np.uint8), TOL["f32"])
    assert dx_half == dx0 == dx1
    print(f"cfg1 worst rel_fro {worst:.2e}")


@pytest.mark.parametrize("r", [0.0, 0.5, 1.0])
def test_bf16_matrix_core_path_several_tiles(ctx, r):
    # every dimension a multiple of 256: 2-3 tiles per side, contraction 4-12 steps of 64
    cfg = wl.scaled(wl.CONFIGS[2], blocks=1, d=512, kv=256, ffn=768, T=512)
    mask = wl.permutation_mask(cfg, r)
    _run_case(ctx, cfg, cfg.T, mask, TOL["bf16"])


def test_bf16_ragged_shapes_fall_to_the_generic_kernel(ctx):
    cfg = wl.scaled(wl.CONFIGS[2], blocks=1, d=264, kv=72, ffn=200, T=100)
    _run_case(ctx, cfg, cfg.T, wl.permutation_mask(cfg, 0.3), TOL["bf16"])
    cfg = wl.scaled(wl.CONFIGS[1], blocks=1, d=33, kv=8, ffn=65, T=7)      # fp32, smaller than one tile
    _run_case(ctx, cfg, cfg.T, wl.permutation_mask(cfg, 0.5), TOL["f32"])
    cfg = wl.scaled(wl.CONFIGS[1], blocks=1, d=8, kv=8, ffn=8, T=1)        # T = 1: outer products
    _run_case(ctx, cfg, cfg.T, np.zeros(7, np.uint8), TOL["f32"])


def test_mixed_eligible_and_ragged_layers_in_one_call(ctx):
    # ffn = 688 is not a multiple of 256: gate/up/down take the generic kernel, q/k/v/o the MFMA one
    cfg = wl.scaled(wl.CONFIGS[2], blocks=2, d=256, kv=256, ffn=688, T=256)
    _run_case(ctx, cfg, cfg.T, wl.permutation_mask(cfg, 0.5), TOL["bf16"])


@pytest.mark.parametrize("dims", [dict(d=256, kv=256, ffn=512, T=256), dict(d=136, kv=40, ffn=72, T=50)])
def test_fp32_accumulation_over_microbatches_with_per_microbatch_masks(ctx, dims):
    # sum_m U_m (.) g_m into fp32 accumulators (App. D.1 update rule); bf16 inputs
    cfg = wl.scaled(wl.CONFIGS[5], blocks=1, microbatches=3, **dims)
    sh = cfg.shapes; T = cfg.T; L = cfg.n_layers
    ratios = [0.2, 0.8, 0.4]
    acc_o = [np.zeros((k, n)) for k, n in sh]
    # device accumulators start at zero; a tensor frozen in every microbatch keeps a canary instead
    masks = [wl.permutation_mask(cfg, ratios[m], microbatch=m) for m in range(3)]
    always = np.minimum.reduce(masks)
    gacc = [canary((k, n), torch.float32) if always[l] else torch.zeros((k, n), device="cuda")
            for l, (k, n) in enumerate(sh)]
    before = [raw_bytes(t) for t in gacc]
    for m in range(3):
        W, X, dY = _inputs(cfg, T, microbatch=m)
        dXo, _ = _oracle_backward(cfg, T, W, X, dY, masks[m], dW0=acc_o, accumulate=True)
        gdX = [torch.empty((T, k), dtype=torch.bfloat16, device="cuda") for k, n in sh]
        tf.tf_stage_backward(ctx, sh, T, tf.TF_BF16, [dev(w, "bf16") for w in W], [dev(x, "bf16") for x in X],
                             [dev(d, "bf16") for d in dY], masks[m], gdX, gacc, tf.TF_F32, accumulate=True)
        torch.cuda.synchronize()
        for l in range(L):
            assert rel_fro(host64(gdX[l]), dXo[l]) <= TOL["bf16"]
            assert_elementwise(host64(gdX[l]), dXo[l], "bf16", f"dX[{l}] microbatch {m}")
    for l in range(L):
        if always[l]:
            assert raw_bytes(gacc[l]) == before[l]
        else:
            e = rel_fro(host64(gacc[l]), acc_o[l])
            assert e <= 1e-5 * 10, f"acc[{l}] rel_fro {e:.3e}"   # fp32 accumulation of bf16 products
            assert_elementwise(host64(gacc[l]), acc_o[l], "f32", f"acc[{l}]", scale=10.0)


@pytest.mark.parametrize("dims", [dict(d=256, kv=256, ffn=512, T=256), dict(d=512, kv=256, ffn=768, T=320),
                                  dict(d=136, kv=40, ffn=72, T=50)])
def test_microbatches_where_a_layers_first_product_overwrites_its_accumulator(ctx, dims):
    # The same sum over microbatches (App. D.1 update rule), with the choice between "=" and "+="
    # made layer by layer: a layer's first unfrozen microbatch of the step overwrites whatever its
    # accumulator holds (here: NaN canaries, which an addition would keep), later ones add.
    cfg = wl.scaled(wl.CONFIGS[5], blocks=1, microbatches=4, **dims)
    sh = cfg.shapes; T = cfg.T; L = cfg.n_layers
    ratios = [0.6, 0.2, 0.8, 0.4]
    masks = [wl.permutation_mask(cfg, ratios[m], microbatch=m) for m in range(4)]
    for mk in masks:
        mk[5] = 1                            # one layer stays frozen in every microbatch
    always = np.minimum.reduce(masks)
    assert always.sum() == 1 and (masks[0] & (1 - masks[1])).sum() >= 1     # ... and some layers start late
    acc_o = [np.zeros((k, n)) for k, n in sh]
    gacc = [canary((k, n), torch.float32) for k, n in sh]
    before = [raw_bytes(t) for t in gacc]
    seen = np.zeros(L, np.uint8)             # the layer has been unfrozen in an earlier microbatch
    for m in range(4):
        W, X, dY = _inputs(cfg, T, microbatch=m)
        dXo, _ = _oracle_backward(cfg, T, W, X, dY, masks[m], dW0=acc_o, accumulate=True)
        gdX = [torch.empty((T, k), dtype=torch.bfloat16, device="cuda") for k, n in sh]
        tf.tf_stage_backward_microbatch(ctx, sh, T, tf.TF_BF16, [dev(w, "bf16") for w in W], [dev(x, "bf16") for x in X],
                                        [dev(d, "bf16") for d in dY], masks[m], gdX, gacc, tf.TF_F32, seen.copy())
        torch.cuda.synchronize()
        seen |= (1 - masks[m]).astype(np.uint8)
        for l in range(L):
            assert rel_fro(host64(gdX[l]), dXo[l]) <= TOL["bf16"]
            assert_elementwise(host64(gdX[l]), dXo[l], "bf16", f"dX[{l}] microbatch {m}")
    for l in range(L):
        if always[l]:
            assert raw_bytes(gacc[l]) == before[l]
        else:
            e = rel_fro(host64(gacc[l]), acc_o[l])
            assert e <= 1e-5 * 10, f"acc[{l}] rel_fro {e:.3e}"
            assert_elementwise(host64(gacc[l]), acc_o[l], "f32", f"acc[{l}]", scale=10.0)


def test_microbatch_entry_point_with_nothing_to_add_equals_the_plain_backward(ctx):
    # all accumulate_mask entries 0: the same launches as tf_stage_backward(accumulate = 0), bf16 dW allowed
    cfg = wl.scaled(wl.CONFIGS[2], blocks=1, d=512, kv=256, ffn=768, T=512)
    sh, T, L = cfg.shapes, cfg.T, cfg.n_layers
    mask = wl.permutation_mask(cfg, 0.3)
    W, X, dY = _inputs(cfg, T)
    gW = [dev(w, "bf16") for w in W]; gX = [dev(x, "bf16") for x in X]; gdY = [dev(d, "bf16") for d in dY]
    out = []
    for entry in ("plain", "microbatch"):
        gdX = [canary((T, k), torch.bfloat16) for k, n in sh]
        gdW = [canary((k, n), torch.bfloat16) for k, n in sh]
        if entry == "plain":
            tf.tf_stage_backward(ctx, sh, T, tf.TF_BF16, gW, gX, gdY, mask, gdX, gdW, tf.TF_BF16)
        else:
            tf.tf_stage_backward_microbatch(ctx, sh, T, tf.TF_BF16, gW, gX, gdY, mask, gdX, gdW, tf.TF_BF16, np.zeros(L, np.uint8))
        torch.cuda.synchronize()
        out.append([raw_bytes(t) for t in gdX + gdW])
    assert out[0] == out[1]
    with pytest.raises(tf.TfError) as err:       # an unfrozen layer that adds needs fp32 accumulators
        tf.tf_stage_backward_microbatch(ctx, sh, T, tf.TF_BF16, gW, gX, gdY, mask, gdX, gdW, tf.TF_BF16, 1 - mask)
    assert err.value.code == -3


def test_degenerate_calls(ctx):
    tf.tf_stage_backward(ctx, [], 16, tf.TF_BF16, [], [], [], [], [], [], tf.TF_BF16)      # no layers
    # all frozen, X and dW absent altogether
    cfg = wl.scaled(wl.CONFIGS[2], blocks=1, d=256, kv=256, ffn=256, T=256)
    W, X, dY = _inputs(cfg, cfg.T)
    gdX = [torch.empty((cfg.T, k), dtype=torch.bfloat16, device="cuda") for k, n in cfg.shapes]
    tf.tf_stage_backward(ctx, cfg.shapes, cfg.T, tf.TF_BF16, [dev(w, "bf16") for w in W], None,
                         [dev(d, "bf16") for d in dY], np.ones(7, np.uint8), gdX, None, tf.TF_BF16)
    torch.cuda.synchronize()
    dXo, _ = _oracle_backward(cfg, cfg.T, W, X, dY, np.ones(7, np.uint8))
    for l in range(7):
        assert rel_fro(host64(gdX[l]), dXo[l]) <= TOL["bf16"]
        assert_elementwise(host64(gdX[l]), dXo[l], "bf16", f"dX[{l}]")
    # errors are reported, not raised as faults
    with pytest.raises(tf.TfError) as ei:
        tf.tf_stage_backward(ctx, cfg.shapes, 0, tf.TF_BF16, gdX, gdX, gdX, None, gdX, gdX, tf.TF_BF16)
    assert ei.value.code == -2
    with pytest.raises(ValueError):     # binding refuses a buffer smaller than the shape says
        tf.tf_stage_backward(ctx, [(512, 512)], 256, tf.TF_BF16, [gdX[0]], [gdX[0]], [gdX[0]], None,
                             [gdX[0]], [gdX[0]], tf.TF_BF16)
    with pytest.raises(tf.TfError) as ei:     # an output that is also an input is refused before anything runs
        tf.tf_stage_backward(ctx, [(256, 256)], 256, tf.TF_BF16, [gdX[0]], [gdX[1]], [gdX[2]], None,
                             [gdX[0]], [gdX[3]], tf.TF_BF16)
    assert ei.value.code == -8


def test_pointer_tables_give_the_same_bytes_as_lists(ctx):
    """The binding's pre-marshalled pointer tables are marshalling only: the same call through
    them writes the same bytes."""
    cfg = wl.scaled(wl.CONFIGS[2], blocks=1, d=512, kv=256, ffn=768, T=512)
    sh, T = cfg.shapes, cfg.T
    W, X, dY = _inputs(cfg, T)
    mask = wl.permutation_mask(cfg, 0.5)
    gW, gX, gdY = ([dev(a, cfg.dtype) for a in t] for t in (W, X, dY))
    out = []
    for wrap in (list, tf.PtrTable):
        gdX = [canary((T, k), torch.bfloat16) for k, n in sh]
        gdW = [canary((k, n), torch.bfloat16) for k, n in sh]
        tf.tf_stage_backward(ctx, sh, T, tf.TF_BF16, wrap(gW), wrap(gX), wrap(gdY), mask, wrap(gdX), wrap(gdW), tf.TF_BF16)
        torch.cuda.synchronize()
        out.append([raw_bytes(t) for t in gdX + gdW])
    assert out[0] == out[1]


def test_more_layers_than_one_grouped_launch_holds(ctx):
    """77 small layers on the matrix cores: 64 problem descriptors per launch, so both halves of
    the backward take a second launch (the weight-gradient half because 70 layers stay
    unfrozen); several contraction lengths so that the cost order differs from the layer order."""
    cfg = wl.scaled(wl.CONFIGS[2], blocks=11, d=256, kv=512, ffn=768, T=256)
    mask = np.zeros(cfg.n_layers, np.uint8)
    mask[[0, 9, 30, 31, 64, 65, 76]] = 1
    _run_case(ctx, cfg, cfg.T, mask, TOL["bf16"])
