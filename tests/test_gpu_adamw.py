"""GPU parity of tf_masked_adamw / tf_stability_update against the fp64 oracle.
Bounds: p, m, v, E, A within relative Frobenius 1e-5 per tensor; bf16 copy
within 1e-2; every frozen element / tensor bit-identical in every buffer;
tensor selection from the scores identical (App. D.1; Sec. 2.3)."""
import numpy as np
import pytest
import torch

import oracle
import workloads as wl
import paper_2602_05754_amd as tf
from gpu_util import canary, dev, host64, raw_bytes, rel_fro

pytestmark = pytest.mark.gpu

# hyper-parameters as the binary32 values the library receives
HP = {k: float(np.float32(v)) for k, v in dict(lr=1e-4, beta1=0.9, beta2=0.95, eps=1e-8, weight_decay=0.1).items()}
DECAY = float(np.float32(0.99))


@pytest.fixture(scope="module")
def ctx():
    c = tf.Context(0)
    yield c
    c.close()


class State:
    """One tensor's host (fp64, oracle) and device (fp32) state, same starting bytes."""

    def __init__(self, rs, n, zero_state, grad_dtype):
        f32 = lambda a: np.ascontiguousarray(a, dtype=np.float32)
        self.n = n
        self.p0 = f32(rs.standard_normal(n) * 0.02)
        z = np.zeros(n, np.float32)
        self.m0 = z.copy() if zero_state else f32(rs.standard_normal(n) * 3e-4)
        self.v0 = z.copy() if zero_state else f32(np.square(rs.standard_normal(n) * 1e-3))
        self.E0 = z.copy() if zero_state else f32(rs.standard_normal(n) * 1e-5)
        self.A0 = z.copy() if zero_state else f32(np.abs(rs.standard_normal(n)) * 1e-4 + np.abs(self.E0))
        self.low0 = wl.round_to_bf16(self.p0)
        self.grad_dtype = grad_dtype
        self.h = {k: getattr(self, k + "0").astype(np.float64) for k in ("p", "m", "v", "E", "A", "low")}
        self.d = {k: dev(getattr(self, k + "0"), "bf16" if k == "low" else "f32") for k in ("p", "m", "v", "E", "A", "low")}

    def grad(self, rs):
        g = np.ascontiguousarray(rs.standard_normal(self.n) * 1e-3, dtype=np.float32)
        if self.grad_dtype == "bf16":
            g = wl.round_to_bf16(g)
        return g


def _check(states, frozen_elem, tensor_mask, before_bytes, label=""):
    for i, s in enumerate(states):
        for k in ("p", "m", "v", "E", "A", "low"):
            got = host64(s.d[k]); ref = s.h[k]
            if tensor_mask is not None and tensor_mask[i]:
                assert raw_bytes(s.d[k]) == before_bytes[i][k], f"{label} frozen tensor {i} buffer {k} changed"
                continue
            e = rel_fro(got, ref)
            assert e <= (1e-2 if k == "low" else 1e-5), f"{label} tensor {i} {k}: rel_fro {e:.3e}"
            if frozen_elem is not None and frozen_elem[i] is not None:
                f = frozen_elem[i].astype(bool)
                b = np.frombuffer(before_bytes[i][k], dtype=np.uint16 if k == "low" else np.uint32)
                a = np.frombuffer(raw_bytes(s.d[k]), dtype=b.dtype)
                assert np.array_equal(a[f], b[f]), f"{label} frozen elements of tensor {i} buffer {k} changed"
                if k != "low" and (~f).sum() > 100:
                    assert np.mean(a[~f] != b[~f]) > 0.99       # the others did move


@pytest.mark.parametrize("grad_dtype", ["bf16", "f32"])
def test_masked_adamw_with_element_and_tensor_masks(ctx, grad_dtype):
    rs = np.random.default_rng(11)
    sizes = [8192 * 3 + 5, 7, 1_000_003, 4096, 64, 300_000]     # ragged tails, tiny, several blocks
    states = [State(rs, n, zero_state=(i % 2 == 0), grad_dtype=grad_dtype) for i, n in enumerate(sizes)]
    tensor_mask = np.array([0, 0, 0, 1, 0, 1], np.uint8)
    elem = [(rs.random(n) < 0.4).astype(np.uint8) if i in (0, 1, 2) else None for i, n in enumerate(sizes)]
    elem[4] = np.ones(64, np.uint8)                               # every element frozen, tensor not
    bits = [None if e is None else torch.from_numpy(wl.pack_mask_bits(e).view(np.int32)).cuda() for e in elem]
    sums = torch.full((2 * len(sizes),), -7.0, dtype=torch.float64, device="cuda")
    steps = [1, 3, 2, 5, 1, 1]
    for rep in range(2):                                          # two consecutive steps on the same state
        grads = [s.grad(rs) for s in states]
        gdev = [dev(g, grad_dtype) for g in grads]
        before = [{k: raw_bytes(s.d[k]) for k in s.d} for s in states]
        for i, s in enumerate(states):
            if tensor_mask[i]:
                continue
            oracle.masked_adamw(s.h["p"], s.h["m"], s.h["v"], grads[i].astype(np.float64), step=steps[i] + rep,
                                grad_scale=0.125, p_lowp=s.h["low"], elem_frozen=elem[i],
                                ema=s.h["E"], ema_abs=s.h["A"], ema_decay=DECAY, **HP)
        tf.tf_masked_adamw(ctx, sizes, [s.d["p"] for s in states], [s.d["m"] for s in states],
                           [s.d["v"] for s in states], gdev, tf.TF_BF16 if grad_dtype == "bf16" else tf.TF_F32,
                           [t + rep for t in steps], HP["lr"], HP["beta1"], HP["beta2"], HP["eps"],
                           HP["weight_decay"], grad_scale=0.125, p_lowp=[s.d["low"] for s in states],
                           tensor_freeze_mask=tensor_mask, elem_freeze_bits=bits,
                           ema=[s.d["E"] for s in states], ema_abs=[s.d["A"] for s in states],
                           ema_decay=DECAY, score_sums=sums)
        torch.cuda.synchronize()
        _check(states, elem, tensor_mask, before, label=f"step {rep}")
        got = sums.cpu().numpy().reshape(-1, 2)
        for i, s in enumerate(states):
            if tensor_mask[i]:
                assert got[i].tolist() == [-7.0, -7.0]            # frozen tensor: sums left alone
            else:
                se, sa = oracle.score_sums(s.h["E"], s.h["A"])
                assert abs(got[i, 0] - se) <= 1e-5 * max(se, 1e-30) and abs(got[i, 1] - sa) <= 1e-5 * max(sa, 1e-30)


def test_adamw_without_optional_buffers_and_first_step_closed_form(ctx):
    rs = np.random.default_rng(12)
    n = 50_000
    s = State(rs, n, zero_state=True, grad_dtype="bf16")
    g = s.grad(rs)
    tf.tf_masked_adamw(ctx, [n], [s.d["p"]], [s.d["m"]], [s.d["v"]], [dev(g, "bf16")], tf.TF_BF16, [1],
                       HP["lr"], HP["beta1"], HP["beta2"], HP["eps"], HP["weight_decay"])
    torch.cuda.synchronize()
    g64 = g.astype(np.float64)
    exp = s.p0.astype(np.float64) * (1 - HP["lr"] * HP["weight_decay"]) - HP["lr"] * g64 / (np.abs(g64) + HP["eps"])
    assert rel_fro(host64(s.d["p"]), exp) <= 1e-5
    assert raw_bytes(s.d["E"]) == s.E0.tobytes() and raw_bytes(s.d["low"]) == wl.f32_to_bf16_bits(s.low0).tobytes()
    tf.tf_masked_adamw(ctx, [], [], [], [], [], tf.TF_BF16, [], 1e-4, 0.9, 0.95, 1e-8, 0.1)   # no tensors: no-op


def test_all_frozen_leaves_every_byte(ctx):
    rs = np.random.default_rng(13)
    sizes = [10_000, 4099]
    states = [State(rs, n, zero_state=False, grad_dtype="bf16") for n in sizes]
    before = [{k: raw_bytes(s.d[k]) for k in s.d} for s in states]
    gd = [dev(s.grad(rs), "bf16") for s in states]
    args = lambda **kw: tf.tf_masked_adamw(ctx, sizes, [s.d["p"] for s in states], [s.d["m"] for s in states],
                                           [s.d["v"] for s in states], gd, tf.TF_BF16, [2, 2], HP["lr"], HP["beta1"],
                                           HP["beta2"], HP["eps"], HP["weight_decay"],
                                           p_lowp=[s.d["low"] for s in states], ema=[s.d["E"] for s in states],
                                           ema_abs=[s.d["A"] for s in states], ema_decay=DECAY, **kw)
    args(tensor_freeze_mask=[1, 1])
    ones = [torch.full(((n + 31) // 32,), -1, dtype=torch.int32, device="cuda") for n in sizes]
    args(elem_freeze_bits=ones)
    torch.cuda.synchronize()
    for i, s in enumerate(states):
        for k in s.d:
            assert raw_bytes(s.d[k]) == before[i][k]


def test_standalone_stability_update(ctx):
    rs = np.random.default_rng(14)
    sizes = [123_457, 8, 40_000]
    E0 = [np.ascontiguousarray(rs.standard_normal(n) * 1e-5, np.float32) for n in sizes]
    A0 = [np.ascontiguousarray(np.abs(rs.standard_normal(n)) * 1e-4, np.float32) for n in sizes]
    D = [np.ascontiguousarray(rs.standard_normal(n) * 1e-4, np.float32) for n in sizes]
    elem = [(rs.random(sizes[0]) < 0.5).astype(np.uint8), None, None]
    tmask = [0, 0, 1]
    Eh = [a.astype(np.float64) for a in E0]; Ah = [a.astype(np.float64) for a in A0]
    Ed = [dev(a, "f32") for a in E0]; Ad = [dev(a, "f32") for a in A0]
    sums = torch.zeros(6, dtype=torch.float64, device="cuda")
    for i in range(2):
        oracle.stability_update(D[i].astype(np.float64), Eh[i], Ah[i], DECAY, elem_frozen=elem[i])
    bits = [torch.from_numpy(wl.pack_mask_bits(elem[0]).view(np.int32)).cuda(), None, None]
    tf.tf_stability_update(ctx, sizes, [dev(d, "f32") for d in D], Ed, Ad, DECAY, tensor_freeze_mask=tmask,
                           elem_freeze_bits=bits, score_sums=sums)
    torch.cuda.synchronize()
    for i in range(2):
        assert rel_fro(host64(Ed[i]), Eh[i]) <= 1e-5 and rel_fro(host64(Ad[i]), Ah[i]) <= 1e-5
    f = elem[0].astype(bool)
    assert np.array_equal(Ed[0].cpu().numpy()[f], E0[0][f]) and np.array_equal(Ad[0].cpu().numpy()[f], A0[0][f])
    assert raw_bytes(Ed[2]) == E0[2].tobytes() and raw_bytes(Ad[2]) == A0[2].tobytes()
    got = sums.cpu().numpy().reshape(3, 2)
    for i in range(2):
        se, sa = oracle.score_sums(Eh[i], Ah[i])
        assert np.isclose(got[i, 0], se, rtol=1e-5) and np.isclose(got[i, 1], sa, rtol=1e-5)
    sc = tf.tf_stability_scores(got[:2])
    assert np.all(sc >= 0) and np.all(sc <= 1)


def test_warmup_then_lowest_score_selection_matches_the_oracle(ctx):
    # 5 seeded warm-up steps (nothing frozen), then freeze the ceil(r L) lowest-score tensors
    cfg = wl.scaled(wl.CONFIGS[2], blocks=2, d=128, kv=32, ffn=512)
    L = cfg.n_layers; sh = cfg.shapes
    sizes = [k * n for k, n in sh]
    hp = {k: float(np.float32(getattr(cfg, k))) for k in ("lr", "beta1", "beta2", "eps", "weight_decay")}
    P = [wl.gen_weight(cfg, l).reshape(-1) for l in range(L)]
    h = [{k: (P[l].astype(np.float64) if k == "p" else np.zeros(sizes[l])) for k in "pmvEA"} for l in range(L)]
    d = [{k: (dev(P[l], "f32") if k == "p" else torch.zeros(sizes[l], device="cuda")) for k in "pmvEA"} for l in range(L)]
    sums = torch.zeros(2 * L, dtype=torch.float64, device="cuda")
    for step in range(1, 6):
        # per-tensor gradient scale differs so that tensors do not all look alike
        grads = [wl.gen_grad(cfg, l, step) for l in range(L)]
        for l in range(L):
            oracle.masked_adamw(h[l]["p"], h[l]["m"], h[l]["v"], grads[l].astype(np.float64), step=step,
                                ema=h[l]["E"], ema_abs=h[l]["A"], ema_decay=DECAY, **hp)
        tf.tf_masked_adamw(ctx, sizes, [x["p"] for x in d], [x["m"] for x in d], [x["v"] for x in d],
                           [dev(g, "bf16") for g in grads], tf.TF_BF16, [step] * L, hp["lr"], hp["beta1"],
                           hp["beta2"], hp["eps"], hp["weight_decay"], ema=[x["E"] for x in d],
                           ema_abs=[x["A"] for x in d], ema_decay=DECAY, score_sums=sums)
    torch.cuda.synchronize()
    got = tf.tf_stability_scores(sums.cpu().numpy())
    ref = np.array([oracle.tensor_score(*oracle.score_sums(h[l]["E"], h[l]["A"])) for l in range(L)])
    err = np.max(np.abs(got - ref))
    for r in (0.0, 0.25, 0.5, 0.75, 0.9, 1.0):
        n = oracle.n_frozen(r, L)
        assert tf.tf_num_frozen(r, L) == n
        ref_mask = oracle.select_lowest(ref, n)
        srt = np.sort(ref)
        gap = srt[n] - srt[n - 1] if 0 < n < L else np.inf
        assert gap > 100 * err, "selection boundary too tight for this seed"
        assert np.array_equal(tf.tf_select_lowest(got, n), ref_mask)


def test_more_tensors_than_one_launch_holds(ctx):
    """80 tensors, 11 of them frozen: the unfrozen 69 take three launches of at most 32
    descriptors, each of which clears and accumulates its own tensors' sums; two steps in a
    row on the same state (App. D.1; Sec. 2.3)."""
    rs = np.random.default_rng(15)
    n_t = 80
    sizes = [int(x) for x in rs.integers(1, 9000, n_t)]
    sizes[5], sizes[40], sizes[70] = 16384 * 2 + 3, 4096 * 4, 1            # several blocks, exact blocks, one element
    states = [State(rs, n, zero_state=(i % 3 == 0), grad_dtype="bf16") for i, n in enumerate(sizes)]
    tensor_mask = np.zeros(n_t, np.uint8)
    tensor_mask[[0, 7, 31, 32, 33, 50, 63, 64, 65, 78, 79]] = 1
    elem = [(rs.random(n) < 0.5).astype(np.uint8) if i % 4 == 1 else None for i, n in enumerate(sizes)]
    bits = [None if e is None else torch.from_numpy(wl.pack_mask_bits(e).view(np.int32)).cuda() for e in elem]
    sums = torch.full((2 * n_t,), -7.0, dtype=torch.float64, device="cuda")
    steps = [int(x) for x in rs.integers(1, 6, n_t)]
    for rep in range(2):
        grads = [s.grad(rs) for s in states]
        before = [{k: raw_bytes(s.d[k]) for k in s.d} for s in states]
        for i, s in enumerate(states):
            if not tensor_mask[i]:
                oracle.masked_adamw(s.h["p"], s.h["m"], s.h["v"], grads[i].astype(np.float64), step=steps[i] + rep,
                                    p_lowp=s.h["low"], elem_frozen=elem[i], ema=s.h["E"], ema_abs=s.h["A"],
                                    ema_decay=DECAY, **HP)
        tf.tf_masked_adamw(ctx, sizes, [s.d["p"] for s in states], [s.d["m"] for s in states],
                           [s.d["v"] for s in states], [dev(g, "bf16") for g in grads], tf.TF_BF16,
                           [t + rep for t in steps], HP["lr"], HP["beta1"], HP["beta2"], HP["eps"], HP["weight_decay"],
                           p_lowp=[s.d["low"] for s in states], tensor_freeze_mask=tensor_mask, elem_freeze_bits=bits,
                           ema=[s.d["E"] for s in states], ema_abs=[s.d["A"] for s in states], ema_decay=DECAY,
                           score_sums=sums)
        torch.cuda.synchronize()
        _check(states, elem, tensor_mask, before, label=f"step {rep}")
        got = sums.cpu().numpy().reshape(-1, 2)
        for i, s in enumerate(states):
            if tensor_mask[i]:
                assert got[i].tolist() == [-7.0, -7.0], i
            else:
                se, sa = oracle.score_sums(s.h["E"], s.h["A"])
                assert np.isclose(got[i, 0], se, rtol=1e-5, atol=1e-30) and np.isclose(got[i, 1], sa, rtol=1e-5, atol=1e-30), i


def test_standalone_stability_update_with_more_tensors_than_one_launch_holds(ctx):
    rs = np.random.default_rng(16)
    n_t = 75
    sizes = [int(x) for x in rs.integers(1, 6000, n_t)]
    sizes[10] = 16384 + 5
    f32 = lambda a: np.ascontiguousarray(a, np.float32)
    E0 = [f32(rs.standard_normal(n) * 1e-5) for n in sizes]
    A0 = [f32(np.abs(rs.standard_normal(n)) * 1e-4) for n in sizes]
    D = [f32(rs.standard_normal(n) * 1e-4) for n in sizes]
    tmask = np.zeros(n_t, np.uint8); tmask[[3, 31, 32, 64, 74]] = 1
    elem = [(rs.random(n) < 0.3).astype(np.uint8) if i % 5 == 2 else None for i, n in enumerate(sizes)]
    bits = [None if e is None else torch.from_numpy(wl.pack_mask_bits(e).view(np.int32)).cuda() for e in elem]
    Eh = [a.astype(np.float64) for a in E0]; Ah = [a.astype(np.float64) for a in A0]
    Ed = [dev(a, "f32") for a in E0]; Ad = [dev(a, "f32") for a in A0]
    sums = torch.full((2 * n_t,), -3.0, dtype=torch.float64, device="cuda")
    tf.tf_stability_update(ctx, sizes, [dev(d, "f32") for d in D], Ed, Ad, DECAY, tensor_freeze_mask=tmask,
                           elem_freeze_bits=bits, score_sums=sums)
    torch.cuda.synchronize()
    got = sums.cpu().numpy().reshape(n_t, 2)
    for i in range(n_t):
        if tmask[i]:
            assert raw_bytes(Ed[i]) == E0[i].tobytes() and raw_bytes(Ad[i]) == A0[i].tobytes(), i
            assert got[i].tolist() == [-3.0, -3.0], i
            continue
        oracle.stability_update(D[i].astype(np.float64), Eh[i], Ah[i], DECAY, elem_frozen=elem[i])
        assert rel_fro(host64(Ed[i]), Eh[i]) <= 1e-5 and rel_fro(host64(Ad[i]), Ah[i]) <= 1e-5, i
        if elem[i] is not None:
            f = elem[i].astype(bool)
            assert np.array_equal(Ed[i].cpu().numpy()[f], E0[i][f]) and np.array_equal(Ad[i].cpu().numpy()[f], A0[i][f]), i
        se, sa = oracle.score_sums(Eh[i], Ah[i])
        assert np.isclose(got[i, 0], se, rtol=1e-5, atol=1e-30) and np.isclose(got[i, 1], sa, rtol=1e-5, atol=1e-30), i


def test_frozen_bf16_copies_under_the_rounded_master_promise(ctx):
    """With tf_assume_lowp_is_rounded_master the stored bf16 copy of a frozen element in a partly
    frozen mask word is not read again but rounded from the unchanged master weight: the same bits
    whenever the copy was the rounding of p, as here (two steps, the second on copies the first wrote)."""
    rs = np.random.default_rng(19)
    sizes = [32 * 1000 + 17, 4096, 70_001]
    states = [State(rs, n, zero_state=False, grad_dtype="bf16") for n in sizes]
    elem = [(rs.random(n) < 0.6).astype(np.uint8) for n in sizes]
    elem[1][:2048] = 1                                             # 64 wholly frozen words
    bits = [torch.from_numpy(wl.pack_mask_bits(e).view(np.int32)).cuda() for e in elem]
    ctx.assume_lowp_is_rounded_master(True)
    try:
        for rep in range(2):
            grads = [s.grad(rs) for s in states]
            before = [{k: raw_bytes(s.d[k]) for k in s.d} for s in states]
            for i, s in enumerate(states):
                oracle.masked_adamw(s.h["p"], s.h["m"], s.h["v"], grads[i].astype(np.float64), step=1 + rep,
                                    p_lowp=s.h["low"], elem_frozen=elem[i], ema=s.h["E"], ema_abs=s.h["A"],
                                    ema_decay=DECAY, **HP)
            tf.tf_masked_adamw(ctx, sizes, [s.d["p"] for s in states], [s.d["m"] for s in states],
                               [s.d["v"] for s in states], [dev(g, "bf16") for g in grads], tf.TF_BF16, [1 + rep] * 3,
                               HP["lr"], HP["beta1"], HP["beta2"], HP["eps"], HP["weight_decay"],
                               p_lowp=[s.d["low"] for s in states], elem_freeze_bits=bits,
                               ema=[s.d["E"] for s in states], ema_abs=[s.d["A"] for s in states], ema_decay=DECAY)
            torch.cuda.synchronize()
            _check(states, elem, None, before, label=f"promise, step {rep}")
    finally:
        ctx.assume_lowp_is_rounded_master(False)
