"""GPU parity of the matrix-core GEMM on extents that are not multiples of its 256 x 256 tile
(Sec. 3.2.1: both halves of the backward): the last tile of a problem computes a whole window
that overlaps its neighbour, or the rows around a sub-tensor problem, and stores only its own
part.  Every output element against the oracle (one bf16 rounding of an fp32 sum), rows of frozen
blocks bit-identical, and the kernel kinds that ran are checked so that a silent fall to the
fp32-FMA kernel would fail the test."""
import numpy as np
import pytest
import torch

import oracle
import workloads as wl
import paper_2602_05754_amd as tf
from gpu_util import assert_elementwise, canary, dev, host64, raw_bytes

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx():
    c = tf.Context(0)
    yield c
    c.close()


def _inputs(rs, shapes, T):
    f32 = lambda a: np.ascontiguousarray(a, dtype=np.float32)
    W = [wl.round_to_bf16(f32(rs.standard_normal(s) * 0.02)) for s in shapes]
    X = [wl.round_to_bf16(f32(rs.standard_normal((T, k)))) for k, n in shapes]
    dY = [wl.round_to_bf16(f32(rs.standard_normal((T, n)) * 1e-3)) for k, n in shapes]
    return W, X, dY


def _kinds(ctx, fn):
    ctx.profile_enable(True)
    ctx.profile_collect()
    fn()
    torch.cuda.synchronize()
    kinds = [k for k, _ in ctx.profile_collect()]
    ctx.profile_enable(False)
    return kinds


def _case(ctx, shapes, T, seed, row_masks=None, block_rows=0, dw="bf16", calls=1, expect=None):
    rs = np.random.default_rng(seed)
    L = len(shapes)
    f64 = lambda t: [np.asarray(a, dtype=np.float64) for a in t]
    ref_dW = [np.zeros(s) for s in shapes]
    acc = dw == "f32"
    gdW = [torch.zeros(s, device="cuda") if acc else canary(s, torch.bfloat16) for s in shapes]
    if acc and row_masks is not None:
        for l in range(L):                                          # frozen rows of an accumulator keep a canary
            for b, f in enumerate(row_masks[l] if row_masks[l] is not None else []):
                if f:
                    gdW[l][b * block_rows:(b + 1) * block_rows] = canary((block_rows, shapes[l][1]), torch.float32)
    before = [t.clone() for t in gdW]
    kinds = []
    for c in range(calls):
        W, X, dY = _inputs(rs, shapes, T)
        ref_dX = [np.zeros((T, k)) for k, n in shapes]
        one = [np.zeros(s) for s in shapes]
        if row_masks is None:
            oracle.stage_backward(shapes, T, f64(W), f64(X), f64(dY), np.zeros(L, np.uint8), ref_dX, one)
        else:
            oracle.stage_backward_blocks(shapes, T, f64(W), f64(X), f64(dY), None, row_masks, block_rows, ref_dX, one)
        for l in range(L):
            ref_dW[l] += one[l]
        gdX = [canary((T, k), torch.bfloat16) for k, n in shapes]
        gW, gX, gdY = ([dev(a, "bf16") for a in t] for t in (W, X, dY))
        kinds += _kinds(ctx, lambda: tf.tf_stage_backward_blocks(
            ctx, shapes, T, tf.TF_BF16, gW, gX, gdY, None, row_masks, block_rows if row_masks is not None else 0,
            gdX, gdW, tf.TF_F32 if acc else tf.TF_BF16, accumulate=acc))
        for l in range(L):
            assert_elementwise(host64(gdX[l]), ref_dX[l], "bf16", f"dX[{l}] {shapes[l]} T={T} call {c}")
    for l, (k, n) in enumerate(shapes):
        rm = row_masks[l] if row_masks is not None and row_masks[l] is not None else None
        keep = np.zeros(k, bool) if rm is None else np.repeat(np.asarray(rm, bool), block_rows)
        got = host64(gdW[l])
        assert_elementwise(got[~keep], ref_dW[l][~keep], dw, f"dW[{l}] {shapes[l]} T={T}", scale=10.0)
        if keep.any():
            kk = torch.from_numpy(keep).cuda()
            assert raw_bytes(gdW[l][kk]) == raw_bytes(before[l][kk]), f"frozen rows of dW[{l}] were touched"
    if expect is not None:
        assert set(kinds) == set(expect), kinds
    return kinds


def test_token_counts_that_are_no_multiple_of_the_tile(ctx):
    shapes = [(512, 256), (256, 768), (1024, 512)]
    # 960 tokens = 3 tiles and 192 rows, 15 contraction steps for the weight gradients: all on the matrix cores
    _case(ctx, shapes, 960, seed=1, expect={"dx_mfma", "dw_mfma"})
    # 1000 tokens: input gradients on the matrix cores (their contraction is N_l); the weight
    # gradients' contraction, 1000, is no multiple of 64 and takes the fp32-FMA kernel
    _case(ctx, shapes, 1000, seed=2, expect={"dx_mfma", "dw_generic"})
    # 264 tokens: one whole tile and a window of 8 new rows
    _case(ctx, shapes, 264, seed=3, expect={"dx_mfma", "dw_generic"})


def test_feature_counts_that_are_no_multiple_of_the_tile(ctx):
    # K = 328 / 520 / 688 and N = 328 / 264: last windows of 72, 8, 176 rows or columns
    shapes = [(328, 256), (520, 328), (256, 264), (688, 512)]
    k = _case(ctx, shapes, 256, seed=4)
    # dX of layer 0 contracts over N = 256 and has 328 columns: matrix cores; layer 1 contracts over 328: generic
    assert "dx_mfma" in k and "dx_generic" in k and "dw_mfma" in k and "dw_generic" not in k


@pytest.mark.parametrize("block_rows", [128, 64])
def test_row_blocks_smaller_than_a_tile_stay_on_the_matrix_cores(ctx, block_rows):
    shapes = [(1024, 512), (384, 256), (256, 256), (768, 512)]
    rs = np.random.default_rng(block_rows)
    masks = [(rs.random(k // block_rows) < 0.45).astype(np.uint8) for k, n in shapes]
    per = 128 // block_rows
    masks[1] = np.repeat(np.array([0, 1, 1], np.uint8), per)       # one run of 128 rows at the start of the tensor
    masks[2] = np.repeat(np.array([1, 0], np.uint8), per)          # ... and one at its end
    k = _case(ctx, shapes, 192, seed=5, row_masks=masks, block_rows=block_rows, expect={"dx_generic", "dw_mfma"})
    assert k.count("dw_mfma") >= 1


def test_fp32_accumulation_on_partial_tiles(ctx):
    shapes = [(328, 264), (640, 256), (256, 520)]
    masks = [None, np.array([0, 1, 0, 0, 1], np.uint8), np.array([0, 1], np.uint8)]
    _case(ctx, shapes, 128, seed=6, row_masks=masks, block_rows=128, dw="f32", calls=3)
