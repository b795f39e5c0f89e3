"""tf_reconcile_mask_static, the entry point that allocates nothing (its rank-search state is a
static device array), against tf_reconcile_mask on the same inputs, through the C ABI: masks
and statistics bit for bit (Alg. 2: integer work), on two calls in a row, the second with a
smaller input, so that whatever the first call left in the shared array must not matter; the
existing entry point's result is itself checked against the oracle."""
import numpy as np
import pytest
import torch

import oracle
import workloads as wl
import paper_2602_05754_amd as tf

pytestmark = pytest.mark.gpu


def _device_words(base):
    return [torch.from_numpy(wl.pack_mask_bits(b).view(np.int32)).cuda() for b in base]


def test_static_scratch_entry_point_matches_the_allocating_one():
    ctx = tf.Context(0)
    try:
        rs = np.random.default_rng(2024)
        # first call: 40 tensors (two launches per pass), additions; second: 3 small tensors, removals
        cases = [([int(n) for n in rs.integers(1, 90000, size=40)], 0.3, 0.6, 0xABCDEF),
                 ([1000, 33, 70001], 0.7, 0.2, 17)]
        for numel, density, r, seed in cases:
            base = [(rs.random(n) < density).astype(np.uint8) for n in numel]
            nf = int(r * sum(numel))
            out = {}
            for name, fn in (("alloc", tf.tf_reconcile_mask), ("static", tf.tf_reconcile_mask_static)):
                words = _device_words(base)
                stats = torch.full((3,), -1, dtype=torch.int64, device="cuda")
                fn(ctx, numel, words, nf, seed, stats=stats)
                torch.cuda.synchronize()
                out[name] = ([w.cpu().numpy().view("<u4") for w in words], stats.cpu().numpy())
            for a, b in zip(out["alloc"][0], out["static"][0]):
                assert np.array_equal(a, b)
            assert np.array_equal(out["alloc"][1], out["static"][1])
            ref, count = oracle.reconcile_mask(base, numel, nf, seed)
            got = [oracle.unpack_bits(w, n) for w, n in zip(out["static"][0], numel)]
            assert all(np.array_equal(g, e) for g, e in zip(got, ref)) and out["static"][1][0] == count
            assert sum(int(g.sum()) for g in got) == nf
        # the limit: 2^32 elements or more are refused before anything is launched
        with pytest.raises(tf.TfError) as e:
            tf.tf_reconcile_mask_static(ctx, [1 << 31, 1 << 31], [4096, 4096], 0, 1)
        assert e.value.code == -2
    finally:
        ctx.close()
