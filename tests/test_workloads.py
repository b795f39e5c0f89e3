"""Input generators: shapes of the paper's LLaMA workloads (Table exp_setup),
bf16 storage format, mask draws."""
import numpy as np
import torch

import workloads as wl


def test_stage_shapes_and_parameter_counts():
    assert wl.CONFIGS[1].n_params == 1_581_056 and wl.CONFIGS[1].n_layers == 14
    assert wl.CONFIGS[2].n_params == 243_269_632 and wl.CONFIGS[2].n_layers == 28
    assert wl.CONFIGS[3].n_params == 1_744_830_464 and wl.CONFIGS[3].n_layers == 56
    assert wl.CONFIGS[3].block_shapes == [(4096, 4096), (4096, 1024), (4096, 1024), (4096, 4096),
                                          (4096, 14336), (4096, 14336), (14336, 4096)]
    assert (wl.CONFIGS[1].T, wl.CONFIGS[2].T, wl.CONFIGS[3].T, wl.CONFIGS[5].T) == (256, 8192, 4096, 1024)


def test_bf16_format_matches_torch():
    rs = np.random.default_rng(0)
    x = (rs.standard_normal(10000) * np.exp(rs.uniform(-30, 30, 10000))).astype(np.float32)
    x[:4] = [0.0, -0.0, np.inf, -np.inf]
    bits = wl.f32_to_bf16_bits(x)
    t = torch.from_numpy(x).to(torch.bfloat16)
    assert np.array_equal(bits, t.view(torch.int16).numpy().view(np.uint16))
    assert np.array_equal(wl.bf16_bits_to_f32(bits), t.to(torch.float32).numpy())
    assert np.isnan(wl.bf16_bits_to_f32(wl.f32_to_bf16_bits(np.array([np.nan], np.float32))))[0]


def test_generators_are_seeded_and_have_the_stated_distribution():
    cfg = wl.scaled(wl.CONFIGS[2], d=256, kv=64, ffn=512, blocks=1)
    W, X, dY = wl.gen_layer(cfg, 4, T=512)
    W2, X2, dY2 = wl.gen_layer(cfg, 4, T=512)
    assert W.tobytes() == W2.tobytes() and X.tobytes() == X2.tobytes() and dY.tobytes() == dY2.tobytes()
    assert W.shape == (256, 512) and X.shape == (512, 256) and dY.shape == (512, 512)
    assert abs(W.std() - 0.02) < 1e-3 and abs(X.std() - 1) < 2e-2 and abs(dY.std() - 1e-3) < 5e-5
    assert np.array_equal(W, wl.round_to_bf16(W))        # representable in bf16
    _, X3, _ = wl.gen_layer(cfg, 4, T=512, microbatch=1)
    assert not np.array_equal(X, X3)


def test_masks():
    cfg = wl.CONFIGS[1]
    m = wl.permutation_mask(cfg, 0.5)
    assert m.dtype == np.uint8 and m.sum() == 7 and m.size == 14
    assert wl.permutation_mask(cfg, 0.0).sum() == 0 and wl.permutation_mask(cfg, 1.0).sum() == 14
    # nested in r for one permutation
    assert np.all(wl.permutation_mask(cfg, 0.75) >= m)
    e = wl.bernoulli_elem_mask(wl.CONFIGS[4], 0, 200000, 0.3)
    assert abs(e.mean() - 0.3) < 5e-3
    # mean of a masked gradient under independent masks is p (.) g  (Lemma "mean_masked", App. D)
    g = np.random.default_rng(1).standard_normal(200000)
    assert abs(np.mean((1 - e) * g) - 0.7 * g.mean()) < 1e-2
    words = wl.pack_mask_bits(e[:1000 + 7])
    assert words.dtype == np.uint32 and words.size == (1007 + 31) // 32
    for j in (0, 1, 31, 32, 33, 500, 1006):
        assert (int(words[j >> 5]) >> (j & 31)) & 1 == e[j]
    assert int(words[-1]) >> (1007 & 31) == 0
    assert abs(wl.frozen_param_fraction(cfg, np.ones(14, np.uint8)) - 1.0) < 1e-15
