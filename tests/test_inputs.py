"""The seeded input generator: determinism, slicing, distribution, bf16 rounding."""
import numpy as np
import torch

from paper_2602_07306_amd import inputs as I


def test_streams_are_deterministic_and_sliceable():
    k = I.stream_key(3, I.KIND_WG, 2, 5)
    x = I.standard_normals(k, 0, 4096)
    assert np.array_equal(x, I.standard_normals(k, 0, 4096))
    for s, c in [(1, 7), (5, 11), (100, 1), (4095, 1), (0, 1)]:
        assert np.array_equal(I.standard_normals(k, s, c), x[s:s + c])
    assert not np.array_equal(x, I.standard_normals(I.stream_key(3, I.KIND_WG, 2, 6), 0, 4096))
    a = I.normal_tensor(k, (64, 64), 0.02, chunk=1000, workers=3)
    b = I.normal_tensor(k, (64, 64), 0.02, chunk=1 << 20, workers=1)
    assert np.array_equal(a, b)


def test_normals_have_the_stated_distribution():
    x = I.standard_normals(I.stream_key(0, I.KIND_EMBED), 0, 1 << 20)
    assert abs(x.mean()) < 4e-3 and abs(x.std() - 1) < 3e-3
    assert abs((x ** 4).mean() - 3) < 0.05 and abs((x ** 3).mean()) < 0.02
    assert abs(np.mean(np.abs(x) < 1) - 0.682689) < 2e-3
    # the two normals of one counter are uncorrelated
    assert abs(np.mean(x[0::2] * x[1::2])) < 4e-3
    w = I.normal_tensor(I.stream_key(0, I.KIND_WQ), (512, 512), 0.02)
    assert w.dtype == np.float32 and abs(w.std() - 0.02) < 2e-4


def test_polynomials_track_libm():
    u = np.linspace(1e-9, 1.0, 100001)
    assert np.max(np.abs(I._log_poly(u) - np.log(u))) < 1e-13
    a = np.linspace(-np.pi / 4, np.pi / 4, 100001)
    c, s = I._sincos_poly(a)
    assert np.max(np.abs(c - np.cos(a))) < 1e-15 and np.max(np.abs(s - np.sin(a))) < 1e-15


def test_bf16_rounding_is_round_to_nearest_even():
    x = np.random.default_rng(0).normal(size=100000).astype(np.float32)
    x[:4] = [1.0, 1.00390625, 1.01171875, -1.00390625]        # exact ties
    ref = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(I.bf16_bits(x), ref)
    assert np.array_equal(I.bf16_to_f32(I.bf16_bits(x)),
                          torch.from_numpy(x).to(torch.bfloat16).float().numpy())


def test_tokens_are_uniform_ids():
    t = I.make_tokens(1, 4, 1024, 32000)
    assert t.shape == (4, 1024) and t.dtype == np.int32 and t.min() >= 0 and t.max() < 32000
    assert len(np.unique(t)) > 3500
    assert np.array_equal(t, I.make_tokens(1, 4, 1024, 32000))


def test_make_weights_shapes_and_rounding():
    cfg = I.config_tiny()
    W = I.make_weights(cfg, 0)
    assert W["wq"].shape == (2, 4, 128, 128) and W["wd"].shape == (2, 4, 512, 128)
    assert W["embed"].shape == (512, 128) and W["head"].shape == (128, 512)
    import dataclasses
    Wb = I.make_weights(dataclasses.replace(cfg, dtype=I.PT_BF16, n_layers=1, block_depth=1), 0)
    assert np.array_equal(Wb["wq"][0, 0], I.round_to_dtype(W["wq"][0, 0], I.PT_BF16))
    assert np.all((Wb["wq"].view(np.uint32) & 0xFFFF) == 0)


def test_expert_streams_and_lazy_weights():
    """PT-MoE weights: one stream per (tensor, track, layer, expert), distinct from each other and from the dense
    streams; LazyWeights generates exactly the tensors of make_weights, one at a time."""
    cfg = I.PTConfig(n_tracks=2, n_layers=2, block_depth=1, d_model=32, n_heads=2, n_kv_heads=1, head_dim=16,
                     d_ffn=32, vocab=64, max_batch=1, max_seq=8, dtype=I.PT_BF16, n_experts=3, top_k=2)
    W = I.make_weights(cfg, 9)
    assert W["wg"].shape == (2, 2, 3, 32, 32) and W["wd"].shape == (2, 2, 3, 32, 32) and W["wr"].shape == (2, 2, 32, 3)
    flat = [W["wu"][i, l, e].tobytes() for i in range(2) for l in range(2) for e in range(3)]
    assert len(set(flat)) == len(flat)
    dense = I.make_weights(I.PTConfig(**{**cfg.__dict__, "n_experts": 0, "top_k": 0}), 9)
    assert not np.array_equal(dense["wu"][0, 0], W["wu"][0, 0, 0])          # expert 0 is not the dense stream
    assert np.array_equal(dense["wq"], W["wq"])                              # the attention half is unchanged
    assert I.stream_key(9, I.KIND_WU, 1, I.expert_layer(1, 2)) != I.stream_key(9, I.KIND_WU, 1, 1)
    seen = []
    L = I.LazyWeights(cfg, 9, on_tensor=lambda name, i, l: seen.append((name, i, l)))
    for name in ("wq", "wk", "wv", "wo"):
        assert np.array_equal(L[name][1, 0], W[name][1, 0])
    for name in ("wg", "wu", "wd"):
        assert np.array_equal(L[name][0, 1, 2], W[name][0, 1, 2])
    assert np.array_equal(L["wr"][1, 1], W["wr"][1, 1])
    for name in ("embed", "head", "gf"):
        assert np.array_equal(L[name], W[name])
    assert np.array_equal(L["g2"][0, 0], W["g2"][0, 0])
    assert ("wq", 1, 0) in seen and ("wd", 0, 1) in seen
