"""Host-side checks of the synthetic workload generator (no method arithmetic in it)."""
import numpy as np
import pytest
import torch

from paper_2407_12820_amd import workloads as wl


def test_bf16_rounding_matches_torch():
    x = np.random.default_rng(0).standard_normal(100000).astype(np.float32) * 100
    x[:4] = [1.00390625, 1.01171875, 0.0, -3.0e-39]  # exact ties (both parities), zero, subnormal
    bits = wl.f32_to_bf16_bits(x)
    ref = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    np.testing.assert_array_equal(bits, ref)
    np.testing.assert_array_equal(wl.bf16_bits_to_f32(bits), torch.from_numpy(x).to(torch.bfloat16).float().numpy())


@pytest.mark.parametrize("name,want", [("tiny_f32", 603136), ("llama8b_32k", 27656192), ("llama8b_128k", 56074240),
                                       ("batch8_32k", 225673216), ("llama70b_128k", 232833024)])
def test_algorithmic_bytes(name, want):
    assert wl.CONFIGS[name].algorithmic_bytes() == want


def test_code_bytes_over_key_bytes_ratio():
    # Section 4.1: codes take h_kv*m*s*b/8 bytes against 2*h_kv*s*d_h bytes of fp16
    # keys, i.e. m*b/(16*d_h): 1/64 for m=4, b=8.  With one byte per code the ratio
    # is m/(2*d_h): 1/128 for m=2.
    for name, ratio in [("llama8b_128k", 1 / 128), ("llama70b_128k", 1 / 64)]:
        w = wl.CONFIGS[name]
        units = w.batch * w.n_kv_heads
        assert (units * w.n_tokens * w.pq_m) / (2 * units * w.n_tokens * w.head_dim) == ratio


def test_selection_sizes():
    assert [wl.CONFIGS[n].topk for n in wl.CONFIG_ORDER] == [512, 6553, 13107, 6553, 13107]
    assert all(wl.CONFIGS[n].n_init == 4 and wl.CONFIGS[n].n_local == 64 for n in wl.CONFIG_ORDER)


def test_generate_is_seeded_and_shaped():
    w = wl.get("llama8b_128k", n_tokens=2048)
    assert w.topk == 204 and w.plant_count == 20
    a, b, c = wl.generate(w, 3), wl.generate(w, 3, threads=1), wl.generate(w, 4)
    for key in ("q", "k", "v"):
        np.testing.assert_array_equal(a[key], b[key])
        assert not np.array_equal(a[key], c[key])
    assert a["k"].shape == (1, 8, 2048, 128) and a["k"].dtype == np.uint16
    assert a["q"].shape == (1, 32, 128)
    pos = a["planted"][0, 0]
    assert pos.min() >= w.n_init and pos.max() < w.n_tokens - w.n_local and len(set(pos.tolist())) == 20
    # planted keys lean towards the group's mean query
    qbar = wl.to_f32(a["q"], "bf16")[0, :4].mean(0)
    kf = wl.to_f32(a["k"], "bf16")[0, 0]
    assert (kf[pos] @ qbar).mean() > 10 * abs((np.delete(kf, pos, 0) @ qbar).mean())


def test_outlier_channels_and_init_indices():
    w = wl.get("llama8b_32k", n_tokens=1024)
    d = wl.generate(w, 1)
    kf = wl.to_f32(d["k"], "bf16")
    for g in range(w.n_kv_heads):
        sd = kf[0, g].std(0)
        ch = d["outlier_channels"][0, g]
        assert np.all(sd[ch] > 6) and np.all(np.delete(sd, ch) < 1.3)
    init = wl.kmeans_init_indices(w, 1)
    assert init.shape == (1, 8, 2, 64) and init.dtype == np.int32
    assert all(len(set(init[0, g, j].tolist())) == 64 for g in range(8) for j in range(2))
    assert init.min() >= 0 and init.max() < 1024
