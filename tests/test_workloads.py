"""Seeded generators: determinism, bf16 rounding rule, config shapes."""
import numpy as np

from workloads import round_to_bf16, bf16_bits, bits_to_f32, gemm_inputs, gemm_cases, layer_inputs, LayerShape


def test_bf16_rounding_nearest_even():
    # 1 + 2^-8 is exactly half-way between bf16 neighbours 1 and 1+2^-7 -> ties to even (1.0)
    x = np.array([1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, 1.0 + 2.0 ** -9, -1.0 - 2.0 ** -8, 0.0, 3.0e38], dtype=np.float32)
    r = round_to_bf16(x)
    assert r[0] == 1.0 and r[1] == np.float32(1.0 + 2.0 ** -6) and r[2] == 1.0 and r[3] == -1.0 and r[4] == 0.0
    bits = bf16_bits(r[:5])
    assert np.array_equal(bits_to_f32(bits), r[:5])
    # brute force: nearest representable among neighbours
    rng = np.random.default_rng(0)
    v = rng.standard_normal(1000).astype(np.float32)
    rv = round_to_bf16(v)
    lo = (v.view(np.uint32) & 0xFFFF0000).view(np.float32)
    hi = ((v.view(np.uint32) & 0xFFFF0000) + 0x10000).view(np.float32)
    best = np.where(np.abs(v - lo) <= np.abs(hi - v), lo, hi)
    ties = np.abs(v - lo) == np.abs(hi - v)
    assert np.array_equal(rv[~ties], best[~ties])


def test_seeded_and_deterministic():
    a1, b1 = gemm_inputs(3, "abt", 8, 16, 4, "bf16")
    a2, b2 = gemm_inputs(3, "abt", 8, 16, 4, "bf16")
    assert np.array_equal(a1, a2) and np.array_equal(b1, b2)
    assert a1.shape == (8, 16) and b1.shape == (4, 16)
    a3, _ = gemm_inputs(4, "abt", 8, 16, 4, "bf16")
    assert not np.array_equal(a1, a3)
    assert np.array_equal(round_to_bf16(a1), a1)


def test_config_shapes():
    c3 = gemm_cases("config3")
    assert len(c3) == 6 and all(g.flops_per_device == 19327352832 for g in c3)
    c1 = {g.form: g for g in gemm_cases("config1")}
    assert (c1["ab"].M, c1["ab"].K, c1["ab"].N) == (32, 64, 256)
    assert (c1["abt"].M, c1["abt"].K, c1["abt"].N) == (32, 256, 64)
    assert (c1["atb"].M, c1["atb"].K, c1["atb"].N) == (64, 32, 256)
    c4 = {g.name: g for g in gemm_cases("config4")}
    assert sum(g.flops_per_device for g in c4.values() if g.form == "ab") == 24 * 8 * 1024 * 4096 ** 2 // 16


def test_layer_inputs_recipe():
    shp = LayerShape(2, 4, 8, 2, 2)
    t = layer_inputs(7, shp, "bf16")
    assert t["x"].shape == (8, 8) and t["w_qkv"].shape == (8, 24) and t["w2"].shape == (32, 8)
    assert np.all(t["ln1_g"] == 1) and np.all(t["b1"] == 0)
    tp = layer_inputs(7, shp, "bf16", perturb_affine=True)
    assert np.array_equal(tp["x"], t["x"]) and not np.all(tp["ln1_g"] == 1)
