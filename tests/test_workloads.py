"""The seeded input generators: shapes, determinism, bf16 exactness."""
import numpy as np
import torch

from paper_2601_21896_amd import workloads as wl


def test_paper_shape_constants():
    assert wl.C1.H == 1536 and wl.C1.Lc == 4680 and wl.C1.n == 32760 and wl.C1.k == 16380
    assert wl.C4.H == 5120 and wl.C4.Lc == 10800 and wl.C4.n == 75600 and wl.C4.k == 22680
    assert wl.C0.H == 128 and wl.C0.Lc == 64 and wl.C0.n == 256 and wl.C0.k == 128


def test_round_to_bf16_matches_library_cast():
    rng = np.random.default_rng(0)
    a = (rng.standard_normal(100000) * 10.0 ** rng.integers(-20, 20, 100000)).astype(np.float32)
    want = torch.from_numpy(a).to(torch.bfloat16).to(torch.float32).numpy()
    got = wl.round_to_bf16(a)
    assert np.array_equal(got, want)
    bits = wl.bf16_bits(got)
    back = (bits.astype(np.uint32) << 16).view(np.float32)
    assert np.array_equal(back, got)


def test_generator_is_deterministic_and_structured():
    cfg = wl.scaled(wl.C1, frame_tokens=40, cache_frames=5, k=100)
    a = wl.make_layer_inputs(cfg)
    b = wl.make_layer_inputs(cfg)
    for key in ("W1", "X_cache", "K_cache", "V_chunk", "Q"):
        assert np.array_equal(a[key], b[key])
        assert np.array_equal(wl.round_to_bf16(a[key]), a[key])        # bf16-representable
    assert a["K_cache"].shape == (200, 12, 128) and a["Q"].shape == (120, 12, 128)
    assert a["W1"].shape == (256, 1536) and a["W2"].shape == (1, 256)
    assert int(a["salient"].sum()) == 20
    sal = a["X_cache"][a["salient"]].mean()
    rest = a["X_cache"][~a["salient"]].mean()
    assert 1.9 < sal - rest < 2.1
    c = wl.make_layer_inputs(cfg, structure="coherent")
    m = c["salient"].reshape(5, 40)
    assert np.all(m == m[0:1]) and int(m[0].sum()) == 4


def test_c0_is_fp32_without_salient_offset():
    d = wl.make_layer_inputs(wl.C0)
    assert d["X_cache"].shape == (256, 128) and not d["salient"].any()
    assert not np.array_equal(wl.round_to_bf16(d["Q"]), d["Q"])
    assert abs(float(d["W1"].std()) - 0.02) < 0.002
