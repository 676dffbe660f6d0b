"""The seeded input generators: determinism, storage formats and the prescribed spectra."""
import numpy as np

from paper_2605_16341_amd import synth


def test_bf16_bits_roundtrip_and_rounding():
    v = np.array([1.0, -2.5, 1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, 3.0e-5], dtype=np.float32)
    bits = synth.f32_to_bf16_bits(v)
    assert bits[:4].tolist() == [0x3F80, 0xC020, 0x3F80, 0x3F82]
    back = synth.bf16_bits_to_f32(bits)
    assert np.all(np.abs(back - v) <= np.abs(v) * 2.0 ** -8)
    assert np.array_equal(synth.f32_to_bf16_bits(back), bits)


def test_streams_are_deterministic_and_order_free():
    a = synth.power_law_stream(96, 64, 7, out_dtype="bf16")
    b = synth.power_law_stream(96, 64, 7, out_dtype="bf16")
    g3 = a.gradient(3)
    a.gradient(0)
    assert np.array_equal(g3, b.gradient(3)) and g3.dtype == np.uint16
    assert not np.array_equal(a.gradient(1), a.gradient(2))
    c = synth.power_law_stream(96, 64, 8, out_dtype="bf16")
    assert not np.array_equal(c.gradient(3), g3)


def test_power_law_spectrum_and_noise_share():
    m, n = 160, 120
    s = synth.power_law_stream(m, n, 11, exponent=0.5, noise_energy=0.05, rms=1e-2, out_dtype="f32")
    sig = np.linalg.svd(s.signal.astype(np.float64), compute_uv=False)
    ratio = sig[:60] / sig[0]
    assert np.allclose(ratio, np.arange(1, 61) ** -0.5, rtol=1e-4)
    g = s.gradient_f32(0).astype(np.float64)
    total = np.sum(g * g)
    assert abs(total / (m * n * 1e-4) - 1.0) < 0.05
    noise = g - s.signal
    assert abs(np.sum(noise * noise) / total - 0.05) < 0.01


def test_inverse_index_stream_matches_its_recipe():
    s = synth.inverse_index_stream(64, 64, 5, noise_std=0.01)
    sig = np.linalg.svd(s.signal.astype(np.float64), compute_uv=False)
    assert np.allclose(sig[:20], 1.0 / np.arange(1, 21), rtol=1e-4)
    noise = s.gradient_f32(2) - s.signal
    assert abs(noise.std() - 0.01) < 1e-3


def test_initial_state_formats():
    st = synth.initial_state(128, 96, 16, 3, x_dtype="bf16")
    assert st.X.dtype == np.uint16 and st.M.dtype == np.float32 and st.Q.shape == (96, 16)
    assert not st.M.any()
    q = st.Q.astype(np.float64)
    assert np.allclose(q.T @ q, np.eye(16), atol=1e-6)
    x = synth.bf16_bits_to_f32(st.X)
    assert abs(x.std() - 0.02) < 2e-3
    st2 = synth.initial_state(64, 64, 8, 3, x_dtype="f32", momentum_std=0.02)
    assert st2.X.dtype == np.float32 and abs(st2.M.std() - 0.02) < 3e-3


def test_workload_table_matches_the_benchmark_configurations():
    w = synth.WORKLOADS
    assert w["C1"].shapes == ((256, 256),) and w["C1"].r == 16 and w["C1"].x_dtype == "f32" and w["C1"].steps == 5
    assert w["C2"].shapes == ((4096, 4096),) and w["C2"].r == 256 and w["C2"].steps == 20
    assert len(w["C3"].shapes) == 96 and w["C3"].r == 512
    assert sorted(set(w["C3"].shapes)) == [(2048, 2048), (2048, 6144), (2048, 8192), (8192, 2048)]
    assert w["C4"].shapes == ((4096, 6144), (4096, 4096), (4096, 14336), (4096, 14336), (14336, 4096))
    assert w["C4"].r == 1024
    assert [w[f"C5-r{r}"].r for r in (16, 64, 256, 1024, 2048)] == [16, 64, 256, 1024, 2048]
    assert all(x.mu == 0.95 for x in w.values())
