"""Pins for the oracle's MLP curve estimator (Appendix A.3: three-layer perceptron
32-128-128-64 from the first tenth of the minimum distance curve to the rest) and the
thresholds derived from it (Section 4.1 steps 1-2).

The network is a plain definition once the representation is fixed; the pins are a library
matrix product, hand-set weights for which the result has a closed form (a constant output,
an exact power law, a neuron that ReLU must switch off), libm for the fixed-order ln / exp, and
the interplay with the rest of the threshold rule (measured boundaries, clamp, monotone)."""
import math

import numpy as np
import pytest

from oracle import ref

SIZES = [(32, 128), (128,), (128, 128), (128,), (128, 64), (64,)]


def pack(W1, b1, W2, b2, W3, b3):
    return np.concatenate([np.asarray(a, dtype=np.float32).reshape(-1) for a in (W1, b1, W2, b2, W3, b3)])


def zeros():
    return [np.zeros(s, dtype=np.float32) for s in SIZES]


def power_curve(m, A, e):
    c = np.empty(m + 1, dtype=np.float32)
    c[0] = np.inf
    c[1:] = (A * np.arange(1, m + 1, dtype=np.float64) ** (-e)).astype(np.float32)
    return c


def inputs_of(mdc, m):
    idx = np.maximum(1, (m * np.arange(1, 33)) // 32)
    return np.log(mdc[idx].astype(np.float64) / np.float64(mdc[m]))


@pytest.mark.parametrize("v", [1.0, 1.0000001, 1.5, 2.0, 3.75, 1e-3, 12345.678, 1e12, 2.0 ** 0.5])
def test_fixed_order_ln_and_exp_against_libm(v):
    assert ref.ln_fixed(v) == pytest.approx(math.log(v), rel=1e-14, abs=1e-16)
    y = math.log(v)
    assert ref.exp_fixed(y) == pytest.approx(v, rel=1e-14)
    assert ref.exp_fixed(-y) == pytest.approx(1.0 / v, rel=1e-14)


def test_forward_pass_against_a_library_matrix_product():
    rng = np.random.Generator(np.random.PCG64(5))
    parts = [rng.normal(0, 0.2, s).astype(np.float32) for s in SIZES]
    m = 51
    mdc = power_curve(m, 3.0, 1.1)
    mdc[1:] *= rng.uniform(0.9, 1.1, m).astype(np.float32)
    mdc[1:] = np.minimum.accumulate(mdc[1:])            # a curve never rises
    out = ref.mlp_curve(mdc, m, pack(*parts))
    W1, b1, W2, b2, W3, b3 = [a.astype(np.float64) for a in parts]
    h1 = np.maximum(inputs_of(mdc, m) @ W1 + b1, 0.0)
    h2 = np.maximum(h1 @ W2 + b2, 0.0)
    want = h2 @ W3 + b3
    assert np.allclose(out, want, rtol=1e-11, atol=1e-12)
    assert (h1 == 0).any() and (h1 > 0).any()           # both sides of the ReLU are exercised


def test_transposed_weights_would_fail():
    # a network that reads ONE input and feeds ONE output: only the stated layout finds them
    parts = zeros()
    parts[0][31, 7] = 1.0      # input 31 -> hidden neuron 7
    parts[2][7, 100] = 2.0     # hidden 7 -> hidden 100
    parts[4][100, 5] = -3.0    # hidden 100 -> output 5
    m = 64
    mdc = power_curve(m, 1.0, 1.0)
    out = ref.mlp_curve(mdc, m, pack(*parts))
    assert np.all(out == 0.0)                            # input 31 is ln(mdc[m] / mdc[m]) = 0
    parts[0][:] = 0
    parts[0][0, 7] = 1.0       # input 0 = ln(mdc[2]/mdc[64])
    out = ref.mlp_curve(mdc, m, pack(*parts))
    want = -6.0 * math.log(float(mdc[2]) / float(mdc[m]))
    assert out[5] == pytest.approx(want, rel=1e-13)
    assert np.count_nonzero(out) == 1


def test_relu_switches_a_negative_neuron_off():
    parts = zeros()
    parts[0][0, 3] = -1.0      # hidden 3 would be -input0 < 0
    parts[2][3, 3] = 1.0
    parts[4][3, 0] = 1.0
    parts[5][:] = 0.25
    mdc = power_curve(40, 2.0, 0.9)
    assert np.all(ref.mlp_curve(mdc, 40, pack(*parts)) == 0.25)


def test_constant_output_gives_closed_form_thresholds():
    # out_j = c for all j: the curve is mdc[m] * exp(c * min(u, 1)) with u the position in units of
    # the output grid -- boundaries beyond the first grid point sit at mdc[m] * exp(c)
    parts = zeros()
    c = -0.75
    parts[5][:] = c
    n, m = 1000, 100
    mdc = power_curve(m, 5.0, 1.0)
    prm = ref.MdpsParams(nseg=6, bias=1.1, level_scale=[1, 1, 1.2, 1, 1, 1], mlp=pack(*parts))
    thr = ref.mdps_thresholds(mdc, n, m, prm)
    base = float(mdc[m]) * math.exp(c) * 1.1 * 1.1
    want = [base, base, base * 1.2, base, base, base]
    want = np.minimum.accumulate(np.array(want))
    assert np.allclose(thr, want.astype(np.float32), rtol=2e-7)


def test_power_law_network_recovers_the_power_law():
    # hand-set weights that continue an exact power law: out_j = -ln(x_j/m) / ln(m/i_0) * input_0
    n, m, e, A = 4000, 400, 1.3, 7.0
    mdc = power_curve(m, A, e)
    i0 = max(1, m // 32)
    parts = zeros()
    parts[0][0, 0] = 1.0
    parts[2][0, 0] = 1.0
    xj = m + (n - 1 - m) * np.arange(1, 65) / 64.0
    parts[4][0, :] = (-np.log(xj / m) / math.log(m / i0)).astype(np.float32)
    prm = ref.MdpsParams(nseg=6, mlp=pack(*parts))
    thr = ref.mdps_thresholds(mdc, n, m, prm)
    bl = [min(max(n * l // 6, 1), n - 1) for l in range(1, 7)]
    want = np.array([A * b ** (-e) for b in bl])
    # linear interpolation of a logarithm on a 64-point grid: well below a percent
    assert np.allclose(thr, want, rtol=5e-3)
    assert np.all(np.diff(thr) <= 0)


def test_boundaries_inside_the_prefix_stay_measured():
    parts = zeros()
    parts[5][:] = -5.0
    n, m = 60, 30                     # p = 0.5: boundaries 10, 20, 30 are measured
    mdc = power_curve(m, 1.0, 1.0)
    prm = ref.MdpsParams(p=0.5, nseg=6, mlp=pack(*parts))
    thr = ref.mdps_thresholds(mdc, n, m, prm)
    assert thr[0] == mdc[10] and thr[1] == mdc[20] and thr[2] == mdc[30]
    assert thr[5] == pytest.approx(float(mdc[m]) * math.exp(-5.0), rel=1e-6)


def test_sampling_with_the_mlp_equals_the_literal_transcription():
    from paper_2507_23480_amd import inputs
    rng = np.random.Generator(np.random.PCG64(9))
    parts = [rng.normal(0, 0.05, s).astype(np.float32) for s in SIZES]
    parts[5][:] = -np.linspace(0.1, 2.0, 64)             # a falling curve whatever the rest adds
    prm = ref.MdpsParams(nseg=4, bias=1.05, mlp=pack(*parts))
    xyz = inputs.uniform_cube(77, 600)
    a, ia = ref.mdps_sample(xyz, 200, prm)
    b, ib = ref.mdps_literal(xyz, 200, prm)
    assert np.array_equal(a, b) and np.array_equal(ia.thr2, ib.thr2)
    assert len(set(a.tolist())) == 200


def test_committed_weights_predict_the_curves_of_a_workload():
    """The trained estimator of the object-classification stage on that workload's own clouds
    (the test split of the training), curves from the oracle's exact FPS: the error of the
    estimated curve stays in the range reported when it was trained, and the training module's
    numpy network is the oracle's network."""
    from paper_2507_23480_amd import inputs, mlp_estimator
    wl = inputs.WORKLOADS["C2"]
    n = wl.stages[0].n
    m = mlp_estimator.prefix_len(n)
    w = mlp_estimator.weights()["C2/0"]
    batch = inputs.make_batch("C2")
    curves = np.stack([ref.fps_exact(batch[b], n)[1] for b in range(wl.B)])
    x, y = mlp_estimator.representation(curves, n, m)
    assert mlp_estimator.mape(w, x, y) < 6.0
    for b in range(3):
        out = ref.mlp_curve(curves[b], m, w)
        assert np.allclose(out, mlp_estimator.forward(w, x[b:b + 1])[0], rtol=1e-9, atol=1e-11)
    assert mlp_estimator.table()["C2"][0]["mape_percent_workload"] < 6.0


def test_exponent_outside_the_range_is_clamped():
    """ref_exp_fixed brings its argument into [-700, 700] first (NaN counts as -700), so that the
    scaling by a power of two stays exact whatever a network puts out: beyond the range the
    result is that of the nearest end, pinned here against libm's exp at the two ends."""
    top, bottom = math.exp(700.0), math.exp(-700.0)        # 1.0142320547350045e+304, 9.85967654375977e-305
    assert top == pytest.approx(1.0142320547350045e304, rel=1e-15)
    assert bottom == pytest.approx(9.85967654375977e-305, rel=1e-15)
    assert ref.exp_fixed(700.0) == pytest.approx(top, rel=1e-13)
    assert ref.exp_fixed(-700.0) == pytest.approx(bottom, rel=1e-13)
    for y in (700.0000001, 1e4, 1e300, math.inf):
        assert ref.exp_fixed(y) == ref.exp_fixed(700.0)
    for y in (-700.0000001, -1e4, -1e300, -math.inf, math.nan):
        assert ref.exp_fixed(y) == ref.exp_fixed(-700.0)
    # just inside the range nothing is clamped
    assert ref.exp_fixed(699.5) == pytest.approx(math.exp(699.5), rel=1e-13)
    assert ref.exp_fixed(699.5) < ref.exp_fixed(700.0)


def test_inputs_whose_ratio_is_not_a_finite_number_at_least_one_read_as_zero():
    """A curve that has fallen to 0 at the end of the prefix (every remaining point coincides with
    a sample) makes the ratios mdc[i] / mdc[m] infinite or 0/0, and a rising curve (never produced
    by exact FPS) makes them smaller than 1: all such inputs read as 0.  Hand-set network in which
    any input other than 0 would show: W1 = 1 everywhere, b1 = 1/2, W2 = identity, W3 = 1/128,
    b3[j] = j/64  ->  with all inputs 0: h1 = h2 = 1/2, out[j] = 128 * (1/2) * (1/128) + j/64."""
    parts = zeros()
    parts[0][:] = 1.0
    parts[1][:] = 0.5
    parts[2][:] = np.eye(128, dtype=np.float32)
    parts[4][:] = 1.0 / 128.0
    parts[5][:] = np.arange(64, dtype=np.float32) / 64.0
    w = pack(*parts)
    want = 0.5 + np.arange(64) / 64.0
    m = 64
    dead = power_curve(m, 2.0, 1.0)
    dead[m] = 0.0                        # ratios +inf
    dead[40:m] = 0.0                     # ... and 0/0 for the inputs taken there
    assert np.array_equal(ref.mlp_curve(dead, m, w), want)
    rising = np.full(m + 1, 1.0, dtype=np.float32)
    rising[m] = 2.0                      # every ratio 1/2 < 1
    assert np.array_equal(ref.mlp_curve(rising, m, w), want)
    # the same network on a falling curve does see its inputs (so the zeros above are the rule's doing)
    live = power_curve(m, 2.0, 1.0)
    assert np.all(ref.mlp_curve(live, m, w) > want + 1.0)
    # thresholds from a dead prefix: mdc[m] * exp(.) = 0 for every boundary beyond the prefix,
    # which the clamp raises to the smallest normal binary32 number
    n = 640
    prm = ref.MdpsParams(nseg=6, bias=1.2, mlp=w)
    thr = ref.mdps_thresholds(dead, n, m, prm)
    assert np.all(thr == np.float32(1.17549435e-38))
