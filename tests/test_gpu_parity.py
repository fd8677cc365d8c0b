"""GPU parity: the HIP library (through its C ABI) against the CPU oracle, element by element,
on the same seeded inputs.

Gates
  * offline weight codes and scales: bit-identical
  * int32 accumulators: bit-exact given identical int8 operands
  * activation codes (teacher-forced per layer: the oracle's fp32 input and scale go in):
    at most 0.1 % differ, each by at most 1 LSB
  * final outputs: max-abs <= 2e-3 against the oracle's quantized forward
  * calibrated scales: within 1e-5 relative
"""
import sys

import numpy as np
import pytest

import paper_2508_13478_amd as dhq
from oracle import dhq_oracle as o
from paper_2508_13478_amd import synth

pytestmark = pytest.mark.gpu

OUT_TOL = 2e-3          # max-abs on final outputs
CODE_RATE = 1e-3        # fraction of codes allowed to differ (by 1 LSB)


def _say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def _torch():
    import torch
    return torch


def _dev(a):
    torch = _torch()
    return torch.from_numpy(np.ascontiguousarray(a)).to("cuda")


class Case:
    """A network quantized by both sides, with the oracle's calibrated scales given to the library."""

    def __init__(self, dims, coords, W, b, bits=8, omega0=30.0, dump=True):
        self.dims, self.coords, self.W, self.b, self.bits = list(dims), coords, W, b, bits
        self.net = o.quantize_net(dims, omega0, bits, bits, W, b)
        res = o.forward(self.net, coords, calibrate=True, dump=dump)
        self.out, self.dump = res if dump else (res, None)
        self.model = dhq.Model(dims, omega0, W, b, bits, bits)
        self.model.set_act_scales(self.net.s_a)


_cache = {}


def case(name, **kw):
    key = (name, tuple(sorted(kw.items())))
    if key not in _cache:
        wl, coords, W, b = synth.make(name)
        stride = kw.pop("stride", 1)
        _cache[key] = Case(wl.dims, coords[::stride], W, b, **kw)
    return _cache[key]


def int_matmul(codes, Wq):
    """codes Wq^T over the integers, for operands that did not come from the oracle (the oracle is
    only ever fed seeded inputs): float64 products and sums of int8 values are exact far beyond int32."""
    return (codes.astype(np.float64) @ Wq.astype(np.float64).T).astype(np.int64).astype(np.int32)


def int_unrotate(acc):
    """acc H over the integers (H: Sylvester-Hadamard matrix of the row length), same remark."""
    from scipy.linalg import hadamard
    return (acc.astype(np.float64) @ hadamard(acc.shape[1]).astype(np.float64)).astype(np.int64).astype(np.int32)


def code_stats(got, exp):
    d = np.abs(got.astype(np.int32) - exp.astype(np.int32))
    return float((d != 0).mean()), int(d.max()) if d.size else 0


# --------------------------------------------------------------------------- offline step
@pytest.mark.parametrize("name", ["C1", "C2"])
def test_weight_codes_and_scales_bit_identical(name):
    _say(f"weights {name}")
    cs = case(name)
    sw, sa = cs.model.scales()
    assert np.array_equal(sw, cs.net.s_w)
    assert np.array_equal(sa, cs.net.s_a)
    for l in range(len(cs.dims) - 1):
        assert np.array_equal(cs.model.weight_codes(l), cs.net.Wq[l]), f"layer {l}"


@pytest.mark.parametrize("bits", [4, 6])
def test_weight_codes_odd_shapes_and_low_bits(bits):
    dims = [3, 48, 100, 5]
    W, b = synth.siren_init(dims, 30.0, 4242)
    net = o.quantize_net(dims, 30.0, bits, bits, W, b)
    m = dhq.Model(dims, 30.0, W, b, bits, bits)
    sw, _ = m.scales()
    assert np.array_equal(sw, net.s_w)
    for l in range(3):
        assert np.array_equal(m.weight_codes(l), net.Wq[l])
    assert not m.has_fused()


# ------------------------------------------------------------- integer GEMM, teacher-forced
@pytest.mark.parametrize("name,rows", [("C1", 4096), ("C2", 4096 + 77)])
def test_gemm_accumulators_bit_exact(name, rows):
    torch = _torch()
    cs = case(name)
    for l in range(len(cs.dims) - 1):
        _say(f"gemm {name} layer {l} rows {rows}")
        codes = cs.dump.codes[l][:rows]
        acc = cs.model.gemm_i8(l, _dev(codes))
        torch.cuda.synchronize()
        assert np.array_equal(acc.cpu().numpy(), cs.dump.acc[l][:rows]), f"layer {l}"


def test_gemm_extreme_operands_and_ragged_rows():
    """All codes at +-qmax against a full-width layer, and row counts around the tile sizes."""
    torch = _torch()
    cs = case("C2")
    l = 2
    Wq = cs.net.Wq[l]
    rng = np.random.default_rng(3)
    for rows in (1, 31, 32, 33, 127, 129, 300):
        _say(f"gemm ragged rows {rows}")
        codes = rng.choice(np.array([-127, 127], dtype=np.int8), size=(rows, Wq.shape[1]))
        if rows == 1:
            codes[0] = np.where(Wq[5] >= 0, 127, -127)       # drives accumulator 5 to its maximum
        acc = cs.model.gemm_i8(l, _dev(codes))
        torch.cuda.synchronize()
        assert np.array_equal(acc.cpu().numpy(), o.igemm(codes, Wq))


# ------------------------------------------------ one layer, teacher-forced with oracle inputs
@pytest.mark.parametrize("name", ["C1", "C2"])
def test_layer_teacher_forced(name):
    torch = _torch()
    cs = case(name)
    L = len(cs.dims) - 1
    rows = min(cs.coords.shape[0], 20000 + 13)
    for l in range(L):
        _say(f"layer {name} {l}")
        x = cs.coords[:rows] if l == 0 else cs.dump.act[l - 1][:rows]
        codes, acc, act = cs.model.forward_debug(_dev(x), l)
        torch.cuda.synchronize()
        codes, acc, act = codes.cpu().numpy(), acc.cpu().numpy(), act.cpu().numpy()
        rate, mx = code_stats(codes, cs.dump.codes[l][:rows])
        _say(f"  code mismatch rate {rate:.2e} max {mx}")
        assert rate <= CODE_RATE and mx <= 1
        # the library's accumulators are exact for the codes it produced
        assert np.array_equal(acc, int_matmul(codes, cs.net.Wq[l]))
        # where the codes agree the accumulators do too, and the epilogue matches
        same = (codes == cs.dump.codes[l][:rows]).all(axis=1)
        assert np.array_equal(acc[same], cs.dump.acc[l][:rows][same])
        err = np.abs(act[same].astype(np.float64) - cs.dump.act[l][:rows][same]).max()
        _say(f"  epilogue max-abs err {err:.2e}")
        assert err <= 2e-5


# ------------------------------------------------------------------------------ whole path
# Free-running, a +-1 LSB code difference (allowed above) early in the network changes every
# later layer's input for that coordinate; the sine layers amplify it and the final value of
# that coordinate can move by more than OUT_TOL although both evaluations are valid quantized
# forwards.  So the end-to-end gate is:
#   * every coordinate whose codes agree with the oracle's at every layer: |err| <= OUT_TOL
#     (checked by replaying the library's own layer chain through the debug hook);
#   * coordinates beyond OUT_TOL: at most FLIP_FRAC of all (scaled with the number of codes a
#     coordinate passes through, relative to the C2 network, because every code is one more
#     chance of a rounding-boundary difference), each with a code difference upstream, each
#     within FLIP_BOUND (ten times OUT_TOL: the size of the quantization error itself, which
#     is what a flipped code perturbs).
FLIP_FRAC = 1e-3
FLIP_BOUND = 2e-2


def flip_frac(dims):
    codes = sum(1 << (k - 1).bit_length() if k > 1 else 1 for k in dims[:-1])
    return FLIP_FRAC * max(1.0, codes / 1026.0)


def _coords_with_code_diffs(cs, n):
    """Replays the layer-by-layer path free-running through dhq_forward_debug and returns a
    boolean mask of coordinates where any layer's codes differ from the oracle's."""
    torch = _torch()
    diff = np.zeros(n, dtype=bool)
    for start in range(0, n, 65536):
        stop = min(n, start + 65536)
        x = _dev(cs.coords[start:stop])
        for l in range(len(cs.dims) - 1):
            codes, _, act = cs.model.forward_debug(x, l)
            d = np.abs(codes.cpu().numpy().astype(np.int32) - cs.dump.codes[l][start:stop].astype(np.int32))
            diff[start:stop] |= (d != 0).any(axis=1)
            x = act
    torch.cuda.synchronize()
    return diff


# A code may legitimately differ from the oracle's only where the exact rotated activation lies
# within the fp32 path's own error of a rounding boundary.  That error is dominated by the sine
# layer before it: the argument in revolutions reaches |t| ~ 10 where one fp32 ulp is 1e-6
# revolutions = 6e-6 rad, so an activation is off by up to ~6e-6 (rms ~1e-6) and a sum of Kp = 256
# of them with signs by ~2e-5 rms.  BOUNDARY_EPS (un-normalised units, i.e. before the 1/sqrt(Kp))
# is five times that; the transform's own rounding (a few ulp of |x^| <= 100, ~1e-5) fits inside.
BOUNDARY_EPS = 1e-4


def _near_boundary(net, dmp, bits):
    """Per coordinate: does any in-range code of any layer come from a rotated activation within
    BOUNDARY_EPS of a rounding boundary?  (dmp.rot holds the oracle's exact, normalised x^.)"""
    qm = (1 << (bits - 1)) - 1
    near = np.zeros(dmp.rot[0].shape[0], dtype=bool)
    for l, rot in enumerate(dmp.rot):
        t = rot / float(net.s_a[l])
        dist = np.abs(t - np.floor(t) - 0.5)                    # in quantization steps
        eps = BOUNDARY_EPS / (float(net.s_a[l]) * np.sqrt(rot.shape[1]))
        near |= ((dist < eps) & (np.abs(t) < qm)).any(axis=1)          # boundaries lie at +-(k + 0.5), k < qmax
    return near


def _assert_close(out, exp, strict=False, frac=FLIP_FRAC):
    """Free-running comparison of final values: strict max-abs, or max-abs on all but the
    small fraction of coordinates that a code difference may have moved."""
    err = np.abs(np.asarray(out, dtype=np.float64) - exp).max(axis=1)
    if strict:
        assert err.max() <= OUT_TOL
    else:
        assert (err > OUT_TOL).mean() <= frac and err.max() <= FLIP_BOUND
    return err


# ---------------------------------------------------------------- the fused kernels, free-running
# The whole-network kernels expose nothing but their final values, so their chain of codes is
# replayed through dhq_forward_debug_fused, which runs one layer of the same device code on given
# input codes: layer 0's quantizer through the layer-by-layer hook (the same two-point butterfly
# and quantizer), then layer after layer on the codes the previous one produced.  That the replay
# is what the whole-network launch computed is checked on its last link: the output layer's
# accumulators of the replayed codes, dequantized, must give the launch's outputs.
def fused_chain(model, net, coords):
    """Codes of every layer's input as the fused kernels produce them free-running, and the
    final values they imply.  coords: (n <= 65536, K0) numpy."""
    torch = _torch()
    L = len(net.dims) - 1
    codes = [model.forward_debug(_dev(coords), 0)[0]]
    for l in range(L - 1):
        _, nxt, _ = model.forward_debug_fused(codes[l], l)
        codes.append(nxt)
    acc = model.gemm_i8(L - 1, codes[L - 1])
    torch.cuda.synchronize()
    acc = acc.cpu().numpy()
    scale = float(net.s_a[L - 1]) * float(net.s_w[L - 1])
    if net.two_sided:
        acc = int_unrotate(acc)
        scale /= np.sqrt(float(acc.shape[1]))
    out = acc[:, : net.dims[-1]].astype(np.float64) * scale + net.bias[L - 1].astype(np.float64)
    return [c.cpu().numpy() for c in codes], out


def first_differences(got_codes, exp_codes):
    """Free-running code comparison.  A coordinate's codes of layer l are a teacher-forced
    comparison exactly as long as all its earlier codes agree with the oracle's (the layer then saw
    the oracle's input).  Returns (mask of coordinates with any difference, number of codes compared
    under that condition, number of those that differ, largest such difference)."""
    n = got_codes[0].shape[0]
    agree = np.ones(n, dtype=bool)
    compared = differing = 0
    worst = 0
    for g, e in zip(got_codes, exp_codes):
        d = np.abs(g.astype(np.int32) - e.astype(np.int32))[agree]
        compared += d.size
        differing += int((d != 0).sum())
        worst = max(worst, int(d.max()) if d.size else 0)
        agree[agree] = (d == 0).all(axis=1)
    return ~agree, compared, differing, worst


def check_fused_against_oracle(model, net, coords, out, exp, dump, label, bound=None):
    """The end-to-end gate of a whole-network launch `out` on `coords` (oracle: exp, dump):
      * the replayed chain reproduces the launch;
      * codes compared while a coordinate still agrees with the oracle: <= 0.1 % differ, each by 1 LSB;
      * every coordinate without a code difference is within OUT_TOL, i.e. every excess is explained
        by a code difference upstream; no value is further off than FLIP_BOUND (or `bound`, for a network whose own
        quantization error is not that of the sine networks).
    Returns (err per coordinate, mask of coordinates with a code difference)."""
    chain, chain_out = fused_chain(model, net, coords)
    assert np.abs(chain_out - out.astype(np.float64)).max() <= 1e-6, f"{label}: the replayed chain is not what the launch computed"
    diff, compared, differing, worst = first_differences(chain, dump.codes)
    err = np.abs(out.astype(np.float64) - exp).max(axis=1)
    over = err > OUT_TOL
    _say(f"  {label}: {differing} of {compared} codes differ where the input agreed ({differing / compared:.2e}, max {worst} LSB); "
         f"{diff.sum()} of {err.size} coords with a code difference, {over.sum()} beyond {OUT_TOL}; "
         f"max err without any: {err[~diff].max() if (~diff).any() else 0.0:.3e}, overall {err.max():.3e}")
    assert worst <= 1 and differing <= CODE_RATE * compared
    assert not (over & ~diff).any()
    assert err.max() <= (FLIP_BOUND if bound is None else bound)
    return err, diff


def _check_forward(cs, flags, label, strict=False):
    torch = _torch()
    out = cs.model.forward(_dev(cs.coords), flags=flags)
    torch.cuda.synchronize()
    out = out.cpu().numpy()
    assert np.isfinite(out).all()
    err = np.abs(out.astype(np.float64) - cs.out).max(axis=1)
    over = err > OUT_TOL
    _say(f"  {label}: max-abs err {err.max():.3e}, {over.sum()} of {err.size} coords beyond {OUT_TOL} "
         f"(|out| max {np.abs(cs.out).max():.3f})")
    if strict:
        assert not over.any()
        return out
    assert over.mean() <= flip_frac(cs.dims) and err.max() <= FLIP_BOUND
    if flags == dhq.DHQ_LAYERWISE and cs.dump is not None:
        diff = _coords_with_code_diffs(cs, err.size)
        _say(f"  {label}: {diff.sum()} coords with a code difference somewhere; "
             f"max err without any: {err[~diff].max():.3e}")
        assert err[~diff].max() <= OUT_TOL        # identical codes -> the tolerance holds strictly
        assert diff[over].all()                   # every excess is explained by a code difference
    if flags == dhq.DHQ_FUSED and cs.dump is not None and err.size <= 65536:
        check_fused_against_oracle(cs.model, cs.net, cs.coords, out, cs.out, cs.dump, label)
    return out


@pytest.mark.parametrize("name", ["C1", "C2"])
def test_forward_layerwise(name):
    _say(f"forward layerwise {name}")
    _check_forward(case(name), dhq.DHQ_LAYERWISE, "layerwise", strict=(name == "C1"))


@pytest.mark.parametrize("name", ["C1", "C2"])
def test_forward_fused(name):
    _say(f"forward fused {name}")
    cs = case(name)
    assert cs.model.has_fused()
    a = _check_forward(cs, dhq.DHQ_FUSED, "fused", strict=(name == "C1"))
    b = _check_forward(cs, dhq.DHQ_LAYERWISE, "layerwise", strict=(name == "C1"))
    d = np.abs(a - b).max(axis=1)
    _say(f"  fused vs layerwise: max-abs {d.max():.3e}, {(d > OUT_TOL).sum()} coords beyond {OUT_TOL}")
    assert (d > OUT_TOL).mean() <= FLIP_FRAC
    # running it again gives the same bits (no atomics, no races)
    c = _check_forward(cs, dhq.DHQ_FUSED, "fused again")
    assert np.array_equal(a, c)


@pytest.mark.parametrize("wide_kernel", [1, 2], ids=["one-wave", "two-waves"])
def test_forward_fused_width_512(wide_kernel):
    """The C5 network (hidden width 512, six sine layers) on a strided sample of its grid:
    each of the two fused kernels for wide layers against the oracle and against the layer-by-layer path."""
    _say(f"forward fused width 512, kernel {wide_kernel}")
    cs = case("C5", stride=811)          # 5172 coordinates: 40 full tiles of 128 and a ragged one
    assert cs.model.has_fused()
    cs.model.select_wide_kernel(wide_kernel)
    for l in range(len(cs.dims) - 1):
        assert np.array_equal(cs.model.weight_codes(l), cs.net.Wq[l]), f"layer {l}"
    a = _check_forward(cs, dhq.DHQ_FUSED, "fused-512")
    b = _check_forward(cs, dhq.DHQ_LAYERWISE, "layerwise-512")
    d = np.abs(a - b).max(axis=1)
    _say(f"  fused vs layerwise: max-abs {d.max():.3e}, {(d > OUT_TOL).sum()} coords beyond {OUT_TOL}")
    # two paths with independently rounded transforms: either may have moved a coordinate
    assert (d > OUT_TOL).mean() <= 2 * flip_frac(cs.dims)
    c = _check_forward(cs, dhq.DHQ_FUSED, "fused-512 again")
    assert np.array_equal(a, c)
    # teacher-forced layers through the debug hook (wide WHT and GEMM shapes of the layer-by-layer path)
    torch = _torch()
    for l in (1, len(cs.dims) - 2):
        x = cs.dump.act[l - 1]
        codes, acc, act = cs.model.forward_debug(_dev(x), l)
        torch.cuda.synchronize()
        rate, mx = code_stats(codes.cpu().numpy(), cs.dump.codes[l])
        _say(f"  layer {l}: code mismatch rate {rate:.2e} max {mx}")
        assert rate <= CODE_RATE and mx <= 1
        assert np.array_equal(acc.cpu().numpy(), int_matmul(codes.cpu().numpy(), cs.net.Wq[l]))
    cs.model.select_wide_kernel(0)   # the cached model goes back to the library's default


@pytest.mark.parametrize("name,bits,wide_kernel", [("C3", 8, 0), ("C4", 4, 0), ("C4", 6, 0), ("C4", 8, 0), ("C5", 8, 1), ("C5", 8, 2)])
def test_full_grid_sampled_outputs(name, bits, wide_kernel):
    """The full-size grids, in the launch configuration the benchmark times (one fused launch
    over the whole grid, static scales).  The oracle cannot run millions of coordinates, but
    with static scales every coordinate is independent: it calibrates the scales on a strided
    sub-grid (an oracle-only step), and the library's outputs are compared with the oracle's
    on a random sample of coordinates plus the first and last tiles."""
    torch = _torch()
    _say(f"full grid {name} bits {bits}")
    wl, coords, W, b = synth.make(name)
    n = coords.shape[0]
    net = o.quantize_net(wl.dims, wl.omega0, bits, bits, W, b)
    o.forward(net, coords[:: max(1, n // 8192)], calibrate=True)
    model = dhq.Model(wl.dims, wl.omega0, W, b, bits, bits)
    model.set_act_scales(net.s_a)
    assert model.has_fused()
    if wide_kernel:
        model.select_wide_kernel(wide_kernel)   # hidden width 512: the kernel with one wave per SIMD, then the one with two
    x = _dev(coords)
    out = model.forward(x, flags=dhq.DHQ_FUSED)
    torch.cuda.synchronize()
    rng = np.random.default_rng(17)
    idx = np.unique(np.concatenate([rng.integers(0, n, 6000), np.arange(0, 300), np.arange(n - 300, n)]))
    got = out[torch.from_numpy(idx).to("cuda")].cpu().numpy()
    exp, dmp = o.forward(net, coords[idx], dump=True)
    # every excess tied to a code difference in the kernel's own chain, the differing codes held to the
    # code gate (0.1 %, 1 LSB) where they are teacher-forced comparisons
    err, diff = check_fused_against_oracle(model, net, coords[idx], got, exp, dmp, f"{name} {bits} bits")
    over = err > OUT_TOL
    # coordinates that share their first-layer codes share everything after them; at 4 bits the
    # whole grid collapses to about a hundred such cases, so the coordinates that moved are
    # reported over distinct cases.  Their number is bounded by the cases with a code difference,
    # which the code gate above bounds; it is printed, not fitted with a threshold of its own.
    _, case_of = np.unique(dmp.codes[0], axis=0, return_inverse=True)
    case_of = np.asarray(case_of).reshape(-1)
    n_cases = int(case_of.max()) + 1
    _say(f"  {idx.size} sampled coords ({n_cases} distinct cases): {np.unique(case_of[over]).size} cases beyond {OUT_TOL}, "
         f"{np.unique(case_of[diff]).size} with a code difference")
    # properties that hold at any size: finite everywhere, and a coordinate's value does not
    # depend on which launch or tile it was computed in
    assert bool(torch.isfinite(out).all())
    sub = model.forward(_dev(coords[idx]), flags=dhq.DHQ_FUSED)
    torch.cuda.synchronize()
    assert np.array_equal(sub.cpu().numpy(), got)
    model.close()


@pytest.mark.parametrize("bits", [4, 6])
def test_forward_low_bits(bits):
    _say(f"forward bits {bits}")
    wl, coords, W, b = synth.make("C1")
    cs = Case(wl.dims, coords, W, b, bits=bits)
    _check_forward(cs, dhq.DHQ_LAYERWISE, f"layerwise b{bits}")
    _check_forward(cs, dhq.DHQ_FUSED, f"fused b{bits}")


def test_forward_ragged_and_tiny_sizes():
    """Row counts around every tile size of both paths; each coordinate is independent under
    static scales, so the oracle's rows for the full grid are the expected values."""
    torch = _torch()
    cs = case("C1")
    for n in (1, 2, 31, 33, 255, 256, 257, 1000):
        _say(f"ragged n={n}")
        for flags in (dhq.DHQ_LAYERWISE, dhq.DHQ_FUSED):
            out = cs.model.forward(_dev(cs.coords[:n]), flags=flags)
            torch.cuda.synchronize()
            assert np.abs(out.cpu().numpy().astype(np.float64) - cs.out[:n]).max() <= OUT_TOL
    # n = 0 is a successful no-op
    empty = torch.empty((0, 2), dtype=torch.float32, device="cuda")
    out = cs.model.forward(empty)
    assert out.shape == (0, 3)


def test_forward_generic_shape_layerwise_only():
    """Non power-of-two fan-ins (zero-padding), fan-out that is no multiple of 32."""
    _say("generic shape")
    dims = [3, 48, 100, 5]
    rng = np.random.default_rng(8)
    W, b = synth.siren_init(dims, 30.0, 99)
    coords = rng.uniform(-1, 1, size=(3001, 3)).astype(np.float32)
    cs = Case(dims, coords, W, b)
    _check_forward(cs, dhq.DHQ_LAYERWISE, "generic layerwise")
    _check_forward(cs, dhq.DHQ_AUTO, "generic auto")
    with pytest.raises(dhq.DhqError) as e:
        cs.model.forward(_dev(coords), flags=dhq.DHQ_FUSED)
    assert e.value.status == dhq.DHQ_EUNSUPPORTED


# Sixteen layers is the most a model may have, 512 the widest dimension.  Free-running differences
# grow with depth (a code that differs in layer 2 perturbs every layer after it, and after fifteen
# sine layers the perturbation has passed through fifteen more quantizers), so at this depth the
# strict statements are the teacher-forced ones: every layer's codes within the rate, its
# accumulators exact.  End to end: every coordinate within FLIP_BOUND, every coordinate whose codes
# agree with the oracle's at all layers within OUT_TOL, and the typical coordinate far inside it.
@pytest.mark.parametrize("dims", [[4] + [256] * 15 + [32], [2] + [512] * 15 + [3], [512] * 17], ids=["256x15", "512x15", "512-512x15-512"])
def test_sixteen_layers_and_widest_dimensions(dims):
    torch = _torch()
    _say(f"limits: {dims[0]}-{dims[1]}x{len(dims) - 2}-{dims[-1]}")
    W, b = synth.siren_init(dims, 30.0, 1000 + len(dims) + dims[1])
    rng = np.random.default_rng(5)
    coords = rng.uniform(-1, 1, size=(1500 + 7, dims[0])).astype(np.float32)
    cs = Case(dims, coords, W, b)
    L = len(dims) - 1
    assert cs.model.has_fused() == (dims[0] <= 4)
    for l in range(L):
        assert np.array_equal(cs.model.weight_codes(l), cs.net.Wq[l]), f"weight codes of layer {l}"
    worst = 0.0
    for l in range(L):
        x = coords if l == 0 else cs.dump.act[l - 1]
        codes, acc, act = cs.model.forward_debug(_dev(x), l)
        torch.cuda.synchronize()
        codes, acc = codes.cpu().numpy(), acc.cpu().numpy()
        rate, mx = code_stats(codes, cs.dump.codes[l])
        worst = max(worst, rate)
        assert rate <= CODE_RATE and mx <= 1, f"layer {l}"
        assert np.array_equal(acc, int_matmul(codes, cs.net.Wq[l])), f"layer {l}"
    _say(f"  teacher-forced: worst code mismatch rate {worst:.2e}")
    diff = _coords_with_code_diffs(cs, coords.shape[0])
    paths = [("layerwise", dhq.DHQ_LAYERWISE)] + ([("fused", dhq.DHQ_FUSED)] if cs.model.has_fused() else [])
    for label, flags in paths:
        out = cs.model.forward(_dev(coords), flags=flags)
        torch.cuda.synchronize()
        err = np.abs(out.cpu().numpy().astype(np.float64) - cs.out).max(axis=1)
        _say(f"  {label}: max-abs err {err.max():.3e}, median {np.median(err):.3e}, {(err > OUT_TOL).sum()} of {err.size} "
             f"beyond {OUT_TOL}; {diff.sum()} coords with a code difference somewhere")
        assert err.max() <= FLIP_BOUND and np.median(err) <= OUT_TOL / 4
        if flags == dhq.DHQ_LAYERWISE:
            assert err[~diff].max() <= OUT_TOL and diff[err > OUT_TOL].all()
    cs.model.close()


def test_clamp_outside_calibrated_range():
    """Coordinates beyond the calibration grid drive codes into the clamp."""
    _say("clamp")
    torch = _torch()
    cs = case("C1")
    rng = np.random.default_rng(2)
    coords = rng.uniform(-3, 3, size=(2000, 2)).astype(np.float32)
    exp = o.forward(cs.net, coords)
    for flags in (dhq.DHQ_LAYERWISE, dhq.DHQ_FUSED):
        out = cs.model.forward(_dev(coords), flags=flags)
        torch.cuda.synchronize()
        _assert_close(out.cpu().numpy(), exp)


# ------------------------------------------------------------------------------ calibration
@pytest.mark.parametrize("name", ["C1", "C2"])
def test_calibrate_matches_oracle_scales(name):
    _say(f"calibrate {name}")
    torch = _torch()
    cs = case(name)
    m = dhq.Model(cs.dims, 30.0, cs.W, cs.b, cs.bits, cs.bits)
    with pytest.raises(dhq.DhqError) as e:
        m.forward(_dev(cs.coords[:10]))
    assert e.value.status == dhq.DHQ_ENOSCALE
    m.calibrate(_dev(cs.coords))
    _, sa = m.scales()
    rel = np.abs(sa.astype(np.float64) - cs.net.s_a) / cs.net.s_a
    _say(f"  scales rel err {rel}")
    assert (rel <= 1e-5).all()
    out = m.forward(_dev(cs.coords))
    torch.cuda.synchronize()
    _assert_close(out.cpu().numpy(), cs.out, strict=(name == "C1"))


def test_error_paths():
    torch = _torch()
    cs = case("C1")
    with pytest.raises(dhq.DhqError) as e:
        cs.model.set_act_scales([0.1, 0.0, 0.1, 0.1])
    assert e.value.status == dhq.DHQ_EINVAL
    with pytest.raises(dhq.DhqError):
        cs.model.set_act_scales([0.1, float("nan"), 0.1, 0.1])
    cs.model.set_act_scales(cs.net.s_a)
    x = torch.zeros((4, 2), device="cuda")
    with pytest.raises(dhq.DhqError):
        dhq.dhq_forward(cs.model.handle, x, torch.empty((4, 3), device="cuda"), flags=7)
    with pytest.raises(dhq.DhqError):
        dhq.dhq_forward_debug(cs.model.handle, x, 9)
