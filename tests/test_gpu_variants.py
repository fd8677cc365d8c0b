"""GPU parity of the two variants built on top of the base path, against the CPU oracle:

  * two-sided rotation (Eq. 4-5 as printed): weights rotated over input and output features,
    the output side undone exactly in int32 after the GEMM;
  * dynamic activation scales (Sec. 3.3): every layer's scale measured on line on the batch.

Same gates as the base path: integer stages bit-exact, codes <= 0.1 % off by <= 1 LSB when
teacher-forced, final values within 2e-3 (see test_gpu_parity.py for the free-running rule).
"""
import numpy as np
import pytest

import paper_2508_13478_amd as dhq
from oracle import dhq_oracle as o
from paper_2508_13478_amd import synth
from test_gpu_parity import (CODE_RATE, FLIP_BOUND, OUT_TOL, _dev, _say, _torch, code_stats, flip_frac, int_matmul,
                             int_unrotate)

pytestmark = pytest.mark.gpu


class TwoSided:
    def __init__(self, dims, coords, W, b, bits=8, omega0=30.0):
        self.dims, self.coords = list(dims), coords
        self.net = o.quantize_net(dims, omega0, bits, bits, W, b, two_sided=True)
        self.out, self.dump = o.forward(self.net, coords, calibrate=True, dump=True)
        self.model = dhq.Model(dims, omega0, W, b, bits, bits, mode=dhq.DHQ_ROTATE_BOTH)
        self.model.set_act_scales(self.net.s_a)


_cache = {}


def two_sided(name, stride=1):
    if (name, stride) not in _cache:
        wl, coords, W, b = synth.make(name)
        _cache[(name, stride)] = TwoSided(wl.dims, coords[::stride], W, b)
    return _cache[(name, stride)]


def _gate(out, exp, dims, strict, label):
    err = np.abs(out.astype(np.float64) - exp).max(axis=1)
    over = err > OUT_TOL
    _say(f"  {label}: max-abs err {err.max():.3e}, {over.sum()} of {err.size} coords beyond {OUT_TOL}")
    if strict:
        assert not over.any()
    else:
        assert over.mean() <= flip_frac(dims) and err.max() <= FLIP_BOUND


# ------------------------------------------------------------------------ two-sided rotation
@pytest.mark.parametrize("name", ["C1", "C2"])
def test_two_sided_weight_codes_bit_identical(name):
    _say(f"two-sided weights {name}")
    cs = two_sided(name)
    sw, sa = cs.model.scales()
    assert np.array_equal(sw, cs.net.s_w) and np.array_equal(sa, cs.net.s_a)
    for l in range(len(cs.dims) - 1):
        q = cs.model.weight_codes(l)
        assert q.shape == cs.net.Wq[l].shape and np.array_equal(q, cs.net.Wq[l]), f"layer {l}"
    assert cs.model.has_fused()


def test_two_sided_weight_codes_odd_shapes():
    dims = [3, 48, 100, 5]
    W, b = synth.siren_init(dims, 30.0, 4242)
    for bits in (4, 6, 8):
        net = o.quantize_net(dims, 30.0, bits, bits, W, b, two_sided=True)
        m = dhq.Model(dims, 30.0, W, b, bits, bits, mode=dhq.DHQ_ROTATE_BOTH)
        sw, _ = m.scales()
        assert np.array_equal(sw, net.s_w)
        for l in range(3):
            assert np.array_equal(m.weight_codes(l), net.Wq[l])


@pytest.mark.parametrize("name", ["C1", "C2"])
def test_two_sided_layers_teacher_forced(name):
    torch = _torch()
    cs = two_sided(name)
    rows = min(cs.coords.shape[0], 20000 + 13)
    for l in range(len(cs.dims) - 1):
        _say(f"two-sided layer {name} {l}")
        M = cs.dims[l + 1]
        # integer GEMM alone on the oracle's codes: rotated accumulators, bit-exact
        acc_r = cs.model.gemm_i8(l, _dev(cs.dump.codes[l][:rows]))
        torch.cuda.synchronize()
        assert np.array_equal(acc_r.cpu().numpy(), cs.dump.acc[l][:rows])
        # the whole layer on the oracle's fp32 input
        x = cs.coords[:rows] if l == 0 else cs.dump.act[l - 1][:rows]
        codes, z, act = cs.model.forward_debug(_dev(x), l)
        torch.cuda.synchronize()
        codes, z, act = codes.cpu().numpy(), z.cpu().numpy(), act.cpu().numpy()
        rate, mx = code_stats(codes, cs.dump.codes[l][:rows])
        _say(f"  code mismatch rate {rate:.2e} max {mx}")
        assert rate <= CODE_RATE and mx <= 1
        # the un-rotation is exact for the codes the library produced
        assert np.array_equal(z, int_unrotate(int_matmul(codes, cs.net.Wq[l])))
        same = (codes == cs.dump.codes[l][:rows]).all(axis=1)
        err = np.abs(act[same].astype(np.float64) - cs.dump.act[l][:rows][same]).max()
        _say(f"  epilogue max-abs err {err:.2e}")
        assert act.shape[1] == M and err <= 2e-5


@pytest.mark.parametrize("name", ["C1", "C2"])
def test_two_sided_forward(name):
    torch = _torch()
    _say(f"two-sided forward {name}")
    cs = two_sided(name)
    lw = cs.model.forward(_dev(cs.coords), flags=dhq.DHQ_LAYERWISE)
    fu = cs.model.forward(_dev(cs.coords), flags=dhq.DHQ_FUSED)
    auto = cs.model.forward(_dev(cs.coords))             # picks the fused kernel
    torch.cuda.synchronize()
    lw, fu = lw.cpu().numpy(), fu.cpu().numpy()
    assert np.array_equal(fu, auto.cpu().numpy())
    _gate(lw, cs.out, cs.dims, name == "C1", "two-sided layer-by-layer")
    _gate(fu, cs.out, cs.dims, name == "C1", "two-sided fused")
    d = np.abs(lw - fu).max(axis=1)
    _say(f"  fused vs layer-by-layer: max-abs {d.max():.3e}, {(d > OUT_TOL).sum()} coords beyond {OUT_TOL}")
    assert (d > OUT_TOL).mean() <= flip_frac(cs.dims)


@pytest.mark.parametrize("dims", [[2, 32, 32, 3], [3, 64, 64, 64, 1], [4, 128, 128, 2], [2, 256, 256, 256, 256, 256, 4],
                                  [2, 64, 64, 5], [3, 128, 128, 128, 12], [2, 256, 256, 256, 17], [4, 32, 32, 32]])
def test_two_sided_fused_shapes_and_ragged_rows(dims):
    torch = _torch()
    W, b = synth.siren_init(dims, 30.0, 31 + len(dims))
    rng = np.random.default_rng(dims[1])
    x = rng.uniform(-1, 1, size=(3000 + 45, dims[0])).astype(np.float32)
    net = o.quantize_net(dims, 30.0, 8, 8, W, b, two_sided=True)
    exp = o.forward(net, x, calibrate=True)
    m = dhq.Model(dims, 30.0, W, b, mode=dhq.DHQ_ROTATE_BOTH)
    assert m.has_fused()
    m.set_act_scales(net.s_a)
    for n in (1, 257, x.shape[0]):
        _say(f"two-sided fused dims {dims} n={n}")
        out = m.forward(_dev(x[:n]), flags=dhq.DHQ_FUSED)
        torch.cuda.synchronize()
        _gate(out.cpu().numpy(), exp[:n], dims, False, f"n={n}")
    # a fan-out above 32 has no fused kernel
    dims33 = dims[:-1] + [33]
    W33, b33 = synth.siren_init(dims33, 30.0, 7)
    assert not dhq.Model(dims33, 30.0, W33, b33, mode=dhq.DHQ_ROTATE_BOTH).has_fused()


def test_two_sided_sixteen_layers():
    """The deepest model the library takes, two-sided: the un-rotation's int32 sums are largest here
    relative to nothing (they do not grow with depth), but every layer's descriptor slot is used.
    Strict statements teacher-forced per layer; end to end as in the one-sided test of the limits."""
    torch = _torch()
    dims = [4] + [256] * 15 + [4]
    W, b = synth.siren_init(dims, 30.0, 1016)
    rng = np.random.default_rng(6)
    coords = rng.uniform(-1, 1, size=(1500 + 7, 4)).astype(np.float32)
    cs = TwoSided(dims, coords, W, b)
    assert cs.model.has_fused()
    for l in range(len(dims) - 1):
        _say(f"two-sided 16 layers: layer {l}")
        assert np.array_equal(cs.model.weight_codes(l), cs.net.Wq[l])
        x = coords if l == 0 else cs.dump.act[l - 1]
        codes, z, act = cs.model.forward_debug(_dev(x), l)
        torch.cuda.synchronize()
        codes, z = codes.cpu().numpy(), z.cpu().numpy()
        rate, mx = code_stats(codes, cs.dump.codes[l])
        assert rate <= CODE_RATE and mx <= 1
        assert np.array_equal(z, int_unrotate(int_matmul(codes, cs.net.Wq[l])))
    x = _dev(coords)
    for label, flags in (("layerwise", dhq.DHQ_LAYERWISE), ("fused", dhq.DHQ_FUSED)):
        out = cs.model.forward(x, flags=flags)
        torch.cuda.synchronize()
        err = np.abs(out.cpu().numpy().astype(np.float64) - cs.out).max(axis=1)
        _say(f"  {label}: max-abs err {err.max():.3e}, median {np.median(err):.3e}, {(err > OUT_TOL).sum()} of {err.size} beyond {OUT_TOL}")
        assert err.max() <= FLIP_BOUND and np.median(err) <= OUT_TOL / 4
    # the per-layer kernels of the dynamic mode at this depth: same bits as the whole-network kernel with their scales
    dyn = cs.model.forward(x, flags=dhq.DHQ_FUSED | dhq.DHQ_DYNAMIC)
    cs.model.set_act_scales(cs.model.dynamic_scales())
    sta = cs.model.forward(x, flags=dhq.DHQ_FUSED)
    torch.cuda.synchronize()
    assert np.array_equal(dyn.cpu().numpy(), sta.cpu().numpy())
    cs.model.close()


def test_two_sided_forward_odd_shapes_ragged_rows_and_chunks():
    torch = _torch()
    dims = [3, 48, 100, 5]
    W, b = synth.siren_init(dims, 30.0, 4242)
    rng = np.random.default_rng(8)
    for n in (1, 129, 70001):                      # 70001 rows: more than one workspace chunk
        _say(f"two-sided odd shapes n={n}")
        x = rng.uniform(-1, 1, size=(n, 3)).astype(np.float32)
        net = o.quantize_net(dims, 30.0, 8, 8, W, b, two_sided=True)
        exp = o.forward(net, x, calibrate=True)
        m = dhq.Model(dims, 30.0, W, b, mode=dhq.DHQ_ROTATE_BOTH)
        m.set_act_scales(net.s_a)
        out = m.forward(_dev(x))
        torch.cuda.synchronize()
        _gate(out.cpu().numpy(), exp, dims, n < 1000, f"n={n}")


# ---------------------------------------------------------------------------- dynamic scales
@pytest.mark.parametrize("name,mode", [("C1", dhq.DHQ_ROTATE_IN), ("C2", dhq.DHQ_ROTATE_IN), ("C3", dhq.DHQ_ROTATE_IN),
                                       ("C2", dhq.DHQ_ROTATE_BOTH)])
def test_dynamic_forward_equals_calibrate_then_static(name, mode):
    """On the same batch the on-line scales are the calibrated ones, so the two runs give the
    same bits; against the oracle (which measures its scales the same way) the usual gates hold."""
    torch = _torch()
    _say(f"dynamic {name} mode {mode}")
    wl, coords, W, b = synth.make(name)
    if name == "C3":
        coords = coords[:100000 + 37]                    # more than one workspace chunk, ragged
    x = _dev(coords)
    m = dhq.Model(wl.dims, wl.omega0, W, b, mode=mode)
    dyn = m.forward(x, flags=dhq.DHQ_LAYERWISE | dhq.DHQ_DYNAMIC)   # no static scales needed
    s_dyn = m.dynamic_scales()
    m.calibrate(x)
    _, s_cal = m.scales()
    sta = m.forward(x, flags=dhq.DHQ_LAYERWISE)
    torch.cuda.synchronize()
    assert np.array_equal(s_dyn, s_cal)
    assert np.array_equal(dyn.cpu().numpy(), sta.cpu().numpy())
    net = o.quantize_net(wl.dims, wl.omega0, 8, 8, W, b, two_sided=(mode == dhq.DHQ_ROTATE_BOTH))
    exp = o.forward(net, coords, calibrate=True)
    rel = np.abs(s_dyn.astype(np.float64) - net.s_a) / net.s_a
    _say(f"  scale rel err max {rel.max():.2e}")
    assert rel.max() <= 1e-5
    # the oracle ran with its own scales; a last-bit difference in a scale moves codes that sit on a
    # rounding boundary, which the free-running gate allows for
    _gate(dyn.cpu().numpy(), exp, wl.dims, False, "dynamic vs oracle")


@pytest.mark.parametrize("name", ["C1", "C2", "C3"])
def test_dynamic_per_layer_fused_equals_static_fused_with_its_scales(name):
    """The one-kernel-per-layer realisation of the dynamic mode: it runs the fused kernel's own
    arithmetic, so a static fused forward with the scales it measured gives the same bits; the scales
    agree with the oracle's (and with the layer-by-layer dynamic path's) to fp32 rounding."""
    torch = _torch()
    _say(f"dynamic per-layer fused {name}")
    wl, coords, W, b = synth.make(name)
    if name == "C3":
        coords = coords[:100000 + 37]                    # several passes per workgroup, ragged tail
    x = _dev(coords)
    m = dhq.Model(wl.dims, wl.omega0, W, b)
    dyn = m.forward(x, flags=dhq.DHQ_FUSED | dhq.DHQ_DYNAMIC)
    s_dyn = m.dynamic_scales()
    auto = m.forward(x, flags=dhq.DHQ_DYNAMIC)                      # AUTO picks the same kernels
    lw = m.forward(x, flags=dhq.DHQ_LAYERWISE | dhq.DHQ_DYNAMIC)
    s_lw = m.dynamic_scales()
    m.set_act_scales(s_dyn)
    sta = m.forward(x, flags=dhq.DHQ_FUSED)
    torch.cuda.synchronize()
    assert np.array_equal(dyn.cpu().numpy(), sta.cpu().numpy())
    assert np.array_equal(dyn.cpu().numpy(), auto.cpu().numpy())
    net = o.quantize_net(wl.dims, wl.omega0, 8, 8, W, b)
    exp = o.forward(net, coords, calibrate=True)
    rel = np.abs(s_dyn.astype(np.float64) - net.s_a) / net.s_a
    _say(f"  scale rel err vs oracle max {rel.max():.2e}; vs layer-by-layer {np.abs(s_dyn / s_lw - 1).max():.2e}")
    assert rel.max() <= 1e-5 and np.abs(s_dyn / s_lw - 1).max() <= 1e-5
    _gate(dyn.cpu().numpy(), exp, wl.dims, False, "dynamic per-layer fused vs oracle")
    d = np.abs(dyn.cpu().numpy() - lw.cpu().numpy()).max(axis=1)
    assert (d > OUT_TOL).mean() <= 2 * 1e-3
    m.close()


@pytest.mark.parametrize("dims", [[2, 32, 32, 3], [3, 64, 64, 64, 5], [4, 128, 128, 2], [1, 256, 256, 32], [2, 64, 1],
                                  [3, 512, 512, 5], [2, 512, 512, 512, 512, 32]])
def test_dynamic_per_layer_fused_shapes_and_ragged_rows(dims):
    torch = _torch()
    W, b = synth.siren_init(dims, 30.0, 123 + len(dims))
    m = dhq.Model(dims, 30.0, W, b)
    net = o.quantize_net(dims, 30.0, 8, 8, W, b)
    rng = np.random.default_rng(dims[1] + 1)
    for n in (1, 257, 3000 + 11):
        _say(f"dynamic per-layer fused dims {dims} n={n}")
        xs = rng.uniform(-1, 1, size=(n, dims[0])).astype(np.float32)
        exp = o.forward(net, xs, calibrate=True)
        dyn = m.forward(_dev(xs), flags=dhq.DHQ_FUSED | dhq.DHQ_DYNAMIC)
        s_dyn = m.dynamic_scales()
        torch.cuda.synchronize()
        assert (np.abs(s_dyn.astype(np.float64) - net.s_a) / net.s_a).max() <= 1e-5
        _gate(dyn.cpu().numpy(), exp, dims, False, f"dims {dims} n={n}")
    m.close()


@pytest.mark.parametrize("bits", [8, 6])
def test_dynamic_per_layer_fused_width_512_equals_static_fused_with_its_scales(bits):
    """Width 512: one launch per layer of the two-wave whole-network kernel's own layer code, so a static forward of
    that kernel with the scales measured on line gives the same bits.  The C5 network on a strided part of its
    grid: several passes per workgroup, a ragged last tile."""
    torch = _torch()
    wl, coords, W, b = synth.make("C5")
    coords = np.ascontiguousarray(coords[::113][:128 * 290 + 77])
    _say(f"dynamic per-layer fused C5 network, {coords.shape[0]} coords, {bits} bits")
    x = _dev(coords)
    m = dhq.Model(wl.dims, wl.omega0, W, b, bits, bits)
    dyn = m.forward(x, flags=dhq.DHQ_FUSED | dhq.DHQ_DYNAMIC)
    s_dyn = m.dynamic_scales()
    auto = m.forward(x, flags=dhq.DHQ_DYNAMIC)                      # AUTO picks the same kernels
    lw = m.forward(x, flags=dhq.DHQ_LAYERWISE | dhq.DHQ_DYNAMIC)
    s_lw = m.dynamic_scales()
    m.set_act_scales(s_dyn)
    m.select_wide_kernel(2)
    sta = m.forward(x, flags=dhq.DHQ_FUSED)
    torch.cuda.synchronize()
    assert np.array_equal(dyn.cpu().numpy(), sta.cpu().numpy())
    assert np.array_equal(dyn.cpu().numpy(), auto.cpu().numpy())
    sub = slice(0, None, 4)                                          # the oracle on a quarter of them, with the scales of all
    net = o.quantize_net(wl.dims, wl.omega0, bits, bits, W, b)
    o.forward(net, coords, calibrate=True)
    exp = o.forward(net, coords[sub])
    rel = np.abs(s_dyn.astype(np.float64) - net.s_a) / net.s_a
    _say(f"  scale rel err vs oracle max {rel.max():.2e}; vs layer-by-layer {np.abs(s_dyn / s_lw - 1).max():.2e}")
    # a layer's maximum is one coordinate's value: at 6 bits a code that fp32 and fp64 round differently upstream of
    # that coordinate moves it (and the scale with it) by a fraction of a quantization step; at 8 bits none does here
    tol = 1e-5 if bits == 8 else 1e-2
    assert rel[:2].max() <= 1e-5 and rel.max() <= tol and np.abs(s_dyn / s_lw - 1).max() <= tol
    if bits == 8:
        _gate(dyn.cpu().numpy()[sub], exp, wl.dims, False, "dynamic per-layer fused width 512 vs oracle")
        d = np.abs(dyn.cpu().numpy() - lw.cpu().numpy()).max(axis=1)
        assert (d > OUT_TOL).mean() <= 2 * flip_frac(wl.dims)
    else:
        # with a scale that differs in the third digit the last quantizer's codes differ for a share of the coordinates:
        # both are valid forwards with on-line scales; the outputs stay within the quantization error of each other
        err = np.abs(dyn.cpu().numpy()[sub].astype(np.float64) - exp).max(axis=1)
        _say(f"  against the oracle with its own scales: max {err.max():.2e}, median {np.median(err):.1e}, {(err > OUT_TOL).sum()} of {err.size} beyond {OUT_TOL}")
        assert err.max() <= FLIP_BOUND and np.median(err) <= 1e-3
    m.close()


@pytest.mark.parametrize("bits", [4, 6])
def test_dynamic_per_layer_fused_low_bits(bits):
    torch = _torch()
    _say(f"dynamic per-layer fused bits {bits}")
    wl, coords, W, b = synth.make("C1")
    m = dhq.Model(wl.dims, wl.omega0, W, b, bits, bits)
    net = o.quantize_net(wl.dims, wl.omega0, bits, bits, W, b)
    exp = o.forward(net, coords, calibrate=True)
    x = _dev(coords)
    dyn = m.forward(x, flags=dhq.DHQ_FUSED | dhq.DHQ_DYNAMIC)
    s_dyn = m.dynamic_scales()
    m.set_act_scales(s_dyn)
    sta = m.forward(x, flags=dhq.DHQ_FUSED)
    torch.cuda.synchronize()
    assert np.array_equal(dyn.cpu().numpy(), sta.cpu().numpy())
    assert (np.abs(s_dyn.astype(np.float64) - net.s_a) / net.s_a).max() <= 1e-5
    _gate(dyn.cpu().numpy(), exp, wl.dims, False, f"bits {bits}")
    m.close()


@pytest.mark.parametrize("name", ["C1", "C2"])
def test_dynamic_per_layer_fused_two_sided_equals_static_fused_with_its_scales(name):
    """The same cut for the two-sided variant: one kernel per layer that runs the two-sided fused
    kernel's arithmetic, hence the same bits as that kernel with the measured scales."""
    torch = _torch()
    _say(f"dynamic per-layer fused two-sided {name}")
    wl, coords, W, b = synth.make(name)
    x = _dev(coords)
    m = dhq.Model(wl.dims, wl.omega0, W, b, mode=dhq.DHQ_ROTATE_BOTH)
    dyn = m.forward(x, flags=dhq.DHQ_FUSED | dhq.DHQ_DYNAMIC)
    s_dyn = m.dynamic_scales()
    auto = m.forward(x, flags=dhq.DHQ_DYNAMIC)
    lw = m.forward(x, flags=dhq.DHQ_LAYERWISE | dhq.DHQ_DYNAMIC)
    s_lw = m.dynamic_scales()
    m.set_act_scales(s_dyn)
    sta = m.forward(x, flags=dhq.DHQ_FUSED)
    torch.cuda.synchronize()
    assert np.array_equal(dyn.cpu().numpy(), sta.cpu().numpy())
    assert np.array_equal(dyn.cpu().numpy(), auto.cpu().numpy())
    net = o.quantize_net(wl.dims, wl.omega0, 8, 8, W, b, two_sided=True)
    exp = o.forward(net, coords, calibrate=True)
    rel = np.abs(s_dyn.astype(np.float64) - net.s_a) / net.s_a
    _say(f"  scale rel err vs oracle max {rel.max():.2e}; vs layer-by-layer {np.abs(s_dyn / s_lw - 1).max():.2e}")
    assert rel.max() <= 1e-5 and np.abs(s_dyn / s_lw - 1).max() <= 1e-5
    _gate(dyn.cpu().numpy(), exp, wl.dims, False, "dynamic per-layer fused two-sided vs oracle")
    d = np.abs(dyn.cpu().numpy() - lw.cpu().numpy()).max(axis=1)
    assert (d > OUT_TOL).mean() <= 2 * 1e-3
    m.close()


@pytest.mark.parametrize("dims", [[2, 32, 32, 3], [3, 64, 64, 64, 1], [4, 128, 128, 2], [1, 256, 256, 4]])
def test_dynamic_per_layer_fused_two_sided_shapes_and_ragged_rows(dims):
    torch = _torch()
    W, b = synth.siren_init(dims, 30.0, 223 + len(dims))
    m = dhq.Model(dims, 30.0, W, b, mode=dhq.DHQ_ROTATE_BOTH)
    net = o.quantize_net(dims, 30.0, 8, 8, W, b, two_sided=True)
    rng = np.random.default_rng(dims[1] + 2)
    for n in (1, 257, 3000 + 11):
        _say(f"dynamic per-layer fused two-sided dims {dims} n={n}")
        xs = rng.uniform(-1, 1, size=(n, dims[0])).astype(np.float32)
        exp = o.forward(net, xs, calibrate=True)
        dyn = m.forward(_dev(xs), flags=dhq.DHQ_FUSED | dhq.DHQ_DYNAMIC)
        s_dyn = m.dynamic_scales()
        torch.cuda.synchronize()
        assert (np.abs(s_dyn.astype(np.float64) - net.s_a) / net.s_a).max() <= 1e-5
        _gate(dyn.cpu().numpy(), exp, dims, False, f"dims {dims} n={n}")
    m.close()


@pytest.mark.parametrize("mode", [dhq.DHQ_ROTATE_IN, dhq.DHQ_ROTATE_BOTH], ids=["one_sided", "two_sided"])
def test_dynamic_whole_batch_buffers_beyond_4_gib(mode):
    """4.2 million coordinates through a 256-wide network: each whole-batch buffer of transformed
    activations is 4.3 GB, so byte offsets pass 2^32.  The batch is 64 copies of one block of 65 573
    coordinates plus a ragged piece of it: its per-tensor maxima are the block's, so the oracle's
    calibrating forward on the block gives the scales and every row's expected value.  Checked: the
    copies come out bit-identical to the first block wherever they sit, the per-layer kernels give
    the bits of the whole-network kernel with their scales, scales and values match the oracle's."""
    torch = _torch()
    dims = [2, 256, 256, 256, 3]
    nb, copies, tail = 65536 + 37, 64, 37
    _say(f"dynamic beyond 4 GiB, mode {mode}, n = {nb * copies + tail}")
    W, b = synth.siren_init(dims, 30.0, 4096)
    rng = np.random.default_rng(12)
    block = rng.uniform(-1, 1, size=(nb, 2)).astype(np.float32)
    net = o.quantize_net(dims, 30.0, 8, 8, W, b, two_sided=(mode == dhq.DHQ_ROTATE_BOTH))
    exp = o.forward(net, block, calibrate=True)
    xb = _dev(block)
    x = torch.cat([xb] * copies + [xb[:tail]])
    n = x.shape[0]
    assert n * 256 * 4 > (1 << 32)
    m = dhq.Model(dims, 30.0, W, b, mode=mode)
    dyn = m.forward(x, flags=dhq.DHQ_FUSED | dhq.DHQ_DYNAMIC)
    s_dyn = m.dynamic_scales()
    lw = m.forward(x, flags=dhq.DHQ_LAYERWISE | dhq.DHQ_DYNAMIC)
    s_lw = m.dynamic_scales()
    m.set_act_scales(s_dyn)
    sta = m.forward(x, flags=dhq.DHQ_FUSED)
    torch.cuda.synchronize()
    for out, label in ((dyn, "per-layer fused"), (lw, "layer by layer")):
        first = out[:nb]
        for k in range(1, copies):
            assert bool((out[k * nb:(k + 1) * nb] == first).all()), f"{label}: copy {k}"
        assert bool((out[copies * nb:] == first[:tail]).all()), f"{label}: ragged piece"
    assert bool((dyn == sta).all())
    rel = np.abs(s_dyn.astype(np.float64) - net.s_a) / net.s_a
    _say(f"  scale rel err vs oracle max {rel.max():.2e}; vs layer-by-layer {np.abs(s_dyn / s_lw - 1).max():.2e}")
    assert rel.max() <= 1e-5 and np.abs(s_dyn / s_lw - 1).max() <= 1e-5
    _gate(dyn[:nb].cpu().numpy(), exp, dims, False, "per-layer fused, first block vs oracle")
    _gate(lw[:nb].cpu().numpy(), exp, dims, False, "layer by layer, first block vs oracle")
    m.close()


def test_dynamic_width_512_at_the_full_size_of_the_largest_workload():
    """The C5 network with on-line scales on as many coordinates as its grid has (4.2 million: 128 passes for every
    workgroup of the per-layer kernels, each whole-batch buffer 8.6 GB), in the launch configuration bench.py
    times with --variant dynamic.  The batch is 128 copies of one block of 32 813 coordinates of the grid plus a
    ragged piece, so that the oracle's calibrating forward on the block gives the scales and every expected value."""
    torch = _torch()
    wl, coords, W, b = synth.make("C5")
    nb, copies, tail = 32768 + 45, 128, 19
    block = np.ascontiguousarray(coords[::127][:nb])
    assert block.shape[0] == nb
    _say(f"dynamic width 512 at full size, n = {nb * copies + tail}")
    net = o.quantize_net(wl.dims, wl.omega0, 8, 8, W, b)
    exp = o.forward(net, block, calibrate=True)
    xb = _dev(block)
    x = torch.cat([xb] * copies + [xb[:tail]])
    m = dhq.Model(wl.dims, wl.omega0, W, b)
    dyn = m.forward(x, flags=dhq.DHQ_FUSED | dhq.DHQ_DYNAMIC)
    s_dyn = m.dynamic_scales()
    m.set_act_scales(s_dyn)
    m.select_wide_kernel(2)
    sta = m.forward(x, flags=dhq.DHQ_FUSED)
    torch.cuda.synchronize()
    first = dyn[:nb]
    for k in range(1, copies):
        assert bool((dyn[k * nb:(k + 1) * nb] == first).all()), f"copy {k}"
    assert bool((dyn[copies * nb:] == first[:tail]).all()), "ragged piece"
    assert bool((dyn == sta).all())
    rel = np.abs(s_dyn.astype(np.float64) - net.s_a) / net.s_a
    _say(f"  scale rel err vs oracle max {rel.max():.2e}")
    assert rel.max() <= 1e-5
    _gate(first.cpu().numpy(), exp, wl.dims, False, "per-layer kernels at full size, first block vs oracle")
    m.close()


def test_dynamic_scales_follow_the_batch_and_workspace_grows():
    torch = _torch()
    wl, coords, W, b = synth.make("C2")
    m = dhq.Model(wl.dims, wl.omega0, W, b)
    small = _dev(coords[:1000])
    out_small = m.forward(small, flags=dhq.DHQ_DYNAMIC)            # AUTO | DYNAMIC -> one kernel per layer
    s_small = m.dynamic_scales()
    full = m.forward(_dev(coords), flags=dhq.DHQ_DYNAMIC)          # the workspace grows here
    s_full = m.dynamic_scales()
    out_small2 = m.forward(small, flags=dhq.DHQ_DYNAMIC)           # and is reused here
    torch.cuda.synchronize()
    assert np.isfinite(full.cpu().numpy()).all()
    assert (s_small <= s_full).all() and (s_small < s_full).any()  # a subset cannot have a larger absmax
    assert np.array_equal(out_small.cpu().numpy(), out_small2.cpu().numpy())
    net = o.quantize_net(wl.dims, wl.omega0, 8, 8, W, b)
    exp = o.forward(net, coords[:1000], calibrate=True)
    _gate(out_small.cpu().numpy(), exp, wl.dims, False, "dynamic subset vs oracle")


def test_dynamic_all_zero_layer_input_gets_scale_one():
    torch = _torch()
    dims = [2, 64, 3]
    W, b = synth.siren_init(dims, 30.0, 77)
    m = dhq.Model(dims, 30.0, W, b)
    x = np.zeros((300, 2), dtype=np.float32)
    out = m.forward(_dev(x), flags=dhq.DHQ_DYNAMIC)
    s = m.dynamic_scales()
    torch.cuda.synchronize()
    assert s[0] == 1.0
    net = o.quantize_net(dims, 30.0, 8, 8, W, b)
    exp = o.forward(net, x, calibrate=True)
    assert net.s_a[0] == 1.0
    assert np.abs(out.cpu().numpy() - exp).max() <= OUT_TOL


def test_variant_flags_are_checked():
    wl, coords, W, b = synth.make("C1")
    m = dhq.Model(wl.dims, wl.omega0, W, b)
    x = _dev(coords[:64])
    for flags, status in ((8, dhq.DHQ_EINVAL), (3, dhq.DHQ_EINVAL)):
        with pytest.raises(dhq.DhqError) as e:
            m.forward(x, flags=flags)
        assert e.value.status == status
    # the per-layer fused kernels of the dynamic mode exist where the whole-network kernels do: two-sided up to width 256
    # and fan-out 32
    wide_dims = [2, 512, 512, 3]
    Ww, bw = synth.siren_init(wide_dims, 30.0, 3)
    out33 = list(wl.dims[:-1]) + [33]
    W33, b33 = synth.siren_init(out33, 30.0, 3)
    for mm in (dhq.Model(out33, wl.omega0, W33, b33, mode=dhq.DHQ_ROTATE_BOTH), dhq.Model(wide_dims, 30.0, Ww, bw, mode=dhq.DHQ_ROTATE_BOTH)):
        with pytest.raises(dhq.DhqError) as e:
            mm.forward(x, flags=dhq.DHQ_FUSED | dhq.DHQ_DYNAMIC)
        assert e.value.status == dhq.DHQ_EUNSUPPORTED
        mm.close()
    with pytest.raises(dhq.DhqError) as e:
        m.forward(x)                                           # static path without scales
    assert e.value.status == dhq.DHQ_ENOSCALE
    with pytest.raises(dhq.DhqError) as e:
        dhq.Model(wl.dims, wl.omega0, W, b, mode=2)
    assert e.value.status == dhq.DHQ_EINVAL


# --------------------------------------------- floating-point activations (W32A32, W8A32)
FLOAT_TOL = 1e-6    # fp32 MFMA accumulation + hardware sine against the fp64 oracle (outputs are O(0.1); measured 1.3e-7)


@pytest.mark.parametrize("name", ["C1", "C2"])
def test_w32a32_forward(name):
    torch = _torch()
    _say(f"W32A32 {name}")
    wl, coords, W, b = synth.make(name)
    exp, _ = o.mlp_float(wl.dims, wl.omega0, W, b, coords)
    m = dhq.Model(wl.dims, wl.omega0, W, b, mode=dhq.DHQ_W32A32)
    assert m.has_fused()
    out = m.forward(_dev(coords))
    again = m.forward(_dev(coords), flags=dhq.DHQ_FUSED)
    torch.cuda.synchronize()
    err = np.abs(out.cpu().numpy().astype(np.float64) - exp).max()
    _say(f"  max-abs err {err:.3e}")
    assert err <= FLOAT_TOL
    assert np.array_equal(out.cpu().numpy(), again.cpu().numpy())


@pytest.mark.parametrize("dims", [[2, 32, 32, 3], [3, 64, 64, 64, 5], [4, 128, 128, 2], [1, 256, 256, 32], [2, 64, 1]])
def test_w32a32_shapes_and_ragged_rows(dims):
    torch = _torch()
    W, b = synth.siren_init(dims, 30.0, 99 + len(dims))
    m = dhq.Model(dims, 30.0, W, b, mode=dhq.DHQ_W32A32)
    rng = np.random.default_rng(dims[1])
    for n in (1, 129, 5000 + 17):
        _say(f"W32A32 dims {dims} n={n}")
        x = rng.uniform(-1, 1, size=(n, dims[0])).astype(np.float32)
        exp, _ = o.mlp_float(dims, 30.0, W, b, x)
        out = m.forward(_dev(x))
        torch.cuda.synchronize()
        assert np.abs(out.cpu().numpy().astype(np.float64) - exp).max() <= FLOAT_TOL


FLOAT_TOL_WIDE = 4e-6   # the same arithmetic with up to 512 terms per sum and up to sixteen layers (measured 1e-6)


@pytest.mark.parametrize("dims", [[2, 32, 32, 3], [3, 48, 100, 5], [2, 512, 512, 512, 3], [512, 512, 512], [1, 1, 1], [7, 9, 300, 33, 2],
                                  [4] + [256] * 15 + [32], [2, 64, 1], [129, 5]])
def test_w32a32_layer_by_layer_any_shape(dims):
    """The layer-by-layer fp32 path: every shape the library accepts (widths that are no multiple of 8 or
    32, one to sixteen layers, 512 on every side), ragged rows, more rows than one workspace chunk; on
    the shapes that also have the whole-network kernel the two paths are compared as well."""
    torch = _torch()
    W, b = synth.siren_init(dims, 30.0, 199 + len(dims) + dims[0])
    m = dhq.Model(dims, 30.0, W, b, mode=dhq.DHQ_W32A32)
    rng = np.random.default_rng(dims[0] + 3)
    for n in (1, 129, 5000 + 17, 70001):
        if n == 70001 and max(dims) > 128:
            continue                                            # the oracle would take too long
        _say(f"W32A32 layer by layer dims {dims[:3]}.. ({len(dims) - 1} layers) n={n}")
        x = rng.uniform(-1, 1, size=(n, dims[0])).astype(np.float32)
        exp, _ = o.mlp_float(dims, 30.0, W, b, x)
        out = m.forward(_dev(x), flags=dhq.DHQ_LAYERWISE)
        torch.cuda.synchronize()
        err = np.abs(out.cpu().numpy().astype(np.float64) - exp).max()
        _say(f"  max-abs err {err:.2e} (|out| max {np.abs(exp).max():.2f})")
        # a 512-wide input layer with the input layer's initialisation drives the sine argument to tens of
        # revolutions, where one fp32 unit in the last place is already 4e-6 revolutions
        tol = FLOAT_TOL_WIDE if dims[0] <= 8 else 5e-5
        assert out.shape == exp.shape and err <= tol
        auto = m.forward(_dev(x))
        torch.cuda.synchronize()
        if m.has_fused():
            assert np.abs(auto.cpu().numpy() - out.cpu().numpy()).max() <= 2 * FLOAT_TOL_WIDE
        else:
            assert np.array_equal(auto.cpu().numpy(), out.cpu().numpy())
    m.close()


@pytest.mark.parametrize("bits", [4, 8])
def test_w8a32_layer_by_layer_odd_shape(bits):
    torch = _torch()
    dims = [3, 48, 100, 5]
    _say(f"W8A32 layer by layer bits {bits}")
    W, b = synth.siren_init(dims, 30.0, 4242)
    rng = np.random.default_rng(bits)
    x = rng.uniform(-1, 1, size=(3001, 3)).astype(np.float32)
    exp, _, _ = o.mlp_w8a32(dims, 30.0, bits, W, b, x)
    m = dhq.Model(dims, 30.0, W, b, bits, bits, mode=dhq.DHQ_W8A32)
    out = m.forward(_dev(x))
    torch.cuda.synchronize()
    assert np.abs(out.cpu().numpy().astype(np.float64) - exp).max() <= FLOAT_TOL_WIDE
    m.close()


@pytest.mark.parametrize("bits", [4, 6, 8])
def test_w8a32_forward(bits):
    torch = _torch()
    _say(f"W8A32 bits {bits}")
    wl, coords, W, b = synth.make("C2")
    coords = coords[::3]
    exp, _, Wt = o.mlp_w8a32(wl.dims, wl.omega0, bits, W, b, coords)
    m = dhq.Model(wl.dims, wl.omega0, W, b, bits, 8, mode=dhq.DHQ_W8A32)
    sw, sa = m.scales()
    for l in range(len(wl.dims) - 1):
        q, s = o.quantize_weights(W[l], bits)
        assert sw[l] == s and np.array_equal(m.weight_codes(l), q)
    assert (sa == 0).all()
    out = m.forward(_dev(coords))
    torch.cuda.synchronize()
    err = np.abs(out.cpu().numpy().astype(np.float64) - exp).max()
    ref, _ = o.mlp_float(wl.dims, wl.omega0, W, b, coords)
    _say(f"  max-abs err vs oracle {err:.3e}; weight-quantization effect {np.abs(exp - ref).max():.3e}")
    assert err <= FLOAT_TOL


def test_float_modes_refuse_what_they_do_not_have():
    wl, coords, W, b = synth.make("C1")
    m = dhq.Model(wl.dims, wl.omega0, W, b, mode=dhq.DHQ_W32A32)
    x = _dev(coords[:64])
    for call in (lambda: m.calibrate(x), lambda: m.set_act_scales(np.ones(4, np.float32)),
                 lambda: m.forward(x, flags=dhq.DHQ_DYNAMIC), lambda: m.forward(x, flags=dhq.DHQ_LAYERWISE | dhq.DHQ_DYNAMIC),
                 lambda: m.weight_codes(0), lambda: m.forward_debug(x, 0), lambda: m.dynamic_scales()):
        with pytest.raises(dhq.DhqError) as e:
            call()
        assert e.value.status == dhq.DHQ_EUNSUPPORTED
    # shapes without a whole-network fp32 kernel run layer by layer and refuse DHQ_FUSED
    for dims in ([2, 512, 512, 3], [2, 48, 48, 3], [2, 64, 128, 3], [5, 64, 64, 3]):
        Wd, bd = synth.siren_init(dims, 30.0, 5)
        md = dhq.Model(dims, 30.0, Wd, bd, mode=dhq.DHQ_W8A32)
        assert not md.has_fused()
        with pytest.raises(dhq.DhqError) as e:
            md.forward(_dev(np.zeros((8, dims[0]), np.float32)), flags=dhq.DHQ_FUSED)
        assert e.value.status == dhq.DHQ_EUNSUPPORTED
        md.close()
    with pytest.raises(dhq.DhqError) as e:
        dhq.Model(wl.dims, wl.omega0, W, b, mode=dhq.DHQ_W8A32 | dhq.DHQ_ROTATE_BOTH)
    assert e.value.status == dhq.DHQ_EUNSUPPORTED


# ------------------------------------------------ wide layers, full-size grids, graph replay
def test_variants_on_width_512():
    """Two-sided rotation and dynamic scales on the C5 network (512-wide layers: the widest
    transform, un-rotation and GEMM shapes of the layer-by-layer path) on a strided sample."""
    torch = _torch()
    wl, coords, W, b = synth.make("C5")
    coords = coords[::1201]                                  # 3493 coordinates
    for two in (False, True):
        _say(f"width 512 two_sided={two}")
        net = o.quantize_net(wl.dims, wl.omega0, 8, 8, W, b, two_sided=two)
        exp = o.forward(net, coords, calibrate=True)
        m = dhq.Model(wl.dims, wl.omega0, W, b, mode=dhq.DHQ_ROTATE_BOTH if two else dhq.DHQ_ROTATE_IN)
        if two:
            for l in range(len(wl.dims) - 1):
                assert np.array_equal(m.weight_codes(l), net.Wq[l])
        dyn = m.forward(_dev(coords), flags=dhq.DHQ_LAYERWISE | dhq.DHQ_DYNAMIC)
        s_dyn = m.dynamic_scales()
        m.set_act_scales(net.s_a)
        sta = m.forward(_dev(coords), flags=dhq.DHQ_LAYERWISE)
        torch.cuda.synchronize()
        assert (np.abs(s_dyn.astype(np.float64) - net.s_a) / net.s_a).max() <= 1e-5
        _gate(sta.cpu().numpy(), exp, wl.dims, False, "static")
        _gate(dyn.cpu().numpy(), exp, wl.dims, False, "dynamic")
        m.close()


@pytest.mark.parametrize("mode_name", ["w32a32", "w8a32", "two_sided"])
def test_full_grid_sampled_outputs_of_the_variants(mode_name):
    """C4's 1024 x 1024 grid (1 048 576 coordinates) in one call, as the benchmark times it; the
    oracle evaluates a random sample of coordinates plus the first and last tiles one by one."""
    torch = _torch()
    _say(f"full grid C4 {mode_name}")
    wl, coords, W, b = synth.make("C4")
    n = coords.shape[0]
    rng = np.random.default_rng(23)
    idx = np.unique(np.concatenate([rng.integers(0, n, 5000), np.arange(0, 300), np.arange(n - 300, n)]))
    if mode_name == "two_sided":
        net = o.quantize_net(wl.dims, wl.omega0, 8, 8, W, b, two_sided=True)
        o.forward(net, coords[:: n // 8192], calibrate=True)
        exp = o.forward(net, coords[idx])
        m = dhq.Model(wl.dims, wl.omega0, W, b, mode=dhq.DHQ_ROTATE_BOTH)
        m.set_act_scales(net.s_a)
        assert m.has_fused()
    elif mode_name == "w8a32":
        exp, _, _ = o.mlp_w8a32(wl.dims, wl.omega0, 8, W, b, coords[idx])
        m = dhq.Model(wl.dims, wl.omega0, W, b, mode=dhq.DHQ_W8A32)
    else:
        exp, _ = o.mlp_float(wl.dims, wl.omega0, W, b, coords[idx])
        m = dhq.Model(wl.dims, wl.omega0, W, b, mode=dhq.DHQ_W32A32)
    out = m.forward(_dev(coords))
    torch.cuda.synchronize()
    assert bool(torch.isfinite(out).all())
    got = out[torch.from_numpy(idx).to("cuda")].cpu().numpy()
    if mode_name == "two_sided":
        _gate(got, exp, wl.dims, False, "sampled")
    else:
        err = np.abs(got.astype(np.float64) - exp).max()
        _say(f"  {idx.size} sampled coords: max-abs err {err:.3e}")
        assert err <= FLOAT_TOL
    sub = m.forward(_dev(coords[idx]))                       # a coordinate's value does not depend on the launch
    torch.cuda.synchronize()
    assert np.array_equal(sub.cpu().numpy(), got)
    m.close()


SWEEP_WIDTHS = [1, 2, 3, 5, 8, 9, 16, 17, 31, 32, 33, 48, 64, 65, 100, 128, 129, 200, 256, 257, 300, 511, 512]


def _sweep_case(i):
    """Seeded random network shape, bit width, rotation mode and row count (case i of the sweep)."""
    rng = np.random.default_rng(20250813 + i)
    bits = int(rng.choice([4, 6, 8]))
    mode = int(rng.choice([dhq.DHQ_ROTATE_IN, dhq.DHQ_ROTATE_BOTH]))
    n = int(rng.choice([1, 7, 255, 257, 1000, 3001]))
    if i >= 60:   # shapes the fused kernels take: equal power-of-two hidden widths, small fan-in and fan-out
        L = int(rng.integers(2, 7))
        widths = [32, 64, 128, 256] if mode == dhq.DHQ_ROTATE_BOTH else [32, 64, 128, 256, 512]   # two-sided fused: up to 256
        dims = [int(rng.integers(1, 5))] + [int(rng.choice(widths))] * (L - 1)
        dims.append(int(rng.choice([1, 2, 3, 4, 7, 32])))
        return dims, bits, mode, n, rng
    L = int(rng.integers(1, 6))
    dims = [int(rng.integers(1, 5)) if rng.random() < 0.7 else int(rng.choice(SWEEP_WIDTHS))]
    same, w = rng.random() < 0.4, int(rng.choice(SWEEP_WIDTHS))
    dims += [w if same else int(rng.choice(SWEEP_WIDTHS)) for _ in range(L - 1)]
    dims.append(int(rng.choice([1, 2, 3, 4, 5, 32, 33, 100])))
    return dims, bits, mode, n, rng


@pytest.mark.parametrize("block", range(6))
def test_random_shapes_bits_modes_and_row_counts(block):
    """Ninety seeded random configurations (sixty of any shape: one to five layers, widths from 1 to 512
    that are and are not powers of two or multiples of 32; thirty of the shapes the fused kernels
    take; 4 / 6 / 8 bits, either rotation mode, row counts around the tile sizes), each through static
    and dynamic scales on the automatically chosen and on the layer-by-layer path.  Weight codes
    bit-identical; every coordinate none of whose codes sits at a rounding boundary within the
    tolerance, and few of the others beyond it."""
    from test_gpu_parity import _near_boundary
    torch = _torch()
    for i in range(15 * block, 15 * block + 15):
        dims, bits, mode, n, rng = _sweep_case(i)
        _say(f"sweep case {i}: dims {dims} bits {bits} mode {mode} n {n}")
        W, b = synth.siren_init(dims, 30.0, 7000 + i)
        x = rng.uniform(-1, 1, size=(n, dims[0])).astype(np.float32)
        net = o.quantize_net(dims, 30.0, bits, bits, W, b, two_sided=(mode == dhq.DHQ_ROTATE_BOTH))
        exp, dmp = o.forward(net, x, calibrate=True, dump=True)
        near = _near_boundary(net, dmp, bits)
        m = dhq.Model(dims, 30.0, W, b, bits, bits, mode=mode)
        assert m.has_fused() or i < 60
        for l in range(len(dims) - 1):
            assert np.array_equal(m.weight_codes(l), net.Wq[l]), f"case {i}: weight codes of layer {l}"
        m.set_act_scales(net.s_a)
        for flags in (dhq.DHQ_AUTO, dhq.DHQ_LAYERWISE, dhq.DHQ_DYNAMIC, dhq.DHQ_DYNAMIC | dhq.DHQ_LAYERWISE):
            out = m.forward(_dev(x), flags=flags)
            torch.cuda.synchronize()
            out = out.cpu().numpy()
            assert out.shape == exp.shape and np.isfinite(out).all()
            err = np.abs(out.astype(np.float64) - exp).max(axis=1)
            over = err > OUT_TOL
            assert not (over & ~near).any(), f"case {i} flags {flags}: max-abs err {err.max():.3e}"
            assert over.sum() <= max(2, flip_frac(dims) * n), f"case {i} flags {flags}: {over.sum()} of {n} beyond {OUT_TOL}"
        m.close()


def test_models_give_back_their_device_memory():
    """Every kernel family's model (packed weights, workspaces, the whole-batch buffers of the dynamic
    mode) is created, used and freed repeatedly; the device's free memory must not drift."""
    torch = _torch()
    rng = np.random.default_rng(3)
    families = [([2, 64, 64, 3], dhq.DHQ_ROTATE_IN), ([2, 256, 256, 3], dhq.DHQ_ROTATE_BOTH), ([2, 512, 512, 3], dhq.DHQ_ROTATE_IN),
                ([3, 48, 100, 5], dhq.DHQ_ROTATE_BOTH), ([2, 128, 128, 3], dhq.DHQ_W32A32), ([2, 128, 128, 3], dhq.DHQ_W8A32),
                ([3, 48, 100, 5], dhq.DHQ_W32A32)]
    nets = [(dims, mode) + synth.siren_init(dims, 30.0, 50 + i) for i, (dims, mode) in enumerate(families)]
    xs = {k: _dev(rng.uniform(-1, 1, size=(70001, k)).astype(np.float32)) for k in (2, 3)}

    def one_round():
        for dims, mode, W, b in nets:
            m = dhq.Model(dims, 30.0, W, b, mode=mode)
            x = xs[dims[0]]
            if mode in (dhq.DHQ_W32A32, dhq.DHQ_W8A32):
                m.forward(x)
                m.forward(x, flags=dhq.DHQ_LAYERWISE)
            else:
                m.calibrate(x)
                m.forward(x)
                m.forward(x, flags=dhq.DHQ_LAYERWISE)
                m.forward(x, flags=dhq.DHQ_DYNAMIC)
                m.forward(x, flags=dhq.DHQ_DYNAMIC | dhq.DHQ_LAYERWISE)
            torch.cuda.synchronize()
            m.close()

    one_round()                                   # code objects loaded, torch's allocator warmed up
    torch.cuda.synchronize()
    free0 = torch.cuda.mem_get_info()[0]
    for rep in range(5):
        _say(f"create/use/free round {rep}")
        one_round()
    torch.cuda.synchronize()
    free1 = torch.cuda.mem_get_info()[0]
    _say(f"  free device memory before {free0 >> 20} MiB, after {free1 >> 20} MiB")
    assert free0 - free1 <= (16 << 20)            # one leaked workspace would be hundreds of MiB


@pytest.mark.parametrize("variant", ["fused", "layerwise", "two_sided", "dynamic", "dynamic_fused", "dynamic_fused_two_sided",
                                     "w32a32", "w32a32_layerwise", "fused_512", "dynamic_fused_512"])
def test_forward_replays_from_a_captured_graph(variant):
    """dhq_forward only enqueues kernels (no memset, no allocation, no synchronisation once the
    workspace exists), so a stream capture of it replays to the same bits as the eager call --
    several times, with eager work and synchronisations in between."""
    torch = _torch()
    _say(f"graph replay {variant}")
    wl, coords, W, b = synth.make("C1")
    x = _dev(coords)
    dims = list(wl.dims)
    if variant.endswith("_512"):                             # the two-wave width-512 kernels, whole network and per layer
        dims = [2, 512, 512, 512, 3]
        W, b = synth.siren_init(dims, wl.omega0, 512)
    mode = {"two_sided": dhq.DHQ_ROTATE_BOTH, "dynamic_fused_two_sided": dhq.DHQ_ROTATE_BOTH,
            "w32a32": dhq.DHQ_W32A32, "w32a32_layerwise": dhq.DHQ_W32A32}.get(variant, dhq.DHQ_ROTATE_IN)
    flags = {"fused": dhq.DHQ_FUSED, "layerwise": dhq.DHQ_LAYERWISE, "dynamic": dhq.DHQ_LAYERWISE | dhq.DHQ_DYNAMIC,
             "dynamic_fused": dhq.DHQ_FUSED | dhq.DHQ_DYNAMIC,
             "dynamic_fused_two_sided": dhq.DHQ_FUSED | dhq.DHQ_DYNAMIC,
             "fused_512": dhq.DHQ_FUSED, "dynamic_fused_512": dhq.DHQ_FUSED | dhq.DHQ_DYNAMIC,
             "w32a32_layerwise": dhq.DHQ_LAYERWISE}.get(variant, dhq.DHQ_AUTO)
    m = dhq.Model(dims, wl.omega0, W, b, mode=mode)
    if not variant.startswith("w32a32"):
        m.calibrate(x)
    out = torch.empty((x.shape[0], dims[-1]), dtype=torch.float32, device="cuda")
    eager = m.forward(x, flags=flags).clone()                # also grows the dynamic workspace before capture
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(s):
        with torch.cuda.graph(g, stream=s):
            dhq.dhq_forward(m.handle, x, out, s, flags)
    torch.cuda.current_stream().wait_stream(s)
    for rep in range(3):
        out.zero_()
        scratch = m.forward(x[: 100 + rep], flags=flags)     # eager work on the same model in between
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert np.array_equal(out.cpu().numpy(), eager.cpu().numpy()), f"replay {rep}"
        assert bool(torch.isfinite(scratch).all())
    m.close()
