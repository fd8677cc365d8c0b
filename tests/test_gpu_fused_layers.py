"""The gates of the layer-by-layer parity tests applied to the whole-network (fused) kernels,
which are the ones the benchmark times.  Those kernels keep every intermediate in registers and
rotate differently from the layer-by-layer path (the 32-point factor of the transform runs on
the matrix unit over two binary16 pieces of each activation), so they are checked through their
own test hook, dhq_forward_debug_fused: one layer of the kernel's own device code on the
ORACLE's input codes (teacher-forced), returning the integer accumulators, the un-normalised
transform x^ of the layer's output and the codes the next quantizer makes of it.

Per layer:
  * accumulators: bit-exact against the oracle's integer GEMM on the same codes;
  * x^: max |x^_gpu - sqrt(Kp) x^_oracle| <= XHAT_TOL(Kp)  (the oracle rotates in fp64);
  * codes: at most 0.1 % differ from the oracle's, each by at most 1 LSB;
  * every differing code is a legitimate one: the oracle's own x^ / s_a lies within the x^ error
    MEASURED on that layer (in code units, plus the rounding of the fp32 multiplier) of the
    rounding boundary between the two codes.  This is a complete check -- no estimate of where
    boundaries are "near" -- and it ties every difference to arithmetic noise of known size.
"""
import sys

import numpy as np
import pytest

import paper_2508_13478_amd as dhq
from oracle import dhq_oracle as o
from paper_2508_13478_amd import synth

pytestmark = pytest.mark.gpu

CODE_RATE = 1e-3


def xhat_tol(kp):
    """Bound on |x^_gpu - sqrt(Kp) x^_oracle| for a layer input of Kp rotated features.

    x^ un-normalised is a sum of Kp activations with signs.  One activation a = sin(2 pi t) carries
    at most d = 2 pi 2^-24 |t| (fp32 rounding of the argument t = acc c1 + b, |t| <= 16 revolutions
    on these networks) + 1.2e-7 (hardware sine) + 2^-21 (the two binary16 pieces) + 6e-8 (fp32
    rounding of a itself) ~ 6.6e-6, and the sums add up to sqrt(Kp)-fold rounding of partial sums
    of size <= Kp: 2^-24 Kp log2(Kp) / 2.  The errors of different activations are independent, so
    the bound is taken at four standard deviations of their sum rather than at the (never
    attained) worst case Kp d: 4 sqrt(Kp) d / sqrt(3) + 2^-24 Kp log2(Kp) / 2."""
    d = 2 * np.pi * 2.0 ** -24 * 16 + 1.2e-7 + 2.0 ** -21 + 6e-8
    return 4.0 * np.sqrt(kp) * d / np.sqrt(3.0) + 2.0 ** -24 * kp * np.log2(max(kp, 2)) / 2


def _say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def _dev(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a)).to("cuda")


def _sample(side, rows, seed):
    """rows coordinates of the side x side grid: the first and last grid rows' pixels plus seeded random ones."""
    grid = synth.grid_coords(side)
    idx = (synth.splitmix64(seed, 0, rows) % np.uint64(grid.shape[0])).astype(np.int64)
    idx[: min(64, rows)] = np.arange(min(64, rows))
    idx[-1] = grid.shape[0] - 1
    return grid[idx]


# name, dims, grid side, bits, two-sided, wavelet spread, rows (not a multiple of any tile size);
# hidden width 512 has two whole-network kernels (dhq_select_wide_kernel): every such case runs on both
_CASES = [
    ("C1", synth.WORKLOADS["C1"].dims, 64, 8, False, None, 4096),
    ("C2", synth.WORKLOADS["C2"].dims, 256, 8, False, None, 8192 + 77),
    ("C4-4bit", synth.WORKLOADS["C4"].dims, 1024, 4, False, None, 4096 + 33),
    ("C4-6bit", synth.WORKLOADS["C4"].dims, 1024, 6, False, None, 4096 + 33),
    ("C5", synth.WORKLOADS["C5"].dims, 2048, 8, False, None, 4096 + 50),
    ("C5-4bit", synth.WORKLOADS["C5"].dims, 2048, 4, False, None, 1024 + 50),
    ("C5-6bit", synth.WORKLOADS["C5"].dims, 2048, 6, False, None, 1024 + 50),
    ("C2-two-sided", synth.WORKLOADS["C2"].dims, 256, 8, True, None, 4096 + 77),
    ("128x3-two-sided-6bit", (2, 128, 128, 128, 3), 128, 6, True, None, 2048 + 5),
    ("C2-wavelet", synth.WORKLOADS["C2"].dims, 256, 8, False, 10.0, 4096 + 77),
    ("C5-wavelet", synth.WORKLOADS["C5"].dims, 2048, 8, False, 10.0, 1024 + 50),
]
CASES = []
for _c in _CASES:
    if _c[1][1] == 512:
        CASES.append((_c[0] + "-one-wave",) + _c[1:] + (1,))
        CASES.append((_c[0] + "-two-waves",) + _c[1:] + (2,))
    else:
        CASES.append(_c + (0,))


@pytest.mark.parametrize("name,dims,side,bits,two_sided,s0,rows,wide_kernel", CASES, ids=[c[0] for c in CASES])
def test_fused_layer_teacher_forced(name, dims, side, bits, two_sided, s0, rows, wide_kernel):
    import torch
    dims = list(dims)
    seed = synth.WORKLOADS[name.split("-")[0]].seed if name.split("-")[0] in synth.WORKLOADS else 0x5EED
    W, b = synth.siren_init(dims, 30.0, seed)
    coords = _sample(side, rows, seed ^ 0xABCDEF)
    net = o.quantize_net(dims, 30.0, bits, bits, W, b, two_sided=two_sided, gabor_s0=s0)
    _, dump = o.forward(net, coords, calibrate=True, dump=True)
    mode = dhq.DHQ_ROTATE_BOTH if two_sided else dhq.DHQ_ROTATE_IN
    model = dhq.Model(dims, 30.0, W, b, bits, bits, mode=mode, wavelet_s0=s0)
    model.set_act_scales(net.s_a)
    assert model.has_fused()
    if wide_kernel:
        model.select_wide_kernel(wide_kernel)
    L = len(dims) - 1
    qm = o.qmax(bits)
    total_codes = total_diff = 0
    for l in range(L - 1):
        xhat, codes, acc = model.forward_debug_fused(_dev(dump.codes[l]), l)
        torch.cuda.synchronize()
        xhat, codes, acc = xhat.cpu().numpy().astype(np.float64), codes.cpu().numpy(), acc.cpu().numpy()
        kp = xhat.shape[1]
        # (i) the integer stage
        assert np.array_equal(acc, o.igemm(dump.codes[l], net.Wq[l])), f"{name} layer {l}: accumulators"
        # (ii) the transformed activations, un-normalised
        ref = dump.rot[l + 1] * np.sqrt(float(kp))
        err = float(np.abs(xhat - ref).max())
        rms = float(np.sqrt(((xhat - ref) ** 2).mean()))
        tol = xhat_tol(kp)
        # (iii) the codes
        exp = dump.codes[l + 1].astype(np.int32)
        d = codes.astype(np.int32) - exp
        ndiff = int((d != 0).sum())
        total_codes += d.size
        total_diff += ndiff
        _say(f"{name} layer {l}: x^ max err {err:.3e} rms {rms:.3e} (tol {tol:.3e}, max |x^| {np.abs(ref).max():.1f}); "
             f"codes differing {ndiff} of {d.size} ({ndiff / d.size:.2e})")
        assert err <= tol, f"{name} layer {l}: x^ error {err} > {tol}"
        assert np.abs(d).max() <= 1 and ndiff <= CODE_RATE * d.size
        # every differing code sits on a rounding boundary of the oracle's own value, within the noise
        # measured above: u = x^ / s_a in code units, boundary between the two codes at min(c) + 1/2
        if ndiff:
            s_a = float(net.s_a[l + 1])
            u = dump.rot[l + 1] / s_a
            where = np.nonzero(d)
            boundary = np.minimum(codes[where].astype(np.float64), exp[where].astype(np.float64)) + 0.5
            slack = err / (s_a * np.sqrt(float(kp))) + (qm + 1) * 2.0 ** -23
            dist = np.abs(u[where] - boundary)
            assert (dist <= slack).all(), f"{name} layer {l}: a code differs {dist.max():.3e} LSB from its boundary, noise {slack:.3e}"
            assert (np.abs(exp[where]) <= qm).all() and (np.abs(codes[where].astype(np.int32)) <= qm).all()
    _say(f"{name}: {total_diff} of {total_codes} codes differ ({total_diff / max(total_codes, 1):.2e})")
    model.close()


def test_fused_hook_rejects_what_it_cannot_do():
    import torch
    dims = [3, 48, 100, 5]            # no whole-network kernel for this shape
    W, b = synth.siren_init(dims, 30.0, 1)
    m = dhq.Model(dims, 30.0, W, b, 8, 8)
    m.set_act_scales(np.ones(3, np.float32))
    x = torch.zeros((8, 4), dtype=torch.int8, device="cuda")
    with pytest.raises(dhq.DhqError) as e:
        m.forward_debug_fused(x, 0)
    assert e.value.status == dhq.DHQ_EUNSUPPORTED
    m.close()
    dims = [2, 64, 64, 3]
    W, b = synth.siren_init(dims, 30.0, 2)
    m = dhq.Model(dims, 30.0, W, b, 8, 8)
    x = torch.zeros((8, 2), dtype=torch.int8, device="cuda")
    with pytest.raises(dhq.DhqError) as e:
        m.forward_debug_fused(x, 0)
    assert e.value.status == dhq.DHQ_ENOSCALE
    m.set_act_scales(np.ones(3, np.float32))
    with pytest.raises(dhq.DhqError) as e:
        m.forward_debug_fused(torch.zeros((8, 64), dtype=torch.int8, device="cuda"), 2)   # the output layer
    assert e.value.status == dhq.DHQ_EUNSUPPORTED
    m.close()
