"""CPU-only checks of the C-ABI library: it loads, exports what include/dhq.h declares,
and rejects bad arguments before touching a GPU."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import paper_2508_13478_amd as dhq

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "dhq.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(dhq_[a-z0-9_]+)\s*\(", text)))


def test_library_loads_and_exports_every_declared_symbol():
    L = dhq.lib()
    declared = _declared_symbols()
    assert "dhq_quantize_weights" in declared and "dhq_forward" in declared
    assert set(declared) == set(dhq.EXPORTS)
    for name in declared:
        assert hasattr(L, name), name
    assert dhq.dhq_version() >= 100
    assert dhq.dhq_strerror(0) == "ok"
    assert "scale" in dhq.dhq_strerror(dhq.DHQ_ENOSCALE)


def test_quantize_weights_rejects_bad_arguments_without_gpu():
    L = dhq.lib()
    dims = (C.c_int32 * 3)(2, 8, 3)
    W = [np.zeros((8, 2), np.float32), np.zeros((3, 8), np.float32)]
    b = [np.zeros(8, np.float32), np.zeros(3, np.float32)]
    Wp = (C.POINTER(C.c_float) * 2)(*[w.ctypes.data_as(C.POINTER(C.c_float)) for w in W])
    bp = (C.POINTER(C.c_float) * 2)(*[x.ctypes.data_as(C.POINTER(C.c_float)) for x in b])
    h = C.c_void_p()

    def call(desc):
        return L.dhq_quantize_weights(C.byref(desc), Wp, bp, C.byref(h))

    assert call(dhq.dhq_net_desc(2, dims, 30.0, 5, 8)) == dhq.DHQ_EINVAL          # bits not in {4,6,8}
    assert call(dhq.dhq_net_desc(2, dims, 30.0, 8, 3)) == dhq.DHQ_EINVAL
    assert call(dhq.dhq_net_desc(0, dims, 30.0, 8, 8)) == dhq.DHQ_EINVAL          # no layers
    assert call(dhq.dhq_net_desc(17, dims, 30.0, 8, 8)) == dhq.DHQ_EUNSUPPORTED   # too deep
    big = (C.c_int32 * 3)(2, 1024, 3)
    assert call(dhq.dhq_net_desc(2, big, 30.0, 8, 8)) == dhq.DHQ_EUNSUPPORTED     # too wide
    zero = (C.c_int32 * 3)(2, 0, 3)
    assert call(dhq.dhq_net_desc(2, zero, 30.0, 8, 8)) == dhq.DHQ_EINVAL
    assert L.dhq_quantize_weights(None, Wp, bp, C.byref(h)) == dhq.DHQ_EINVAL
    assert h.value is None


def test_null_model_is_rejected():
    L = dhq.lib()
    assert L.dhq_forward(None, None, 0, None, None, 0) == dhq.DHQ_EINVAL
    assert L.dhq_set_act_scales(None, None) == dhq.DHQ_EINVAL
    assert L.dhq_has_fused(None) == dhq.DHQ_EINVAL
    L.dhq_free(None)  # a no-op


def test_product_package_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_2508_13478_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                text = open(os.path.join(dirpath, f)).read()
                assert not re.search(r"^\s*(from|import)\s+oracle", text, flags=re.M), f
                assert "dhq_oracle" not in text and "dhqo_" not in text, f
    for f in ("dhq_oracle.c", "dhq_oracle.py"):
        text = open(os.path.join(ROOT, "oracle", f)).read()
        assert "paper_2508_13478_amd" not in text and "libdhq.so" not in text


def test_wide_register_map_check_catches_violations():
    """The build refuses a width-512 kernel whose compiler-generated code touches the
    accumulation registers the kernel addresses by number, or whose allocation is too small."""
    from paper_2508_13478_amd import build as b
    ok = "\n".join([
        "_Z21dhq_fused_wide_kernelILi512EEv9wide_args: ; @kernel",
        "\tv_mov_b32_e32 v5, v3",
        "\t;;#ASMSTART",
        "\tv_mfma_f32_32x32x16_f16 a[0x10:0x1f], v[16:19], v[20:23], 0",
        "\tglobal_load_dwordx4 a[224:227], v1, s[2:3]",
        "\t;;#ASMEND",
        "\tv_add_f32_e32 v1, v2, v3 ; a200 in a comment does not count",
        ".Lfunc_end0:",
        "\t.amdhsa_kernel _Z21dhq_fused_wide_kernelILi512EEv9wide_args",
        "\t.amdhsa_next_free_vgpr 468",
        "\t.amdhsa_accum_offset 212",
        "\t.end_amdhsa_kernel",
    ])
    b.check_wide_register_map(ok)
    for planted in ("\tv_accvgpr_read_b32 v5, a0", "\tds_write_b128 v1, a[156:163]", "\tscratch_store_dword off, a[0xff], off"):
        bad = ok.replace("\tv_add_f32_e32", planted + "\n\tv_add_f32_e32")
        with pytest.raises(RuntimeError):
            b.check_wide_register_map(bad)
    with pytest.raises(RuntimeError):
        b.check_wide_register_map(ok.replace("accum_offset 212", "accum_offset 216"))
    with pytest.raises(RuntimeError):
        b.check_wide_register_map("nothing here")
    # the float kernels keep their activations in a128 and up; another function's registers do not matter
    flt = ok.replace("dhq_fused_wide_kernelILi512EEv9wide_args", "dhq_float_kernelILi256EEv10float_args").replace("_Z21", "_Z16")
    flt = flt.replace("\tv_mov_b32_e32 v5, v3", "\tv_accvgpr_write_b32 a127, v3")
    assert b.check_fixed_agprs(flt, "dhq_float_kernel", 128) == 1
    with pytest.raises(RuntimeError):
        b.check_fixed_agprs(flt.replace("a127", "a128"), "dhq_float_kernel", 128)
    other = "helper_function:\n\tv_accvgpr_write_b32 a200, v1\n" + ok
    b.check_wide_register_map(other)


def test_packing_index_maps(tmp_path):
    """The maps behind the fused kernels' offline packing (which rotated feature a lane's register holds,
    where a feature's bias sits) are permutations and agree with the MFMA accumulator layout."""
    import subprocess
    from paper_2508_13478_amd import build as b
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    exe = str(tmp_path / "index_maps_check")
    subprocess.run([b._hipcc(), "--offload-arch=gfx950", "-O1", "-w", "-I", os.path.join(root, "include"), "-I", b.CSRC,
                    os.path.join(root, "tests", "c", "index_maps_check.hip"), "-o", exe], check=True)
    r = subprocess.run([exe], capture_output=True, text=True)
    assert r.returncode == 0, r.stdout + r.stderr
    assert "index_maps ok" in r.stdout


def test_two_sided_int32_bound_is_enforced_before_the_device_is_touched():
    """One non-zero weight in a 512 x 512 layer rotates into 512 x 512 equal codes of +-127; with
    all activation codes at 127 the un-rotated sum reaches 127 * 127 * 512 * 512 > 2^31.  The
    oracle reports the overflow when it happens, the library refuses the weights up front."""
    from oracle import dhq_oracle as o
    W = np.zeros((512, 512), dtype=np.float32)
    W[0, 0] = 1.0
    b = np.zeros(512, dtype=np.float32)
    with pytest.raises(dhq.DhqError) as e:
        dhq.dhq_quantize_weights_mode([512, 512], 30.0, 8, 8, dhq.DHQ_ROTATE_BOTH, [W], [b])
    assert e.value.status == dhq.DHQ_EUNSUPPORTED
    Wq, s_w = o.quantize_weights_two_sided(W, 8)
    assert (np.abs(Wq) == 127).all()
    a = np.zeros((1, 512), dtype=np.float32)
    a[0, 0] = 1.0                                   # rotates into 512 equal values -> all codes 127
    with pytest.raises(o.OracleError):
        o.layer_two_sided(a, 512, Wq, s_w, b, None, 8, False, 30.0)
    # the same weights are fine one-sided, and a 256-wide layer stays inside int32 even in the worst case
    W2 = np.zeros((256, 256), dtype=np.float32)
    W2[0, 0] = 1.0
    r = o.layer_two_sided(a[:, :256], 256, *o.quantize_weights_two_sided(W2, 8), b[:256], None, 8, False, 30.0)
    assert np.abs(r["unrot"]).max() == 127 * 127 * 256 * 256


def _build_c_abi_check(tmp_path):
    import subprocess
    dhq.lib()
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    libdir = os.path.dirname(dhq.LIB_PATH)
    exe = str(tmp_path / "c_abi_check")
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-Werror", "-pedantic", "-I", os.path.join(root, "include"),
                    os.path.join(root, "tests", "c", "c_abi_check.c"), "-o", exe, "-L", libdir, "-l:libdhq.so",
                    "-L/opt/rocm/lib", "-lamdhip64", "-lm", "-Wl,-rpath," + libdir, "-Wl,-rpath,/opt/rocm/lib"], check=True)
    return exe


def test_header_is_plain_c_and_entry_points_link_from_c(tmp_path):
    """include/dhq.h compiled as C99 with warnings as errors, linked against libdhq.so and run:
    version, status names and the argument checks that are decided before the device is touched."""
    import subprocess
    exe = _build_c_abi_check(tmp_path)
    r = subprocess.run([exe], capture_output=True, text=True)
    assert r.returncode == 0, r.stdout + r.stderr
    assert "c_abi_check ok" in r.stdout


@pytest.mark.gpu
def test_c_program_runs_a_forward(tmp_path):
    """The same C program with a device present: quantize, calibrate, forward (static, dynamic and the
    non-allocating entry point) from plain C, against the closed form of its tiny network."""
    import subprocess
    exe = _build_c_abi_check(tmp_path)
    r = subprocess.run([exe, "forward"], capture_output=True, text=True)
    assert r.returncode == 0, r.stdout + r.stderr
    assert "c_abi_check forward ok" in r.stdout and "c_abi_check ok" in r.stdout
