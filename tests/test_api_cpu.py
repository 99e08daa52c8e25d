"""Host-side behaviour of the C ABI that needs no GPU: the library loads, exports
what include/gemm.h declares, validates descriptors and picks kernels."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def g():
    import paper_2603_12440_amd as g
    if not os.path.exists(g.library_path()):
        from paper_2603_12440_amd.build import build_library
        build_library()
    g.load_library()
    return g


def test_every_declared_symbol_is_exported(g):
    header = open(os.path.join(ROOT, "include", "gemm.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    names = set(re.findall(r"\b(gemm_[a-z_]+)\s*\(", header))
    assert {"gemm_create", "gemm_run", "gemm_destroy", "gemm_status_string", "gemm_plan_info",
            "gemm_create_config", "gemm_config_count", "gemm_config_name", "gemm_tune",
            "gemm_create_splitk", "gemm_workspace_bytes", "gemm_run_workspace",
            "gemm_set_autotune", "gemm_autotune_entries", "gemm_autotune_clear"} <= names
    rope = open(os.path.join(ROOT, "include", "rope.h")).read()
    rope = re.sub(r"/\*.*?\*/", "", rope, flags=re.S)
    rope_names = set(re.findall(r"\b(rope_[a-z_]+)\s*\(", rope))
    assert rope_names == {"rope_apply"}
    probe = open(os.path.join(ROOT, "include", "probe.h")).read()
    probe = re.sub(r"/\*.*?\*/", "", probe, flags=re.S)
    probe_names = set(re.findall(r"\b(probe_[a-z0-9_]+)\s*\(", probe))
    assert probe_names == {"probe_mfma_peak", "probe_mfma16_peak", "probe_read_peak"}
    lib = ctypes.CDLL(g.library_path())
    for n in names | rope_names | probe_names:
        assert hasattr(lib, n), n


def test_binding_exposes_the_same_names(g):
    for n in ("gemm_create", "gemm_run", "gemm_destroy", "gemm_status_string", "gemm_plan_info",
              "gemm_create_config", "gemm_config_count", "gemm_config_name", "gemm_tune",
              "gemm_create_splitk", "gemm_workspace_bytes", "gemm_run_workspace", "rope_apply",
              "gemm_set_autotune", "gemm_autotune_entries", "gemm_autotune_clear"):
        assert callable(getattr(g, n))


def test_probe_argument_checks_need_no_device(g):
    for call, want in [(lambda: g.probe_mfma16_peak(g.BF16, 0, stream=0), -1),
                       (lambda: g.probe_mfma16_peak(g.F8E4M3, 0x1000, stream=0), -4),
                       (lambda: g.probe_mfma_peak(g.BF16, 0, stream=0), -1),
                       (lambda: g.probe_mfma_peak(g.F32, 0x1000, stream=0), -4),
                       (lambda: g.probe_mfma_peak(7, 0x1000, stream=0), -4),
                       (lambda: g.probe_mfma_peak(g.BF16, 0x1002, stream=0), -5),
                       (lambda: g.probe_read_peak(0, 1 << 30, 0x1000, stream=0), -1),
                       (lambda: g.probe_read_peak(0x10000, 1 << 20, 0x1000, stream=0), -2),      # too small
                       (lambda: g.probe_read_peak(0x10000, (1 << 30) + 16, 0x1000, stream=0), -2),
                       (lambda: g.probe_read_peak(0x10008, 1 << 30, 0x1000, stream=0), -5)]:
        with pytest.raises(g.GemmError) as e:
            call()
        assert e.value.status == want


def test_splitk_plans(g):
    """Split-K planning is host work: slices, workspace size, what it refuses."""
    p = g.gemm_create_splitk(g.GemmDesc(512, 512, 32768))
    assert "kernel=splitk_16+mfma16_128x128" in p.info() and "grid=256,1,1" in p.info()   # 16 tiles x 16 slices, persistent
    assert g.gemm_workspace_bytes(p) == 16 * 512 * 512 * 4
    # a split-K plan cannot run without its workspace
    with pytest.raises(g.GemmError) as e:
        g.gemm_run(p, 0x1000, 0x2000, 0x3000, stream=0)
    assert e.value.status == -11
    with pytest.raises(g.GemmError) as e:
        g.gemm_run_workspace(p, 0x1000, 0x2000, 0x3000, None, 0x4000, 1024, stream=0)
    assert e.value.status == -11                       # too small
    with pytest.raises(g.GemmError) as e:
        g.gemm_run_workspace(p, 0x1000, 0x2000, 0x3000, None, 0x4004, 1 << 40, stream=0)
    assert e.value.status == -11                       # not 16-byte aligned
    g.gemm_destroy(p)
    p = g.gemm_create_splitk(g.GemmDesc(256, 256, 4096), splits=4)
    assert "kernel=splitk_4+" in p.info() and g.gemm_workspace_bytes(p) == 4 * 256 * 256 * 4
    g.gemm_destroy(p)
    # many tiles already: the built-in choice does not split
    p = g.gemm_create_splitk(g.GemmDesc(8192, 8192, 8192))
    assert "kernel=splitk_1+" in p.info()
    g.gemm_destroy(p)
    p = g.gemm_create(g.GemmDesc(512, 512, 512))
    assert g.gemm_workspace_bytes(p) == 0
    g.gemm_destroy(p)
    def status(**kw):
        splits = kw.pop("splits", 0)
        try:
            g.gemm_destroy(g.gemm_create_splitk(g.GemmDesc(**kw), splits))
        except g.GemmError as e:
            return e.status
        return 0
    assert status(M=256, N=256, K=4096, splits=3) == -4          # 4096 is not a multiple of 8*3
    assert status(M=256, N=256, K=4096, splits=-1) == -2
    assert status(M=256, N=256, K=4096, batch=2) == -4
    assert status(M=256, N=256, K=4096, dtype=g.F32, layout_b=g.ROW_MAJOR) == -4
    assert status(M=256, N=256, K=4096, layout_a=g.COL_MAJOR) == -4
    assert status(M=0, N=256, K=4096) == -2


def test_rope_argument_checks_need_no_device(g):
    """Everything rope_apply rejects is rejected on the host, before any device call."""
    def status(desc, tensors, cos=0x1000, sin=0x2000):
        try:
            g.rope_apply(desc, tensors, cos, sin, stream=0)
        except g.GemmError as e:
            return e.status
        return 0
    t = g.RopeTensor(0x10000, 0x20000, heads=4)
    ok = dict(batch=2, seq=8, head_dim=64)
    assert status(g.RopeDesc(**ok), [g.RopeTensor(0, 0x20000, heads=4)]) == -1
    assert status(g.RopeDesc(**ok), [t], cos=0) == -1
    assert status(g.RopeDesc(batch=2, seq=8, head_dim=63), [t]) == -2          # odd head_dim
    assert status(g.RopeDesc(batch=0, seq=8, head_dim=64), [t]) == -2
    assert status(g.RopeDesc(**ok), [t, t, t]) == -2                            # at most two tensors
    assert status(g.RopeDesc(**ok), [g.RopeTensor(0x10000, 0x20000, heads=0)]) == -2
    assert status(g.RopeDesc(**ok, dtype=5), [t]) == -8
    assert status(g.RopeDesc(**ok, dtype=g.BF16, table_dtype=g.F16), [t]) == -4
    assert status(g.RopeDesc(**ok, table_stride_b=100), [t]) == -3              # tables of batches overlap
    assert status(g.RopeDesc(**ok), [g.RopeTensor(0x10000, 0x20000, heads=4, x_strides=(0, 64, 0))]) == -3
    assert status(g.RopeDesc(**ok), [g.RopeTensor(0x10000, 0x20000, heads=4, x_strides=(2048, 32, 256))]) == -3
    assert status(g.RopeDesc(**ok), [g.RopeTensor(0x10001, 0x20000, heads=4)]) == -5
    assert status(g.RopeDesc(**ok), [t], cos=0x1002) == -5                      # fp32 table, 2-byte aligned


def _status(g, **kw):
    try:
        p = g.gemm_create(g.GemmDesc(**kw))
    except g.GemmError as e:
        return e.status
    g.gemm_destroy(p)
    return 0


def test_descriptor_validation(g):
    ok = dict(M=64, N=64, K=64)
    assert _status(g, **ok) == 0
    assert _status(g, M=0, N=64, K=64) == -2
    assert _status(g, M=64, N=-1, K=64) == -2
    assert _status(g, M=64, N=64, K=0) == -2
    assert _status(g, **ok, batch=0) == -2
    assert _status(g, **ok, lda=63) == -3            # row-major A needs lda >= K
    assert _status(g, **ok, ldb=10) == -3
    assert _status(g, **ok, ldc=1) == -3
    assert _status(g, **ok, batch=2, stride_c=10) == -3   # overlapping output batches
    assert _status(g, **ok, batch=2, stride_bias=3, epilogue=g.EPI_BIAS) == -3
    assert _status(g, **ok, dtype=g.BF16, dtype_b=g.F16) == -4
    assert _status(g, **ok, dtype=g.F32, dtype_c=g.BF16) == -4
    assert _status(g, **ok, dtype_bias=g.BF16) == -4
    assert _status(g, **ok, epilogue=11) == -8
    assert _status(g, **ok, epilogue=-1) == -8
    # the scale is checked exactly where an epilogue uses it
    for e in (g.EPI_SWISH_SCALE, g.EPI_SIGMOID_SCALE_RESIDUAL):
        assert _status(g, **ok, epilogue=e, scale=float("nan")) == -10
        assert _status(g, **ok, epilogue=e, scale=float("inf")) == -10
        assert _status(g, **ok, epilogue=e, scale=-2.5) == 0
    assert _status(g, **ok, epilogue=g.EPI_RELU, scale=float("nan")) == 0
    assert "scale" in g.gemm_status_string(-10)
    assert _status(g, **ok, layout_a=2) == -8
    assert _status(g, **ok, dtype=4) == -8
    # 8-bit E4M3 operands: results are bf16 or fp32; only the matrix-core kernels take them
    assert _status(g, **ok, dtype=g.F8E4M3) == 0
    assert _status(g, **ok, dtype=g.F8E4M3, dtype_c=g.F32) == 0
    assert _status(g, **ok, dtype=g.F8E4M3, dtype_c=g.F8E4M3) == -4
    assert _status(g, **ok, dtype=g.F8E4M3, dtype_c=g.F16) == -4
    assert _status(g, M=64, N=64, K=72, dtype=g.F8E4M3) == -4          # K not a multiple of 16
    assert _status(g, **ok, dtype=g.F8E4M3, layout_b=g.ROW_MAJOR) == -4
    assert _status(g, M=1 << 31, N=64, K=64) == -2


def test_null_handling(g):
    lib = g.load_library()
    out = ctypes.c_void_p(123)
    assert lib.gemm_create(None, ctypes.byref(out)) == -1 and not out.value
    assert lib.gemm_create(ctypes.byref(g.GemmDesc(8, 8, 8)), None) == -1
    assert lib.gemm_destroy(None) == 0
    assert lib.gemm_run(None, 16, 16, 16, None, None) == -1
    assert lib.gemm_plan_info(None, None, 0) == -1
    p = g.gemm_create(g.GemmDesc(64, 64, 64))
    assert lib.gemm_run(p.handle, None, 16, 16, None, None) == -1
    assert lib.gemm_run(p.handle, 16, 16, 16, 16, None) == -1     # bias given, epilogue has none
    assert lib.gemm_run(p.handle, 16, 24, 32, None, None) == -5   # MFMA path wants 16-byte alignment
    g.gemm_destroy(p)
    q = g.gemm_create(g.GemmDesc(64, 64, 64, epilogue=g.EPI_BIAS))
    assert lib.gemm_run(q.handle, 16, 16, 16, None, None) == -1   # bias missing
    g.gemm_destroy(q)
    best = ctypes.c_int(5)
    assert lib.gemm_tune(None, 16, 16, 16, None, None, 0.0, ctypes.byref(best), None) == -1
    assert lib.gemm_tune(ctypes.byref(g.GemmDesc(8, 8, 8)), 16, 16, 16, None, None, 0.0, None, None) == -1
    assert lib.gemm_tune(ctypes.byref(g.GemmDesc(0, 8, 8)), 16, 16, 16, None, None, 0.0,
                         ctypes.byref(best), None) == -2 and best.value == -1
    for s in range(-9, 1):
        assert g.gemm_status_string(s) not in ("", "unknown status")
    assert g.gemm_status_string(-99) == "unknown status"


def test_kernel_choice(g):
    def kernel(**kw):
        p = g.gemm_create(g.GemmDesc(**kw))
        info = p.info()
        g.gemm_destroy(p)
        return info
    assert "kernel=mfma16_256x256x64_w2x4" in kernel(M=8192, N=8192, K=8192)
    assert "_p " in kernel(M=8192, N=8192, K=8192) and "grid=256,1,1" in kernel(M=8192, N=8192, K=8192)   # persistent workgroups
    assert "_p " not in kernel(M=8192, N=8192, K=8200) and "grid=1024,1,1" in kernel(M=8192, N=8192, K=8200)
    # wave quantisation: 384 tiles of 256x256 are 1.5 rounds of the 256 CUs: one whole round on the big
    # tile, the remaining third of the columns as a second launch
    q = kernel(M=4096, N=6144, K=4096)
    assert "kernel=mfma16_256x256" in q and "grid=256,1,1" in q and "columns=4096.." in q
    assert "kernel=mfma16_256x256" in kernel(M=4096, N=4096, K=14336)
    # one round and an eighth: the whole round on the big tile, the rest as a second launch
    two = kernel(M=4096, N=4608, K=4096)
    assert "kernel=mfma16_256x256" in two and "columns=0..4095" in two and "columns=4096.." in two
    assert "kernel=skinny_m1_w8_g1" in kernel(M=1, N=8192, K=8192)
    assert "kernel=skinny_m1_w8_g2" in kernel(M=1, N=28672, K=8192)
    for m in (2, 3, 4, 5, 8, 16):
        assert "kernel=skinnydirect_d2_b512_w4" in kernel(M=m, N=8192, K=8192)
        assert "kernel=skinnydirect_d2_b512_w4" in kernel(M=m, N=28672, K=8192)
    assert "kernel=skinny_m4_w" in kernel(M=3, N=8192, K=8192, lda=(1 << 27))      # panel offsets need 32 bits
    assert "grid=256,1,1" in kernel(M=1, N=8192, K=8192)
    assert "kernel=mfma8_256x256x128" in kernel(M=8192, N=8192, K=8192, dtype=g.F8E4M3)
    assert "kernel=mfma8_" in kernel(M=4, N=8192, K=8192, dtype=g.F8E4M3)      # no skinny fp8 kernel
    assert "kernel=f32small_16x16x256" in kernel(M=256, N=256, K=256, dtype=g.F32, layout_b=g.ROW_MAJOR)
    assert "kernel=f32small_16x16x256" in kernel(M=512, N=512, K=512, dtype=g.F32, layout_b=g.ROW_MAJOR)
    assert "kernel=simt_32x32x64" in kernel(M=512, N=512, K=512, layout_b=g.ROW_MAJOR)      # 16-bit, general layout
    assert "kernel=f32mfma_64x64x32" in kernel(M=1024, N=1024, K=1024, dtype=g.F32, layout_b=g.ROW_MAJOR)
    assert "kernel=general_mfma32_64x64x16" in kernel(M=1024, N=1022, K=1024, dtype=g.F32, layout_b=g.ROW_MAJOR)
    assert "kernel=f32mfma_64x64x32" in kernel(M=2048, N=2048, K=2048, dtype=g.F32, layout_b=g.ROW_MAJOR)
    assert "kernel=f32mfma_128x128x32" in kernel(M=4096, N=4096, K=4096, dtype=g.F32, layout_b=g.ROW_MAJOR)
    assert "kernel=general_mfma32_128x128x16" in kernel(M=4096, N=4096, K=4098, dtype=g.F32, layout_b=g.ROW_MAJOR)
    # 16-bit operands the tiled kernels cannot take go to the general kernel
    assert "kernel=simt" in kernel(M=256, N=256, K=256, layout_a=g.COL_MAJOR)
    assert "kernel=simt" in kernel(M=256, N=256, K=100)            # K not a multiple of 8
    assert "kernel=simt" in kernel(M=256, N=256, K=256, lda=257)   # rows not 16-byte aligned
    assert "kernel=general_mfma32" in kernel(M=2048, N=2048, K=2048, layout_a=g.COL_MAJOR)
    assert "kernel=mfma" in kernel(M=512, N=512, K=128, batch=64)
    assert "kernel=mfma" in kernel(M=17, N=64, K=64)


def test_config_table(g):
    names = g.config_names()
    assert len(names) == g.gemm_config_count() and len(set(names)) == len(names)
    assert g.gemm_config_name(-1) is None and g.gemm_config_name(len(names)) is None
    d = g.GemmDesc(256, 256, 256, dtype=g.F32, layout_b=g.ROW_MAJOR)
    for i, n in enumerate(names):
        try:
            p = g.gemm_create_config(d, i)
        except g.GemmError as e:
            assert e.status == -9 and not n.startswith(("simt", "general_", "f32"))     # fp32 only runs on the general kernels
        else:
            assert n.startswith(("simt", "general_", "f32")) and n in p.info()
            g.gemm_destroy(p)
    with pytest.raises(g.GemmError):
        g.gemm_create_config(d, len(names))
    d16 = g.GemmDesc(32, 4096, 4096)
    with pytest.raises(g.GemmError):                                # skinny kernels stop at M = 16
        g.gemm_create_config(d16, names.index("skinnydirect_d2_b512_w4"))


def test_build_guard_flags_kernels_that_use_scratch_memory():
    """The build refuses a library in which a kernel keeps data in scratch memory or spills vector
    registers (scalar registers parked in vector-register lanes are fine)."""
    from paper_2603_12440_amd.build import kernels_with_scratch
    remarks = "\n".join([
        "a.hpp:1:1: remark: Function Name: kernel_ok [-Rpass-analysis=kernel-resource-usage]",
        "a.hpp:1:1: remark:     VGPRs: 128 [-Rpass-analysis=kernel-resource-usage]",
        "a.hpp:1:1: remark:     ScratchSize [bytes/lane]: 0 [-Rpass-analysis=kernel-resource-usage]",
        "a.hpp:1:1: remark:     SGPRs Spill: 19 [-Rpass-analysis=kernel-resource-usage]",
        "a.hpp:1:1: remark:     VGPRs Spill: 0 [-Rpass-analysis=kernel-resource-usage]",
        "a.hpp:1:1: remark: Function Name: kernel_stack [-Rpass-analysis=kernel-resource-usage]",
        "a.hpp:1:1: remark:     ScratchSize [bytes/lane]: 1408 [-Rpass-analysis=kernel-resource-usage]",
        "a.hpp:1:1: remark:     VGPRs Spill: 0 [-Rpass-analysis=kernel-resource-usage]",
        "a.hpp:1:1: remark: Function Name: kernel_spill [-Rpass-analysis=kernel-resource-usage]",
        "a.hpp:1:1: remark:     ScratchSize [bytes/lane]: 60 [-Rpass-analysis=kernel-resource-usage]",
        "a.hpp:1:1: remark:     VGPRs Spill: 50 [-Rpass-analysis=kernel-resource-usage]",
        "warning: something else",
    ])
    assert kernels_with_scratch(remarks) == ["kernel_stack", "kernel_spill"]
    assert kernels_with_scratch("") == []


def test_tuning_mode_switch_and_environment(g):
    """Tuning mode is off by default, follows GEMM_TUNE at first use, and the switch returns the
    previous setting; the table of remembered problems starts empty (no device needed)."""
    import subprocess, sys
    code = ("import paper_2603_12440_amd as g; "
            "print(int(g.gemm_set_autotune(True)), int(g.gemm_set_autotune(False)), int(g.gemm_set_autotune(False)), "
            "g.gemm_autotune_entries())")
    def run(env_value):
        env = dict(os.environ)
        env.pop("GEMM_TUNE", None)
        if env_value is not None:
            env["GEMM_TUNE"] = env_value
        out = subprocess.run([sys.executable, "-c", code], cwd=ROOT, env=env, capture_output=True, text=True)
        assert out.returncode == 0, out.stderr
        return out.stdout.split()
    assert run(None) == ["0", "1", "0", "0"]
    assert run("0") == ["0", "1", "0", "0"]
    assert run("") == ["0", "1", "0", "0"]
    assert run("1") == ["1", "1", "0", "0"]
    g.gemm_autotune_clear()
    assert g.gemm_autotune_entries() == 0


def test_overflowing_extents_are_refused(g):
    """major x ld beyond 2^62 elements cannot be addressed: BAD_LD, decided without overflow."""
    for kw in (dict(M=1 << 30, N=64, K=64, lda=1 << 40), dict(M=64, N=1 << 30, K=64, ldb=1 << 40),
               dict(M=1 << 30, N=64, K=64, ldc=1 << 40)):
        with pytest.raises(g.GemmError) as e:
            g.gemm_create(g.GemmDesc(**kw))
        assert e.value.status == -3, kw


def test_gemm_log_names_the_kernel():
    """GEMM_LOG=1: one line per plan on stderr with the kernel and tile it got."""
    import subprocess
    import sys
    code = ("import paper_2603_12440_amd as g; p = g.gemm_create(g.GemmDesc(8192, 8192, 8192)); g.gemm_destroy(p); "
            "p = g.gemm_create(g.GemmDesc(1, 8192, 8192)); g.gemm_destroy(p)")
    for env_val, want in (("1", 2), ("0", 0)):
        r = subprocess.run([sys.executable, "-c", code], capture_output=True, text=True, cwd=ROOT,
                           env=dict(os.environ, GEMM_LOG=env_val))
        assert r.returncode == 0, r.stderr
        lines = [l for l in r.stderr.splitlines() if l.startswith("[mi355gemm] plan")]
        assert len(lines) == want, r.stderr
        if want:
            assert "8192 x 8192 x 8192" in lines[0] and "kernel=mfma16_256x256" in lines[0]
            assert "kernel=skinny_m1" in lines[1]
