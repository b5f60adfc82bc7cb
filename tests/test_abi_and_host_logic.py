"""CPU-only checks of the boundary and the host logic: the shared library loads, exports every
symbol include/dsmoe.h declares, validates configurations without touching a GPU, and the host
threshold policies and input generators behave as documented."""
import ctypes
import os
import re

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "dsmoe.h")
LIB = os.path.join(ROOT, "paper_2508_18376_amd", "libdsmoe.so")


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = re.findall(r"\b((?:dsmoe|moe)_[a-z_0-9]+)\s*\(", text)
    return sorted(set(names))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(LIB):
        from paper_2508_18376_amd.build import build
        build(force=True)
    return ctypes.CDLL(LIB)


def test_every_declared_symbol_is_exported(lib):
    names = declared_functions()
    assert {"moe_partition_weights", "moe_route_and_mask", "moe_dualsparse_forward", "dsmoe_create",
            "dsmoe_workspace_bytes", "dsmoe_packed_bytes"} <= set(names)
    for n in names:
        assert hasattr(lib, n), "header declares %s but the library does not export it" % n


def cfg_struct(**kw):
    from paper_2508_18376_amd.binding import _Config
    base = dict(d_model=128, d_ff=256, n_experts=8, top_k=2, n_part=2, n_shared=0, d_ff_shared=0, expert_lo=0,
                expert_hi=8, renorm_combine=0, max_tokens=64, dtype=0)
    base.update(kw)
    return _Config(**base)


def create(lib, **kw):
    lib.dsmoe_create.restype = ctypes.c_int
    out = ctypes.c_void_p()
    c = cfg_struct(**kw)
    rc = lib.dsmoe_create(ctypes.byref(c), ctypes.byref(out))
    return rc, out


BAD = [dict(d_ff=255), dict(n_part=0), dict(n_part=9), dict(top_k=0), dict(top_k=9), dict(top_k=17, n_experts=32, expert_hi=32),
       dict(n_experts=0, expert_hi=0), dict(n_experts=513, expert_hi=513), dict(expert_lo=3, expert_hi=3), dict(expert_hi=9),
       dict(expert_lo=-1), dict(max_tokens=0), dict(dtype=2), dict(n_shared=1, d_ff_shared=0), dict(n_shared=-1),
       dict(renorm_combine=2), dict(d_model=0), dict(tall_items=2), dict(tall_items=-2)]


@pytest.mark.parametrize("kw", BAD, ids=[str(b) for b in BAD])
def test_create_rejects_bad_configurations(lib, kw):
    rc, out = create(lib, **kw)
    assert rc == -1 and not out.value


def test_create_sizes_and_path_selection(lib):
    lib.dsmoe_packed_bytes.restype = ctypes.c_size_t
    lib.dsmoe_workspace_bytes.restype = ctypes.c_size_t
    lib.dsmoe_uses_mfma.restype = ctypes.c_int
    lib.dsmoe_packed_bytes.argtypes = lib.dsmoe_workspace_bytes.argtypes = lib.dsmoe_uses_mfma.argtypes = [ctypes.c_void_p]
    lib.dsmoe_destroy.argtypes = [ctypes.c_void_p]
    # fp32 layers and odd bf16 shapes take the generic kernels, regular bf16 shapes the MFMA kernels
    rc, c1 = create(lib)
    assert rc == 0 and lib.dsmoe_uses_mfma(c1) == 0
    assert lib.dsmoe_packed_bytes(c1) >= 3 * 8 * 128 * 256 * 4
    rc, c2 = create(lib, d_model=4096, d_ff=14336, n_part=4, max_tokens=4096, dtype=1)
    assert rc == 0 and lib.dsmoe_uses_mfma(c2) == 1
    assert lib.dsmoe_packed_bytes(c2) == 3 * 8 * 4096 * 14336 * 2 + 256  # no padding for this shape; + the W2 scale record
    ws = lib.dsmoe_workspace_bytes(c2)
    rows = 4096 * 2 + 8 * 256
    assert ws >= rows * 14336 * 2 + rows * 4096 * 4 and ws < 2 * (rows * 14336 * 2 + rows * 4096 * 4)
    rc, c3 = create(lib, d_model=72, d_ff=80, dtype=1)
    assert rc == 0 and lib.dsmoe_uses_mfma(c3) == 0
    rc, c4 = create(lib, d_model=2048, d_ff=1408, n_experts=64, expert_hi=64, top_k=6, n_shared=2, d_ff_shared=1408,
                    max_tokens=8192, dtype=1)
    assert rc == 0 and lib.dsmoe_uses_mfma(c4) == 1
    for c in (c1, c2, c3, c4):
        assert lib.dsmoe_destroy(c) == 0
    assert lib.dsmoe_destroy(None) == -1


def test_null_arguments_are_errors_not_crashes(lib):
    lib.dsmoe_create.restype = ctypes.c_int
    assert lib.dsmoe_create(None, None) == -1
    rc, ctx = create(lib)
    lib.moe_dualsparse_forward.restype = ctypes.c_int
    lib.moe_dualsparse_forward.argtypes = [ctypes.c_void_p] * 5 + [ctypes.c_int32] + [ctypes.c_void_p] * 3
    assert lib.moe_dualsparse_forward(ctx, None, None, None, None, 4, None, None, None) == -1
    lib.moe_route_and_mask.restype = ctypes.c_int
    lib.moe_route_and_mask.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int32] + [ctypes.c_void_p] * 6
    assert lib.moe_route_and_mask(ctx, None, -1, None, None, None, None, None, None) == -1
    lib.moe_partition_weights.restype = ctypes.c_int
    lib.moe_partition_weights.argtypes = [ctypes.c_void_p] * 10
    assert lib.moe_partition_weights(ctx, *([None] * 9)) == -1
    lib.dsmoe_profile_begin.restype = ctypes.c_int
    lib.dsmoe_profile_begin.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_int]
    assert lib.dsmoe_profile_begin(ctx, 3, 10) == -1 and lib.dsmoe_profile_begin(ctx, 1, 0) == -1
    lib.dsmoe_strerror.restype = ctypes.c_char_p
    msgs = {lib.dsmoe_strerror(c) for c in (0, -1, -2, -3, -4, -99)}
    assert len(msgs) == 6 and all(m for m in msgs)


def test_plan_layout_is_inside_the_workspace(lib):
    lib.dsmoe_plan_layout.restype = ctypes.c_int
    lib.dsmoe_workspace_bytes.restype = ctypes.c_size_t
    rc, ctx = create(lib, d_model=256, d_ff=512, max_tokens=1000, dtype=1)
    from paper_2508_18376_amd.binding import DSMOE_PLAN_FIELDS
    header = open(os.path.join(ROOT, "include", "dsmoe.h")).read()
    assert "#define DSMOE_PLAN_FIELDS %d" % DSMOE_PLAN_FIELDS in header  # the binding sizes its buffer by this
    out = (ctypes.c_int64 * DSMOE_PLAN_FIELDS)()
    assert lib.dsmoe_plan_layout(ctx, out) == DSMOE_PLAN_FIELDS == 14
    ws = lib.dsmoe_workspace_bytes(ctx)
    offs = [out[i] for i in (0, 1, 2, 3, 4, 5, 6, 7, 11, 12, 13)]
    assert all(0 <= o < ws and o % 256 == 0 for o in offs) and len(set(offs)) == len(offs)
    assert out[9] == 256 and out[8] % out[9] == 0 and out[8] >= 1000 * 2


# ------------------------------------------------------------------ host policies and generators
def test_dual_thresholds_and_rate_calibration():
    from paper_2508_18376_amd.thresholds import dual_thresholds, tau_for_drop_rate, load_aware, tau_capping_rows
    np.testing.assert_allclose(dual_thresholds(0.08, 2), [0.07, 0.09], atol=1e-7)
    np.testing.assert_allclose(dual_thresholds(0.12, 1), [0.12], atol=1e-7)
    th4 = dual_thresholds(0.3, 4)
    assert np.all(np.diff(th4) > 0) and abs(th4[0] - 0.29) < 1e-6 and abs(th4[3] - 0.31) < 1e-6
    rng = np.random.default_rng(0)
    n = rng.beta(2, 5, size=20000)
    for rate in (0.125, 0.25, 0.5):
        th = tau_for_drop_rate(n, 2, rate)
        got = np.mean([(n < t).mean() for t in th])
        assert abs(got - rate) < 0.02
        assert min(np.abs(n[:, None] - th[None, :].astype(np.float64)).min(axis=0)) > 1e-7
    assert np.all(tau_for_drop_rate(n, 4, 0.0) == 0)
    # load-aware rule: overloaded experts get the maximum, underloaded ones proportionally less
    tab = load_aware(np.array([200, 100, 50, 50]), np.array([0.1, 0.12]))
    np.testing.assert_allclose(tab[0], [0.1, 0.12], rtol=1e-6)
    np.testing.assert_allclose(tab[1], [0.1, 0.12], rtol=1e-6)
    np.testing.assert_allclose(tab[2], [0.05, 0.06], rtol=1e-6)
    cap = tau_capping_rows(n, 1, 5000)
    assert abs((n >= cap[0]).sum() - 5000) < 150
    assert np.all(tau_capping_rows(n[:100], 2, 500) == 0)


def test_generators_are_seeded_and_order_independent():
    from synth import LAYERS, LayerSpec, make_layer, make_logits, zipf_logit_bias, bf16_bits_to_f32
    spec = LayerSpec("g", T=32, D=16, F=24, E=4, K=2, P=2, dtype="bf16", seed=5, n_shared=1, F_sh=8)
    a, b = make_layer(spec, threads=1), make_layer(spec, threads=4)
    for k in a:
        assert np.array_equal(a[k], b[k]), k
    assert np.array_equal(make_logits(spec), a["logits"])
    assert a["w1"].dtype == np.uint16 and a["w1"].shape == (4, 16, 24) and a["sh_w2"].shape == (1, 8, 16)
    assert abs(bf16_bits_to_f32(a["w1"]).std() - 0.02) < 0.004
    for e in range(4):
        assert sorted(a["perm"][e]) == list(range(24))
    c5 = LAYERS["C5"]
    bias = zipf_logit_bias(c5)
    assert abs(np.exp(bias).sum() - 1.0) < 1e-5 and bias.argmax() == 0 and c5.resident == (0, 2)
    assert [LAYERS[k].T for k in ("C1", "C2", "C3", "C4", "C5")] == [64, 4096, 8192, 8192, 16384]


def test_later_entry_points_validate_before_touching_the_gpu(lib):
    """Bad arguments of the reconstruction / threshold / router / transformation calls are refused
    on the host (no GPU is present in this test)."""
    vp, i32 = ctypes.c_void_p, ctypes.c_int32
    rc, ctx = create(lib, max_tokens=64)
    assert rc == 0
    fake = ctypes.c_void_p(4096)       # non-null, 256-byte aligned; never dereferenced by a refused call
    odd = ctypes.c_void_p(4096 + 8)    # misaligned workspace
    lib.moe_profile_importance.restype = ctypes.c_int
    lib.moe_profile_importance.argtypes = [vp, vp, vp, vp, i32, i32, vp, vp, vp]
    assert lib.moe_profile_importance(ctx, fake, fake, fake, 4, 4, fake, fake, None) == -1    # metric 0..3
    assert lib.moe_profile_importance(ctx, fake, fake, fake, 65, 0, fake, fake, None) == -1   # T > max_tokens
    assert lib.moe_profile_importance(ctx, fake, fake, fake, 4, 0, fake, odd, None) == -1     # workspace alignment
    assert lib.moe_profile_importance(ctx, fake, None, fake, 4, 0, fake, fake, None) == -1    # x missing
    lib.moe_importance_to_perm.restype = ctypes.c_int
    lib.moe_importance_to_perm.argtypes = [vp, vp, vp, vp]
    assert lib.moe_importance_to_perm(ctx, None, fake, None) == -1
    lib.moe_select_thresholds.restype = ctypes.c_int
    lib.moe_select_thresholds.argtypes = [vp, vp, i32, vp, i32, i32, vp, vp, vp, vp]
    assert lib.moe_select_thresholds(ctx, fake, 4, fake, 3, 0, fake, None, fake, None) == -1   # 3 does not divide 8 experts
    assert lib.moe_select_thresholds(ctx, fake, 4, fake, 0, 0, fake, None, fake, None) == -1
    assert lib.moe_select_thresholds(ctx, fake, 4, fake, 1, -1, fake, None, fake, None) == -1  # negative row budget
    assert lib.moe_select_thresholds(ctx, fake, 4, None, 1, 0, fake, None, fake, None) == -1   # tau_max missing
    assert lib.moe_select_thresholds(ctx, fake, 65, fake, 1, 0, fake, None, fake, None) == -1
    lib.moe_thresholds_for_drop_rate.restype = ctypes.c_int
    lib.moe_thresholds_for_drop_rate.argtypes = [vp, vp, i32, ctypes.c_double, ctypes.POINTER(i32), vp, vp, vp, vp]
    offs = (i32 * 2)(-41, 41)
    assert lib.moe_thresholds_for_drop_rate(ctx, fake, 4, 1.5, offs, fake, None, fake, None) == -1             # rate in [0, 1]
    assert lib.moe_thresholds_for_drop_rate(ctx, fake, 4, float("nan"), offs, fake, None, fake, None) == -1
    assert lib.moe_thresholds_for_drop_rate(ctx, fake, 4, 0.25, (i32 * 2)(0, 5000), fake, None, fake, None) == -1  # offset off the grid
    assert lib.moe_thresholds_for_drop_rate(ctx, fake, 4, 0.25, None, fake, None, fake, None) == -1
    lib.moe_pack_router.restype = lib.moe_router_logits.restype = ctypes.c_int
    lib.moe_pack_router.argtypes = [vp, vp, vp, vp]
    lib.moe_router_logits.argtypes = [vp, vp, vp, i32, vp, vp]
    assert lib.moe_pack_router(ctx, None, fake, None) == -1
    assert lib.moe_router_logits(ctx, None, fake, 4, fake, None) == -1
    assert lib.moe_router_logits(ctx, fake, fake, 4, None, None) == -1
    assert lib.moe_router_logits(ctx, fake, odd, 4, fake, None) == -1                          # x must be 16-byte aligned
    lib.moe_dualsparse_forward_routed.restype = ctypes.c_int
    lib.moe_dualsparse_forward_routed.argtypes = [vp, vp, vp, vp, vp, i32, vp, vp, vp, vp]
    assert lib.moe_dualsparse_forward_routed(ctx, fake, None, fake, fake, 4, fake, None, fake, None) == -1
    assert lib.moe_dualsparse_forward_routed(ctx, fake, fake, fake, fake, 65, fake, None, fake, None) == -1
    lib.moe_transform_complete.restype = ctypes.c_int
    lib.moe_transform_complete.argtypes = [vp] * 12
    assert lib.moe_transform_complete(ctx, None, None, fake, fake, None, None, fake, fake, fake, None, None) == -1   # w1 missing
    assert lib.moe_transform_complete(ctx, fake, fake, fake, fake, None, None, fake, fake, fake, None, None) == -1   # wg without wg_out
    assert lib.moe_transform_complete(ctx, None, fake, fake, fake, fake, None, fake, fake, fake, None, None) == -1   # perm needs a workspace
    lib.dsmoe_router_packed_bytes.restype = ctypes.c_size_t
    lib.dsmoe_router_packed_bytes.argtypes = [vp]
    assert lib.dsmoe_router_packed_bytes(ctx) == 128 * 8 * 4          # fp32 layer: W_g widened to float, [D][E]
    rc, c2 = create(lib, d_model=4096, d_ff=14336, n_part=4, max_tokens=64, dtype=1)
    assert lib.dsmoe_router_packed_bytes(c2) == 4096 * 32 * 2         # MFMA operand order, experts padded to 32
    lib.dsmoe_destroy.argtypes = [vp]
    lib.dsmoe_destroy(ctx)
    lib.dsmoe_destroy(c2)


def test_build_script_is_importable_without_the_library():
    """A fresh tree has no libdsmoe.so: importing the package or its build script must not need it
    (only the first use of the binding does, and that fails loudly)."""
    import subprocess
    import sys
    code = ("import sys, paper_2508_18376_amd, paper_2508_18376_amd.build, paper_2508_18376_amd.thresholds; "
            "assert 'paper_2508_18376_amd.binding' not in sys.modules; print('ok')")
    out = subprocess.run([sys.executable, "-c", code], cwd=ROOT, capture_output=True, text=True)
    assert out.returncode == 0 and out.stdout.strip() == "ok", out.stderr


def test_build_refuses_register_spills_in_the_gemm_kernels():
    """The build reads the compiler's resource remarks and fails when one of the MFMA GEMM kernels
    uses scratch memory (a spill inside their main loops stalls the load queue): the parser that
    decides it, on a remark text of the compiler's format."""
    from paper_2508_18376_amd import build
    remarks = "\n".join([
        "a.hip:1:1: remark: Function Name: _ZN5dsmoe17gemm1_mfma_kernelILb0EEEvNS_6LayoutEi [-Rpass-analysis=kernel-resource-usage]",
        "a.hip:1:1: remark:     VGPRs: 256 [-Rpass-analysis=kernel-resource-usage]",
        "a.hip:1:1: remark:     ScratchSize [bytes/lane]: 20 [-Rpass-analysis=kernel-resource-usage]",
        "a.hip:1:1: remark: Function Name: _ZN5dsmoe17gemm2_mfma_kernelILb1EEEvNS_6LayoutEi [-Rpass-analysis=kernel-resource-usage]",
        "a.hip:1:1: remark:     ScratchSize [bytes/lane]: 0 [-Rpass-analysis=kernel-resource-usage]",
        "a.hip:1:1: remark: Function Name: _ZN5dsmoe11some_helperEv [-Rpass-analysis=kernel-resource-usage]",
        "a.hip:1:1: remark:     ScratchSize [bytes/lane]: 64 [-Rpass-analysis=kernel-resource-usage]",
    ])
    bad = build._scratch_users(remarks, build.NO_SCRATCH["gemm_mfma.hip"])
    assert len(bad) == 1 and "gemm1_mfma_kernel" in bad[0] and "20" in bad[0]
    assert build._scratch_users(remarks.replace(": 20 ", ": 0 "), build.NO_SCRATCH["gemm_mfma.hip"]) == []


def test_header_is_plain_c(lib, tmp_path):
    """include/dsmoe.h is the boundary: it must compile as C (no C++ or HIP types in the
    signatures) and a C program must link against the library's entry points."""
    import shutil
    import subprocess
    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("no C compiler")
    src = tmp_path / "use_dsmoe.c"
    src.write_text(
        '#include "dsmoe.h"\n'
        "#include <stdio.h>\n"
        "int main(void) {\n"
        "  dsmoe_config c = {0};\n"
        "  dsmoe_ctx* ctx = 0;\n"
        "  int rc = dsmoe_create(&c, &ctx);  /* an all-zero configuration is refused, without a GPU */\n"
        '  printf("%d %s\\n", rc, dsmoe_strerror(rc));\n'
        "  return rc == 0;\n"
        "}\n")
    inc = os.path.join(ROOT, "include")
    obj = tmp_path / "use_dsmoe.o"
    r = subprocess.run([gcc, "-std=c99", "-Wall", "-Werror", "-pedantic", "-I", inc, "-c", str(src), "-o", str(obj)],
                       capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
    exe = tmp_path / "use_dsmoe"
    libdir = os.path.dirname(LIB)
    r = subprocess.run([gcc, str(obj), "-o", str(exe), "-L", libdir, "-l:libdsmoe.so", "-Wl,-rpath," + libdir,
                        "-Wl,--allow-shlib-undefined"], capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
    r = subprocess.run([str(exe)], capture_output=True, text=True, timeout=120)
    assert r.returncode == 0 and r.stdout.split()[0] != "0", (r.returncode, r.stdout, r.stderr)
