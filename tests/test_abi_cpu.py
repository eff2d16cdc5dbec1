"""Boundary checks that need no GPU: the library loads, exports every symbol the header
declares, and rejects bad arguments on the host before any launch."""
import ctypes
import os
import re

import pytest

import paper_2302_05045_amd as samo

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE = 0x10000  # non-null, 16-byte aligned; never dereferenced on these paths


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "samo.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(samo_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = _declared_symbols()
    assert {"samo_build_index", "samo_decompress", "samo_gather_grads", "samo_adam_step",
            "samo_fused_step", "samo_fused_step_batched"} <= set(names)
    handle = ctypes.CDLL(samo.LIB_PATH)
    for name in names:
        assert hasattr(handle, name), name
    assert set(names) == set(samo._SIGNATURES), "binding and header disagree"


def test_abi_version_and_strings():
    L = samo.lib()
    assert L.samo_abi_version() == 4
    assert samo.status_string(0) == "ok"
    for s in range(-8, 0):
        assert samo.status_string(s) not in ("ok", "unknown status")
    assert samo.status_string(-99) == "unknown status"


def test_seg_ptr_len():
    L = samo.lib()
    assert L.samo_seg_ptr_len(0) == 1
    assert L.samo_seg_ptr_len(1) == 2
    assert L.samo_seg_ptr_len(1024) == 2
    assert L.samo_seg_ptr_len(1025) == 3
    assert L.samo_seg_ptr_len(2**31 - 1) == 2**21 + 1
    assert L.samo_seg_ptr_len(2**31) == -1
    assert L.samo_seg_ptr_len(-1) == -1


def _cfg(**kw):
    base = dict(step=1, lr=1e-4, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.0, decoupled_wd=0)
    base.update(kw)
    return samo.adam_cfg(**base)


def test_size_and_null_rejection():
    L = samo.lib()
    big = 2**31
    assert L.samo_decompress(FAKE, FAKE, FAKE, 1, FAKE, big, None) == samo.SAMO_ERR_SIZE
    assert L.samo_decompress(FAKE, FAKE, FAKE, 5, FAKE, 4, None) == samo.SAMO_ERR_SIZE
    assert L.samo_decompress(FAKE, FAKE, FAKE, -1, FAKE, 4, None) == samo.SAMO_ERR_SIZE
    assert L.samo_decompress(None, FAKE, FAKE, 1, FAKE, 4, None) == samo.SAMO_ERR_NULL
    assert L.samo_decompress(FAKE, None, FAKE, 1, FAKE, 4, None) == samo.SAMO_ERR_NULL
    assert L.samo_decompress(FAKE, FAKE, None, 1, FAKE, 4, None) == samo.SAMO_ERR_NULL
    assert L.samo_decompress(FAKE, FAKE, FAKE, 1, None, 4, None) == samo.SAMO_ERR_NULL
    assert L.samo_decompress(FAKE, None, None, 3, FAKE, 4, None) == samo.SAMO_ERR_SIZE  # dense needs nnz == n
    assert L.samo_decompress(FAKE + 4, FAKE, FAKE, 1, FAKE, 4, None) == samo.SAMO_ERR_ALIGN
    assert L.samo_decompress(FAKE, FAKE, FAKE, 1, FAKE + 2, 4, None) == samo.SAMO_ERR_ALIGN
    assert L.samo_build_index(FAKE, big, FAKE, 1, FAKE, FAKE, None) == samo.SAMO_ERR_SIZE
    assert L.samo_build_index(None, 8, FAKE, 8, FAKE, FAKE, None) == samo.SAMO_ERR_NULL
    assert L.samo_build_index(FAKE, 8, None, 8, FAKE, FAKE, None) == samo.SAMO_ERR_NULL
    assert L.samo_build_index(FAKE, 8, FAKE, -1, FAKE, FAKE, None) == samo.SAMO_ERR_SIZE
    jobs = (samo.IndexJob * 2)()
    jobs[0].mask, jobs[0].n, jobs[0].seg_ptr, jobs[0].nnz = FAKE, 8, FAKE, FAKE
    jobs[1].mask, jobs[1].n, jobs[1].seg_ptr, jobs[1].nnz = FAKE, 2**31, FAKE, FAKE
    assert L.samo_build_index_batched(jobs, 2, None) == samo.SAMO_ERR_SIZE     # second job bad: nothing launched
    jobs[1].n, jobs[1].idx_capacity = 8, 4
    assert L.samo_build_index_batched(jobs, 2, None) == samo.SAMO_ERR_NULL     # capacity without idx
    assert L.samo_build_index_batched(None, 1, None) == samo.SAMO_ERR_NULL
    assert L.samo_build_index_batched(None, 0, None) == samo.SAMO_OK
    assert L.samo_count_nonzero(FAKE, 8, None, FAKE, None) == samo.SAMO_ERR_NULL
    assert L.samo_count_nonzero(FAKE + 1, 8, FAKE, FAKE, None) == samo.SAMO_ERR_ALIGN
    assert L.samo_gather_grads(FAKE, 8, None, 4, 1.0, FAKE, None) == samo.SAMO_ERR_NULL
    assert L.samo_gather_grads(None, 8, FAKE, 4, 1.0, FAKE, None) == samo.SAMO_ERR_NULL
    assert L.samo_stream_copy(FAKE, FAKE, 24, None) == samo.SAMO_ERR_SIZE
    assert L.samo_mfma_rate_probe(-1, FAKE, 1, None, None) == samo.SAMO_ERR_SIZE
    assert L.samo_mfma_rate_probe(1, FAKE, 1 << 17, None, None) == samo.SAMO_ERR_SIZE
    assert L.samo_mfma_rate_probe(1, None, 1, None, None) == samo.SAMO_ERR_NULL
    assert L.samo_validate_index(FAKE, 4, 8, None, None, None) == samo.SAMO_ERR_NULL


@pytest.mark.parametrize("kw", [dict(step=0), dict(beta1=1.0), dict(beta2=-0.1), dict(eps=0.0), dict(eps=float("nan")),
                                dict(lr=float("inf")), dict(weight_decay=-1.0)])
def test_bad_adam_hyperparameters(kw):
    L = samo.lib()
    cfg = _cfg(**kw)
    assert L.samo_adam_step(FAKE, FAKE, FAKE, FAKE, 4, ctypes.byref(cfg), None) == samo.SAMO_ERR_ARG
    assert L.samo_fused_step(FAKE, FAKE, 8, FAKE, FAKE, 4, FAKE, FAKE, FAKE, 1.0, ctypes.byref(cfg), None) \
        == samo.SAMO_ERR_ARG


@pytest.mark.parametrize("scale", [0.0, -1.0, float("inf"), float("nan")])
def test_bad_loss_scale(scale):
    L = samo.lib()
    cfg = _cfg()
    assert L.samo_gather_grads(FAKE, 8, FAKE, 4, scale, FAKE, None) == samo.SAMO_ERR_ARG
    assert L.samo_fused_step(FAKE, FAKE, 8, FAKE, FAKE, 4, FAKE, FAKE, FAKE, scale, ctypes.byref(cfg), None) \
        == samo.SAMO_ERR_ARG


def test_sgd_and_new_single_layer_entries_reject_bad_arguments():
    L = samo.lib()
    good = samo.sgd_cfg(0.1, 0.9, 0.0)
    assert L.samo_sgd_step(FAKE, FAKE, FAKE, 4, None, None) == samo.SAMO_ERR_NULL
    assert L.samo_sgd_step(FAKE, None, FAKE, 4, ctypes.byref(good), None) == samo.SAMO_ERR_NULL
    for bad in (samo.sgd_cfg(float("nan")), samo.sgd_cfg(0.1, 1.0), samo.sgd_cfg(0.1, -0.1), samo.sgd_cfg(0.1, 0.9, -1.0)):
        assert L.samo_sgd_step(FAKE, FAKE, FAKE, 4, ctypes.byref(bad), None) == samo.SAMO_ERR_ARG
        assert L.samo_fused_sgd_step(FAKE, FAKE, 8, FAKE, FAKE, 4, FAKE, FAKE, 1.0, ctypes.byref(bad), None) \
            == samo.SAMO_ERR_ARG
    assert L.samo_gather_grads_fp16(FAKE, 8, FAKE, 4, None, 0, None) == samo.SAMO_ERR_NULL
    assert L.samo_gather_grads_fp16(FAKE, 8, FAKE, 9, FAKE, 0, None) == samo.SAMO_ERR_SIZE
    assert L.samo_gather_grads_fp16(FAKE, 8, FAKE, 4, FAKE + 2, 0, None) == samo.SAMO_ERR_ALIGN
    cfg = _cfg()
    assert L.samo_adam_expand_step(None, FAKE, 8, FAKE, FAKE, 4, FAKE, FAKE, FAKE, 1.0, ctypes.byref(cfg), None) \
        == samo.SAMO_ERR_NULL
    assert L.samo_adam_expand_step(FAKE, FAKE, 8, FAKE, FAKE, 4, FAKE, FAKE, FAKE, 0.0, ctypes.byref(cfg), None) \
        == samo.SAMO_ERR_ARG
    assert L.samo_grad_stats_batched(None, 0, 1.0, FAKE, FAKE, 16, None) == samo.SAMO_ERR_NULL
    assert L.samo_plan_stats_workspace_bytes(None, None) == samo.SAMO_ERR_NULL


def test_null_cfg_and_plan():
    L = samo.lib()
    assert L.samo_adam_step(FAKE, FAKE, FAKE, FAKE, 4, None, None) == samo.SAMO_ERR_NULL
    assert L.samo_fused_step_batched(None, 1.0, ctypes.byref(_cfg()), None, None) == samo.SAMO_ERR_NULL
    out = samo.PlanDesc()
    ws, ws_bytes = FAKE, 1 << 20
    bad = (samo.LayerDesc * 1)()
    bad[0].n, bad[0].nnz = 8, 9
    assert L.samo_plan_init(bad, 1, ws, ws_bytes, None, ctypes.byref(out)) == samo.SAMO_ERR_SIZE
    bad[0].nnz = 4
    bad[0].idx, bad[0].seg_ptr = FAKE, FAKE
    assert L.samo_plan_init(bad, 1, ws, ws_bytes, None, ctypes.byref(out)) == samo.SAMO_ERR_NULL      # p missing
    bad[0].p = FAKE + 8
    assert L.samo_plan_init(bad, 1, ws, ws_bytes, None, ctypes.byref(out)) == samo.SAMO_ERR_ALIGN
    bad[0].p = FAKE
    assert L.samo_plan_init(bad, 1, ws, 16, None, ctypes.byref(out)) == samo.SAMO_ERR_WORKSPACE
    assert L.samo_plan_init(bad, 1, None, ws_bytes, None, ctypes.byref(out)) == samo.SAMO_ERR_WORKSPACE
    assert not out.d_layers and out.num_layers == 0


def test_plan_workspace_size_follows_the_layer_sizes():
    """Host arithmetic only: descriptors (104 bytes each), two start tables, one 8-byte record per
    tile and per 256-element chunk, every table padded to 256 bytes."""
    L = samo.lib()
    need = ctypes.c_size_t()
    d = (samo.LayerDesc * 2)()
    d[0].n, d[0].nnz, d[0].idx, d[0].seg_ptr = 1 << 20, 100_000, FAKE, FAKE          # pruned
    d[1].n, d[1].nnz = 5000, 5000                                                     # dense: one tile per segment
    assert L.samo_plan_workspace_bytes(d, 2, ctypes.byref(need)) == samo.SAMO_OK
    tiles = -(-(6144 * 1024 + 24 * 100_000) // 32768) + 5
    chunks = -(-100_000 // 256) + -(-5000 // 256)
    pad = lambda x: -(-x // 256) * 256
    assert need.value == pad(2 * ctypes.sizeof(samo.LayerDesc)) + 2 * pad(3 * 8) + pad(8 * tiles) + pad(8 * chunks)
    # a model that keeps less than 7 % of its elements is cut into heavier tiles: 65536, or 49152 with an fp32 dense
    # side; the size reported before the arrays are known is that of the lighter ones
    d[0].nnz, d[1].n, d[1].nnz = 50_000, 0, 0
    assert L.samo_plan_workspace_bytes(d, 2, ctypes.byref(need)) == samo.SAMO_OK
    tiles = -(-(6144 * 1024 + 24 * 50_000) // 49152)
    assert need.value == pad(2 * ctypes.sizeof(samo.LayerDesc)) + 2 * pad(3 * 8) + pad(8 * tiles) + pad(8 * -(-50_000 // 256))
    assert L.samo_plan_workspace_bytes(d, 0, ctypes.byref(need)) == samo.SAMO_OK and need.value == 2 * 256
    assert samo.samo_index_workspace_bytes(1025) == 12
    assert L.samo_static_scratch_bytes() == 16 << 20


def test_library_is_stateless_no_allocation_copy_or_synchronisation():
    """The shared library imports no HIP call that allocates, frees, copies or synchronises, and reads
    no environment variable: every entry point only launches kernels on the caller's stream."""
    import subprocess
    out = subprocess.run(["nm", "-D", "--undefined-only", samo.LIB_PATH], capture_output=True, text=True, check=True).stdout
    imported = set(line.split()[-1].split("@")[0] for line in out.splitlines() if line.strip())
    assert "hipLaunchKernel" in imported or any(s.startswith("hipLaunchKernel") or s.startswith("__hipPushCallConfiguration")
                                                for s in imported)
    banned = [s for s in imported if re.match(r"hip(Malloc|Free|Memcpy|Memset|DeviceSynchronize|StreamSynchronize|"
                                              r"HostMalloc|HostFree|EventSynchronize|StreamCreate|ExtMalloc)", s)]
    assert not banned, banned
    assert "getenv" not in imported and "secure_getenv" not in imported


def test_memory_model_matches_paper_formulas(golden_dir):
    from conftest import read_golden
    gold = read_golden(golden_dir + "/memory_model.txt")
    phi, nnz = 2_516_582_400, 251_658_240
    d, s, r = samo.samo_memory_model(phi, nnz)
    assert d == int(gold["default_bytes_per_param"]) * phi
    assert s == int(gold["samo_bytes_per_kept_param"]) * nnz + int(gold["samo_bytes_per_param"]) * phi
    assert round(100 * (d - s) / d) == int(gold["saved_percent_at_0.9"])
    assert r == 16 * nnz + 2 * phi
    with pytest.raises(samo.SamoError):
        samo.samo_memory_model(10, 11)


def test_binding_refuses_cpu_tensors():
    import torch
    with pytest.raises(TypeError):
        samo.samo_decompress(torch.zeros(4), torch.zeros(4, dtype=torch.int32), torch.zeros(2, dtype=torch.int32),
                             torch.zeros(8, dtype=torch.float16))


def test_header_is_plain_c(tmp_path):
    """include/samo.h is a C header: it compiles on its own as C99 and as C++17, pedantically,
    and a C translation unit can name every type and take the address of every entry point."""
    import re
    import subprocess
    header = os.path.join(ROOT, "include", "samo.h")
    names = sorted(set(re.findall(r"\b(samo_[a-z0-9_]+)\s*\(", open(header).read())))
    assert "samo_fused_step_batched" in names and "samo_build_index" in names
    src = tmp_path / "use_samo.c"
    body = "\n".join("    p[%d] = (void (*)(void))%s;" % (i, n) for i, n in enumerate(names))
    src.write_text('#include "samo.h"\n'
                   "void (*p[%d])(void);\n" % len(names) +
                   "int use(void) {\n"
                   "    samo_adam_cfg a; samo_sgd_cfg s; samo_grad_stats g; samo_step_guard q; samo_index_job j; samo_layer l;\n"
                   "    (void)a; (void)s; (void)g; (void)q; (void)j; (void)l;\n" + body + "\n    return SAMO_OK;\n}\n")
    inc = "-I" + os.path.join(ROOT, "include")
    subprocess.check_call(["gcc", "-std=c99", "-Wall", "-Wextra", "-Werror", "-pedantic", inc, "-c", str(src),
                           "-o", str(tmp_path / "use_samo.o")])
    subprocess.check_call(["g++", "-std=c++17", "-Wall", "-Wextra", "-Werror", "-pedantic", inc, "-x", "c++", "-c",
                           str(src), "-o", str(tmp_path / "use_samo_cpp.o")])


def test_weight_gradient_kernels_touch_m0_only_in_their_lds_copies(tmp_path):
    """The direct-to-LDS copies of wgrad.hip set M0 from inline assembly, which cannot declare that
    register clobbered; the kernels are right only as long as the compiler itself never uses M0 in
    them.  Checked on the generated ISA after every build (so a compiler change shows here and not
    as wrong numbers): in the whole device code of wgrad.hip, M0 appears only as the destination of
    `s_mov_b32 m0, <sgpr>`, each followed by `s_nop 0` and `global_load_lds_dwordx4` — exactly the
    copy helper's three instructions."""
    import subprocess
    from paper_2302_05045_amd import _build
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    asm = tmp_path / "wgrad.s"
    subprocess.check_call([hipcc] + [f for f in _build.FLAGS if f not in ("-shared", "-fPIC")] +
                          ["-S", "--cuda-device-only", "-I", os.path.join(ROOT, "include"), "-I", _build.CSRC,
                           os.path.join(_build.CSRC, "wgrad.hip"), "-o", str(asm)],
                          stdout=subprocess.DEVNULL, stderr=subprocess.DEVNULL)
    lines = [ln.split(";")[0].strip() for ln in asm.read_text().splitlines()]
    code = [ln for ln in lines if ln and not ln.startswith(".") and not ln.endswith(":")]
    uses = [i for i, ln in enumerate(code) if re.search(r"\bm0\b", ln)]
    assert len(uses) >= 16, "the copy helper's M0 writes are expected in four kernels"
    for i in uses:
        assert re.fullmatch(r"s_mov_b32 m0, s\d+", code[i]), code[i]
        assert code[i + 1] == "s_nop 0" and code[i + 2].startswith("global_load_lds_dwordx4 "), code[i:i + 3]
    assert sum(ln.startswith("global_load_lds_dwordx4 ") for ln in code) == len(uses)


def test_host_side_of_the_library_under_sanitizers(tmp_path):
    """The library's host code (argument validation, status strings, byte accounting) built with
    AddressSanitizer and UBSan and driven through every entry point with arguments it must reject
    before enqueueing anything (tests/abi_sanitizer_driver.c): no GPU needed, nothing dereferenced."""
    import subprocess
    from paper_2302_05045_amd import _build
    exe = str(tmp_path / "abi_san")
    obj = str(tmp_path / "driver.o")
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    clang = os.path.join(os.path.dirname(os.path.realpath(hipcc)), "..", "llvm", "bin", "clang")
    if not os.path.exists(clang):
        clang = "/opt/rocm/llvm/bin/clang"
    inc = ["-I", os.path.join(ROOT, "include")]
    # the driver is C (it also checks that the header serves a C caller), same compiler family as
    # hipcc so that both halves share one sanitizer runtime
    subprocess.check_call([clang, "-std=c99", "-O1", "-g", "-fsanitize=address,undefined", "-Wall", "-Werror"] + inc +
                          ["-c", os.path.join(ROOT, "tests", "abi_sanitizer_driver.c"), "-o", obj])
    srcs = [os.path.join(_build.CSRC, s) for s in _build.SOURCES]
    cmd = [hipcc, "-O1", "-g", "-std=c++17", "--offload-arch=gfx950",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined"] + inc + \
          ["-I", _build.CSRC] + srcs + ["-x", "none", obj, "-o", exe]
    subprocess.check_call(cmd, stdout=subprocess.DEVNULL, stderr=subprocess.DEVNULL)
    out = subprocess.run([exe], capture_output=True, text=True,
                         env=dict(os.environ, ASAN_OPTIONS="detect_leaks=0:protect_shadow_gap=0"))
    assert out.returncode == 0, (out.stdout + out.stderr)[-3000:]
    assert "all rejected as documented" in out.stdout
