"""The C-ABI library loads and exports every entry point that include/gmpgr_ann.h declares, and
argument errors that are detected before any HIP call come back as error codes (no GPU needed)."""
import ctypes
import os
import re
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "gmpgr_ann.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ann_[a-z_0-9]+)\s*\(", text)))


@pytest.fixture(scope="module")
def lib():
    import paper_2502_11490_amd as ann

    if not os.path.exists(ann.lib_path()):
        from paper_2502_11490_amd.build import build

        build()
    return ann.load_library()


def test_header_and_library_agree(lib):
    names = _declared()
    assert len(names) >= 12
    for n in names:
        assert hasattr(lib, n), f"{n} declared in the header but not exported"
    from paper_2502_11490_amd.binding import EXPORTS

    assert sorted(EXPORTS) == names, "the Python binding must cover exactly the declared entry points"


def test_errors_detected_before_any_device_work(lib):
    out = ctypes.c_void_p()
    assert lib.ann_graph_load(None, None, 10, 4, 8, 0, 0, None, ctypes.byref(out)) == -1
    assert b"null" in lib.ann_last_error()
    assert lib.ann_graph_load(ctypes.c_void_p(16), ctypes.c_void_p(16), 0, 4, 8, 0, 0, None, ctypes.byref(out)) == -1
    assert lib.ann_graph_load(ctypes.c_void_p(16), ctypes.c_void_p(16), 10, 65, 8, 0, 0, None, ctypes.byref(out)) == -1
    assert lib.ann_graph_load(ctypes.c_void_p(16), ctypes.c_void_p(16), 10, 4, 8, 7, 0, None, ctypes.byref(out)) == -1
    assert lib.ann_graph_load(ctypes.c_void_p(18), ctypes.c_void_p(16), 10, 4, 8, 0, 0, None, ctypes.byref(out)) == -1
    assert out.value is None
    assert lib.ann_search_workspace_bytes(None, None, 4, 1, 1, 1, 1, 0) == 0
    assert lib.ann_mlp_load(0, None, None, None, None, 4, 0, 0, None, ctypes.byref(out)) == -1
    dims = (ctypes.c_int32 * 2)(8, 3)
    Wp = (ctypes.c_void_p * 1)(None)
    hw = (ctypes.c_float * 3)(0.5, 0.3, 0.2)
    assert lib.ann_mlp_load(1, dims, Wp, Wp, hw, 4, 0, 0, None, ctypes.byref(out)) == -1   # null layer arrays
    assert lib.ann_mlp_load(1, dims, Wp, Wp, hw, 8, 0, 0, None, ctypes.byref(out)) == -1   # d_user >= dims[0]
    assert lib.ann_search_stats(None, None, None) == -1
    assert lib.ann_profile_read(None, None) == -1
    # a graph handle needs no device work: borrowed pointers, checked shapes
    assert lib.ann_graph_load(ctypes.c_void_p(256), ctypes.c_void_p(512), 10, 4, 8, 0, 0, None, ctypes.byref(out)) == 0
    g = ctypes.c_void_p(out.value)
    assert lib.ann_search_workspace_bytes(g, None, 4, 1, 1, 1, 1, 0) == 0
    lib.ann_graph_free(g)


def test_errors_of_the_later_entry_points_without_a_device(lib):
    """Open stream, allocation-free pair scoring, exhaustive search, progress time limit, pair scoring, noise,
    quantiser: every
    argument error that can be seen before a HIP call comes back as ANN_EINVAL with a reason."""
    vp = ctypes.c_void_p
    out = vp()
    assert lib.ann_stream_open(None, None, 8, 2, 1, 1, 4, 3, 0, vp(256), vp(256), vp(256), vp(256), vp(256), 1 << 20, None,
                               ctypes.byref(out)) == -1
    assert b"null" in lib.ann_last_error() and out.value is None
    assert lib.ann_stream_open(None, None, 0, 2, 1, 1, 4, 3, 0, vp(256), vp(256), vp(256), vp(256), vp(256), 1 << 20, None,
                               ctypes.byref(out)) == -1
    assert b"capacity" in lib.ann_last_error()
    assert lib.ann_stream_open(None, None, 8, 2, 1, 1, 4, 3, 0, vp(256), vp(256), vp(256), vp(256), vp(256), 1 << 20, None,
                               None) == -1
    assert lib.ann_stream_submit(None, 1) == -1 and lib.ann_stream_step(None, 1) == -1 and lib.ann_stream_drain(None) == -1
    assert lib.ann_stream_close(None) == 0          # closing nothing is not an error
    assert lib.ann_search_stream_workspace_bytes(None, None, 8, 0, 1, 1, 4, 3, 0) == 0
    assert lib.ann_score_pairs_noalloc(None, None, vp(256), 1, 4, vp(256), vp(256), vp(256), None) == -1
    assert lib.ann_score_pairs(None, None, vp(256), 1, 4, vp(256), vp(256), vp(256), 0, None) == -1
    assert lib.ann_brute_force(None, None, vp(256), 1, 4, vp(256), vp(256), None, 0, None) == -1 and b"null" in lib.ann_last_error()
    assert lib.ann_rerank(None, None, vp(256), 1, None, 8, 4, vp(256), vp(256), None, 0, None) == -1 and b"cand_dev" in lib.ann_last_error()
    assert lib.ann_rerank(None, None, vp(256), 1, vp(256), 70000, 4, vp(256), vp(256), None, 0, None) == -1
    assert lib.ann_rerank_workspace_bytes(None, None, 4, 8, 4) == 0 and lib.ann_brute_force_workspace_bytes(None, None, 4, 4) == 0
    assert lib.ann_set_progress_timeout(ctypes.c_double(-1.0)) == -1
    assert lib.ann_set_progress_timeout(ctypes.c_double(float("nan"))) == -1
    assert lib.ann_set_progress_timeout(ctypes.c_double(600.0)) == 0
    assert lib.ann_users_add_noise(vp(256), vp(256), 4, 0, 0, ctypes.c_double(1.0), 1, 0, None) == -1       # d < 1
    assert lib.ann_users_add_noise(vp(256), vp(256), 4, 8, 2, ctypes.c_double(1.0), 1, 0, None) == -1       # 8-bit users
    assert lib.ann_users_add_noise(vp(256), vp(256), 4, 8, 0, ctypes.c_double(-1.0), 1, 0, None) == -1      # sigma < 0
    assert lib.ann_users_add_noise(None, None, 0, 8, 0, ctypes.c_double(1.0), 1, 0, None) == 0              # nothing to do
    assert lib.ann_quantize_e4m3(vp(256), 3, 16, ctypes.c_float(1.0), vp(256), None) == -1                  # fp16 source
    assert lib.ann_quantize_e4m3(vp(256), 0, 16, ctypes.c_float(0.0), vp(256), None) == -1                  # scale 0
    assert lib.ann_quantize_e4m3(None, 0, 0, ctypes.c_float(1.0), None, None) == 0
    # a graph handle and a search plan need no device: limits of the plan
    g = vp()
    assert lib.ann_graph_load(vp(256), vp(512), 1000, 32, 8, 0, 0, None, ctypes.byref(g)) == 0
    assert lib.ann_search_workspace_bytes(g, None, 4, 1, 1, 1, 1, 0) == 0 and b"null" in lib.ann_last_error()
    assert lib.ann_search_walkers_workspace_bytes(g, None, 4, 1, 0, 1) == 0 and b"T >= 1" in lib.ann_last_error()
    lib.ann_graph_free(g)


def test_binding_checks_shapes_before_the_library_is_called():
    """The binding refuses tensors whose shapes the C entry points could not check (bare pointers), on CPU tensors
    already: no GPU needed to see the refusal."""
    import torch

    import paper_2502_11490_amd.binding as b

    class FakeMlp:
        handle, dims, d_user, dtype = None, [8, 3], 4, b.ANN_F32

    class FakeGraph:
        handle = None

    users = torch.zeros(5, 4)
    with pytest.raises(ValueError, match="rows"):
        b.ann_search(FakeGraph(), FakeMlp(), users, torch.zeros(6, 2, dtype=torch.int32), 1, 4, 3, 1,
                     workspace=torch.zeros(8, dtype=torch.uint8))
    with pytest.raises(ValueError, match=r"\[Q\]\[4\]"):
        b.ann_search(FakeGraph(), FakeMlp(), torch.zeros(5, 3), torch.zeros(5, 2, dtype=torch.int32), 1, 4, 3, 1,
                     workspace=torch.zeros(8, dtype=torch.uint8))
    with pytest.raises(ValueError, match="out_ids"):
        b.ann_search(FakeGraph(), FakeMlp(), users, torch.zeros(5, 2, dtype=torch.int32), 1, 4, 3, 1,
                     workspace=torch.zeros(8, dtype=torch.uint8), out_ids=torch.zeros(5, 2, dtype=torch.int32),
                     out_scores=torch.zeros(5, 3))
    with pytest.raises(ValueError, match="one int32 per query"):
        b.ann_search_ragged(FakeGraph(), FakeMlp(), users, torch.zeros(5, 2, dtype=torch.int32),
                            torch.zeros(4, dtype=torch.int32), torch.zeros(5, dtype=torch.int32),
                            torch.zeros(5, dtype=torch.int32), 2, 8, 3, 4, workspace=torch.zeros(8, dtype=torch.uint8),
                            out_ids=torch.zeros(5, 3, dtype=torch.int32), out_scores=torch.zeros(5, 3))
    with pytest.raises(ValueError, match="pairs"):
        b.ann_score_pairs(FakeGraph(), FakeMlp(), users, torch.zeros(7, dtype=torch.int32), torch.zeros(6, dtype=torch.int32))


def test_missing_library_is_loud(monkeypatch):
    import paper_2502_11490_amd.binding as b

    monkeypatch.setattr(b, "_lib", None)
    monkeypatch.setattr(b, "_LIB_PATH", "/nonexistent/libgmpgr_ann.so")
    with pytest.raises(FileNotFoundError):
        b.load_library()


def test_generated_assembly_is_up_to_date(tmp_path):
    """The .inc files next to the kernels are written by the generator scripts beside them: what is committed
    must be what the scripts write."""
    import importlib.util
    import shutil
    csrc = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "paper_2502_11490_amd", "csrc")
    for script, inc in (("gen_stream_asm.py", "mlp_mfma_stream_asm.inc"), ("gen_f8_wide_asm.py", "mlp_mfma_f8_wide_asm.inc")):
        work = tmp_path / script.replace(".py", "")
        work.mkdir()
        shutil.copy(os.path.join(csrc, script), work / script)
        spec = importlib.util.spec_from_file_location(script[:-3], str(work / script))
        mod = importlib.util.module_from_spec(spec)
        spec.loader.exec_module(mod)
        mod.main()   # writes the .inc next to the copied script
        assert (work / inc).read_text() == open(os.path.join(csrc, inc)).read(), f"{inc} is stale: run {script}"


@pytest.mark.parametrize("source,kernel,min_statements", [("mlp_mfma_stream.hip", "mlp_mfma2_stream_kernel", 18),
                                                          ("mlp_mfma_f8.hip", "mlp_mfma2_f8_wide_kernel", 4)])
def test_kernels_keep_accumulation_registers_to_their_assembly(tmp_path, source, kernel, min_statements):
    """The widest bf16 / fp16 kernel and the wide 8-bit kernel name their 256 accumulation registers outright
    inside their assembly statements and only list them as clobbered, so nothing the compiler generates between
    two statements may touch one (a spill into them, a copy through them): in the kernel's compiled code every
    accumulation register sits between the markers of an assembly statement, and nothing is spilled."""
    import shutil
    import subprocess
    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(hipcc):
        pytest.skip("no hipcc here")
    csrc = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "paper_2502_11490_amd", "csrc")
    out = tmp_path / "kernel.s"
    from paper_2502_11490_amd import build
    flags = [f for f in build.FLAGS if f not in ("-shared", "-fPIC")]
    subprocess.run([hipcc] + flags + ["-S", "--cuda-device-only", os.path.join(csrc, source), "-o", str(out)],
                   check=True, capture_output=True)
    text = out.read_text()
    # the bodies of this kernel's instantiations: from each "<mangled name>:" label to the end-of-function label
    bodies = re.findall(r"^(_Z\w*" + kernel + r"\w*):[^\n]*\n(.*?)^\.Lfunc_end\d+:", text, re.S | re.M)
    assert bodies, "kernel not found in the compiled code"
    for name, body in bodies:
        inside, statements, outside = False, 0, []
        for line in body.split("\n"):
            if "#ASMSTART" in line:
                inside, statements = True, statements + 1
            elif "#ASMEND" in line:
                inside = False
            elif not inside:
                code = line.split(";")[0]
                if re.search(r"\ba\[?\d+", code) or "accvgpr" in code or "scratch_" in code:
                    outside.append(line.strip())
        assert statements >= min_statements, (name, statements)
        assert not outside, (name, outside[:5])


def test_bench_refuses_more_than_one_gpu():
    """The library runs on one GPU; the benchmark says so instead of launching anything."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0
    assert "one GPU" in r.stderr or "--gpus 1" in r.stderr
    assert not r.stdout.strip()


def test_the_abi_from_plain_c(lib, tmp_path):
    """tests/c_abi_check.c: the header compiles as C99 with warnings as errors, every entry point links with the
    header's prototype, and the argument errors come back from C as they do through ctypes."""
    import paper_2502_11490_amd as ann

    libdir = os.path.dirname(ann.lib_path())
    exe = str(tmp_path / "c_abi_check")
    cmd = ["gcc", "-std=c99", "-Wall", "-Wextra", "-Werror", "-I", os.path.join(ROOT, "include"),
           os.path.join(ROOT, "tests", "c_abi_check.c"), "-o", exe, "-L", libdir, "-lgmpgr_ann",
           f"-Wl,-rpath,{libdir}", "-Wl,-rpath,/opt/rocm/lib"]
    res = subprocess.run(cmd, capture_output=True, text=True)
    assert res.returncode == 0, res.stderr
    run = subprocess.run([exe], capture_output=True, text=True, timeout=120)
    assert run.returncode == 0 and "c abi ok" in run.stdout, run.stdout + run.stderr


def test_committed_traffic_summaries_belong_to_the_sources_in_the_tree():
    """bench.py reads the counter traffic of the scoring kernel and of the round kernel at the timed point from
    profiles/ and nulls a figure whose summary was taken on other kernel sources: the committed ones must match."""
    import sys

    sys.path.insert(0, ROOT)
    import bench

    assert bench.recorded_traffic("C3", 64, 8192) is not None, "profiles/c3_W64_L8192_hbm_traffic.txt: scoring kernels changed"
    assert bench.recorded_traffic("C3", 64, 8192, "round") is not None, "same file: search_kernels.hip or keys.h changed"
    assert bench.recorded_traffic("C3", 8, 1024) is not None and bench.recorded_traffic("C3", 8, 1024, "round") is not None
    assert bench.recorded_traffic("C3", 32, 8192) is None   # no such measurement
