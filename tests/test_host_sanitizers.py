"""Host code under AddressSanitizer and UndefinedBehaviorSanitizer (CPU only; GPU sanitizers are not
used):
  * the oracle, rebuilt with -fsanitize=address,undefined, runs its pins;
  * the HIP library's host side (argument validation, tile planning, table upload staging, Sec. 3.2
    schedule state), rebuilt with both sanitizers on the host pass only, runs the host-side ABI tests.
Each runs in a child process with the sanitizer's runtime preloaded (the interpreter itself is not
instrumented): a sanitizer report aborts the child, which fails the test."""
import os
import subprocess
import sys
import textwrap

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _run(code, tmp_path, asan_runtime=None):
    script = tmp_path / "child.py"
    script.write_text(textwrap.dedent(code))
    env = dict(os.environ, UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1")
    if asan_runtime:
        # the runtime goes in front of whatever is preloaded already; leaks are the interpreter's business
        env["LD_PRELOAD"] = asan_runtime + (":" + env["LD_PRELOAD"] if env.get("LD_PRELOAD") else "")
        env["ASAN_OPTIONS"] = "detect_leaks=0:halt_on_error=1:abort_on_error=1:verify_asan_link_order=0"
    p = subprocess.run([sys.executable, str(script)], cwd=ROOT, env=env, capture_output=True, text=True, timeout=900)
    assert p.returncode == 0, p.stdout[-2000:] + p.stderr[-4000:]
    assert "runtime error" not in p.stderr and "AddressSanitizer" not in p.stderr
    return p.stdout


def test_the_address_sanitizer_set_up_sees_an_overrun(tmp_path):
    """The preloaded runtime really checks the instrumented library: a tiny C function that writes one
    element past a heap array makes the child abort."""
    src = tmp_path / "overrun.c"
    src.write_text("#include <stdlib.h>\nint overrun(int n) { int* a = malloc(n * sizeof(int)); a[n] = 1; "
                   "int v = a[n]; free(a); return v; }\n")
    so = tmp_path / "overrun.so"
    subprocess.run(["gcc", "-O0", "-g", "-fsanitize=address", "-shared", "-fPIC", "-o", str(so), str(src)], check=True)
    rt = subprocess.run(["gcc", "-print-file-name=libasan.so"], capture_output=True, text=True).stdout.strip()
    script = tmp_path / "child.py"
    script.write_text(f"import ctypes as C\nC.CDLL({str(so)!r}).overrun(8)\nprint('survived')\n")
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:verify_asan_link_order=0")
    env["LD_PRELOAD"] = rt + (":" + env["LD_PRELOAD"] if env.get("LD_PRELOAD") else "")
    p = subprocess.run([sys.executable, str(script)], env=env, capture_output=True, text=True, timeout=120)
    assert p.returncode != 0 and "heap-buffer-overflow" in p.stderr and "survived" not in p.stdout


def test_oracle_pins_under_asan_and_ubsan(tmp_path):
    so = tmp_path / "ref_san.so"
    subprocess.run(["g++", "-O1", "-g", "-std=c++17", "-ffp-contract=off", "-fopenmp", "-fsanitize=address,undefined",
                    "-fno-sanitize-recover=all", "-shared", "-fPIC", "-I", os.path.join(ROOT, "oracle"), "-o", str(so),
                    os.path.join(ROOT, "oracle", "cocodc_ref.cpp")], check=True)
    asan = subprocess.run(["g++", "-print-file-name=libasan.so"], capture_output=True, text=True).stdout.strip()
    assert os.path.isabs(asan), "g++'s AddressSanitizer runtime is not installed"
    out = _run(f"""
        import ctypes as C, inspect, sys
        sys.path.insert(0, {ROOT!r}); sys.path.insert(0, {os.path.join(ROOT, 'tests')!r})
        import oracle
        oracle.lib()
        lib = C.CDLL({str(so)!r})
        for name in dir(oracle._lib):
            pass
        for name in ("pseudograd", "outer_nesterov", "delay_compensate", "fragment_scores", "select_fragments",
                     "sync_step", "sync_step_mt", "sync_plan", "fragment_scores_segmented", "sync_step_segmented",
                     "pseudograd_bf16", "sync_step_bf16", "select_fragments_bytes", "sync_event", "sync_step_bf16_segmented", "sync_event_bf16", "sync_event_segmented", "sync_event_bf16_segmented"):
            getattr(lib, "cocodc_ref_" + name).restype = C.c_int
        lib.cocodc_ref_round_bf16.restype = C.c_uint16
        lib.cocodc_ref_round_bf16.argtypes = [C.c_double]
        lib.cocodc_ref_widen_bf16.restype = C.c_double
        lib.cocodc_ref_widen_bf16.argtypes = [C.c_uint16]
        lib.cocodc_ref_round_f16.restype = C.c_uint16
        lib.cocodc_ref_round_f16.argtypes = [C.c_double]
        lib.cocodc_ref_widen_f16.restype = C.c_double
        lib.cocodc_ref_widen_f16.argtypes = [C.c_uint16]
        oracle._lib = lib
        import test_oracle_pins as a, test_oracle_segments as b, test_oracle_bf16 as c, test_oracle_loop as d
        n = 0
        for mod in (a, b, c, d):
            for k in sorted(dir(mod)):
                fn = getattr(mod, k)
                if not k.startswith("test_") or "exhaustive" in k or "every_pattern" in k:
                    continue
                params = list(inspect.signature(fn).parameters)
                if params == ["ref"]:
                    fn(oracle); n += 1
                elif params == ["ref", "amplified"]:
                    fn(oracle, True); fn(oracle, False); n += 1
        print("pins run:", n)
        """, tmp_path, asan_runtime=asan)
    assert int(out.strip().split()[-1]) >= 40


def test_library_host_side_under_asan_and_ubsan(tmp_path):
    sys.path.insert(0, ROOT)
    from paper_2504_17672_amd import build as hip_build
    import glob
    import pytest
    rt = glob.glob("/opt/rocm*/lib/llvm/lib/clang/*/lib/linux/libclang_rt.asan-x86_64.so")
    if not rt:
        pytest.skip("clang's shared AddressSanitizer runtime is not installed")
    so = tmp_path / "libcocodc_san.so"
    hip_build.build(extra=["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
                           "-Xarch_host", "-fno-sanitize-recover=all", "-g",
                           "-shared-libsan", "-Wl,-rpath," + os.path.dirname(rt[0])], out=str(so))
    out = _run(f"""
        import importlib.util, os, sys, types
        ROOT = {ROOT!r}
        sys.path.insert(0, ROOT); sys.path.insert(0, os.path.join(ROOT, "tests"))
        import paper_2504_17672_amd as pkg
        src = open(os.path.join(ROOT, "paper_2504_17672_amd", "binding.py")).read()
        SO = {str(so)!r}
        src = src.replace('LIB_PATH = os.path.join(_HERE, "libcocodc.so")', "LIB_PATH = " + repr(SO))
        mod = types.ModuleType("paper_2504_17672_amd.binding")
        mod.__file__ = os.path.join(ROOT, "paper_2504_17672_amd", "binding.py")
        exec(compile(src, mod.__file__, "exec"), mod.__dict__)
        sys.modules["paper_2504_17672_amd.binding"] = mod
        pkg.binding = mod
        assert mod.LIB_PATH.endswith("libcocodc_san.so")
        import oracle
        import test_abi_host as t, test_host_tile_plan as p
        t.test_workspace_size(mod)
        t.test_planner_golden_and_ranges(mod)
        t.test_planner_agrees_with_oracle_on_a_grid(mod, oracle)
        t.test_status_strings(mod)
        t.test_invalid_arguments_are_rejected_before_any_device_work(mod)
        t.test_loop_step_rejects_bad_buffers_before_any_device_work(mod)
        t.test_bf16_entry_points_reject_bad_arguments_before_any_device_work(mod)
        t.test_segmented_event_rejects_bad_arguments_before_any_device_work(mod)
        p.test_boundary_tables(mod)
        import random
        for seed in range(200):
            rng = random.Random(seed)
            n_used = rng.randrange(1, 300000)
            K = rng.randrange(1, 9)
            p.check_plan(mod, p.random_table(rng, n_used, rng.randrange(1, 40), K), K,
                         n_used + ((1 << 24) if seed % 2 else 0))
        # Sec. 3.2 schedule state (host only: create, plan, observe, due, state, destroy)
        rc, loop = mod.cocodc_loop_create([(0, 10), (10, 10), (20, 10), (30, 10)], 40, mod.hparams(5, 100), 0.4, 1.0, 5.0)
        assert rc == 0 and mod.cocodc_loop_plan(loop) == (0, 8, 12)
        assert mod.cocodc_loop_observe(loop, 1.0, 2.5, 1.0) == 0 and mod.cocodc_loop_plan(loop) == (0, 16, 6)
        assert mod.cocodc_loop_due(loop, 5) == (0, [])
        assert mod.cocodc_loop_state(loop) == (0, [0] * 4, [0] * 4, [-1] * 4)
        mod.cocodc_loop_destroy(loop)
        print("host checks done")
        """, tmp_path, asan_runtime=rt[0])
    assert "host checks done" in out
