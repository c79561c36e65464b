"""The oracle's C sources under AddressSanitizer and UndefinedBehaviorSanitizer (host code only, CPU).

The pin tests are run once more, in a child process, against a build of the same sources with
-fsanitize=address,undefined: an out-of-bounds access, a use of uninitialised stack through a bad index, a signed
overflow or an invalid shift in the oracle aborts that process and fails this test.
"""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_oracle_pins_pass_under_address_and_undefined_behaviour_sanitizers():
    sys.path.insert(0, ROOT)
    import oracle
    oracle.build_sanitized()
    env = dict(os.environ)
    env[oracle.SANITIZED_ENV] = "1"
    # the runtime has to be in the process before the sanitized library is loaded; whatever is preloaded already stays
    env["LD_PRELOAD"] = " ".join(p for p in (oracle.sanitizer_preload(), env.get("LD_PRELOAD", "")) if p)
    # python itself is not instrumented: its own allocations are not reported as leaks, and the link order of an
    # uninstrumented main program is not an error
    env["ASAN_OPTIONS"] = "detect_leaks=0:verify_asan_link_order=0:abort_on_error=1"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    env["OMP_NUM_THREADS"] = "4"
    pins = [os.path.join(ROOT, "tests", f) for f in ("test_oracle_pins.py", "test_block_oracle_pins.py",
                                                     "test_quantizer_oracle_pins.py")]
    p = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", *pins], env=env, cwd=ROOT,
                       capture_output=True, text=True, timeout=900)
    assert p.returncode == 0, p.stdout[-3000:] + p.stderr[-3000:]
    assert "passed" in p.stdout and "failed" not in p.stdout
    # the child really ran the sanitized build
    probe = subprocess.run([sys.executable, "-c",
                            "import oracle; oracle.half_to_double(0x3c00); print(oracle._lib._name)"],
                           env=env, cwd=ROOT, capture_output=True, text=True, timeout=300)
    assert probe.returncode == 0, probe.stderr[-2000:]
    assert probe.stdout.strip().endswith("libptqtp_oracle_san.so")


def test_the_sanitizer_set_up_catches_a_planted_overread(tmp_path):
    # the same flags, preload and options on a four-line C function that reads one element past its buffer:
    # the child process must die, or a clean run of the pins above would prove nothing
    sys.path.insert(0, ROOT)
    import oracle
    src = tmp_path / "overread.c"
    src.write_text("#include <stdint.h>\n"
                   "int64_t sum_one_too_many(const int32_t *a, int64_t n) {\n"
                   "    int64_t s = 0;\n"
                   "    for (int64_t i = 0; i <= n; ++i) s += a[i];\n"
                   "    return s;\n"
                   "}\n")
    lib = tmp_path / "liboverread.so"
    subprocess.check_call(["gcc", "-O1", "-g", "-std=c11", "-fPIC", "-shared", "-fsanitize=address,undefined",
                           "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer", "-o", str(lib), str(src)])
    env = dict(os.environ)
    env["LD_PRELOAD"] = " ".join(p for p in (oracle.sanitizer_preload(), env.get("LD_PRELOAD", "")) if p)
    env["ASAN_OPTIONS"] = "detect_leaks=0:verify_asan_link_order=0:abort_on_error=1"
    code = ("import ctypes, sys\n"
            f"lib = ctypes.CDLL({str(lib)!r})\n"
            "lib.sum_one_too_many.restype = ctypes.c_int64\n"
            "lib.sum_one_too_many.argtypes = [ctypes.c_void_p, ctypes.c_int64]\n"
            "libc = ctypes.CDLL(None)\n"
            "libc.malloc.restype = ctypes.c_void_p\n"
            "libc.malloc.argtypes = [ctypes.c_size_t]\n"
            "buf = libc.malloc(400)\n"
            "ctypes.memset(buf, 0, 400)\n"
            "print(lib.sum_one_too_many(buf, int(sys.argv[1])))\n")
    good = subprocess.run([sys.executable, "-c", code, "99"], env=env, capture_output=True, text=True, timeout=120)
    assert good.returncode == 0 and good.stdout.strip() == "0", good.stderr[-2000:]
    bad = subprocess.run([sys.executable, "-c", code, "100"], env=env, capture_output=True, text=True, timeout=120)
    assert bad.returncode != 0 and "heap-buffer-overflow" in bad.stderr
