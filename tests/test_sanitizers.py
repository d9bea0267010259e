"""The CPU-side code under AddressSanitizer and UndefinedBehaviorSanitizer: the oracle, the input encoder, the
product's header parser and table builder and the host walk-through of the kernels' lane code are compiled with
-fsanitize=address,undefined into one program (tests/sanitize/san_driver.cpp) that decodes intact files of every
layout and extreme shape, files with damaged entropy-coded data, truncated files and files with mutated headers.
Any out-of-bounds access, use of an uninitialised size, signed overflow or misaligned access ends the program with
a non-zero status."""
import os
import subprocess

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = os.path.join(ROOT, "tests", "sanitize")
FLAGS = ["-g", "-O1", "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer"]


def test_cpu_side_code_is_clean_under_asan_and_ubsan():
    exe = os.path.join(SAN, "san_driver")
    objs = []
    for src, cc in ((os.path.join(ROOT, "oracle", "jpeg_oracle.c"), "gcc"),
                    (os.path.join(ROOT, "workloads", "jpeg_encoder.c"), "gcc")):
        obj = os.path.join(SAN, os.path.basename(src) + ".o")
        subprocess.check_call([cc, *FLAGS, "-c", src, "-o", obj])
        objs.append(obj)
    subprocess.check_call(["g++", "-std=c++17", *FLAGS, "-o", exe, os.path.join(SAN, "san_driver.cpp"),
                           os.path.join(ROOT, "tests", "emul", "jpgd_emul.cpp"),
                           os.path.join(ROOT, "paper_2111_09219_amd", "csrc", "jpgd_parse.cpp"), *objs, "-lm"])
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    r = subprocess.run([exe], capture_output=True, text=True, timeout=900, env=env)
    for f in objs + [exe]:
        os.remove(f)
    assert r.returncode == 0, (r.stdout[-2000:], r.stderr[-6000:])
    assert "0 failures" in r.stdout
