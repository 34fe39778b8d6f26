"""Host code under AddressSanitizer and UndefinedBehaviorSanitizer (no GPU).

The host sources of the library (stack, planner, run, run-time-build glue) are compiled with
both sanitizers and linked with the already built kernel objects; `tests/sanitize/host_driver.cpp`
then throws a few thousand random layer lists and plan options at the C ABI -- valid and
invalid -- and checks the answers for consistency.  Any heap error, leak or undefined
behaviour in the planner fails the test.
"""
import os
import subprocess

from paper_1804_08378_amd import build

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CLANG = "/opt/rocm/lib/llvm/bin/clang++"
SAN = ["-fsanitize=address", "-fsanitize=undefined", "-fno-sanitize-recover=undefined"]


def test_host_code_is_clean_under_asan_and_ubsan(tmp_path):
    build.build(force=False)  # the kernel objects come from the normal build
    objdir = os.path.join(build.HERE, "_build")
    kernel_objs = [os.path.join(objdir, s + ".o") for s in build.SOURCES if s.endswith(".hip")]
    assert all(os.path.exists(o) for o in kernel_objs), "run build() first"
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    inc = ["-I", os.path.join(ROOT, "include"), "-I", build.CSRC]
    embed = str(tmp_path / "bs_jit_embed.cpp")
    build.write_embedded_headers(embed)
    objs = []
    procs = []
    for src in [os.path.join(build.CSRC, s) for s in build.SOURCES if s.endswith(".cpp")] + [embed]:
        obj = str(tmp_path / (os.path.basename(src) + ".o"))
        objs.append(obj)
        # plain C++ files: the sanitizers apply to host code only
        procs.append(subprocess.Popen([hipcc, "-O1", "-g", "-std=c++17", "-fPIC", "-fno-gpu-sanitize", *SAN, *inc,
                                       "-c", src, "-o", obj], stdout=subprocess.PIPE, stderr=subprocess.STDOUT))
    for p in procs:
        out, _ = p.communicate()
        assert p.returncode == 0, out.decode()
    lib = str(tmp_path / "libbs_san.so")
    subprocess.run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-fno-gpu-sanitize", *SAN, *objs, *kernel_objs,
                    "-lhiprtc", "-ldl", "-o", lib], check=True, capture_output=True)
    exe = str(tmp_path / "host_driver")
    subprocess.run([CLANG, "-O1", "-g", "-std=c++17", *SAN, *inc, os.path.join(HERE, "sanitize", "host_driver.cpp"),
                    "-L", str(tmp_path), "-lbs_san", "-Wl,-rpath," + str(tmp_path), "-o", exe], check=True,
                   capture_output=True)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    r = subprocess.run([exe, "3000"], capture_output=True, text=True, env=env, timeout=600)
    assert r.returncode == 0, r.stdout[-3000:] + r.stderr[-6000:]
    print(r.stdout.strip())
    assert r.stdout.startswith("ok:"), r.stdout
