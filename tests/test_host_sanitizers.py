"""The host side of the library (packer, layout self-check, latency model) and the C oracle built
with AddressSanitizer and UndefinedBehaviorSanitizer and run on the CPU: tests/native/host_sanitize.cpp
packs every layout, exports, self-checks, compares with the oracle bit for bit and feeds the error
paths; a sanitizer report fails the run.  Device code is not involved: the launch entry point is
linked from a stub, since only its host-side argument checks are reachable without a GPU."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2109_00170_amd", "csrc")


@pytest.mark.skipif(shutil.which("hipcc") is None or shutil.which("gcc") is None, reason="needs hipcc and gcc")
def test_packer_latency_model_and_oracle_under_asan_and_ubsan(tmp_path):
    san = ["-fsanitize=address", "-fsanitize=undefined", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer",
           "-g", "-O1"]
    clang = os.path.join(os.path.dirname(os.path.realpath(shutil.which("hipcc"))), "..", "llvm", "bin", "clang++")
    if not os.path.exists(clang):
        clang = "/opt/rocm/llvm/bin/clang++"
    inc = ["-I", os.path.join(ROOT, "include"), "-I", CSRC, "-I", "/opt/rocm/include", "-D__HIP_PLATFORM_AMD__"]
    exe = str(tmp_path / "host_sanitize")
    stub = tmp_path / "stub.cpp"
    # alcs_sparse_conv's host-side checks (shape against the handle) without any device code
    stub.write_text('#include "alcs_internal.h"\n'
                    'extern "C" int alcs_sparse_conv(const alcs_packed_t *Wp, const float *X, const float *, float *Y,\n'
                    '    int N, int Cin, int Cout, int H, int W, int kernel, int stride, void *) {\n'
                    '  if (!Wp || N < 0 || H <= 0 || W <= 0 || !X || !Y) return ALCS_E_INVALID_ARG;\n'
                    '  if (Cin != Wp->Cin || Cout != Wp->Cout || kernel != Wp->k) return ALCS_E_INVALID_ARG;\n'
                    '  (void)stride; return Wp->dev.blob ? ALCS_E_UNSUPPORTED : ALCS_E_NO_DEVICE; }\n'
                    '// device-side part of the upload (never reached without a GPU)\n'
                    'namespace alcs { int add_channel_records(alcs_packed *, void *) { return ALCS_OK; } }\n')
    oracle_o = str(tmp_path / "oracle.o")
    subprocess.check_call([clang.replace("clang++", "clang"), "-std=c99", "-c", os.path.join(ROOT, "oracle", "alcs_oracle.c"),
                           "-o", oracle_o] + san)
    cmd = [clang, "-std=c++17", os.path.join(ROOT, "tests", "native", "host_sanitize.cpp"),
           os.path.join(CSRC, "alcs_pack.cpp"), os.path.join(CSRC, "alcs_latency.cpp"), str(stub), oracle_o,
           "-o", exe, "-L/opt/rocm/lib", "-lamdhip64", "-Wl,-rpath,/opt/rocm/lib"] + inc + san
    subprocess.check_call(cmd)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    out = subprocess.run([exe], env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, timeout=600)
    text = out.stdout.decode(errors="replace")
    assert out.returncode == 0 and "host sanitize OK" in text, text[-4000:]
    assert "runtime error" not in text and "AddressSanitizer" not in text, text[-4000:]
    # the instrumentation is really there
    syms = subprocess.run(["nm", "-D", "--undefined-only", exe], stdout=subprocess.PIPE).stdout.decode() + \
        subprocess.run(["nm", exe], stdout=subprocess.PIPE).stdout.decode()
    assert "__asan_init" in syms and "__ubsan_handle" in syms
