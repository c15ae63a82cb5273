"""Host code under AddressSanitizer and UndefinedBehaviorSanitizer (CPU only):
  - the C oracle, over a sweep of shapes, ties and degenerate groups (tests/oracle_sanitize_main.c);
  - the host side of the C ABI: argument validation and workspace planning, none of which touches a device
    (tests/abi_sanitize_main.cpp; only the host passes of api.hip and loss.hip are instrumented, the GPU
    code objects are compiled as usual)."""
import glob
import os
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2504_13818_amd", "csrc")


def _run(cmd, **kw):
    p = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, **kw)
    out = "\n".join(l for l in p.stdout.splitlines() if "packed-fp32-ops" not in l and "Woption-ignored" not in l)
    assert p.returncode == 0, f"{' '.join(cmd[:3])} ... failed:\n{out[-3000:]}"
    return out


def test_c_oracle_under_sanitizers(tmp_path):
    exe = str(tmp_path / "oracle_san")
    _run(["gcc", "-O1", "-g", "-fopenmp", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
          "-static-libasan", "-fno-omit-frame-pointer", os.path.join(ROOT, "tests", "oracle_sanitize_main.c"),
          os.path.join(ROOT, "oracle", "pods_oracle.c"), "-o", exe, "-lm"])
    assert "oracle sanitizer run ok" in _run([exe], env=dict(os.environ, OMP_NUM_THREADS="3"))


def test_host_abi_layer_under_sanitizers(tmp_path):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    if not os.path.exists(hipcc):
        pytest.skip("hipcc not available")
    from paper_2504_13818_amd import build as hip_build
    objs = {os.path.basename(o): o for o in glob.glob(os.path.join(hip_build.OBJ, "*.o"))}
    if not all(src.replace(".hip", ".o") in objs for src in hip_build.SOURCES):
        hip_build.build()                       # the uninstrumented objects of the other sources
        objs = {os.path.basename(o): o for o in glob.glob(os.path.join(hip_build.OBJ, "*.o"))}
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host",
           "-fno-sanitize-recover=all"]
    common = [hipcc, *hip_build.COMMON, "-O1", "-g", *san]
    mine = []
    for src, lang in (("api.hip", []), ("loss.hip", []), (os.path.join(ROOT, "tests", "abi_sanitize_main.cpp"), ["-x", "hip"])):
        path = src if os.path.isabs(src) else os.path.join(CSRC, src)
        obj = str(tmp_path / (os.path.basename(path) + ".o"))
        _run([*common, *lang, "-c", path, "-o", obj])
        mine.append(obj)
    others = [o for name, o in objs.items() if name not in ("api.o", "loss.o")]
    exe = str(tmp_path / "abi_san")
    _run([hipcc, "--offload-arch=gfx950", "-fsanitize=address", "-fsanitize=undefined", *mine, *others, "-o", exe])
    assert "abi sanitizer run ok" in _run([exe])
