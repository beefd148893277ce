"""Build libwgkv.so (the C-ABI library) for gfx950 with hipcc, in-tree.

`python -m paper_2512_17452_amd.build --sanitize-host` writes a second library, libwgkv_hostsan.so, whose host
code (argument checks, bookkeeping, launch set-up) is compiled with AddressSanitizer and
UndefinedBehaviorSanitizer; the device code is built as always.  WGKV_LIB makes the Python binding load it.  The
host-only boundary tests under it, from the repository root:

    python -m paper_2512_17452_amd.build --sanitize-host && \
    LD_PRELOAD="$(/opt/rocm/lib/llvm/bin/clang -print-file-name=libclang_rt.asan-x86_64.so)${LD_PRELOAD:+:$LD_PRELOAD}" \
    ASAN_OPTIONS=detect_leaks=0:protect_shadow_gap=0 UBSAN_OPTIONS=halt_on_error=1 \
    WGKV_LIB=paper_2512_17452_amd/libwgkv_hostsan.so python -m pytest tests/test_boundary_host.py -q
"""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
BUILD = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libwgkv.so")
LIB_HOSTSAN = os.path.join(HERE, "libwgkv_hostsan.so")
HOSTSAN_FLAGS = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host",
                 "-fno-omit-frame-pointer", "-g"]
SOURCES = ["wgkv_api.hip", "admit.hip", "attend_decode.hip", "attend_prefill.hip", "attend_prefill_plain.hip", "gate.hip", "gate_mlp.hip", "evict.hip", "evict_scores.hip", "quest.hip", "soft_attn.hip", "probe.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def _compile(src: str, sanitize_host: bool = False) -> str:
    obj = os.path.join(BUILD, src.replace(".hip", ".hostsan.o" if sanitize_host else ".o"))
    cmd = [HIPCC] + FLAGS + (HOSTSAN_FLAGS if sanitize_host else []) + ["-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{r.stdout}\n{r.stderr}")
    warn = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l and l.strip())
    if warn:
        sys.stderr.write(warn + "\n")
    return obj


def build_hostsan() -> str:
    os.makedirs(BUILD, exist_ok=True)
    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as ex:
        objs = list(ex.map(lambda s_: _compile(s_, True), SOURCES))
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-fsanitize=address", "-fsanitize=undefined",
           "-shared-libsan", "-o", LIB_HOSTSAN] + objs
    subprocess.run(cmd, check=True)
    return LIB_HOSTSAN


def build(force: bool = True) -> str:
    srcs = [os.path.join(CSRC, s) for s in SOURCES] + [os.path.join(CSRC, "wgkv_dev.h"),
                                                        os.path.join(HERE, "..", "include", "wgkv.h")]
    if not force and os.path.exists(LIB) and all(os.path.getmtime(LIB) >= os.path.getmtime(s) for s in srcs):
        return LIB
    os.makedirs(BUILD, exist_ok=True)
    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as ex:
        objs = list(ex.map(_compile, SOURCES))
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build_hostsan() if "--sanitize-host" in sys.argv[1:] else build(force=True))
