"""Builds libsparsevila.so (HIP, gfx950 only) and its test build libsparsevila_hooks.so in-tree next to this file."""
from __future__ import annotations

import os
import re
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ_DIR = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libsparsevila.so")
LIB_HOOKS = os.path.join(HERE, "libsparsevila_hooks.so")   # same objects, sv_api.hip compiled with -DSV_TEST_HOOKS
HOOKED_SOURCE = "sv_api.hip"
SOURCES = ["sv_api.hip", "sv_score.hip", "sv_select.hip", "sv_attend.hip", "sv_attend_mfma.hip", "sv_attend_flash.hip", "sv_pack.hip", "sv_mass.hip", "sv_salience.hip", "sv_util.hip"]

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wextra",
    "-Wno-unused-command-line-argument",
    # packed fp32 VALU forms are kept off for every kernel of this library
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    # per-kernel register / scratch / LDS remarks: parsed below, not printed
    "-Rpass-analysis=kernel-resource-usage",
]


# Host-side sanitizers (AddressSanitizer + UndefinedBehaviorSanitizer on the C-ABI layer and the launchers; device
# code is compiled as always).  Used by build_host_sanitized() only.
HOST_SANITIZE = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
                 "-Xarch_host", "-fno-sanitize-recover=undefined", "-Xarch_host", "-fno-omit-frame-pointer", "-g"]
LIB_ASAN = os.path.join(HERE, "libsparsevila_asan.so")


def _compile(src: str, hooks: bool = False, sanitize: bool = False) -> str:
    obj = os.path.join(OBJ_DIR, src.replace(".hip", "_asan.o" if sanitize else "_hooks.o" if hooks else ".o"))
    cmd = [HIPCC, *FLAGS, *(["-DSV_TEST_HOOKS"] if hooks else []), *(HOST_SANITIZE if sanitize else []),
           "-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed for {src}:\n{r.stdout}\n{r.stderr}")
    # the host pass does not know the packed-fp32 feature name; that warning is expected
    noise = "is not a recognized feature for this target"
    msgs, kernel, in_remark = [], "?", False
    for line in r.stderr.splitlines():
        if in_remark and re.match(r"^\s*\d*\s*\|", line):
            continue   # the source lines quoted under a remark
        in_remark = False
        if "[-Rpass-analysis=kernel-resource-usage]" in line:
            in_remark = True
            # No kernel of the library may spill to scratch memory: a kernel that does pays for it at
            # every launch (and so did the launch after it, when it was measured).
            text = line.split("remark:", 1)[-1].strip()
            if text.startswith("Function Name:"):
                kernel = text.split(":", 1)[1].split("[")[0].strip()
            elif text.startswith("ScratchSize [bytes/lane]:"):
                if int(text.split(":")[1].split("[")[0]) != 0:
                    raise RuntimeError(f"{src}: kernel {kernel} uses scratch memory ({text})")
            continue
        if line.strip() and noise not in line:
            msgs.append(line)
    if msgs:
        sys.stderr.write("\n".join(msgs) + "\n")
    return obj


def build(verbose: bool = False) -> str:
    """Compiles every source and links the shared library; always rebuilds."""
    os.makedirs(OBJ_DIR, exist_ok=True)
    with ThreadPoolExecutor(max_workers=8) as ex:
        objs = ex.map(_compile, SOURCES)
        api_hooks = ex.submit(_compile, HOOKED_SOURCE, True)
        objs = list(objs)
        api_hooks = api_hooks.result()
    # The test build differs from the product in one host-side object (two more knob names in sv_api.hip): every
    # kernel object is shared, so what the hooks time and test is the product's device code.
    hooked = [api_hooks if o.endswith(HOOKED_SOURCE.replace(".hip", ".o")) else o for o in objs]
    for lib, parts in ((LIB, objs), (LIB_HOOKS, hooked)):
        cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", lib, *parts]
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError(f"link failed:\n{r.stdout}\n{r.stderr}")
        if verbose:
            print(f"built {lib}")
    return LIB


def build_host_sanitized(verbose: bool = False) -> str:
    """libsparsevila_asan.so: every source with AddressSanitizer and UndefinedBehaviorSanitizer on its HOST code.
    For the CPU-only argument-checking tests (tests/run_sanitizers.sh); load it with SPARSEVILA_LIBRARY=<path> and
    clang's libclang_rt.asan preloaded.  Not built by build()."""
    os.makedirs(OBJ_DIR, exist_ok=True)
    with ThreadPoolExecutor(max_workers=8) as ex:
        objs = list(ex.map(lambda s: _compile(s, sanitize=True), SOURCES))
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-fsanitize=address", "-fsanitize=undefined",
           "-shared-libsan", "-o", LIB_ASAN, *objs]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"link failed:\n{r.stdout}\n{r.stderr}")
    if verbose:
        print(f"built {LIB_ASAN}")
    return LIB_ASAN


if __name__ == "__main__":
    if "--host-sanitize" in sys.argv[1:]:
        build_host_sanitized(verbose=True)
    else:
        build(verbose=True)
