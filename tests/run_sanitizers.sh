#!/bin/bash
# CPU-only sanitizer pass over the code that runs on the host:
#   1. the C oracle (gcc AddressSanitizer + UndefinedBehaviorSanitizer) under its pins and the comparison rules;
#   2. the host side of the HIP library (clang ASan + UBSan on the C-ABI layer and the launchers) under the
#      argument-checking tests, none of which reaches a kernel launch.
# Two runs, because gcc's and clang's sanitizer runtimes cannot share a process.  No GPU is used.
# usage: bash tests/run_sanitizers.sh        (from the repository root; exits non-zero on any finding)
set -e
cd "$(dirname "$0")/.."
export ASAN_OPTIONS=detect_leaks=0:abort_on_error=0:halt_on_error=1
export UBSAN_OPTIONS=print_stacktrace=1:halt_on_error=1

echo "== oracle under gcc ASan + UBSan"
SV_ORACLE_SANITIZE=1 LD_PRELOAD="$(gcc -print-file-name=libasan.so)" \
    python -m pytest tests/test_oracle_pins.py tests/test_oracle_properties.py tests/test_compare_rules.py tests/test_inputs.py -q -x -p no:cacheprovider

echo "== host code of libsparsevila under clang ASan + UBSan"
python -m paper_2510_17777_amd.build --host-sanitize
RT="$(/opt/rocm/lib/llvm/bin/clang --print-file-name=libclang_rt.asan-x86_64.so)"
SPARSEVILA_LIBRARY="$PWD/paper_2510_17777_amd/libsparsevila_asan.so" LD_PRELOAD="$RT" \
    python -m pytest tests/test_abi.py -q -x -p no:cacheprovider
rm -f paper_2510_17777_amd/libsparsevila_asan.so oracle/libsv_oracle_asan.so paper_2510_17777_amd/_build/*_asan.o
echo "sanitizers: clean"
