#!/bin/bash
# Host code under AddressSanitizer and UndefinedBehaviorSanitizer, CPU only: builds the host side of
# the library (csrc/lutgemm_host.cpp: sizes, quantisers, packing) and the C oracle
# (oracle/oracle_gemv.c) with -fsanitize=address,undefined into a temporary directory and runs
# the CPU tests that exercise them against those builds.  Usage: tests/run_host_sanitizers.sh
set -euo pipefail
ROOT="$(cd "$(dirname "${BASH_SOURCE[0]}")/.." && pwd)"
OUT="$(mktemp -d /tmp/lutgemm_san.XXXXXX)"
trap 'rm -rf "$OUT"' EXIT
SAN="-fsanitize=address,undefined -fno-sanitize-recover=undefined -fno-omit-frame-pointer -g -O1"
g++ $SAN -std=c++17 -fPIC -shared -pthread -I "$ROOT/include" -o "$OUT/liblutgemm_host_san.so" \
    "$ROOT/paper_2206_09557_amd/csrc/lutgemm_host.cpp"
gcc $SAN -std=c11 -fPIC -shared -fopenmp -ffp-contract=off -o "$OUT/liboracle_gemv_san.so" "$ROOT/oracle/oracle_gemv.c" -lm
cd "$ROOT"
# (leak detection off: the interpreter itself never frees everything; the device entry points and
# the export check need the full library and are left out)
LD_PRELOAD="$(gcc -print-file-name=libasan.so) $(gcc -print-file-name=libubsan.so)" \
ASAN_OPTIONS=detect_leaks=0:abort_on_error=1 UBSAN_OPTIONS=print_stacktrace=1:halt_on_error=1 \
LUTGEMM_LIB="$OUT/liblutgemm_host_san.so" ORACLE_GEMV_LIB="$OUT/liboracle_gemv_san.so" OMP_NUM_THREADS=4 \
python3 -m pytest tests/test_abi_host.py tests/test_oracle_format.py tests/test_oracle_matvec.py tests/test_oracle_quantizer.py \
    -q -m "not gpu" -k "not exports and not plan_grid and not argument_validation" -p no:cacheprovider "$@"
echo "host sanitizers: clean"
