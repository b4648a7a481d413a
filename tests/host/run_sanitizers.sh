#!/bin/bash
# Builds the library's sources with AddressSanitizer and UndefinedBehaviorSanitizer on the HOST code (the
# device code is compiled as usual) together with the host-only exerciser, and runs it.  No GPU needed.
set -e
here=$(cd "$(dirname "$0")" && pwd)
root=$(cd "$here/../.." && pwd)
out=${TMPDIR:-/tmp}/mona_sanitize
mkdir -p "$out"
src="$root/paper_2605_26842_amd/csrc"
san="-Xarch_host -fsanitize=address -Xarch_host -fsanitize=undefined -Xarch_host -fno-omit-frame-pointer"
objs=""
for f in mona_api state_update ns_gemm adamw; do
  /opt/rocm/bin/hipcc --offload-arch=gfx950 -O1 -g -std=c++17 -fPIC -fno-gpu-rdc \
    -Xclang -target-feature -Xclang -packed-fp32-ops -Wno-unused-command-line-argument $san \
    -c "$src/$f.hip" -o "$out/$f.o" 2>&1 | grep -v "not a recognized feature" || true
  objs="$objs $out/$f.o"
done
/opt/rocm/lib/llvm/bin/clang++ -O1 -g -std=c++17 -fsanitize=address -fsanitize=undefined -fno-omit-frame-pointer \
  -c "$here/sanitize_host_paths.cpp" -o "$out/driver.o"
/opt/rocm/bin/hipcc --offload-arch=gfx950 -fno-gpu-sanitize -fsanitize=address -fsanitize=undefined $objs "$out/driver.o" -o "$out/sanitize_host_paths"
ASAN_OPTIONS=detect_leaks=1:abort_on_error=0 UBSAN_OPTIONS=print_stacktrace=1:halt_on_error=1 "$out/sanitize_host_paths"
