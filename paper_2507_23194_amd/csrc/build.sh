#!/bin/bash
# Builds libgeakcheck.so for gfx950 next to the package (in-tree, no JIT cache).
#   -ffp-contract=off                 the rule's product and sum are rounded separately
#   -packed-fp32-ops (target feature) no packed-FP32 VALU forms
#   -Wno-int-to-pointer-cast          LDS addresses are 32-bit offsets; the host pass of the kernel files sees 64-bit pointers
# The translation units are compiled side by side, then linked.
set -euo pipefail
here="$(cd "$(dirname "${BASH_SOURCE[0]}")" && pwd)"
root="$(cd "$here/../.." && pwd)"
out="$here/../libgeakcheck.so"
obj="$(mktemp -d)"
trap 'rm -rf "$obj"' EXIT
# Digest of the sources the library is built from (this script, the header, every file of csrc/, in
# bytewise path order), compiled in and returned by geak_check_build_id(): tests, the smoke check and
# the benchmark compare it with the digest of the tree they run in, so a stale library is noticed.
build_id="$(cd "$root" && LC_ALL=C ls include/*.h paper_2507_23194_amd/csrc/* | LC_ALL=C sort | xargs cat | sha256sum | cut -c1-16)"
flags=(--offload-arch=gfx950 -O3 -std=c++17 -fPIC -ffp-contract=off
       -Xclang -target-feature -Xclang -packed-fp32-ops
       -Wall -Wno-unused-function -Wno-int-to-pointer-cast -I"$root/include" -I"$here"
       -DGEAK_BUILD_ID="\"$build_id\"" "$@")
pids=()
for src in kernels.hip ulp_kernels.hip verdict_kernel.hip static_scratch.hip timing.hip metrics_host.cpp api.cpp plan_host.cpp; do
    hipcc "${flags[@]}" -c "$here/$src" -o "$obj/${src%.*}.o" &
    pids+=($!)
done
for pid in "${pids[@]}"; do wait "$pid"; done
hipcc --offload-arch=gfx950 -shared -fPIC "$obj"/*.o -o "$out"
echo "built $out (build id $build_id)"
