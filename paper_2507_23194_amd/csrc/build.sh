#!/bin/bash
# Builds libgeakcheck.so for gfx950 next to the package (in-tree, no JIT cache).
#   -ffp-contract=off                 the rule's product and sum are rounded separately
#   -packed-fp32-ops (target feature) no packed-FP32 VALU forms
set -euo pipefail
here="$(cd "$(dirname "${BASH_SOURCE[0]}")" && pwd)"
root="$(cd "$here/../.." && pwd)"
out="$here/../libgeakcheck.so"
hipcc --offload-arch=gfx950 -O3 -std=c++17 -fPIC -shared -ffp-contract=off \
      -Xclang -target-feature -Xclang -packed-fp32-ops \
      -Wall -Wno-unused-function \
      -I"$root/include" -I"$here" \
      "$here/kernels.hip" "$here/ulp_kernels.hip" "$here/verdict_kernel.hip" "$here/metrics_host.cpp" "$here/api.cpp" "$here/plan_host.cpp" \
      -o "$out" "$@"
echo "built $out"
