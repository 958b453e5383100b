#!/bin/bash
# Builds libadmmq.so for gfx950 next to the Python binding.
set -e
here="$(cd "$(dirname "$0")" && pwd)"
out="$here/../libadmmq.so"
flags="--offload-arch=gfx950 -O3 -std=c++17 -fPIC -Xclang -target-feature -Xclang -packed-fp32-ops -ffp-contract=off -Wno-unused-command-line-argument"
mkdir -p "$here/_build"
pids=()
for f in gemm_tn hessian_bf16 gemm_f16x3 stream factor householder band local_search formats api; do
  /opt/rocm/bin/hipcc $flags -c "$here/$f.hip" -o "$here/_build/$f.o" 2> >(grep -v "packed-fp32-ops" >&2) &
  pids+=($!)
done
for p in "${pids[@]}"; do wait $p; done
/opt/rocm/bin/hipcc --offload-arch=gfx950 -shared -fPIC -pthread -o "$out" "$here"/_build/{gemm_tn,hessian_bf16,gemm_f16x3,stream,factor,householder,band,local_search,formats,api}.o
echo "built $out"
