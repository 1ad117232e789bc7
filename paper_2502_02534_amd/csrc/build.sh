#!/bin/bash
# Builds libspdecode.so for gfx950 next to the Python binding.
set -euo pipefail
here="$(cd "$(dirname "${BASH_SOURCE[0]}")" && pwd)"
out="$here/../libspdecode.so"
flags=(--offload-arch=gfx950 -O3 -std=c++17 -fPIC -fvisibility=hidden -munsafe-fp-atomics
       -Xclang -target-feature -Xclang -packed-fp32-ops
       -Wall -Wno-unused-function)
objs=()
pids=()
mkdir -p "$here/_build"
for src in "$here"/*.hip; do
  obj="$here/_build/$(basename "${src%.hip}").o"
  /opt/rocm/bin/hipcc "${flags[@]}" -c "$src" -o "$obj" &
  pids+=($!)
  objs+=("$obj")
done
for pid in "${pids[@]}"; do wait "$pid"; done
/opt/rocm/bin/hipcc --offload-arch=gfx950 -shared -fPIC -o "$out" "${objs[@]}"
echo "built $out"
