#!/usr/bin/env bash
# Builds libgleam.so (gfx950 only) next to the Python binding.  Usage: build.sh [-j N]
set -euo pipefail
here="$(cd "$(dirname "${BASH_SOURCE[0]}")" && pwd)"
out="$here/../libgleam.so"
obj="$here/../_build"
mkdir -p "$obj"
flags=(-O3 --offload-arch=gfx950 -std=c++17 -fPIC -Xclang -target-feature -Xclang -packed-fp32-ops -Wno-unused-command-line-argument)
pids=()
for f in sense prox prox_bf16 prox_bf16w prox_wino prox_wino3 prox_time prox_thin cg gleam_api; do
  hipcc "${flags[@]}" -c "$here/$f.hip" -o "$obj/$f.o" 2> >(grep -v "packed-fp32-ops' is not a recognized feature" >&2) &
  pids+=($!)
done
for p in "${pids[@]}"; do wait "$p"; done
hipcc --offload-arch=gfx950 -shared -fPIC "$obj"/sense.o "$obj"/prox.o "$obj"/prox_bf16.o "$obj"/prox_bf16w.o "$obj"/prox_wino.o "$obj"/prox_wino3.o "$obj"/prox_time.o "$obj"/prox_thin.o "$obj"/cg.o "$obj"/gleam_api.o -o "$out"
echo "built $out"
