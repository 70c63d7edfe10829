#!/bin/bash
# Builds libmilo.so for gfx950 from the HIP sources next to this script.
set -e
cd "$(dirname "$0")"
OUT=../lib
mkdir -p "$OUT" _build
FLAGS="-O3 --offload-arch=gfx950 -fPIC -std=c++17 -Xclang -target-feature -Xclang -packed-fp32-ops -fhip-fp32-correctly-rounded-divide-sqrt -Wno-unused-command-line-argument"
pids=()
hipcc $FLAGS -ffp-contract=off -c pack.hip -o _build/pack.o & pids+=($!)
hipcc $FLAGS -c gemm_tiled.hip -o _build/gemm_tiled.o & pids+=($!)
hipcc $FLAGS -c gemm_decode.hip -o _build/gemm_decode.o & pids+=($!)
hipcc $FLAGS -c moe.hip -o _build/moe.o & pids+=($!)
hipcc $FLAGS -c api.hip -o _build/api.o & pids+=($!)
for p in "${pids[@]}"; do wait $p; done
hipcc --offload-arch=gfx950 -shared -fPIC -o "$OUT/libmilo.so" _build/pack.o _build/gemm_tiled.o _build/gemm_decode.o _build/moe.o _build/api.o
echo "built $OUT/libmilo.so"
