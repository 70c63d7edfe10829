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
# The decode kernel counts outstanding memory operations by hand (see gemm_decode.hip): between the
# last buffer-to-LDS copy and the hand-written "s_waitcnt vmcnt(N)" there must be exactly N vector
# memory instructions, all of them the weight loads, and none added by the compiler (spills).
hipcc $FLAGS -S --cuda-device-only gemm_decode.hip -o _build/gemm_decode.s
python3 - <<'PY'
import re, sys
txt = open("_build/gemm_decode.s").read()
checked = 0
for m in re.finditer(r"^(_ZN4milo18w3lr_decode_kernel\S*):[^\n]*\n(.*?)s_endpgm", txt, re.S | re.M):
    name, body = m.group(1), m.group(2).split("\n")
    for i, line in enumerate(body):
        w = re.search(r"s_waitcnt vmcnt\((\d+)\)", line)
        if not (w and i > 0 and "ASMSTART" in body[i - 1]):
            continue
        n = int(w.group(1))
        if n == 0:
            continue                      # waiting for everything is always safe
        j = i - 1
        vmem = []
        while j >= 0 and not ("buffer_load" in body[j] and " lds" in body[j]):
            if re.match(r"\s+(buffer_|global_|scratch_|flat_)", body[j]):
                vmem.append(body[j].split()[0])
            j -= 1
        if j < 0:
            continue                      # a wait that does not guard an LDS copy (wait_vmem)
        if len(vmem) != n or any(not v.startswith("buffer_load") for v in vmem):
            sys.exit("%s: %d memory instructions between the LDS copies and s_waitcnt vmcnt(%d): %r"
                     % (name, len(vmem), n, vmem))
        checked += 1
if checked == 0:
    sys.exit("decode kernel: no guarded LDS copy found; the check is out of date")
print("decode kernel: %d guarded LDS copies verified" % checked)
PY
hipcc --offload-arch=gfx950 -shared -fPIC -o "$OUT/libmilo.so" _build/pack.o _build/gemm_tiled.o _build/gemm_decode.o _build/moe.o _build/api.o
echo "built $OUT/libmilo.so"
