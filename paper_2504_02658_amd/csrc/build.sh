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
VMEM = re.compile(r"\s+(buffer_|global_|scratch_|flat_)")
for m in re.finditer(r"^(_ZN4milo18w3lr_decode_kernel\S*):[^\n]*\n(.*?)s_endpgm", txt, re.S | re.M):
    name, body = m.group(1), m.group(2).split("\n")
    for i, line in enumerate(body):
        w = re.search(r"s_waitcnt vmcnt\((\d+)\)", line)
        if not (w and i > 0 and "ASMSTART" in body[i - 1]) or int(w.group(1)) == 0:
            continue                      # only hand-written partial waits are of interest
        n = int(w.group(1))
        # walk back over exactly n vector memory instructions: none may be a spill or a store,
        # and the one before them must be a buffer-to-LDS copy (the data this wait is for)
        j, seen = i - 1, []
        while j >= 0 and len(seen) < n:
            if VMEM.match(body[j]):
                seen.append(body[j].split()[0] + (" lds" if " lds" in body[j] else ""))
            j -= 1
        while j >= 0 and not VMEM.match(body[j]):
            j -= 1
        bad = [v for v in seen if not v.startswith("buffer_load")]
        if bad or j < 0 or " lds" not in body[j]:
            sys.exit("%s: s_waitcnt vmcnt(%d) does not sit %d loads after an LDS copy: %r / %r"
                     % (name, n, n, seen, body[j] if j >= 0 else None))
        checked += 1
if checked == 0:
    sys.exit("decode kernel: no guarded LDS copy found; the check is out of date")
print("decode kernel: %d hand-counted waits verified" % checked)
PY
# The tiled kernel counts outstanding memory operations by hand too; it is safe as long as the
# compiler adds none of its own, i.e. as long as no variant uses scratch memory.
hipcc $FLAGS -S --cuda-device-only gemm_tiled.hip -o _build/gemm_tiled.s
python3 - <<'PY'
import re, sys
txt = open("_build/gemm_tiled.s").read()
bad = []
for m in re.finditer(r"\.name:\s+(\S*w3lr_tiled_kernel\S*)(.*?)\.wavefront_size", txt, re.S):
    scratch = int(re.search(r"\.private_segment_fixed_size:\s+(\d+)", m.group(2)).group(1))
    if scratch:
        bad.append((m.group(1), scratch))
if bad:
    sys.exit("tiled kernel variants use scratch memory: %r" % bad)
print("tiled kernel: no scratch memory")
PY
hipcc --offload-arch=gfx950 -shared -fPIC -o "$OUT/libmilo.so" _build/pack.o _build/gemm_tiled.o _build/gemm_decode.o _build/moe.o _build/api.o
echo "built $OUT/libmilo.so"
