#!/bin/bash
# Builds libmilo.so for gfx950 from the HIP sources next to this script.
set -e
cd "$(dirname "$0")"
OUT=../lib
mkdir -p "$OUT" _build
FLAGS="-O3 --offload-arch=gfx950 -fPIC -std=c++17 -Xclang -target-feature -Xclang -packed-fp32-ops -fhip-fp32-correctly-rounded-divide-sqrt -Wno-unused-command-line-argument"
# the decode kernel's leading scalar arguments are placed in registers at wave start (see gemm_decode.hip)
PRELOAD="-mllvm -amdgpu-kernarg-preload-count=11"
pids=()
hipcc $FLAGS -ffp-contract=off -c pack.hip -o _build/pack.o & pids+=($!)
hipcc $FLAGS -ffp-contract=off -c compress.hip -o _build/compress.o & pids+=($!)
hipcc $FLAGS -c gemm_tiled.hip -o _build/gemm_tiled.o & pids+=($!)
hipcc $FLAGS $PRELOAD -c gemm_decode.hip -o _build/gemm_decode.o & pids+=($!)
hipcc $FLAGS -c moe.hip -o _build/moe.o & pids+=($!)
hipcc $FLAGS -c api.hip -o _build/api.o & pids+=($!)
hipcc $FLAGS -c gemm_static.hip -o _build/gemm_static.o & pids+=($!)
# the same two GEMM kernels with every hand-counted wait replaced by a wait for everything
hipcc $FLAGS -DMILO_FULL_WAITS -c gemm_tiled.hip -o _build/gemm_tiled_fw.o & pids+=($!)
hipcc $FLAGS $PRELOAD -DMILO_FULL_WAITS -c gemm_decode.hip -o _build/gemm_decode_fw.o & pids+=($!)
for p in "${pids[@]}"; do wait $p; done
# The decode kernel counts outstanding memory operations by hand (see gemm_decode.hip): a streaming
# wave requests in a fixed order (per chunk XC buffer-to-LDS copies of activations and per row block a
# 16-byte and a 12-byte load of weights) and waits with "s_waitcnt vmcnt(N)".  The compiler must not
# reorder these requests; memory operations of its own (register spills) after a counted request only
# make a counted wait longer, never too short, but they must stay out of the streaming loop.
hipcc $FLAGS $PRELOAD -S --cuda-device-only gemm_decode.hip -o _build/gemm_decode.s
python3 - <<'PY'
import re, sys
txt = open("_build/gemm_decode.s").read()
VMEM = re.compile(r"\s+(buffer_|global_|scratch_|flat_)(\S+)")
checked = 0
for m in re.finditer(r"^(_ZN4milo18w3lr_decode_kernelILi(\d+)ELi(\d+)ELi(\d+)E\S*):[^\n]*\n(.*?)^\.Lfunc_end", txt, re.S | re.M):
    name = m.group(1)
    R, LR, XC = (int(m.group(i)) for i in (2, 3, 4))
    body = m.group(5).split("\n")
    ev = []
    for i, line in enumerate(body):
        w = re.search(r"s_waitcnt vmcnt\((\d+)\)", line)
        if w and i > 0 and "ASMSTART" in body[i - 1]:
            if int(w.group(1)) > 0:
                ev.append(int(w.group(1)))
            continue
        v = VMEM.match(line)
        if v:
            ev.append(v.group(1) + v.group(2) + (" lds" if " lds" in line else ""))
    unit = ["buffer_load_dwordx4", "buffer_load_dwordx3"]
    xcp = ["buffer_load_dwordx4 lds"] * XC
    nz = lambda seq: [x for x in seq if x != 0]
    want = xcp + unit * R                                           # first chunk, up front
    want += nz([2 * (R - 1)]) + xcp + unit                          # loop: unit 0, next activations, next unit 0
    for b in range(1, R):
        want += [2 * (R - 1) + XC] + unit                           #       unit b, next unit b
    want += nz([2 * (R - 1 - b) for b in range(R)])                 # last chunk
    # the streaming loop is the one place with counted waits: its whole sequence must appear as it is
    # (what a T worker does before it, when it goes on to stream, is complete by then: it ends with a
    # wait for everything)
    found = any(ev[i:i + len(want)] == want for i in range(len(ev) - len(want) + 1))
    counted = [e for e in ev if isinstance(e, int)]
    if not found or counted != [e for e in want if isinstance(e, int)]:
        sys.exit("%s: requests and waits of the streaming loop are not in the counted order:\n%r\nexpected\n%r" % (name, ev, want))
    checked += 1
if checked == 0:
    sys.exit("decode kernel: nothing checked; the check is out of date")
print("decode kernel: request order around the hand-counted waits verified in %d variants" % checked)
PY
# The tiled kernel counts outstanding memory operations by hand too (in its K loop); that is safe as
# long as the compiler adds none of its own there: no scratch access may sit between the barriers
# around a hand-written wait for a non-zero count (a wait for zero assumes nothing).  (Its cold path that forms T may spill; it only waits for zero.)
hipcc $FLAGS -S --cuda-device-only gemm_tiled.hip -o _build/gemm_tiled.s
python3 - <<'PY'
import re, sys
txt = open("_build/gemm_tiled.s").read()
bad, n, waits = [], 0, 0
for m in re.finditer(r"^(_ZN4milo17w3lr_tiled_kernel\S*):[^\n]*\n(.*?)^\.Lfunc_end", txt, re.S | re.M):
    n += 1
    body = m.group(2).split("\n")
    bars = [i for i, l in enumerate(body) if re.match(r"\s+s_barrier", l)]
    for i, l in enumerate(body):
        w = re.search(r"s_waitcnt vmcnt\((\d+)\)", l)
        if not (i > 0 and "ASMSTART" in body[i - 1] and w):
            continue
        if int(w.group(1)) == 0:
            continue        # waits for everything: valid whatever else is in flight
        waits += 1
        lo = max([b for b in bars if b < i] or [0])
        hi = min([b for b in bars if b > i] or [len(body)])
        if any(re.match(r"\s+scratch_", x) for x in body[lo:hi]):
            bad.append((m.group(1), i))
if bad or n == 0 or waits == 0:
    sys.exit("tiled kernel: scratch access inside the K loop (or nothing checked): %r" % bad[:4])
print("tiled kernel: no scratch access around %d hand-counted waits in %d variants" % (waits, n))
PY
hipcc --offload-arch=gfx950 -shared -fPIC -o "$OUT/libmilo.so" _build/pack.o _build/gemm_tiled.o _build/gemm_decode.o _build/moe.o _build/api.o _build/gemm_static.o _build/compress.o
hipcc --offload-arch=gfx950 -shared -fPIC -o "$OUT/libmilo_fullwaits.so" _build/pack.o _build/gemm_tiled_fw.o _build/gemm_decode_fw.o _build/moe.o _build/api.o _build/gemm_static.o _build/compress.o
# Every kernel the host code launches must have its launch stub in the library (a stub that the
# compiler failed to emit only shows up as an undefined symbol when the library is loaded).
for lib in libmilo.so libmilo_fullwaits.so; do
    if nm -u "$OUT/$lib" | grep -q "__device_stub__"; then
        echo "$lib has undefined kernel launch stubs:" >&2
        nm -u "$OUT/$lib" | grep "__device_stub__" >&2
        exit 1
    fi
done
echo "built $OUT/libmilo.so and $OUT/libmilo_fullwaits.so"
