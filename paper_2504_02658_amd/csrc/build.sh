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
# The decode kernel counts outstanding memory operations by hand (see gemm_decode.hip): all loads
# of a piece are issued in a fixed order (per chunk eight buffer-to-LDS copies, then per row block
# a 16-byte and a 12-byte load) before the first hand-written "s_waitcnt vmcnt(N)",
# and the compiler must neither reorder them nor add memory operations of its own (spills).
hipcc $FLAGS -S --cuda-device-only gemm_decode.hip -o _build/gemm_decode.s
python3 - <<'PY'
import re, sys
txt = open("_build/gemm_decode.s").read()
checked = 0
VMEM = re.compile(r"\s+(buffer_|global_|scratch_|flat_)(\S+)")
CPW = 2
for m in re.finditer(r"^(_ZN4milo18w3lr_decode_kernelILi(\d+)ELi(\d+)\S*):[^\n]*\n(.*?)^\.Lfunc_end", txt, re.S | re.M):
    name, R, body = m.group(1), int(m.group(2)), m.group(4).split("\n")
    meta = re.search(r"\.name:\s+%s\b(.*?)\.wavefront_size" % re.escape(name), txt, re.S)
    if int(re.search(r"\.private_segment_fixed_size:\s+(\d+)", meta.group(1)).group(1)):
        sys.exit("%s uses scratch memory" % name)
    total = CPW * (8 + 2 * R)
    first = total - (8 + 2)
    hits = [i for i, line in enumerate(body)
            if i > 0 and "ASMSTART" in body[i - 1] and re.search(r"s_waitcnt vmcnt\(%d\)" % first, line)]
    if not hits:
        sys.exit("%s: no hand-written s_waitcnt vmcnt(%d) found" % (name, first))
    for i in hits:
        seen, j = [], i - 1
        while j >= 0 and len(seen) < total:
            v = VMEM.match(body[j])
            if v:
                seen.append(v.group(1) + v.group(2) + (" lds" if " lds" in body[j] else ""))
            j -= 1
        seen.reverse()
        unit = ["buffer_load_dwordx4", "buffer_load_dwordx3"]
        want = (["buffer_load_dwordx4 lds"] * 8 + unit * R) * CPW
        if seen != want:
            sys.exit("%s: the loads before s_waitcnt vmcnt(%d) are not in the counted order:\n%r" % (name, first, seen))
        checked += 1
if checked == 0:
    sys.exit("decode kernel: nothing checked; the check is out of date")
print("decode kernel: load order before %d hand-counted wait sequences verified" % checked)
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
hipcc --offload-arch=gfx950 -shared -fPIC -o "$OUT/libmilo.so" _build/pack.o _build/gemm_tiled.o _build/gemm_decode.o _build/moe.o _build/api.o
# Every kernel the host code launches must have its launch stub in the library (a stub that the
# compiler failed to emit only shows up as an undefined symbol when the library is loaded).
if nm -u "$OUT/libmilo.so" | grep -q "__device_stub__"; then
    echo "libmilo.so has undefined kernel launch stubs:" >&2
    nm -u "$OUT/libmilo.so" | grep "__device_stub__" >&2
    exit 1
fi
echo "built $OUT/libmilo.so"
