"""Builds ``libtictac.so`` from ``csrc/`` with hipcc for gfx950 (cross-compiles without a GPU)."""

from __future__ import annotations

import glob
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libtictac.so")

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-munsafe-fp-atomics",
    "-Wall", "-Wno-unused-function",
]


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


def is_stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    deps = sources() + glob.glob(os.path.join(CSRC, "*.h")) + glob.glob(os.path.join(ROOT, "include", "*.h"))
    return any(os.path.getmtime(f) > t for f in deps)


# Kernels whose waits for memory are counted by hand ("s_waitcnt vmcnt(N)" in inline asm): the count is right only
# while the compiler issues exactly the memory instructions the source shows between two such waits.  For each
# kernel (by a piece of its mangled name): N, and what must lie between consecutive hand-written waits.
#   "level": exactly `loads` 16-byte loads and `stores` stores, nothing else that counts (N = 7 levels of them)
#   "request": after the stores that follow a wait come `loads` 16-byte loads in straight-line code (the request
#              the wait is counted for); up to the next wait only loads follow (a load whose value is used has
#              been waited for, and everything older with it: memory instructions of a wave complete in order)
COUNTED_WAITS = {
    "16propagate_levelsILi": {"n": 21, "kind": "level", "loads": 2, "stores": 1},
    "22propagate_levels_batchILi": {"n": 21, "kind": "level", "loads": 2, "stores": 1},
    "24propagate_levels_q_batchILi": {"n": 14, "kind": "level", "loads": 1, "stores": 1},
    "15propagate_nodesILi": {"n": 8, "kind": "request", "loads": 8},
}
_VM_PREFIXES = ("global_", "flat_", "scratch_", "buffer_")


def _functions(asm: str):
    """(name, lines) of every function in the assembly text."""
    name, lines = None, []
    for line in asm.splitlines():
        head = line.split(";")[0].rstrip()
        if head.startswith("_Z") and head.endswith(":"):
            name, lines = head[:-1], []
            continue
        if name is None:
            continue
        lines.append(line)
        if line.strip().startswith(".Lfunc_end"):
            yield name, lines
            name = None


def check_counted_waits(asm: str) -> list:
    """Violations (strings) of the rules above in the device assembly of k1_propagate.hip; [] when it is sound."""
    bad, seen = [], set()
    for name, lines in _functions(asm):
        rule = next((r for key, r in COUNTED_WAITS.items() if key in name), None)
        if rule is None:
            continue
        seen.add(next(key for key in COUNTED_WAITS if key in name))
        in_asm, events = False, []          # ("wait", n) | ("vm", mnemonic) | ("branch",)
        for line in lines:
            t = line.strip()
            if t.startswith(";;#ASMSTART"):
                in_asm = True
            elif t.startswith(";;#ASMEND"):
                in_asm = False
            elif t.startswith("s_waitcnt") and in_asm and "vmcnt(" in t:
                n = int(t.split("vmcnt(")[1].split(")")[0])
                if n > 0:
                    events.append(("wait", n))
            elif t.startswith(_VM_PREFIXES):
                events.append(("vm", t.split()[0]))
            elif t.startswith(("s_cbranch", "s_branch", "s_swappc", "s_setpc")):
                events.append(("branch",))
        if any(e[0] == "vm" and e[1].startswith(("scratch_", "buffer_")) for e in events):
            bad.append(f"{name}: register spills (scratch instructions) in a kernel with counted waits")
        waits = [i for i, e in enumerate(events) if e[0] == "wait"]
        if not waits:
            bad.append(f"{name}: no hand-written wait found")
            continue
        if any(events[i][1] != rule["n"] for i in waits):
            bad.append(f"{name}: a hand-written wait is not vmcnt({rule['n']})")
        if rule["kind"] == "level":
            for a, b in zip(waits, waits[1:]):
                ops = [e[1] for e in events[a + 1:b] if e[0] == "vm"]
                loads = sum(o == "global_load_dwordx4" for o in ops)
                stores = sum(o.startswith("global_store") for o in ops)
                if loads != rule["loads"] or stores != rule["stores"] or len(ops) != loads + stores:
                    bad.append(f"{name}: {ops} between two waits, expected {rule['loads']} loads and "
                               f"{rule['stores']} stores")
                    break
        else:
            for k, a in enumerate(waits):
                b = waits[k + 1] if k + 1 < len(waits) else len(events)
                region = events[a + 1:b]
                stores = [i for i, e in enumerate(region) if e[0] == "vm" and e[1].startswith("global_store")]
                first = (stores[-1] + 1) if stores else 0
                while first < len(region) and region[first][0] != "vm":
                    first += 1
                request = region[first:first + rule["loads"]]
                ok = len(request) == rule["loads"] and all(e == ("vm", "global_load_dwordx4") for e in request)
                ok = ok and all("load" in e[1] for e in region[first + rule["loads"]:] if e[0] == "vm")
                if not ok:
                    bad.append(f"{name}: after a wait, the stores are not followed by {rule['loads']} straight-line "
                               f"16-byte loads and then loads only")
                    break
    for key in COUNTED_WAITS:
        if key not in seen:
            bad.append(f"no kernel matching {key} in the assembly")
    return bad


def device_assembly(source: str) -> str:
    cmd = [HIPCC] + [f for f in FLAGS if f not in ("-shared", "-fPIC")] + \
        ["-I", os.path.join(ROOT, "include"), "-I", CSRC, "--cuda-device-only", "-S", "-o", "-", source]
    return subprocess.run(cmd, check=True, stdout=subprocess.PIPE, stderr=subprocess.DEVNULL, text=True).stdout


def build(verbose: bool = False) -> str:
    cmd = [HIPCC] + FLAGS + ["-I", os.path.join(ROOT, "include"), "-I", CSRC, "-o", LIB] + sources()
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    bad = check_counted_waits(device_assembly(os.path.join(CSRC, "k1_propagate.hip")))
    if bad:
        os.remove(LIB)
        raise RuntimeError("hand-counted memory waits no longer match the generated code:\n  " + "\n  ".join(bad))
    return LIB


if __name__ == "__main__":
    build(verbose=True)
    print(LIB)
