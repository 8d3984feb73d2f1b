"""Ceilings of the units the fused attention kernel uses (instrumentation, not part of the product).

`python -m paper_2012_01114_amd.probe` runs libattnprobe.so on cuda:0 and prints one line per
combination of units: matrix cores, softmax vector work, LDS fragment reads, with constant and with
random operands.  One group = 16 MFMAs of 32x32x16 (one 32 x 32 score block at d_k = 128)."""
from __future__ import annotations

import ctypes as C
import json
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libattnprobe.so")
UNIT_NAMES = {1: "mfma", 2: "softmax valu", 4: "lds reads"}
MFMA_FLOP_PER_GROUP = 16 * 2 * 32 * 32 * 16
N_SIMD = 1024   # 256 compute units x 4


def run(units: int, density: int, waves_per_simd: int, random_operands: bool, iters: int = 2000):
    lib = C.CDLL(LIB_PATH)
    lib.attn_probe_run.restype = C.c_int
    lib.attn_probe_run.argtypes = [C.c_int] * 5 + [C.POINTER(C.c_double)] * 2
    ns, cyc = C.c_double(), C.c_double()
    rc = lib.attn_probe_run(units, density, waves_per_simd, iters, 1 if random_operands else 0, C.byref(ns), C.byref(cyc))
    if rc:
        raise RuntimeError(f"attn_probe_run returned {rc}")
    return ns.value, cyc.value


def run_block(deferred: bool, lds_reads: bool, waves_per_simd: int, iters: int = 4000):
    """One block of the d_k = 64 walk as the kernel issues it (vector phase, then matrix phase), with
    nothing behind it; deferred: the weighted sum of the block before between the exponentials."""
    lib = C.CDLL(LIB_PATH)
    lib.attn_probe_block.restype = C.c_int
    lib.attn_probe_block.argtypes = [C.c_int] * 4 + [C.POINTER(C.c_double)] * 2
    ns, cyc = C.c_double(), C.c_double()
    rc = lib.attn_probe_block(1 if deferred else 0, 1 if lds_reads else 0, waves_per_simd, iters, C.byref(ns), C.byref(cyc))
    if rc:
        raise RuntimeError(f"attn_probe_block returned {rc}")
    return ns.value, cyc.value


def main():
    rows = []
    for density in (1, 2):
        for units in (1, 2, 4, 3, 5, 7):
            for rnd in (False, True):
                for waves in (1, 2):
                    ns, cyc = run(units, density, waves, rnd)
                    name = " + ".join(n for b, n in UNIT_NAMES.items() if units & b)
                    rec = {"units": name, "pairs_per_group": 8 * density, "waves_per_simd": waves,
                           "operands": "random" if rnd else "constant", "ns_per_group_per_simd": round(ns, 1),
                           "cycles_per_group_per_simd": round(cyc, 1), "clock_ghz": round(cyc / ns, 3)}
                    if units & 1:
                        rec["mfma_tflops_chip"] = round(MFMA_FLOP_PER_GROUP * N_SIMD / ns / 1e3, 1)
                    rows.append(rec)
                    print(json.dumps(rec), flush=True)
    for waves in (1, 2, 3):
        for deferred in (False, True):
            for reads in (False, True):
                ns, cyc = run_block(deferred, reads, waves)
                rec = {"block_of_the_walk": "d_k 64", "weighted_sum": "one block late, between the exponentials" if deferred
                       else "in the matrix phase", "lds_reads": reads, "waves_per_simd": waves,
                       "ns_per_block_per_simd": round(ns, 1), "cycles_per_block_of_a_wavefront": round(cyc, 1),
                       "mfma_tflops_chip": round(8 * 2 * 32 * 32 * 16 * N_SIMD / ns / 1e3, 1)}
                rows.append(rec)
                print(json.dumps(rec), flush=True)
    return rows


if __name__ == "__main__":
    main()
