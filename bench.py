"""Benchmark of the whole self-attention call on one MI355X.

One step = one attn_forward: q/k/v projection GEMM and the fused
score/softmax/weighted-sum kernel with redundancy skipping, on synthetic
inputs already resident in HBM.  Prints ONE JSON line.

  value     useful TFLOP/s of the whole call: (projection FLOPs of the rows some
            allowed pair uses + 4*d_k FLOPs per NEEDED pair, i.e. post-skip) /
            wall time per step
  roofline  the dominant kernel (by time) against the bf16 MFMA peak; its
            duration is measured with HIP events recorded by the library on the
            launch stream around every kernel, in a pass of its own after the
            headline pass (which carries no events)
  workloads the same three rates (whole call, projection, attention) for the
            other workloads of the metric
  cpu_baseline  the float64 CPU checker timed on a bounded sample of the same
            workload (reported, not a target)
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

MFMA_BF16_PEAK_TFLOPS = 2500.0   # MI355X dense bf16, published

# HBM/fabric bytes per launch from rocprofv3 counter runs (FETCH_SIZE + WRITE_SIZE, each scaled by what
# the same counter reads for a plain 1 GiB device copy: x2.00 and x1.00; see profiles/).  They hold for
# the kernel sources with the hash below; with other sources the bench line carries null.
TRAFFIC_SOURCES_SHA256 = "39f81de1bce478a69b42e703e25d685277851c6381e0111e8946276781ab65ab"
TRAFFIC_BYTES = {
    "long": {"projection": int((2 * 589960 + 196640) * 1024), "attention": int((2 * 151010 + 65792) * 1024)},
    "causal": {"projection": int((2 * 39037 + 36896) * 1024), "attention": int((2 * 18670 + 12480) * 1024)},
}


def kernel_sources_sha256() -> str:
    """Hash of what libattnring.so is built from (the probe library's source is not part of it)."""
    import glob
    import hashlib
    from paper_2012_01114_amd import build as libbuild
    csrc = os.path.join(ROOT, "paper_2012_01114_amd", "csrc")
    files = sorted([os.path.join(csrc, f) for f in libbuild.SOURCES] + glob.glob(os.path.join(csrc, "*.h")))
    h = hashlib.sha256()
    for f in files:
        h.update(os.path.basename(f).encode())
        with open(f, "rb") as fh:
            h.update(fh.read())
    return h.hexdigest()
METRIC = "useful attention TFLOP/s (post-skip) + % bf16 MFMA peak, 1 MI355X"


def needed_pairs(w, lens, rows_too=False):
    """Pairs phase 1 must touch, all batch items and heads (closed forms).  rows_too: query rows
    past the key length are left out as well."""
    n = w.n
    from paper_2012_01114_amd import inputs
    Ls = [int(L) for L in (lens if lens is not None else [n] * w.batch)]
    if w.scheme == inputs.SCHEME_CAUSAL:
        per = [L * (L + 1) // 2 + (0 if rows_too else (n - L) * L) for L in Ls]
    else:
        per = [(L if rows_too else n) * L for L in Ls]
    return sum(per) * w.n_heads


def cpu_baseline(w, f64, lens, budget_s=12.0, max_heads=256, rows_too=False):
    """Time the CPU checker on (batch, head) pairs, 256 sampled rows each, until about
    `budget_s` seconds of CPU work have been spent."""
    from oracle import attn_oracle as orc
    import numpy as np
    rng = np.random.default_rng(7)
    t_total, flop = 0.0, 0.0
    picks = []
    for s in range(max_heads):
        if t_total >= budget_s:
            break
        b = int(rng.integers(0, w.batch))
        h = int(rng.integers(0, w.n_heads))
        rows = sorted(int(r) for r in rng.choice(w.n, size=min(256, w.n), replace=False))
        t0 = time.perf_counter()
        orc.head_rows(f64["X"], f64["Wq"], f64["Wk"], f64["Wv"], n_heads=w.n_heads, d_k=w.d_k, p=w.p,
                      scheme=w.scheme, scale=w.d_k ** -0.5, b=b, h=h, rows=rows, lens=lens,
                      skip_padded_rows=rows_too)
        t_total += time.perf_counter() - t0
        L = w.n if lens is None else int(lens[b])
        from paper_2012_01114_amd import inputs
        pairs = sum((min(r + 1, L) if w.scheme == inputs.SCHEME_CAUSAL else L) for r in rows
                    if not (rows_too and r >= L))
        flop += 2.0 * w.d_model * w.d_k * (2 * w.n + len(rows)) + 4.0 * w.d_k * pairs
        picks.append((b, h))
    return {"value": flop / t_total / 1e12, "unit": "TFLOP/s", "cores": orc.num_threads(), "kind": "oracle",
            "seconds": round(t_total, 2),
            "sample": f"{len(picks)} (batch, head) pairs, k and v projected for all {w.n} rows, "
                      f"{min(256, w.n)} random query rows each; FLOPs counted for the sample only"}


class Session:
    """One workload resident on the GPU: inputs, context, output buffer."""

    def __init__(self, name, tiles="auto", skip_padded_rows=False, scheme=None, one_weight=False, packed=False):
        """scheme: run the workload's shape under another scheme; one_weight: Wq in all three roles
        (the setting in which the q = k = v scheme and the original definition give the same result);
        packed: the items cut to their lengths and stored back to back (attn_forward_packed)."""
        import torch
        from paper_2012_01114_amd import attnring as ar
        from paper_2012_01114_amd import inputs
        self.ar, self.torch = ar, torch
        self.w = w = inputs.WORKLOADS[name]
        if scheme is not None:
            self.w = w = inputs.with_scheme(w, scheme)
        stored, self.f64 = inputs.make_inputs(w)
        if one_weight:
            stored["Wk"] = stored["Wv"] = stored["Wq"]
        self.lens = stored["lens"]
        dev = torch.device("cuda:0")
        self.X, self.Wq, self.Wk, self.Wv = [stored[k].to(dev) for k in ("X", "Wq", "Wk", "Wv")]
        self.lens_dev = None if self.lens is None else torch.from_numpy(self.lens).to(dev)
        self.out = torch.empty(w.batch, w.n, w.hd, dtype=self.X.dtype, device=dev)
        dt = ar.ATTN_F32 if w.dtype == "f32" else ar.ATTN_BF16
        flags = {"auto": 0, "wide": ar.ATTN_FLAG_WIDE_TILES, "narrow": ar.ATTN_FLAG_NARROW_TILES}[tiles]
        self.packed = packed and self.lens is not None
        self.rows_too = (skip_padded_rows or self.packed) and self.lens is not None
        if self.rows_too:
            flags |= ar.ATTN_FLAG_SKIP_PADDED_ROWS
        if self.packed:
            import numpy as np
            offs = np.concatenate([[0], np.cumsum(self.lens)]).astype(np.int32)
            self.offs_dev = torch.from_numpy(offs).to(dev)
            self.X = torch.cat([self.X[b, :int(L)] for b, L in enumerate(self.lens)], 0).contiguous()
            self.out = torch.empty(int(offs[-1]), w.hd, dtype=self.X.dtype, device=dev)
        self.ctx = ar.attn_init(w.batch, w.n, w.d_model, w.n_heads, w.d_k, w.p, dt, 0.0, flags)
        ar.attn_set_key_lengths(self.ctx, self.lens_dev)
        self.stream = torch.cuda.current_stream(dev)

    def step(self):
        if self.packed:
            self.ar.attn_forward_packed(self.ctx, self.offs_dev, self.X, self.Wq, self.Wk, self.Wv, self.w.scheme,
                                        self.out, self.stream)
            return
        self.ar.attn_forward(self.ctx, self.X, self.Wq, self.Wk, self.Wv, self.w.scheme, self.out, self.stream)

    def flops(self):
        """(attention FLOPs on needed pairs, projection FLOPs of the rows some allowed pair uses)."""
        import numpy as np
        w, lens = self.w, self.lens
        pairs = needed_pairs(w, lens, self.rows_too)
        kv_rows = w.batch * w.n if lens is None else int(np.minimum(np.maximum(lens, 0), w.n).sum())
        q_rows = kv_rows if self.rows_too else w.batch * w.n
        return 4.0 * w.d_k * pairs, 2.0 * (q_rows + 2 * kv_rows) * w.d_model * w.hd, pairs

    def measure(self, steps, warmup, repeats):
        """Headline pass: `repeats` timed regions of exactly `steps` back-to-back calls each, wall clock
        between device synchronisations, nothing else on the stream; the median region counts.
        Then a separate pass of `steps` calls with the library's per-kernel HIP events switched on."""
        torch, ar = self.torch, self.ar
        for _ in range(warmup):
            self.step()
        torch.cuda.synchronize()
        regions = []
        for _ in range(repeats):
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(steps):
                self.step()
            torch.cuda.synchronize()
            regions.append((time.perf_counter() - t0) * 1e3 / steps)
        ar.attn_profile(self.ctx, True)
        for _ in range(steps):
            self.step()
        prof = ar.attn_profile_read(self.ctx)
        ar.attn_profile(self.ctx, False)
        stats = ar.attn_stats(self.ctx)
        regions_sorted = sorted(regions)
        return regions_sorted[len(regions) // 2], regions, prof, stats

    def close(self):
        self.torch.cuda.synchronize()
        self.ar.attn_destroy(self.ctx)
        self.ctx = None


def rates(attn_flop, proj_flop, ms_step, prof):
    """Whole call, projection alone, attention alone: TFLOP/s and share of the bf16 MFMA peak."""
    def one(flop, ms):
        t = flop / (ms * 1e-3) / 1e12
        return {"ms": round(ms, 4), "tflops": round(t, 2), "pct_of_peak": round(100.0 * t / MFMA_BF16_PEAK_TFLOPS, 2)}
    return {"whole_call": one(attn_flop + proj_flop, ms_step),
            "projection": one(proj_flop, prof["ms_projection"]),
            "attention": one(attn_flop, prof["ms_attention"])}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--repeats", type=int, default=5, help="timed regions of --steps calls each; the median counts")
    ap.add_argument("--workload", default="long", help="tiny|encoder|causal|long|padded")
    ap.add_argument("--others", default="causal,encoder,padded",
                    help="workloads timed besides the headline one (GPU only, reported under `workloads`); '' for none")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--skip-padded-rows", action="store_true",
                    help="padded workload: leave the padded vectors out as queries too (ATTN_FLAG_SKIP_PADDED_ROWS); "
                         "the useful FLOPs shrink accordingly")
    ap.add_argument("--tiles", default="auto", choices=["auto", "wide", "narrow"],
                    help="attention kernel choice (default: the library's own)")
    ap.add_argument("--copy-probe", type=int, default=0, metavar="MIB",
                    help="instead of the benchmark, run 10 plain device copies of MIB MiB (reference for "
                         "scaling rocprofv3 FETCH_SIZE / WRITE_SIZE readings)")
    args = ap.parse_args()
    if args.copy_probe:
        import torch
        src = torch.ones(args.copy_probe << 20, dtype=torch.uint8, device="cuda:0")
        dst = torch.empty_like(src)
        for _ in range(10):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_probe_mib": args.copy_probe, "copies": 10}))
        return
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1")

    import torch
    from paper_2012_01114_amd import attnring as ar
    from paper_2012_01114_amd import inputs

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    if not os.path.exists(ar.LIB_PATH):
        from paper_2012_01114_amd import build as libbuild
        libbuild.build()

    ses = Session(args.workload, args.tiles, args.skip_padded_rows)
    w, lens, rows_too = ses.w, ses.lens, ses.rows_too
    ms_step, regions, prof, stats = ses.measure(args.steps, args.warmup, args.repeats)
    attn_flop, proj_flop, pairs = ses.flops()
    assert pairs == stats["pairs_needed"][0], (pairs, stats["pairs_needed"])
    value = (attn_flop + proj_flop) / (ms_step * 1e-3) / 1e12
    f64 = ses.f64
    ses.close()

    kern = {
        "attention": {"flop": attn_flop, "ms": prof["ms_attention"]},
        "projection": {"flop": proj_flop, "ms": prof["ms_projection"]},
    }
    dom = max(kern, key=lambda k: kern[k]["ms"])
    achieved = kern[dom]["flop"] / (kern[dom]["ms"] * 1e-3) / 1e12
    traffic = None
    if args.tiles == "auto" and not rows_too and kernel_sources_sha256() == TRAFFIC_SOURCES_SHA256:
        traffic = TRAFFIC_BYTES.get(w.name, {}).get(dom)
    roofline = {"kernel": dom, "bound": "mfma", "achieved": round(achieved, 2), "peak": MFMA_BF16_PEAK_TFLOPS,
                "unit": "TFLOP/s", "frac": round(achieved / MFMA_BF16_PEAK_TFLOPS, 4), "traffic": traffic,
                "avg_ms": round(kern[dom]["ms"], 4)}
    extra = {k: {"tflops": round(v["flop"] / (v["ms"] * 1e-3) / 1e12, 2), "avg_ms": round(v["ms"], 4),
                 "frac_of_mfma_peak": round(v["flop"] / (v["ms"] * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4)}
             for k, v in kern.items()}
    extra["prepare_avg_ms"] = round(prof["ms_prepare"], 4)

    def describe(w, lens, rows_too):
        return (f"{w.name}: batch {w.batch}, n {w.n}, d_model {w.d_model}, heads {w.n_heads}, "
                f"d_k {w.d_k}, scheme {inputs.SCHEME_NAMES[w.scheme]}, P {w.p}"
                + (", key lengths from seed" if lens is not None else "")
                + (", padded rows left out" if rows_too else ""))

    line = {
        "metric": METRIC, "value": round(value, 2), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_step, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16" if w.dtype == "bf16" else "f32", "data": "synthetic",
        "pct_bf16_mfma_peak": round(100.0 * value / MFMA_BF16_PEAK_TFLOPS, 2),
        "timing": {"repeats": args.repeats, "ms_per_step_each": [round(r, 4) for r in regions],
                   "reported": "median region; per-kernel times from a separate pass with HIP events"},
        "operands": "projection: bf16 x bf16 -> fp32; q, k, v and the exponentials kept in fp16 (same MFMA rate), "
                    "scores and weighted sums accumulate in fp32; out rounded to bf16",
        "config": {"workload": describe(w, lens, rows_too),
                   "needed_pairs": pairs, "full_pairs": stats["pairs_full"],
                   "tiles_executed": stats["tiles_executed"], "tiles_full": stats["tiles_full"]},
        "roofline": roofline,
        "kernels": extra,
    }

    # the other workloads of the metric: GPU only, same protocol, inputs drawn once each
    others = {}
    runs = []
    for name in [n for n in args.others.split(",") if n and n != args.workload]:
        runs.append((name, {}))
        if inputs.WORKLOADS[name].padded:  # the same items without their padded rows, in both layouts
            runs.append((name + "_rows_left_out", {"skip_padded_rows": True}))
            runs.append((name + "_packed", {"packed": True}))
    for label, kw in runs:
        o = Session(label.split("_")[0], **kw)
        o_ms, o_regions, o_prof, o_stats = o.measure(args.steps, args.warmup, args.repeats)
        o_attn, o_proj, o_pairs = o.flops()
        assert o_pairs == o_stats["pairs_needed"][0]
        rec = rates(o_attn, o_proj, o_ms, o_prof)
        rec["ms_per_step"] = round(o_ms, 4)
        rec["workload"] = describe(o.w, o.lens, o.rows_too) + (", stored back to back" if o.packed else "")
        others[label] = rec
        o.close()
        del o
        torch.cuda.empty_cache()
    if others:
        line["workloads"] = others

    # Sec. 4: the q = k = v scheme (each score tile computed once, used for both row blocks) against
    # the original definition on the same inputs, Wq in all three roles; encoder shape
    if args.others:
        rec = {}
        for label, scheme in (("full", inputs.SCHEME_FULL), ("symmetric", inputs.SCHEME_SYMMETRIC)):
            o = Session("encoder", scheme=scheme, one_weight=True)
            o_ms, _, o_prof, o_stats = o.measure(args.steps, args.warmup, args.repeats)
            rec[label] = {"ms_per_step": round(o_ms, 4), "ms_projection": round(o_prof["ms_projection"], 4),
                          "ms_attention": round(o_prof["ms_attention"], 4),
                          "phase1_pairs_needed": o_stats["pairs_needed"][0],
                          "phase1_pairs_scheduled": o_stats["pairs_scheduled"][0],
                          "score_blocks_issued": o_stats["phys_tiles_executed"]}
            o.close()
            del o
            torch.cuda.empty_cache()
        rec["workload"] = "encoder shape, Wq = Wk = Wv"
        line["symmetric_vs_full"] = rec

    if not args.no_cpu_baseline:
        line["cpu_baseline"] = cpu_baseline(w, f64, lens, rows_too=rows_too)
    print(json.dumps(line))


if __name__ == "__main__":
    main()
