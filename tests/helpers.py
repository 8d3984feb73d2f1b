"""Shared plumbing of the GPU parity tests: run the library through its C ABI
binding on seeded inputs and fetch what the CPU checker says for the same inputs."""
import math
import os

import numpy as np

from oracle import attn_oracle as orc
from paper_2012_01114_amd import attnring as ar
from paper_2012_01114_amd import inputs


def tol_check(got, ref, dtype):
    """Parity bar.  f32: |g-r| <= 1e-5*|r| + 1e-5*max|r|.  bf16: |g-r| <= 2e-2."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape
    assert np.all(np.isfinite(got)), "non-finite output"
    err = np.abs(got - ref)
    if dtype == "f32":
        bound = 1e-5 * np.abs(ref) + 1e-5 * np.max(np.abs(ref))
    else:
        bound = np.full_like(ref, 2e-2)
    bad = err > bound
    assert not bad.any(), (f"{int(bad.sum())} of {bad.size} elements out of tolerance; "
                           f"max err {err.max():.3e} at {np.unravel_index(err.argmax(), err.shape)}")
    return float(err.max())


def report_max_err(case, err, dtype):
    """One line per parity case (shown by `pytest -rA`), also appended to the file that
    ATTN_PARITY_LOG names, if set."""
    line = f"[maxerr] {case}: {err:.3e} ({dtype}; bar {'2e-2 abs' if dtype == 'bf16' else '1e-5 rel'})"
    print(line, flush=True)
    path = os.environ.get("ATTN_PARITY_LOG")
    if path:
        with open(path, "a") as fh:
            fh.write(line + "\n")


def expected_phys_blocks(w, scheme, lens=None, skip_padded_rows=False, block=32):
    """Score blocks of `block` x `block` pairs that hold at least one allowed pair, summed over
    batch items and heads, enumerated from the pair predicate itself: pair (i, j) is allowed iff
    j < len, (masked scheme) j <= i, and (padded rows left out) i < len.  Row blocks are the
    32-row groups a wavefront owns, key blocks the 32-key groups it walks."""
    n = w.n
    nb = (n + block - 1) // block
    total = 0
    i = np.arange(n)[:, None]
    j = np.arange(n)[None, :]
    for b in range(w.batch):
        L = n if lens is None else int(min(max(int(lens[b]), 0), n))
        ok = np.broadcast_to(j < L, (n, n)).copy()
        if scheme == inputs.SCHEME_CAUSAL:
            ok &= j <= i
        if skip_padded_rows:
            ok &= i < L
        pad = np.zeros((nb * block, nb * block), dtype=bool)
        pad[:n, :n] = ok
        total += int(pad.reshape(nb, block, nb, block).any(axis=(1, 3)).sum())
    return total * w.n_heads


def expected_sym_blocks(w, tile=128, block=32):
    """q = k = v scheme on the matrix cores: 32 x 32 score blocks computed when every unordered pair
    of 128-row tiles is computed once (Eq. (4): the other orientation reuses it), counting the
    blocks that hold a row and a key below n."""
    n = w.n
    nt = (n + tile - 1) // tile
    total = 0
    for a in range(nt):
        row_blocks = len([r for r in range(tile // block) if a * tile + r * block < n])
        for b in range(a + 1):
            key_blocks = len([c for c in range(tile // block) if b * tile + c * block < n])
            total += row_blocks * key_blocks
    return total * w.batch * w.n_heads


def default_scale(w, scale):
    return (1.0 / math.sqrt(w.d_k)) if scale == 0.0 else scale


class GpuRun:
    """One context + device copies of one workload's inputs."""

    def __init__(self, w, stored, scale=0.0, flags=0):
        import torch
        self.torch = torch
        self.w = w
        dev = torch.device("cuda:0")
        self.dt = ar.ATTN_F32 if w.dtype == "f32" else ar.ATTN_BF16
        self.X = stored["X"].to(dev)
        self.W = [None if stored[k] is None else stored[k].to(dev) for k in ("Wq", "Wk", "Wv")]
        self.lens = None
        if stored.get("lens") is not None:
            self.lens = torch.from_numpy(np.asarray(stored["lens"], dtype=np.int32)).to(dev)
        self.ctx = ar.attn_init(w.batch, w.n, w.d_model, w.n_heads, w.d_k, w.p, self.dt, scale, flags)
        ar.attn_set_key_lengths(self.ctx, self.lens)
        self.out = torch.full((w.batch, w.n, w.hd), float("nan"), dtype=self.X.dtype, device=dev)

    def forward(self, scheme):
        ar.attn_forward(self.ctx, self.X, self.W[0], self.W[1], self.W[2], scheme, self.out)
        stats = ar.attn_stats(self.ctx)          # waits for the stream
        return self.out.to("cpu").to(self.torch.float64).numpy(), stats

    def forward_packed(self, scheme, lens, guard_rows=8):
        """The items cut to `lens` and stored back to back; returns the output laid out as
        [batch][n][...] again (zeros past the lengths) and the counts.  Rows of `out` past the
        last item must come back untouched."""
        torch = self.torch
        lens = [int(L) for L in lens]
        offs = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
        total = int(offs[-1])
        parts = [self.X[b, :L] for b, L in enumerate(lens)]
        Xp = torch.cat(parts, 0).contiguous() if total else self.X[0, :0].contiguous()
        if total == 0:  # an allocation to point at
            Xp = torch.zeros((1, self.w.d_model), dtype=self.X.dtype, device=self.X.device)
        outp = torch.full((total + guard_rows, self.w.hd), float("nan"), dtype=self.X.dtype, device=self.X.device)
        offs_dev = torch.from_numpy(offs).to(self.X.device)
        ar.attn_forward_packed(self.ctx, offs_dev, Xp, self.W[0], self.W[1], self.W[2], scheme, outp)
        stats = ar.attn_stats(self.ctx)
        host = outp.to("cpu").to(torch.float64).numpy()
        assert np.all(np.isnan(host[total:])), "rows past the last item were written"
        assert not np.any(np.isnan(host[:total])), "a row of an item was left unwritten"
        full = np.zeros((self.w.batch, self.w.n, self.w.hd))
        for b, L in enumerate(lens):
            full[b, :L] = host[offs[b]:offs[b] + L]
        return full, stats

    def close(self):
        if self.ctx is not None:
            self.torch.cuda.synchronize()
            ar.attn_destroy(self.ctx)
            self.ctx = None


def oracle_forward(w, f64, scheme, scale, lens=None, **kw):
    return orc.forward(f64["X"], f64["Wq"], f64["Wk"], f64["Wv"], n_heads=w.n_heads, d_k=w.d_k, p=w.p,
                       scheme=scheme, scale=default_scale(w, scale), lens=lens, **kw)


def oracle_counts(w, scheme, lens=None, **kw):
    return orc.counts(batch=w.batch, n=w.n, n_heads=w.n_heads, p=w.p, scheme=scheme, lens=lens, **kw)


def check_counts(stats, ref, noskip=False):
    """Bit-exact comparison of the library's counts with the checker's."""
    assert stats["pairs_full"] == ref["pairs_full"]
    assert stats["pairs_needed"] == ref["pairs_needed"]
    assert stats["pairs_scheduled"] == ref["pairs_scheduled"]
    assert stats["tiles_full"] == ref["tiles_full"]
    if noskip:
        assert stats["tiles_executed"] == ref["tiles_full"]
    else:
        assert stats["tiles_executed"] == ref["tiles_executed"]
        assert stats["pairs_executed"] == ref["pairs_executed"]


def custom_workload(name, B, n, D, H, d, p, dtype, scheme, seed, padded=False, len_lo=0, len_hi=0):
    return inputs.Workload(name, B, n, D, H, d, p, dtype, scheme, seed, padded, len_lo, len_hi)
