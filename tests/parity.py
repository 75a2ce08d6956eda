"""The comparator of the GPU parity tests: one output tensor of the HIP path against the fp64 oracle's.

Three measures, all of ||got - ref||_2 / ||ref||_2 kind, on the same pair of arrays:
  whole   over the whole tensor                           (the bar the benchmark spec states: 1e-5 fp32 I/O, 2e-2 bf16 I/O)
  group   per leading index -- per (b,h) pair of a [B,H,N,d] tensor, per batch entry of a [B,d,L] one --, worst one
  row     per row of the last axis (one token's features): the row's error over the larger of the row's own norm and
          the root-mean-square row norm of the BLOCK rows of the reference around it, worst one

The method reaches the plain causal sum exactly (Sec. 4.1; "lossless", Sec. 4.4), so every row has to agree with the
oracle to rounding, not just the tensor on average: a single wrong token row in a tensor of a million rows moves the
whole-tensor figure by a few parts in a thousand and would pass it.  What "to rounding" means for one row: its
rounding errors are proportional to the terms that were summed, not to the sum.  A row whose terms happen to cancel
(dQ_t = S_t dO_t with a state S_t of nearly equal positive entries and an upstream gradient whose features add up to
almost nothing -- a few rows in every thousand with positive feature maps) is a hundred times shorter than its
neighbours and carries the same absolute error as they do; measured against its own norm alone it reads 0.3 for
every correct implementation.  The neighbouring rows see the same state and terms of the same size, so their
root-mean-square norm is the scale such a row's error is held against; a row that is NOT short is held against its
own norm.  A row that took another row's values, lost a term or was never written is off by about its whole scale
and reads about 1 either way.

Bounds.  bf16 I/O: the final rounding of an output element is uniform in +-2^-9 relative (rms 2^-9/sqrt(3) = 1.1e-3),
the score tile and the carried state are rounded the same way once each as matrix-core operands and enter the two
halves of the sum, so a row of d >= 64 features is expected at (1.1e-3) * sqrt(1 + ~1 + ~1) ~ 2e-3 .. 2.5e-3 with a
spread of about 1/sqrt(2 d) ~ 9 % from row to row (measured: whole 2.3e-3 .. 2.5e-3).  EXPECT (6e-3) leaves 2.5x for
the whole tensor and for every group.  The worst single row among a million is another matter: a row's error is a
weighted sum of d element errors, and where the weights are uneven -- Y = Norm(O) * G with a silu gate, whose few
large entries may sit on small entries of Norm(O) -- the tail reaches 5x the typical row (measured: 1.1e-2 .. 1.3e-2
on the gated outputs, 3e-3 .. 7e-3 on the plain ones).  ROW_BAR is therefore the bar the benchmark spec states for the whole
tensor, 2e-2, now demanded of every single row; a row that is wrong rather than rounded reads 0.1 .. 1.  fp32 I/O:
sums of up to 1e5 terms in fp32 give ~1e-7 .. 5e-7 (worst row 2e-6); every measure is held to the 1e-5 bar.
"""
import numpy as np

BAR = {"f32": 1e-5, "bf16": 2e-2}          # the benchmark spec, whole tensor
EXPECT = {"f32": 2e-6, "bf16": 6e-3}       # what rounding explains (whole tensor and every group), with margin
ROW_BAR = {"f32": 1e-5, "bf16": 2e-2}      # worst single row: the stated bar, row by row
BLOCK = 64                                 # rows whose root-mean-square norm is the scale of a short row

STATS = []       # (name, dtype, whole, worst group, worst row) of every call, for the summary the tests print


def _as_groups(a):
    """[..., rows, d] -> [groups, rows, d]; a 2-D array is one group, a 1-D array one group of one row."""
    if a.ndim == 0:
        return a.reshape(1, 1, 1)
    if a.ndim == 1:
        return a.reshape(1, 1, -1)
    if a.ndim == 2:
        return a.reshape(1, a.shape[0], a.shape[1])
    return a.reshape(-1, a.shape[-2], a.shape[-1])


def measures(got, ref):
    """(whole, worst group, worst row, index of the worst row as (group, row)) for two float64 arrays of one shape."""
    assert got.shape == ref.shape, (got.shape, ref.shape)
    if ref.size == 0:
        return 0.0, 0.0, 0.0, (0, 0)
    g, r = _as_groups(got), _as_groups(ref)
    e2 = np.zeros(r.shape[:2])
    n2 = np.zeros(r.shape[:2])
    step = max(1, (1 << 24) // max(1, r.shape[1] * r.shape[2]))          # groups per slab: bounds the temporaries
    for s in range(0, r.shape[0], step):
        diff = g[s:s + step] - r[s:s + step]
        e2[s:s + step] = np.einsum("gnd,gnd->gn", diff, diff)
        n2[s:s + step] = np.einsum("gnd,gnd->gn", r[s:s + step], r[s:s + step])
    tot_n = float(n2.sum())
    whole = float(np.sqrt(e2.sum() / tot_n)) if tot_n > 0 else (0.0 if float(e2.sum()) == 0 else np.inf)
    gn = n2.sum(axis=1)
    ge = e2.sum(axis=1)
    with np.errstate(divide="ignore", invalid="ignore"):
        grp = np.where(gn > 0, np.sqrt(ge / np.where(gn > 0, gn, 1.0)), np.where(ge > 0, np.inf, 0.0))
    # scale of a row: its own norm, or the rms norm of its block of BLOCK rows if that is larger
    G, N = n2.shape
    nb = (N + BLOCK - 1) // BLOCK
    padded = np.full((G, nb * BLOCK), np.nan)
    padded[:, :N] = n2
    local2 = np.repeat(np.nanmean(padded.reshape(G, nb, BLOCK), axis=2), BLOCK, axis=1)[:, :N]
    den = np.maximum(n2, local2)
    with np.errstate(divide="ignore", invalid="ignore"):
        row = np.where(den > 0, np.sqrt(e2 / np.where(den > 0, den, 1.0)), np.where(e2 > 0, np.inf, 0.0))
    at = np.unravel_index(int(np.argmax(row)), row.shape)
    return whole, float(grp.max()), float(row.max()), (int(at[0]), int(at[1]))


def check(name, got, ref, dtype, to_f64):
    """Assert all three measures; `got` is a tensor of the HIP path (any device), `ref` the oracle's float64 array."""
    g = to_f64(got)
    whole, grp, row, at = measures(g, np.asarray(ref, dtype=np.float64))
    print("   rel-L2 %-12s whole %.3e   worst group %.3e   worst row %.3e at %s" % (name, whole, grp, row, at),
          flush=True)
    STATS.append((name, dtype, whole, grp, row))
    assert np.isfinite(whole) and whole <= BAR[dtype], (name, "whole tensor", whole)
    assert whole <= EXPECT[dtype], (name, "whole tensor", whole, "inside the bar but larger than rounding explains")
    # A group of fewer than BLOCK rows (a sequence of one token, say) averages over nothing and has no neighbours to
    # take a short row's scale from -- dK of a single token is q (v . dO), and the 128 terms of that scalar may
    # cancel --: there the stated bar is what is left to hold every measure to.
    rows_per_group = 1 if np.ndim(ref) < 2 else np.shape(ref)[-2]
    short = rows_per_group < BLOCK
    assert np.isfinite(grp) and grp <= (BAR[dtype] if short else EXPECT[dtype]), (name, "worst (b,h) / leading index", grp)
    assert np.isfinite(row) and row <= (BAR[dtype] if short else ROW_BAR[dtype]), (name, "worst row", row, at)
    return whole
