"""Pins for the CPU oracle: it is checked against things other than itself.

  * the hand-worked fixture in tests/golden/ (pencil evaluation of the paper's
    definitions: Section 5.1 rule row = o + s, Section 5.2 Layout / Notify /
    Dispatch / Combine equations),
  * brute force of the counting-set definition of s (Section 5.2, Prefill Layout),
  * library routines the definitions reduce to (numpy bincount, cumsum, stable argsort,
    take; an fp64 einsum for the combine sum; torch's CPU bf16 rounding),
  * closed forms and invariants (identity expert, power-of-two weights, permutation
    property, contiguity of expert blocks),
  * mutants: plausible mistakes planted in a copy of the oracle's source must each be
    caught by at least one of the checks above.
"""
import json
import os
import subprocess
import sys

import numpy as np
import pytest
from hypothesis import given, settings, strategies as st

import oracle
import workloads as wl


# --------------------------------------------------------------------------- helpers

def bf16(a):
    return wl.f32_to_bf16_bits(np.asarray(a, np.float32))


def unbf16(b):
    return wl.bf16_bits_to_f32(b)


def bf16_order(b):
    """Monotone integer image of bf16 bit patterns (for ulp distances)."""
    b = b.astype(np.int32)
    return np.where(b & 0x8000, 0x8000 - b, b)


def ulp_dist(a, b):
    return np.abs(bf16_order(a) - bf16_order(b))


def brute_s(K, E):
    """Counting-set definition of s, evaluated literally in O(N^2)."""
    flat = K.reshape(-1)
    s = np.full(flat.shape, -1, np.int64)
    for i, e in enumerate(flat):
        if 0 <= e < E:
            s[i] = sum(1 for ip in range(i) if flat[ip] == e)
    return s.reshape(K.shape)


# --------------------------------------------------------------------------- the pin suite
# Each check takes nothing and raises AssertionError on a wrong oracle; the mutant test
# re-runs all of them against deliberately broken copies.

def check_golden():
    g = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "worked_example.json")))
    E, R = g["E"], g["R"]
    X = bf16(g["X"])
    W = np.asarray(g["W"], np.float32)
    scale = np.asarray(g["scale"], np.float32)
    for case, stride in (("tight", 0), ("fixed_stride_4", 4), ("masked", 0)):
        c = g[case]
        K = np.asarray(c.get("K", g["K"]), np.int32)
        pl = oracle.plan(K, E, R, stride)
        assert pl.c_exp.tolist() == c["c_exp"], case
        assert pl.c_rank.tolist() == c["c_rank"], case
        assert pl.expert_offset.tolist() == c["expert_offset"], case
        assert pl.region_base.tolist() == c["region_base"], case
        assert pl.row_map.tolist() == c["row_map"], case
        assert pl.status.tolist() == c["status"] + [0], case
        if "s" in c:
            assert pl.s.tolist() == c["s"], case
        window = oracle.dispatch(X, pl.row_map, pl.window_rows)
        if "window_token" in c:
            assert np.array_equal(window, X[np.asarray(c["window_token"])]), case
        Yexp = oracle.expert_standin(window, K, pl.row_map, scale)
        if "Yexp" in c:
            assert np.array_equal(unbf16(Yexp), np.asarray(c["Yexp"], np.float32)), case
        for comb in (oracle.combine, oracle.combine_f64):
            Y = comb(Yexp, W, pl.row_map)
            assert np.array_equal(unbf16(Y), np.asarray(c["Y"], np.float32)), (case, comb.__name__)
        # the same example in fp32 storage
        Xf = np.asarray(g["X"], np.float32)
        wf = oracle.dispatch(Xf, pl.row_map, pl.window_rows)
        Yf = oracle.combine(oracle.expert_standin(wf, K, pl.row_map, scale), W, pl.row_map)
        assert np.array_equal(Yf, np.asarray(c["Y"], np.float32)), case


def check_plan_against_library(seed=0):
    rng = np.random.default_rng(seed)
    for T, k, E, R, distinct in ((16, 2, 8, 2, True), (37, 3, 12, 4, False), (64, 8, 256, 32, True),
                                 (5, 4, 2, 1, False), (1, 1, 1, 1, False), (33, 1, 6, 6, False)):
        K = wl.random_routing(rng, T, k, E, distinct=distinct)
        pl = oracle.plan(K, E, R)
        flat = K.reshape(-1)
        N = T * k
        Er = E // R
        counts = np.bincount(flat, minlength=E)
        assert np.array_equal(pl.c_exp, counts)
        assert np.array_equal(pl.c_rank, np.bincount(flat // Er, minlength=R))
        assert pl.c_exp.sum() == N and pl.c_rank.sum() == N
        assert np.array_equal(pl.c_rank, counts.reshape(R, Er).sum(axis=1))
        assert np.array_equal(pl.expert_offset, np.concatenate([[0], np.cumsum(counts)]))
        assert np.array_equal(pl.region_base, np.concatenate([[0], np.cumsum(pl.c_rank)]))
        assert np.array_equal(pl.region_base, pl.expert_offset[::Er])
        assert np.array_equal(pl.s, brute_s(K, E))
        order = np.argsort(flat, kind="stable")           # branches in window-row order
        inv = np.empty(N, np.int64)
        inv[order] = np.arange(N)
        assert np.array_equal(pl.row_map.reshape(-1), inv)
        assert np.array_equal(np.sort(pl.row_map.reshape(-1)), np.arange(N))   # a permutation
        # expert blocks are contiguous and stable: expert ids non-decreasing along rows,
        # flat indices increasing inside a block
        by_row = np.argsort(pl.row_map.reshape(-1))
        assert np.all(np.diff(flat[by_row]) >= 0)
        same = np.diff(flat[by_row]) == 0
        assert np.all(np.diff(by_row)[same] > 0)
        assert np.array_equal(pl.status, [0, 0, 0])


def check_masked_and_invalid(seed=1):
    rng = np.random.default_rng(seed)
    T, k, E, R = 41, 4, 12, 3
    K = wl.random_routing(rng, T, k, E, p_masked=0.2, p_invalid=0.1)
    pl = oracle.plan(K, E, R)
    flat = K.reshape(-1)
    valid = (flat >= 0) & (flat < E)
    assert pl.status[0] == np.count_nonzero(~valid & (flat != -1)) and pl.status[0] > 0
    assert np.array_equal(pl.c_exp, np.bincount(flat[valid], minlength=E))
    assert np.array_equal(pl.s, brute_s(K, E))
    assert np.all(pl.row_map.reshape(-1)[~valid] == -1)
    rows = pl.row_map.reshape(-1)[valid]
    assert np.array_equal(np.sort(rows), np.arange(valid.sum()))
    order = np.flatnonzero(valid)[np.argsort(flat[valid], kind="stable")]
    assert np.array_equal(pl.row_map.reshape(-1)[order], np.arange(valid.sum()))


def check_fixed_stride(seed=2):
    rng = np.random.default_rng(seed)
    T, k, E, R = 50, 2, 8, 4
    K = wl.random_routing(rng, T, k, E)
    tight = oracle.plan(K, E, R)
    stride = int(np.sort(tight.c_rank)[1])            # at least two regions overflow or just fit
    pl = oracle.plan(K, E, R, stride)
    Er = E // R
    assert np.array_equal(pl.region_base, np.arange(R + 1) * stride)
    assert np.array_equal(pl.c_exp, tight.c_exp) and np.array_equal(pl.s, tight.s)
    local = tight.expert_offset[:E] - tight.region_base[np.arange(E) // Er]
    assert np.array_equal(pl.expert_offset[:E], local + pl.region_base[np.arange(E) // Er])
    flat = K.reshape(-1)
    want = pl.expert_offset[flat] + pl.s.reshape(-1)
    drop = want >= pl.region_base[flat // Er + 1]
    assert pl.status[1] == drop.sum() == np.maximum(tight.c_rank - stride, 0).sum() and drop.sum() > 0
    assert np.array_equal(pl.row_map.reshape(-1), np.where(drop, -1, want))
    kept = pl.row_map.reshape(-1)[~drop]
    assert len(np.unique(kept)) == len(kept) and kept.max() < R * stride


def check_dispatch(seed=3):
    rng = np.random.default_rng(seed)
    for dtype in (wl.DTYPE_BF16, wl.DTYPE_F32):
        T, H, k, E, R = 29, 24, 3, 10, 5
        X = rng.standard_normal((T, H)).astype(np.float32)
        X = bf16(X) if dtype == wl.DTYPE_BF16 else X
        K = wl.random_routing(rng, T, k, E, p_masked=0.1)
        pl = oracle.plan(K, E, R)
        n = pl.window_rows
        window = oracle.dispatch(X, pl.row_map, n + 3, fill=7)
        flat = K.reshape(-1)
        valid = flat >= 0
        src = np.flatnonzero(valid)[np.argsort(flat[valid], kind="stable")] // k   # library: gather by sort
        assert np.array_equal(window[:n], np.take(X, src, axis=0))
        assert np.all(window[n:] == 7)                                             # nothing else touched
        for i, p in enumerate(pl.row_map.reshape(-1)):
            if p >= 0:
                assert window[p].tobytes() == X[i // k].tobytes()


def _einsum_reference(Yexp_f64, W, row_map):
    rm = np.where(row_map >= 0, row_map, 0)
    g = Yexp_f64[rm] * (row_map >= 0)[..., None]                  # [T,k,H]
    return np.einsum("tk,tkh->th", W.astype(np.float64), g)


def check_combine(seed=4):
    rng = np.random.default_rng(seed)
    T, H, k, E, R = 23, 40, 4, 8, 2
    K = wl.random_routing(rng, T, k, E, distinct=True)
    pl = oracle.plan(K, E, R)
    Xf = rng.standard_normal((T, H)).astype(np.float32)
    X = bf16(Xf)
    window = oracle.dispatch(X, pl.row_map, pl.window_rows)

    # (i) identity expert, one-hot weight in slot j -> Y == X exactly, for every j
    for j in range(k):
        W = np.zeros((T, k), np.float32)
        W[:, j] = 1.0
        assert np.array_equal(oracle.combine(window, W, pl.row_map), X)
    # (ii) identity expert, weights 1/k with k a power of two -> exact
    W = np.full((T, k), 1.0 / k, np.float32)
    assert np.array_equal(oracle.combine(window, W, pl.row_map), X)
    # (iii) identity expert, softmax weights -> within 1 bf16 ulp of X
    lg = rng.standard_normal((T, k))
    W = (np.exp(lg) / np.exp(lg).sum(1, keepdims=True)).astype(np.float32)
    assert ulp_dist(oracle.combine(window, W, pl.row_map), X).max() <= 1
    # (iv) slot-dependent weights and expert-dependent rows: a transposed or shifted index shows up
    scale = np.arange(1, E + 1, dtype=np.float32)
    Yexp = oracle.expert_standin(window, K, pl.row_map, scale)
    closed = unbf16(X).astype(np.float64) * (W.astype(np.float64) * (K + 1)).sum(1, keepdims=True)
    ref = _einsum_reference(unbf16(Yexp).astype(np.float64), W, pl.row_map)
    Y32 = oracle.combine(Yexp, W, pl.row_map)
    Y64 = oracle.combine_f64(Yexp, W, pl.row_map)
    assert np.array_equal(Y64, oracle.f64_to_bf16(ref))          # fp64 path == library einsum, same rounding
    assert ulp_dist(Y32, Y64).max() <= 1                          # fp32 path within 1 ulp of the exact sum
    # Yexp rows were rounded to bf16 (rel. 2^-9 each) before the sum; Y is rounded once more
    assert np.allclose(unbf16(Y32), closed, rtol=3 * 2.0 ** -8, atol=1e-30)
    # (v) fp32 storage: fmaf chain bounded by k roundings of 2^-24 relative to the sum of magnitudes
    Xw = oracle.dispatch(Xf, pl.row_map, pl.window_rows)
    Ye = oracle.expert_standin(Xw, K, pl.row_map, scale)
    Yf = oracle.combine(Ye, W, pl.row_map)
    reff = _einsum_reference(Ye.astype(np.float64), W, pl.row_map)
    mag = _einsum_reference(np.abs(Ye).astype(np.float64), np.abs(W), pl.row_map)
    assert np.all(np.abs(Yf - reff) <= k * 2.0 ** -24 * mag + 1e-45)
    assert np.array_equal(oracle.combine_f64(Ye, W, pl.row_map), reff.astype(np.float32))
    # (vi) masked slots contribute nothing
    Km = K.copy()
    Km[::3, 1] = -1
    plm = oracle.plan(Km, E, R)
    wm = oracle.dispatch(X, plm.row_map, plm.window_rows)
    Yem = oracle.expert_standin(wm, Km, plm.row_map, scale)
    refm = _einsum_reference(unbf16(Yem).astype(np.float64), W, plm.row_map)
    assert np.array_equal(oracle.combine_f64(Yem, W, plm.row_map), oracle.f64_to_bf16(refm))
    assert ulp_dist(oracle.combine(Yem, W, plm.row_map), oracle.f64_to_bf16(refm)).max() <= 1


def check_accumulation_order():
    """fp32, ascending j, fused multiply-add, start at +0: a case where each of these matters.

    Values chosen so that the exact fp32 chain is known by hand:
      w = [1, 1, 1], y = [2^24, 1, -2^24]:  fl(fl(0+2^24)+1) = 2^24 (tie to even), then -2^24 -> 0;
      descending j gives 1 instead; fp64 gives 1.
      w = [-1, 1+2^-12], y = [1+2^-11, 1+2^-12] in fp32 storage: acc = -(1+2^-11) exactly, then the
      product (1+2^-12)^2 = 1+2^-11+2^-24 needs 25 bits; fused: (1+2^-11+2^-24) - (1+2^-11) = 2^-24
      exactly; an unfused multiply rounds the product to 1+2^-11 (tie to even) and the result is 0.
    """
    row_map = np.array([[0, 1, 2]], np.int32)
    Yexp = np.array([[2.0 ** 24], [1.0], [-2.0 ** 24]], np.float32)
    W = np.ones((1, 3), np.float32)
    assert oracle.combine(Yexp, W, row_map)[0, 0] == 0.0
    assert oracle.combine_f64(Yexp, W, row_map)[0, 0] == 1.0
    assert oracle.combine(Yexp[::-1].copy(), W, row_map)[0, 0] == 1.0
    a = np.float32(1 + 2.0 ** -12)
    Yexp = np.array([[np.float32(1 + 2.0 ** -11)], [a]], np.float32)
    W = np.array([[-1.0, a]], np.float32)
    assert oracle.combine(Yexp, W, np.array([[0, 1]], np.int32))[0, 0] == np.float32(2.0 ** -24)
    # all slots masked -> +0
    z = oracle.combine(Yexp, W, np.array([[-1, -1]], np.int32))
    assert z[0, 0] == 0.0 and not np.signbit(z[0, 0])


def check_rounding():
    """The oracle's fp32->bf16 and fp64->bf16 against torch's CPU conversion (independent code)."""
    import torch
    rng = np.random.default_rng(5)
    bits = rng.integers(0, 2 ** 32, size=200_000, dtype=np.uint64).astype(np.uint32)
    special = np.array([0x00000000, 0x80000000, 0x3F808000, 0x3F818000, 0x3F807FFF, 0x3F808001, 0x7F7FFFFF,
                        0x7F7F8000, 0x7F800000, 0xFF800000, 0x00000001, 0x00008000, 0x00018000, 0x007FFFFF,
                        0x0000FFFF, 0x33800000], np.uint32)
    f = np.concatenate([bits, special]).view(np.float32)
    finite = ~np.isnan(f)
    want = torch.from_numpy(f.copy()).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    got = oracle.f32_to_bf16(f)
    assert np.array_equal(got[finite], want[finite])
    nan = oracle.f32_to_bf16(f[~finite])
    assert np.all((nan & 0x7F80) == 0x7F80) and np.all(nan & 0x7F)
    # fp64 -> bf16 must agree with fp32 -> bf16 on values that are exactly fp32
    assert np.array_equal(oracle.f64_to_bf16(f[finite].astype(np.float64)), want[finite])
    # and must round once: 1 + 2^-8 + 2^-40 is above the tie, fp64->fp32->bf16 would round to even (down)
    d = np.array([1 + 2.0 ** -8 + 2.0 ** -40, 1 + 2.0 ** -8, 1 + 3 * 2.0 ** -8, -(1 + 2.0 ** -8 + 2.0 ** -40),
                  2.0 ** -133 * 2.5, 2.0 ** -133 * 2.5000001, 3.4e38, (2 - 2.0 ** -8) * 2.0 ** 127], np.float64)
    assert oracle.f64_to_bf16(d).tolist() == [0x3F81, 0x3F80, 0x3F82, 0xBF81, 0x0002, 0x0003, 0x7F80, 0x7F80]


def check_golden_multi():
    g = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "worked_example.json")))
    E, R = g["E"], g["R"]
    X = bf16(g["X"])
    K = np.asarray(g["K"], np.int32)
    W = np.asarray(g["W"], np.float32)
    scale = np.asarray(g["scale"], np.float32)
    for case in ("multi_source", "multi_source_stride_8"):
        c = g[case]
        pl = oracle.plan_multi(K, np.asarray(c["M"], np.int32), c["me"], E, R, c.get("stride", 0))
        for key in ("c_exp", "c_rank", "expert_offset", "region_base", "row_map", "o_all", "recv_count",
                    "recv_offset"):
            assert getattr(pl, key).tolist() == c[key], (case, key)
        assert pl.status.tolist() == c["status"] + [0], case
        window = oracle.dispatch(X, pl.row_map, pl.window_rows)
        Yexp = oracle.expert_standin(window, K, pl.row_map, scale)
        assert np.array_equal(unbf16(oracle.combine(Yexp, W, pl.row_map)), np.asarray(c["Y"], np.float32)), case


def check_multi_against_library(seed=6):
    rng = np.random.default_rng(seed)
    for T, k, E, R in ((40, 3, 12, 4), (64, 8, 32, 8), (7, 2, 6, 1), (30, 4, 8, 8)):
        Er = E // R
        K = wl.random_routing(rng, T, k, E, p_masked=0.1)
        M = rng.integers(0, 9, size=(R, E)).astype(np.int32)
        single = oracle.plan(K, E, R)
        for me in sorted({0, R // 2, R - 1}):
            pl = oracle.plan_multi(K, M, me, E, R)
            full = M.copy()
            full[me] = single.c_exp                          # own row replaced by the computed counts
            assert np.array_equal(pl.c_exp, single.c_exp) and np.array_equal(pl.s, single.s)
            assert np.array_equal(pl.recv_count, full.sum(0))
            assert np.array_equal(pl.recv_offset, np.concatenate([[0], np.cumsum(full.sum(0))]))
            # sub-blocks in (expert, source) order tile the window: exclusive cumsum of the transposed matrix
            assert np.array_equal(pl.o_all.reshape(-1), np.concatenate([[0], np.cumsum(full.T.reshape(-1))])[:-1])
            assert np.array_equal(pl.expert_offset[:E], pl.o_all[:, me])
            assert pl.expert_offset[E] == full.sum() == pl.region_base[R] == pl.window_rows
            assert np.array_equal(pl.region_base[:R], pl.recv_offset[:E:Er])
            flat = K.reshape(-1)
            valid = flat >= 0
            want = np.where(valid, pl.expert_offset[np.where(valid, flat, 0)] + pl.s.reshape(-1), -1)
            assert np.array_equal(pl.row_map.reshape(-1), want)
            # our rows lie inside our own sub-blocks, each used once
            rows = pl.row_map.reshape(-1)[valid]
            assert len(np.unique(rows)) == len(rows)
            lo = pl.o_all[flat[valid], me]
            assert np.all((rows >= lo) & (rows < lo + single.c_exp[flat[valid]]))
        # no traffic from the other sources: identical to the single-source plan
        z = oracle.plan_multi(K, np.zeros((R, E), np.int32), R - 1, E, R)
        for key in ("c_exp", "c_rank", "expert_offset", "region_base", "s", "row_map", "status"):
            assert np.array_equal(getattr(z, key), getattr(single, key)), key
        assert np.array_equal(z.recv_count, single.c_exp) and np.array_equal(z.recv_offset, single.expert_offset)
        # fixed stride: regions start at d*stride; our dropped branches are those at or past the region's end
        stride = int(full.reshape(R, R, Er).sum(axis=(0, 2)).max()) - 2 if R > 1 else int(full.sum()) - 2
        pf = oracle.plan_multi(K, M, 0, E, R, stride)
        assert np.array_equal(pf.region_base, np.arange(R + 1) * stride)
        full0 = M.copy()
        full0[0] = single.c_exp
        start = np.arange(E) // Er * stride + (np.concatenate([[0], np.cumsum(full0.sum(0))])[:-1]
                                               - np.repeat(np.concatenate([[0], np.cumsum(full0.sum(0))])[:-1][::Er], Er))
        assert np.array_equal(pf.recv_offset[:E], start)
        wantf = np.where(valid, pf.expert_offset[np.where(valid, flat, 0)] + pf.s.reshape(-1), -1)
        dropped = valid & (wantf >= (np.where(valid, flat, 0) // Er + 1) * stride)
        assert np.array_equal(pf.row_map.reshape(-1), np.where(dropped, -1, wantf)) and pf.status[1] == dropped.sum()


def check_row_total_limit(seed=8):
    """Rows are int32.  Blocks of all sources that together hold 2^31 rows or more cannot be laid out:
    status[2] = 1 and nothing is placed; one row fewer is an ordinary plan whose last block ends at 2^31 - 1."""
    rng = np.random.default_rng(seed)
    T, k, E, R = 9, 3, 8, 4
    K = wl.random_routing(rng, T, k, E, p_masked=0.1, p_invalid=0.1)
    single = oracle.plan(K, E, R)
    own = int(single.c_exp.sum())
    for me in (0, 2):
        for excess in (-1, 0, 5, 2 ** 32 + 7):                  # total rows = 2^31 + excess
            M = np.zeros((R, E), np.int64)
            M[me] = 77                                           # own row of M is ignored
            others = 2 ** 31 + excess - own
            rows = [r for r in range(R) if r != me]
            per = others // (len(rows) * E)
            assert per < 2 ** 31
            for r in rows:
                M[r] = per
            M[rows[0], E - 1] += others - per * len(rows) * E
            assert M[rows[0], E - 1] < 2 ** 31
            pl = oracle.plan_multi(K, M.astype(np.int32), me, E, R)
            assert np.array_equal(pl.c_exp, single.c_exp) and np.array_equal(pl.c_rank, single.c_rank)
            assert np.array_equal(pl.s, single.s)
            if excess >= 0:
                assert pl.status.tolist() == [int(single.status[0]), 0, 1], (me, excess)
                assert np.all(pl.row_map == -1)
            else:
                assert pl.status.tolist() == [int(single.status[0]), 0, 0]
                full = M.copy()
                full[me] = single.c_exp
                assert pl.expert_offset[E] == 2 ** 31 - 1 == full.sum()
                assert np.array_equal(pl.recv_offset.astype(np.int64), np.concatenate([[0], np.cumsum(full.sum(0))]))
                placed = pl.row_map.reshape(-1)[pl.s.reshape(-1) >= 0]
                assert placed.min() >= 0 and len(np.unique(placed)) == own


def check_quantised(seed=7):
    """Row-wise quantised dispatch: hand-worked codes, torch's float8_e4m3fn conversion as the library step,
    exact scales, and the dequantisation error bound of the format."""
    import torch
    g = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "worked_example.json")))
    X = bf16(g["X"])
    pl = oracle.plan(np.asarray(g["K"], np.int32), g["E"], g["R"])
    wq, ws = oracle.dispatch_quant(X, pl.row_map, pl.window_rows)
    tok = np.asarray(g["tight"]["window_token"])
    assert wq.tolist() == np.asarray(g["quantised"]["q_token"])[tok].tolist()
    want_scale = (np.asarray(g["quantised"]["scale_numerator"], np.float32) / np.float32(448))[tok]
    assert np.array_equal(ws, want_scale)
    # conversion against an independent implementation, including ties, subnormals and saturation
    rng = np.random.default_rng(seed)
    f = np.concatenate([rng.uniform(-448, 448, 100000), rng.uniform(-0.05, 0.05, 20000),
                        [0.0, -0.0, 448.0, -448.0, 2 ** -9, 2 ** -10, 1.5 * 2 ** -9, 2.5 * 2 ** -9, 2 ** -6, 336.0, 352.0,
                         17.0, 19.0, 447.99997]]).astype(np.float32)
    want = torch.from_numpy(f).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    assert np.array_equal(oracle.f32_to_e4m3(f), want)
    assert oracle.f32_to_e4m3(np.array([1e9, -1e9, np.inf, 448.00003], np.float32)).tolist() == [0x7E, 0xFE, 0x7E, 0x7E]
    # a random batch: same arithmetic spelled with numpy fp32 ops and torch's conversion
    T, H, k, E, R = 19, 48, 3, 6, 3
    Xf = (rng.standard_normal((T, H)) * np.exp(rng.uniform(-3, 3, (T, 1)))).astype(np.float32)
    Xf[5] = 0.0                                                   # an all-zero row: scale 1, codes 0
    Xb = bf16(Xf)
    x = unbf16(Xb)
    K = wl.random_routing(rng, T, k, E, p_masked=0.1)
    pl = oracle.plan(K, E, R)
    wq, ws = oracle.dispatch_quant(Xb, pl.row_map, pl.window_rows + 2, fill=0xAA)
    amax = np.abs(x).max(axis=1)
    scale = np.where(amax == 0, np.float32(1), amax / np.float32(448)).astype(np.float32)
    inv = np.where(amax == 0, np.float32(1), np.float32(448) / np.where(amax == 0, 1, amax)).astype(np.float32)
    q = torch.from_numpy((x * inv[:, None]).astype(np.float32)).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    q = np.where(np.abs(x * inv[:, None]) >= 448, np.where(x < 0, 0xFE, 0x7E), q).astype(np.uint8)   # saturate, not NaN
    for i, p in enumerate(pl.row_map.reshape(-1)):
        if p >= 0:
            assert np.array_equal(wq[p], q[i // k]) and ws[p] == scale[i // k]
    untouched = np.setdiff1d(np.arange(wq.shape[0]), pl.row_map.reshape(-1))
    assert np.all(wq[untouched] == 0xAA) and np.all(ws[untouched] == -1.0)
    deq = torch.from_numpy(wq[:pl.window_rows]).view(torch.float8_e4m3fn).float().numpy() * ws[:pl.window_rows, None]
    src = np.empty(pl.window_rows, np.int64)
    for i, p in enumerate(pl.row_map.reshape(-1)):
        if p >= 0:
            src[p] = i // k
    # half a unit in the last place of the top binade (16 of 448) plus the roundings of scale and inv
    assert np.all(np.abs(deq - x[src]) <= amax[src][:, None] * (16.0 / 448 + 1e-6))


PINS = [check_golden, check_golden_multi, check_row_total_limit, check_quantised, check_multi_against_library, check_plan_against_library, check_masked_and_invalid, check_fixed_stride, check_dispatch,
        check_combine, check_accumulation_order, check_rounding]


@pytest.mark.parametrize("check", PINS, ids=lambda f: f.__name__)
def test_pin(check):
    check()


# --------------------------------------------------------------------------- properties on random tiny shapes

@settings(max_examples=60, deadline=None)
@given(st.integers(0, 12), st.integers(1, 5), st.integers(1, 4), st.integers(1, 4), st.integers(0, 2 ** 31 - 1))
def test_plan_properties(T, k, Er, R, seed):
    E = Er * R
    rng = np.random.default_rng(seed)
    K = wl.random_routing(rng, T, k, E, p_masked=0.15, p_invalid=0.05)
    pl = oracle.plan(K, E, R)
    flat = K.reshape(-1)
    valid = (flat >= 0) & (flat < E)
    assert pl.c_exp.sum() == valid.sum() == pl.c_rank.sum() == pl.expert_offset[E] == pl.region_base[R]
    assert np.array_equal(pl.s, brute_s(K, E))
    placed = pl.row_map.reshape(-1)[valid]
    assert np.array_equal(np.sort(placed), np.arange(valid.sum()))       # every branch placed exactly once
    assert np.all(pl.row_map.reshape(-1)[~valid] == -1)
    H = 8
    X = rng.integers(0, 2 ** 16, size=(T, H)).astype(np.uint16)
    window = oracle.dispatch(X, pl.row_map, pl.window_rows)
    for i in np.flatnonzero(valid):
        assert np.array_equal(window[pl.row_map.reshape(-1)[i]], X[i // k])


def test_identity_expert_restores_input_tiny_config():
    """The tiny configuration: weights sum to 1, identity expert -> Y is X up to the last bit of fp32 sums."""
    w = wl.make(wl.CONFIGS["tiny"])
    cfg = w.cfg
    pl = oracle.plan(w.K, cfg.E, cfg.R)
    assert pl.c_exp.sum() == cfg.T * cfg.k
    window = oracle.dispatch(w.X, pl.row_map, pl.window_rows)
    Y = oracle.combine(window, w.W, pl.row_map)
    assert np.allclose(Y, w.X, rtol=4 * 2.0 ** -24, atol=0)
    # closed form with the index-scaled stand-in: Y_t = X_t * sum_j W_tj (K_tj + 1)
    _, _, _, Y2 = oracle.layer(w.X, w.K, w.W, w.scale, cfg.E, cfg.R)
    closed = w.X.astype(np.float64) * (w.W.astype(np.float64) * (w.K + 1)).sum(1, keepdims=True)
    assert np.allclose(Y2, closed, rtol=4 * 2.0 ** -24, atol=0)


def test_bad_shapes_rejected():
    K = np.zeros((2, 2), np.int32)
    for E, R in ((7, 2), (0, 1), (4, 0)):
        with pytest.raises(ValueError):
            oracle.plan(K, E, R)


# --------------------------------------------------------------------------- mutants

MUTANTS = {
    "s_counts_inclusive": ("s[i] = c_exp[e];\n      c_exp[e] += 1;", "c_exp[e] += 1;\n      s[i] = c_exp[e];"),
    "s_not_stable": ("s[i] = c_exp[e];\n      c_exp[e] += 1;", "c_exp[e] += 1;\n      s[i] = -2 - e;"),   # fixed up below
    "rank_is_mod": ("region_base[e / Er + 1]", "region_base[e % R + 1]"),
    "rank_count_shifted": ("for (int32_t e = r * Er; e < (r + 1) * Er; ++e) acc += c_exp[e];",
                           "for (int32_t e = r * Er + 1; e < (r + 1) * Er + 1 && e < E; ++e) acc += c_exp[e];"),
    "offset_inclusive": ("expert_offset[e] = run;\n      run += c_exp[e];", "run += c_exp[e];\n      expert_offset[e] = run;"),
    "invalid_counted": ("if (e < 0 || e >= E) { status[0] += 1; s[i] = -1; continue; }",
                        "if (e < 0 || e >= E) { s[i] = -1; continue; }"),
    "dispatch_wrong_source": ("(const char *)X + (size_t)t * row_bytes, row_bytes);",
                              "(const char *)X + (size_t)(t ^ (j & 1)) * row_bytes % ((size_t)T * row_bytes), row_bytes);"),
    "combine_weight_transposed": ("acc = fmaf(W[(int64_t)t * k + j], y, acc);",
                                  "acc = fmaf(W[(int64_t)t * k + (k - 1 - j)], y, acc);"),
    "combine_descending": ("      for (int32_t j = 0; j < k; ++j) {\n        const int32_t q = row_map[(int64_t)t * k + j];\n        if (q < 0) continue;\n        const size_t idx = (size_t)q * (size_t)H + (size_t)h;\n        const float y",
                           "      for (int32_t j = k - 1; j >= 0; --j) {\n        const int32_t q = row_map[(int64_t)t * k + j];\n        if (q < 0) continue;\n        const size_t idx = (size_t)q * (size_t)H + (size_t)h;\n        const float y"),
    "combine_unfused": ("acc = fmaf(W[(int64_t)t * k + j], y, acc);",
                        "{ volatile float pr = W[(int64_t)t * k + j] * y; acc = acc + pr; }"),
    "combine_drops_last": ("      float acc = 0.0f;\n      for (int32_t j = 0; j < k; ++j) {",
                           "      float acc = 0.0f;\n      for (int32_t j = 0; j < k - (k > 2); ++j) {"),
    "bf16_truncates": ("u += 0x7FFFu + lsb;", "u += 0u * lsb;"),
    "bf16_half_up": ("u += 0x7FFFu + lsb;", "u += 0x8000u + 0u * lsb;"),
    "f64_double_rounds": ("    uint64_t u;\n    memcpy(&u, &a, 8);\n    const uint64_t lsb = (u >> 45) & 1ull;\n    u += ((1ull << 44) - 1ull) + lsb;\n    u &= ~((1ull << 45) - 1ull);\n    memcpy(&r, &u, 8);",
                          "    r = (double)bf16_to_f32(f32_to_bf16_rne((float)a));"),
    "stride_keeps_overflow": ("if (region_stride_rows > 0 && row >= region_base[e / Er + 1]) {",
                              "if (region_stride_rows > 0 && row > region_base[e / Er + 1]) {"),
}
MUTANTS["row_total_limit_off_by_one"] = ("if (all_rows >= 2147483648LL) {", "if (all_rows > 2147483648LL) {")
MUTANTS["row_total_in_int32"] = ("  int64_t all_rows = 0;", "  int32_t all_rows = 0;")
MUTANTS["multi_own_row_not_replaced"] = ("const int32_t m = r == me ? c_exp[e] : M[(int64_t)r * E + e];",
                                         "const int32_t m = M[(int64_t)r * E + e];")
MUTANTS["multi_sources_reversed"] = ("      for (int32_t r = 0; r < R; ++r) {\n        const int32_t m = r == me",
                                     "      for (int32_t r = R - 1; r >= 0; --r) {\n        const int32_t m = r == me")
MUTANTS["multi_offset_is_block_start"] = ("expert_offset[e] = o_all[(int64_t)e * R + me];", "expert_offset[e] = recv_offset[e];")
MUTANTS["multi_stride_ignored"] = ("    if (region_stride_rows > 0) run = (int32_t)((int64_t)d * region_stride_rows);\n    region_base[d] = run;",
                                   "    region_base[d] = run;")
MUTANTS["quant_truncates"] = ("  v += 0x7FFFFu + lsb;\n  v >>= 20;", "  v += 0u * lsb;\n  v >>= 20;")
MUTANTS["quant_half_up"] = ("  v += 0x7FFFFu + lsb;\n  v >>= 20;", "  v += 0x80000u + 0u * lsb;\n  v >>= 20;")
MUTANTS["quant_scale_is_inverse"] = ("      window_scale[p] = scale;", "      window_scale[p] = inv;")
MUTANTS["quant_amax_signed"] = ("amax = fmaxf(amax, fabsf(bf16_to_f32(x[h])));", "amax = fmaxf(amax, bf16_to_f32(x[h]));")
MUTANTS["quant_bias_off_by_one"] = ("const uint32_t code = v - ((127u - 7u) << 3);", "const uint32_t code = v - ((127u - 8u) << 3);")
# an unstable but otherwise valid placement: reverse order inside each expert block
MUTANTS["s_not_stable"] = ("    row_map[i] = row;\n", "    row_map[i] = expert_offset[e] + (c_exp[e] - 1 - s[i]);\n")


@pytest.mark.parametrize("name", sorted(MUTANTS))
def test_pins_catch_mutant(name, tmp_path):
    src = open(os.path.join(os.path.dirname(oracle.__file__), "moe_oracle.c")).read()
    old, new = MUTANTS[name]
    assert src.count(old) >= 1, f"mutation site for {name} not found in the oracle source"
    mutated = src.replace(old, new, 1)
    c = tmp_path / "mutant.c"
    so = tmp_path / "mutant.so"
    c.write_text(mutated)
    subprocess.check_call(["gcc", "-O2", "-mfma", "-ffp-contract=off", "-shared", "-fPIC", "-o", str(so), str(c), "-lm"])
    # A mutant may scribble over memory, so it runs in a child process; the first failing pin
    # ends the child before later checks can touch bad row maps.
    child = (
        "import ctypes, sys\n"
        f"sys.path.insert(0, {os.path.dirname(os.path.dirname(os.path.abspath(__file__)))!r})\n"
        f"sys.path.insert(0, {os.path.dirname(os.path.abspath(__file__))!r})\n"
        "import oracle, test_oracle_pins as pins\n"
        f"oracle._lib = ctypes.CDLL({str(so)!r})\n"
        "for check in pins.PINS:\n"
        "    try:\n"
        "        check()\n"
        "    except AssertionError:\n"
        "        print('caught by', check.__name__); sys.exit(0)\n"
        "sys.exit(3)\n"
    )
    res = subprocess.run([sys.executable, "-c", child], capture_output=True, text=True, timeout=300)
    assert res.returncode != 3, f"no pin notices the planted mistake '{name}'"
    assert res.returncode == 0, f"mutant '{name}' crashed the checker instead of failing a pin:\n{res.stderr[-2000:]}"


def test_all_cores_build_gives_the_serial_results():
    """The benchmark's all-cores baseline is the same source with the token loops of dispatch and combine
    split over threads: it must reproduce the serial build bit for bit."""
    cfg = wl.CONFIGS["tiny"].with_(T=300, H=256, E=16, R=4, k=4)
    w = wl.make(cfg, seed=5)
    pl = oracle.plan(w.K, cfg.E, cfg.R)
    window = oracle.dispatch(w.X, pl.row_map, pl.window_rows)
    y = oracle.combine(window, w.W, pl.row_map)
    assert oracle.threads() == 1
    with oracle.all_cores():
        assert oracle.threads() >= 1
        pl2 = oracle.plan(w.K, cfg.E, cfg.R)
        window2 = oracle.dispatch(w.X, pl2.row_map, pl2.window_rows)
        y2 = oracle.combine(window2, w.W, pl2.row_map)
    assert oracle.threads() == 1
    assert np.array_equal(pl.row_map, pl2.row_map)
    assert np.array_equal(window, window2) and np.array_equal(y, y2)
