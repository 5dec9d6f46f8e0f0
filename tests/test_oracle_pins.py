"""Pins for the CPU oracle: each routine is checked against something other than itself --
a closed form, a value the paper prints, an invariant the paper states, a library routine, or
brute force written with different tools (numpy in float64 on decoded vectors)."""
import os

import numpy as np
import pytest
import scipy.cluster.vq

import synth
from helpers import (brute_force_sqdist, check_topk, codebooks_from_rows, decode_np, lex_topk, t2n)

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


@pytest.fixture(scope="module")
def small(oracle_lib):
    """N=3000, D=32, M=8 index on Gaussian data with data-row code books and 24 coarse codes."""
    D, M, N, K = 32, 8, 3000, 24
    x = t2n(synth.gaussian(11, 0, N, D))
    cb = codebooks_from_rows(x, M)
    codes = oracle_lib.encode(cb, x)
    coarse = codes[t2n(synth.sample_rows(5, N, K))].copy()
    T = oracle_lib.sym_table(cb)
    a = oracle_lib.assign(T, codes, coarse)
    off, lids = oracle_lib.build_lists(a, K)
    q = t2n(synth.gaussian(12, 0, 16, D))
    return dict(D=D, M=M, N=N, K=K, x=x, cb=cb, codes=codes, coarse=coarse, T=T, a=a, off=off, lids=lids, q=q)


# ---------------------------------------------------------------- worked example (closed form)
def test_hand_example(oracle_lib):
    """D=2, M=2, Z=2.  Code books {0,1} and {0,10}; q=(0.25, 7).  By hand (Sec. 3):
    A = [[0.0625, 0.5625], [49, 9]]; codes (0,0),(1,1),(0,1),(1,0) -> 49.0625, 9.5625, 9.0625, 49.5625."""
    cb = np.array([[[0.0], [1.0]], [[0.0], [10.0]]], dtype=np.float32)
    q = np.array([[0.25, 7.0]], dtype=np.float32)
    A = oracle_lib.lut(cb, q)[0]
    assert A.tolist() == [[0.0625, 0.5625], [49.0, 9.0]]
    codes = np.array([[0, 0], [1, 1], [0, 1], [1, 0]], dtype=np.uint8)
    assert oracle_lib.adc(A, codes).tolist() == [49.0625, 9.5625, 9.0625, 49.5625]
    ids, dist = oracle_lib.linear_scan(A, codes, 3)
    assert ids.tolist() == [2, 1, 0] and dist.tolist() == [9.0625, 9.5625, 49.0625]
    # subset {0, 3}: only members may be returned, padded beyond |S| (Sec. 4, Eq. (3))
    ids, dist = oracle_lib.linear_scan(A, codes, 3, S=np.array([0, 3]))
    assert ids.tolist() == [0, 3, -1] and dist[:2].tolist() == [49.0625, 49.5625] and np.isinf(dist[2])
    # encode of the points themselves (Eq. (1)); (0.5, 5) is equidistant twice -> lowest index
    x = np.array([[0.9, 9.0], [0.1, 1.0], [0.5, 5.0]], dtype=np.float32)
    assert oracle_lib.encode(cb, x).tolist() == [[1, 1], [0, 0], [0, 0]]


def test_hand_example_inverted_index(oracle_lib):
    """Same tables.  Two coarse codes (0,1) and (1,0): d0 = 9.0625 and 49.5625, so list 0 is
    visited first.  Lists W_0 = {1, 2, 4}, W_1 = {0, 3}.  Alg. 2 with one list sees only W_0;
    with a cap of L=2 candidates it scores ids 1 and 2 only (stored order), never id 4."""
    cb = np.array([[[0.0], [1.0]], [[0.0], [10.0]]], dtype=np.float32)
    A = oracle_lib.lut(cb, np.array([[0.25, 7.0]], dtype=np.float32))[0]
    codes = np.array([[0, 0], [1, 1], [0, 1], [1, 0], [0, 1]], dtype=np.uint8)
    coarse = np.array([[0, 1], [1, 0]], dtype=np.uint8)
    off = np.array([0, 3, 5], dtype=np.int64)
    lids = np.array([1, 2, 4, 0, 3], dtype=np.int32)
    ks, d0 = oracle_lib.coarse_rank(A, coarse, 2)
    assert ks.tolist() == [0, 1] and d0.tolist() == [9.0625, 49.5625]
    ids, dist, scored = oracle_lib.inverted_index(A, codes, coarse, off, lids, R=3, P=1)
    assert ids.tolist() == [2, 4, 1] and dist.tolist() == [9.0625, 9.0625, 9.5625] and scored == 3
    ids, dist, scored = oracle_lib.inverted_index(A, codes, coarse, off, lids, R=3, P=1, Lcap=2)
    assert ids.tolist() == [2, 1, -1] and scored == 2
    ids, dist, scored = oracle_lib.inverted_index(A, codes, coarse, off, lids, R=5, P=2)
    assert ids.tolist() == [2, 4, 1, 0, 3] and scored == 5
    # target identifiers {0, 4}: list 0 contributes 4 only, list 1 contributes 0
    ids, dist, scored = oracle_lib.inverted_index(A, codes, coarse, off, lids, R=2, P=2, S=np.array([0, 4]))
    assert ids.tolist() == [4, 0] and scored == 2
    ids, dist, scored = oracle_lib.inverted_index(A, codes, coarse, off, lids, R=2, P=1, S=np.array([0, 4]))
    assert ids.tolist() == [4, -1] and scored == 1


# ---------------------------------------------------------------- encode (Eq. 1)
def test_encode_matches_library_vq(small, oracle_lib):
    """Per sub-space Eq. (1) is textbook nearest-centroid: scipy's vq on the slices agrees."""
    M, D = small["M"], small["D"]
    Ds = D // M
    for m in range(M):
        ref, _ = scipy.cluster.vq.vq(small["x"][:, m * Ds:(m + 1) * Ds].astype(np.float64),
                                     small["cb"][m].astype(np.float64))
        got = small["codes"][:, m]
        diff = np.nonzero(ref != got)[0]
        # fp32 vs fp64 may only differ at a near tie
        for n in diff:
            xm = small["x"][n, m * Ds:(m + 1) * Ds].astype(np.float64)
            d = ((small["cb"][m].astype(np.float64) - xm) ** 2).sum(1)
            assert abs(d[ref[n]] - d[got[n]]) <= 1e-6 * d[ref[n]]
        assert len(diff) <= 2


def test_encode_fixed_point_and_tiebreak(small, oracle_lib):
    """Encoding a decoded vector gives the code back; duplicated code words -> lowest index."""
    xhat = oracle_lib.decode(small["cb"], small["codes"][:200])
    assert np.array_equal(oracle_lib.encode(small["cb"], xhat), small["codes"][:200])
    cb = small["cb"].copy()
    cb[:, 200] = cb[:, 3]  # code word 200 duplicates code word 3
    codes = oracle_lib.encode(cb, small["x"][:500])
    assert not np.any(codes == 200)
    with pytest.raises(ValueError):
        oracle_lib.encode(small["cb"][:3], small["x"][:4])  # M=3 does not divide D=32


# ---------------------------------------------------------------- table and ADC (Sec. 3, Eq. 2)
def test_lut_against_float64_numpy(small, oracle_lib):
    cb, q, M = small["cb"], small["q"], small["M"]
    Ds = small["D"] // M
    A32 = oracle_lib.lut(cb, q)
    A64 = oracle_lib.lut(cb, q, f64=True)
    ref = np.stack([[((cb[m].astype(np.float64) - q[i, m * Ds:(m + 1) * Ds].astype(np.float64)) ** 2).sum(1)
                     for m in range(M)] for i in range(len(q))])
    np.testing.assert_allclose(A64, ref, rtol=1e-12)
    np.testing.assert_allclose(A32, ref, rtol=1e-6)
    # the smallest entry of row m sits at the code Eq. (1) gives the query itself
    assert np.array_equal(A32.argmin(axis=2), oracle_lib.encode(cb, q))


def test_adc_equals_distance_to_decoded_vector(small, oracle_lib):
    """Eq. (2) is exactly ||q - decode(code)||^2 because the sub-spaces are disjoint."""
    cb, codes = small["cb"], small["codes"]
    xhat = decode_np(cb, codes)
    for i in range(4):
        q = small["q"][i]
        ref = brute_force_sqdist(q, xhat)
        d32 = oracle_lib.adc(oracle_lib.lut(cb, q)[0], codes)
        d64 = oracle_lib.adc(oracle_lib.lut(cb, q, f64=True)[0], codes)
        np.testing.assert_allclose(d64, ref, rtol=1e-12)
        np.testing.assert_allclose(d32, ref, rtol=2e-6)
    # a query that is itself a decoded vector is at distance 0 from its own code
    q0 = oracle_lib.decode(cb, codes[17:18])[0]
    assert oracle_lib.adc(oracle_lib.lut(cb, q0)[0], codes)[17] == 0.0
    # gathered rows
    ids = np.array([5, 17, 2999], dtype=np.int32)
    A = oracle_lib.lut(cb, small["q"][0])[0]
    assert np.array_equal(oracle_lib.adc(A, codes, ids), oracle_lib.adc(A, codes)[ids])


# ---------------------------------------------------------------- Alg. 1
def test_linear_scan_against_exact_reconstruction(small, oracle_lib):
    cb, codes, N = small["cb"], small["codes"], small["N"]
    xhat = decode_np(cb, codes)
    all_ids = np.arange(N, dtype=np.int32)
    for i in range(6):
        q = small["q"][i]
        A = oracle_lib.lut(cb, q)[0]
        ids, dist = oracle_lib.linear_scan(A, codes, 50)
        ref_i, ref_d = lex_topk(brute_force_sqdist(q, xhat), all_ids, 50)
        check_topk(ids, dist, ref_i, ref_d.astype(np.float32), exact_ids=False,
                   dist_of_id=lambda s: brute_force_sqdist(q, xhat[s]))


def test_linear_scan_order_on_exact_ties(oracle_lib):
    """Identical codes have identical distances; the order is then by identifier."""
    rng = np.random.default_rng(0)
    cb = rng.normal(size=(4, 256, 2)).astype(np.float32)
    base = rng.integers(0, 256, size=(10, 4)).astype(np.uint8)
    codes = np.tile(base, (30, 1))  # every code appears 30 times
    A = oracle_lib.lut(cb, rng.normal(size=(1, 8)).astype(np.float32))[0]
    ids, dist = oracle_lib.linear_scan(A, codes, 45)
    assert np.all(np.diff(dist) >= 0)
    for v in np.unique(dist):
        run = ids[dist == v]
        assert np.all(np.diff(run) > 0)
    # the nearest code's 30 copies come first, ids = j, j+10, j+20, ...
    assert np.array_equal(ids[:30], ids[0] + 10 * np.arange(30))


def test_subset_scan(small, oracle_lib):
    """Results are members of S, equal filter-then-sort, and S = everything is the plain scan."""
    cb, codes, N = small["cb"], small["codes"], small["N"]
    xhat = decode_np(cb, codes)
    q = small["q"][3]
    A = oracle_lib.lut(cb, q)[0]
    for size in (1, 7, 100, 1500):
        S = t2n(synth.sorted_subset(3, size, N, size))
        ids, dist = oracle_lib.linear_scan(A, codes, 20, S=S)
        got = ids[ids >= 0]
        assert np.all(np.isin(got, S)) and len(got) == min(20, size)
        ref_i, ref_d = lex_topk(brute_force_sqdist(q, xhat[S]), S, 20)
        check_topk(ids, dist, ref_i, ref_d.astype(np.float32), exact_ids=False)
    full = oracle_lib.linear_scan(A, codes, 20)
    sub = oracle_lib.linear_scan(A, codes, 20, S=np.arange(N, dtype=np.int32))
    assert np.array_equal(full[0], sub[0]) and np.array_equal(full[1], sub[1])
    ids, dist = oracle_lib.linear_scan(A, codes, 5, S=np.zeros(0, dtype=np.int32))
    assert np.all(ids == -1) and np.all(np.isinf(dist))


# ---------------------------------------------------------------- lists (Sec. 4.1, Eq. 4)
def test_assignment_and_lists(small, oracle_lib):
    cb, codes, coarse, K, N = small["cb"], small["codes"], small["coarse"], small["K"], small["N"]
    # d_S between two PQ codes is the squared distance between their decoded vectors
    xhat, chat = decode_np(cb, codes), decode_np(cb, coarse)
    d = ((xhat[:, None, :] - chat[None, :, :]) ** 2).sum(2)
    ref = d.argmin(1)
    a = small["a"]
    for n in np.nonzero(ref != a)[0]:
        assert abs(d[n, ref[n]] - d[n, a[n]]) <= 1e-5 * d[n, ref[n]]
    assert (ref != a).sum() <= 3
    # symmetric table: zero diagonal, symmetric
    T = small["T"]
    assert np.all(T[:, np.arange(256), np.arange(256)] == 0) and np.array_equal(T, T.transpose(0, 2, 1))
    # a coarse code drawn from the database is its own nearest centre at distance 0
    rows = t2n(synth.sample_rows(5, N, K))
    dd = d[rows, a[rows]]
    assert np.all(dd == 0)
    # posting lists partition the identifiers, ascending inside each list
    off, lids = small["off"], small["lids"]
    assert off[0] == 0 and off[-1] == N and np.array_equal(np.sort(lids), np.arange(N))
    for k in range(K):
        w = lids[off[k]:off[k + 1]]
        assert np.all(a[w] == k) and np.all(np.diff(w) > 0)
    # duplicate coarse codes: ties go to the lower list number
    coarse2 = np.concatenate([coarse, coarse[:1]])
    a2 = oracle_lib.assign(T, codes, coarse2)
    assert not np.any(a2 == K)


# ---------------------------------------------------------------- Alg. 2
def test_coarse_rank_is_adc_over_coarse_codes(small, oracle_lib):
    A = oracle_lib.lut(small["cb"], small["q"][1])[0]
    d0_all = oracle_lib.adc(A, small["coarse"])
    ks, d0 = oracle_lib.coarse_rank(A, small["coarse"], 10)
    ref_k, ref_d = lex_topk(d0_all, np.arange(small["K"], dtype=np.int32), 10)
    assert np.array_equal(ks, ref_k) and np.array_equal(d0, ref_d)


def test_inverted_index_all_lists_equals_linear_scan(small, oracle_lib):
    """Looking at all K lists without a cap scores every item once: the plain scan (Sec. 4.2)."""
    s = small
    for i in range(4):
        A = oracle_lib.lut(s["cb"], s["q"][i])[0]
        ids, dist, scored = oracle_lib.inverted_index(A, s["codes"], s["coarse"], s["off"], s["lids"], R=30, P=s["K"])
        ref = oracle_lib.linear_scan(A, s["codes"], 30)
        assert scored == s["N"] and np.array_equal(ids, ref[0]) and np.array_equal(dist, ref[1])


def test_inverted_index_partial(small, oracle_lib):
    s = small
    xhat = decode_np(s["cb"], s["codes"])
    q = s["q"][2]
    A = oracle_lib.lut(s["cb"], q)[0]
    S = t2n(synth.sorted_subset(9, 0, s["N"], 900))
    prev_kth = np.inf
    for P in (1, 3, 8, s["K"]):
        ks, _ = oracle_lib.coarse_rank(A, s["coarse"], P)
        pool = np.concatenate([s["lids"][s["off"][k]:s["off"][k + 1]] for k in ks])
        ids, dist, scored = oracle_lib.inverted_index(A, s["codes"], s["coarse"], s["off"], s["lids"], R=10, P=P)
        assert scored == len(pool) and np.all(np.isin(ids[ids >= 0], pool))
        ref_i, ref_d = lex_topk(brute_force_sqdist(q, xhat[pool]), pool, 10)
        check_topk(ids, dist, ref_i, ref_d.astype(np.float32), exact_ids=False)
        assert dist[9] <= prev_kth  # more lists never make the 10th distance worse
        prev_kth = dist[9]
        # with target identifiers: brute force over (union of lists) ∩ S
        ids, dist, scored = oracle_lib.inverted_index(A, s["codes"], s["coarse"], s["off"], s["lids"], R=10, P=P, S=S)
        poolS = pool[np.isin(pool, S)]
        assert scored == len(poolS)
        ref_i, ref_d = lex_topk(brute_force_sqdist(q, xhat[poolS]), poolS, 10)
        check_topk(ids, dist, ref_i, ref_d.astype(np.float32), exact_ids=False)
        # candidate cap: exactly the first Lcap members of S in traversal order
        cap = 37
        ids, dist, scored = oracle_lib.inverted_index(A, s["codes"], s["coarse"], s["off"], s["lids"], R=10, P=P,
                                                      S=S, Lcap=cap)
        first = poolS[:cap]
        assert scored == len(first)
        ref_i, ref_d = lex_topk(brute_force_sqdist(q, xhat[first]), first, 10)
        check_topk(ids, dist, ref_i, ref_d.astype(np.float32), exact_ids=False)


def test_num_lists_formula(oracle_lib):
    """ceil(K L / |S|) capped at K; the default L = N/K on the whole database is one list."""
    assert oracle_lib.num_lists(1000, 1000, 10**6) == 1
    assert oracle_lib.num_lists(1000, 5000, 10**6) == 5
    assert oracle_lib.num_lists(1000, 1000, 10**6 - 1) == 2
    assert oracle_lib.num_lists(1000, 1000, 500) == 1000
    assert oracle_lib.num_lists(4096, 2441, 10**7) == 1
    assert oracle_lib.num_lists(16384, 6103 * 64, 10**8) == 64
    assert oracle_lib.num_lists(3, 10**9, 7) == 3  # no overflow in K*L


# ---------------------------------------------------------------- Alg. 3
def test_query_switch(small, oracle_lib):
    s = small
    q = s["q"][5]
    A = oracle_lib.lut(s["cb"], q)[0]
    theta, L, R = 200, 300, 10
    for size, want_mode in ((theta - 1, 0), (theta, 1), (theta + 50, 1), (5, 0)):
        S = t2n(synth.sorted_subset(21, size, s["N"], size))
        ids, dist, mode = oracle_lib.query(s["cb"], q, s["codes"], s["coarse"], s["off"], s["lids"], R, L, theta, S=S)
        assert mode == want_mode
        if mode == 0:
            ref = oracle_lib.linear_scan(A, s["codes"], R, S=S)
        else:
            P = oracle_lib.num_lists(s["K"], L, size)
            ref = oracle_lib.inverted_index(A, s["codes"], s["coarse"], s["off"], s["lids"], R, P, S=S, Lcap=L)[:2]
        assert np.array_equal(ids, ref[0]) and np.array_equal(dist, ref[1])
    # whole database: |S| = N >= theta -> inverted index with ceil(K L / N) lists
    ids, dist, mode = oracle_lib.query(s["cb"], q, s["codes"], s["coarse"], s["off"], s["lids"], R, L, theta)
    assert mode == 1
    P = oracle_lib.num_lists(s["K"], L, s["N"])
    ref = oracle_lib.inverted_index(A, s["codes"], s["coarse"], s["off"], s["lids"], R, P, Lcap=L)
    assert np.array_equal(ids, ref[0])


# ---------------------------------------------------------------- memory model (Sec. 4.1, Table 2)
def test_index_size_matches_paper_table(oracle_lib):
    """(N+K) M log2 Z + 32 N bits.  The paper prints the theoretical sizes (Sec. 5.4 text under
    Table 2): 68 MB for SIFT1M (M=64) and 244 MB for GIST1M (M=240), K=1000, N=10^6."""
    rows = [l.split() for l in open(os.path.join(GOLDEN, "index_size_table2.txt")) if l.strip() and l[0] != "#"]
    assert len(rows) == 2
    for name, N, K, M, theory_mb in rows:
        b = oracle_lib.index_bytes(int(N), int(K), int(M))
        assert b == (int(N) + int(K)) * int(M) + 4 * int(N)
        assert int(b / 1e6) == int(theory_mb), (name, b)


# ---------------------------------------------------------------- complexity (Table 1)
def test_oracle_cost_scales_with_subset_size(oracle_lib):
    """Alg. 1 costs O(M |S|): a 16x larger subset takes several times longer."""
    import time
    rng = np.random.default_rng(1)
    codes = rng.integers(0, 256, size=(400000, 16)).astype(np.uint8)
    A = rng.random((16, 256)).astype(np.float32)
    def t(size):
        S = np.sort(rng.choice(400000, size, replace=False)).astype(np.int32)
        best = 1e9
        for _ in range(3):
            t0 = time.perf_counter(); oracle_lib.linear_scan(A, codes, 10, S=S); best = min(best, time.perf_counter() - t0)
        return best
    assert t(320000) > 4 * t(20000)


# ---------------------------------------------------------------- rotation (Sec. 4.5)
def test_rotation(oracle_lib):
    """y = R x: identity leaves x alone; a permutation matrix permutes coordinates exactly; an
    orthogonal R preserves norms and distances (so PQ after rotating data and query alike is the
    method of Sec. 4.5); agrees with numpy's matmul in float64."""
    rng = np.random.default_rng(2)
    D = 24
    x = rng.normal(size=(50, D)).astype(np.float32)
    assert np.array_equal(oracle_lib.rotate(np.eye(D, dtype=np.float32), x), x)
    perm = rng.permutation(D)
    P = np.zeros((D, D), dtype=np.float32)
    P[np.arange(D), perm] = 1.0
    assert np.array_equal(oracle_lib.rotate(P, x), x[:, perm])
    Rm, _ = np.linalg.qr(rng.normal(size=(D, D)))
    y = oracle_lib.rotate(Rm.astype(np.float32), x)
    np.testing.assert_allclose(y, x.astype(np.float64) @ Rm.T, rtol=1e-5, atol=1e-5)
    np.testing.assert_allclose(np.linalg.norm(y, axis=1), np.linalg.norm(x, axis=1), rtol=1e-5)
    dx = ((x[:, None, :] - x[None, :, :]) ** 2).sum(2)
    dy = ((y[:, None, :] - y[None, :, :]) ** 2).sum(2)
    np.testing.assert_allclose(dy, dx, rtol=1e-4, atol=1e-4)
    # not symmetric in R: a transposed operand would fail here
    A = rng.normal(size=(D, D)).astype(np.float32)
    e0 = np.zeros((1, D), dtype=np.float32); e0[0, 0] = 1.0
    assert np.array_equal(oracle_lib.rotate(A, e0)[0], A[:, 0])
