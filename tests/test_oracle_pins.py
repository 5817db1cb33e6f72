"""Pins for the CPU oracle: each part is checked against something other than itself —
figures the paper prints, exact rational arithmetic, definitions written out on sets,
closed forms, invariants and brute force on tiny inputs."""
import heapq
import math
import os
from fractions import Fraction

import numpy as np
import pytest

import synth
from oracle import csv_oracle as O

GOLD = os.path.join(os.path.dirname(__file__), "golden", "paper_arithmetic.txt")


def _gold():
    out = {}
    for line in open(GOLD):
        if line.startswith("#") or not line.strip():
            continue
        name, val = line.split()[:2]
        out[name] = float(val)
    return out


def _agrees_to_three_digits(x, printed):
    """|x - printed| below one unit of the printed value's third significant digit
    (the paper's FLOP figure is twice its already-rounded multiply-add figure)."""
    unit = 10 ** (math.floor(math.log10(abs(printed))) - 2)
    return abs(x - printed) < unit


def _frac_bf16(bits):
    return Fraction(float(O.bf16_to_f64(np.array([bits], dtype=np.uint16))[0]))


def _small(seed=0, **kw):
    r = synth.small_recipe(**kw)
    head = synth.make_head(r, seed=seed, threads=1)
    h = synth.make_hidden(r, head["centers"], seed=seed)
    return r, head, h


# ------------------------------------------------------------------ printed arithmetic
def test_paper_head_flops_and_footprint():
    g = _gold()
    V, d = int(g["gpt3_vocab"]), int(g["gpt3_hidden"])
    assert O.head_flops(V, d) == 1_235_116_032
    assert _agrees_to_three_digits(O.head_flops(V, d), g["gpt3_flops_printed"])
    assert _agrees_to_three_digits(O.head_flops(V, d) // 2, g["gpt3_macs_printed"])
    assert O.head_flops(V, d) // 2 == 617_558_016
    C, dm = int(g["meta_clusters"]), int(g["meta_hidden"])
    assert O.metadata_bytes(1, dm) == int(g["meta_bytes_per_cluster"])
    assert O.metadata_bytes(C, dm) == 32_792_000
    assert _agrees_to_three_digits(O.metadata_bytes(C, dm) / 1e6, g["meta_total_mb_printed"])
    assert dm * 2 + 4 == int(g["allgather_bytes_per_row_d4096"])


# ------------------------------------------------------------------ full logits
def test_full_logits_exact_rational():
    rng = np.random.default_rng(1)
    V, d, B = 7, 24, 2
    Wb = synth.f32_to_bf16_bits(rng.standard_normal((V, d)).astype(np.float32))
    hb = synth.f32_to_bf16_bits(rng.standard_normal((B, d)).astype(np.float32) * 3)
    b = rng.standard_normal(V).astype(np.float32)
    got = O.full_logits(O.bf16_to_f64(Wb), b, O.bf16_to_f64(hb))
    assert got.shape == (B, V)
    for s in range(B):
        for i in range(V):
            exact = sum(_frac_bf16(Wb[i, j]) * _frac_bf16(hb[s, j]) for j in range(d)) + Fraction(float(b[i]))
            assert abs(got[s, i] - float(exact)) <= 1e-13 * max(1.0, abs(float(exact)))


def test_full_logits_linearity_and_operand_roles():
    rng = np.random.default_rng(2)
    W = rng.standard_normal((5, 3))
    b = rng.standard_normal(5)
    h = rng.standard_normal((2, 3))
    l1 = O.full_logits(W, b, h)
    l2 = O.full_logits(W, b, 4.0 * h)
    assert np.allclose(l2 - b, 4.0 * (l1 - b), rtol=0, atol=1e-12)
    # a unit hidden vector reads off a column of W: catches a transposed operand
    e = np.zeros((1, 3)); e[0, 1] = 1.0
    assert np.array_equal(O.full_logits(W, None, e)[0], W[:, 1])


def test_logsumexp_against_direct_sum_and_shift():
    x = np.array([0.3, -1.2, 2.5, 2.5, -7.0])
    assert math.isclose(O.logsumexp(x), math.log(sum(math.exp(v) for v in x)), rel_tol=1e-14)
    assert math.isclose(O.logsumexp(x + 1000.0), O.logsumexp(x) + 1000.0, rel_tol=1e-14)
    assert O.logsumexp(np.array([])) == -math.inf


# ------------------------------------------------------------------ brute-force top-k
@pytest.mark.parametrize("V", [1, 2, 17, 64])
def test_topk_three_ways(V):
    rng = np.random.default_rng(V)
    x = np.round(rng.standard_normal(V), 1)          # coarse values: ties are common
    for k in sorted({1, 2, V} & set(range(1, V + 1))):
        ids, vals = O.topk_bruteforce(x, k)
        # (a) repeated arg-max scan, smallest id on ties
        left = list(range(V)); scan = []
        for _ in range(k):
            best = left[0]
            for i in left[1:]:
                if x[i] > x[best]:
                    best = i
            scan.append(best); left.remove(best)
        # (b) heap selection on the composite key
        hp = [i for _, i in heapq.nsmallest(k, ((-x[i], i) for i in range(V)))]
        assert list(ids) == scan == hp
        assert np.array_equal(vals, x[ids])


# ------------------------------------------------------------------ index
def test_index_partition_radius_bias():
    r, head, _ = _small(seed=3)
    idx = O.build_index(head["W_bits"], head["b"], head["labels"], r.C, radius_slack=0.0)
    assert sorted(idx.perm.tolist()) == list(range(r.V))                 # a permutation
    assert idx.n.sum() == r.V and np.array_equal(idx.n, np.bincount(head["labels"], minlength=r.C))
    W = O.bf16_to_f64(head["W_bits"])
    for c in range(r.C):
        rows = idx.rows(c)
        assert np.all(head["labels"][rows] == c)                          # every row in its own cluster
        assert np.all(np.diff(rows) > 0)                                  # ascending ids inside
        assert np.allclose(idx.mu[c], W[rows].mean(0), rtol=1e-6, atol=1e-7)
        dist = np.sqrt(((W[rows] - idx.mu[c].astype(np.float64)) ** 2).sum(1))
        assert float(idx.R[c]) >= dist.max()                              # stored radius covers every member
        assert float(idx.R[c]) <= dist.max() * (1 + 2e-7)                 # and is the max, not something larger
        assert idx.bmax[c] == head["b"][rows].max()
    # the default slack only ever enlarges the radius
    idx2 = O.build_index(head["W_bits"], head["b"], head["labels"], r.C)
    assert np.all(idx2.R >= idx.R) and np.all(idx2.R <= idx.R * 1.001 + 1e-3)


def test_lloyd_recovers_planted_labels():
    r, head, _ = _small(seed=4, V=600, d=64, C=6)
    first = np.array([int(np.flatnonzero(head["labels"] == c)[0]) for c in range(r.C)])
    labels, cent = O.lloyd_kmeans(head["W_bits"], first, iters=3)
    assert np.array_equal(labels, head["labels"])
    idx = O.build_index(head["W_bits"], head["b"], labels, r.C)
    assert np.allclose(cent, idx.mu, atol=1e-6)


def test_lloyd_assign_is_nearest_centroid_with_ties():
    W = np.array([[0.0, 0.0], [1.0, 0.0], [0.5, 0.0], [3.0, 4.0]])
    cent = np.array([[0.0, 0.0], [1.0, 0.0], [3.0, 3.0]])
    assert O.lloyd_assign(W, cent).tolist() == [0, 1, 0, 2]               # [0.5,0] ties -> smaller id


# ------------------------------------------------------------------ bounds
@pytest.mark.parametrize("slack", [0.0, 2.0 ** -14])
def test_bound_dominates_every_logit(slack):
    r, head, h = _small(seed=5, steps=6)
    idx = O.build_index(head["W_bits"], head["b"], head["labels"], r.C, radius_slack=slack)
    W = O.bf16_to_f64(head["W_bits"])
    for t in range(h.shape[0]):
        h64 = O.bf16_to_f64(h[t])
        L = O.full_logits(W, head["b"], h64)
        U, hn = O.cluster_bounds(idx, h64)
        assert np.allclose(hn, np.linalg.norm(h64, axis=1))
        assert np.all(L <= U[:, head["labels"]] + 1e-12)                  # Cauchy-Schwarz invariant


def test_bound_homogeneity_and_special_cases():
    r, head, h = _small(seed=6)
    idx = O.build_index(head["W_bits"], head["b"], head["labels"], r.C, radius_slack=0.0)
    h64 = O.bf16_to_f64(h[0])
    U1, _ = O.cluster_bounds(idx, h64)
    U3, _ = O.cluster_bounds(idx, 3.0 * h64)
    bm = idx.bmax.astype(np.float64)
    assert np.allclose(U3 - bm, 3.0 * (U1 - bm), rtol=1e-12, atol=1e-12)
    W = O.bf16_to_f64(head["W_bits"])
    L = O.full_logits(W, head["b"], h64)
    # one cluster per token: zero radius, the bound IS the logit
    idxV = O.build_index(head["W_bits"], head["b"], np.arange(r.V), r.V, radius_slack=0.0)
    UV, _ = O.cluster_bounds(idxV, h64)
    assert np.all(idxV.R == 0) and np.allclose(UV, L, rtol=1e-13, atol=1e-13)
    # a single cluster: one bound above the maximum logit
    idx1 = O.build_index(head["W_bits"], head["b"], np.zeros(r.V, dtype=int), 1, radius_slack=0.0)
    Uo, _ = O.cluster_bounds(idx1, h64)
    assert Uo.shape == (r.B, 1) and np.all(Uo[:, 0] >= L.max(1))


def test_bound_is_attained_when_deviation_aligns_with_h():
    # two rows mu +- r*e0, equal bias, h along e0: the larger logit equals the bound exactly,
    # so neither the radius term nor the bias term can be over- or under-weighted.
    mu = np.array([1.0, 2.0, -0.5, 0.25], dtype=np.float32)
    dev = np.array([0.5, 0, 0, 0], dtype=np.float32)
    Wb = synth.f32_to_bf16_bits(np.stack([mu + dev, mu - dev]))
    b = np.array([0.75, 0.75], dtype=np.float32)
    idx = O.build_index(Wb, b, np.zeros(2, dtype=int), 1, radius_slack=0.0)
    h64 = np.array([[3.0, 0.0, 0.0, 0.0]])
    U, hn = O.cluster_bounds(idx, h64)
    L = O.full_logits(O.bf16_to_f64(Wb), b, h64)
    assert hn[0] == 3.0 and float(idx.R[0]) == 0.5
    assert U[0, 0] == L.max() == 1.5 * 3.0 + 0.75
    # empty clusters never win
    idxe = O.build_index(Wb, b, np.array([0, 2]), 3, radius_slack=0.0)
    Ue, _ = O.cluster_bounds(idxe, h64)
    assert Ue[0, 1] == -math.inf and np.isfinite(Ue[0, [0, 2]]).all()


# ------------------------------------------------------------------ certificates by definition
def _random_problem(seed, V=60, d=8, C=6, bias=True, spread=1.0):
    rng = np.random.default_rng(seed)
    cent = rng.standard_normal((C, d)) * spread
    labels = rng.integers(0, C, V)
    W = cent[labels] + 0.3 * rng.standard_normal((V, d))
    Wb = synth.f32_to_bf16_bits(W.astype(np.float32))
    b = (0.2 * rng.standard_normal(V)).astype(np.float32) if bias else None
    idx = O.build_index(Wb, b, labels, C, radius_slack=0.0)
    hb = synth.f32_to_bf16_bits((rng.standard_normal((1, d)) * 1.5).astype(np.float32))
    h64 = O.bf16_to_f64(hb)
    L = O.full_logits(O.bf16_to_f64(Wb), b, h64)[0]
    U, _ = O.cluster_bounds(idx, h64)
    return idx, U[0], L, labels


def _certs_by_definition(idx, U, L, opened, k, eps):
    """Definition 1 and Theorem 2 (cluster-wise tail) written out on sets, in the linear domain."""
    open_set = set(int(c) for c in opened)
    rest = [c for c in range(idx.C) if c not in open_set and idx.n[c] > 0]
    S = np.concatenate([idx.rows(c) for c in opened]) if len(opened) else np.empty(0, dtype=int)
    vals = np.sort(L[S])[::-1]
    if not rest:
        return True, True
    tk = len(vals) >= k >= 1 and all(U[c] < vals[k - 1] for c in rest)
    Rhat = sum(int(idx.n[c]) * math.exp(U[c]) for c in rest)
    ZS = float(np.sum(np.exp(L[S])))
    sm = len(S) > 0 and eps > 0 and Rhat / (ZS + Rhat) <= eps
    return bool(tk), bool(sm)


@pytest.mark.parametrize("combine", [O.COMBINE_ANY, O.COMBINE_ALL])
def test_alg1_matches_prefix_enumeration(combine):
    checked = 0
    for seed in range(40):
        idx, U, L, _ = _random_problem(seed, spread=1.0 + (seed % 4))
        for k, eps in [(3, 0.05), (1, 0.3), (5, 1e-3), (4, -1.0), (0, 0.2)]:
            got = O.alg1_step(idx, U, L, k, eps, K_max=idx.V, combine=combine)
            order = [c for c in O.cluster_order(U) if idx.n[c] > 0]
            want = None
            for m in range(len(order) + 1):
                tk, sm = _certs_by_definition(idx, U, L, order[:m], k, eps)
                tk_ok = tk if k >= 1 else combine == O.COMBINE_ALL
                sm_ok = sm if eps > 0 else combine == O.COMBINE_ALL
                if (tk_ok and sm_ok) if combine == O.COMBINE_ALL else (tk_ok or sm_ok):
                    want = m
                    break
            assert not got["fallback"] and got["opened"] == want, (seed, k, eps)
            checked += 1
    assert checked == 200


def test_alg1_budget():
    idx, U, L, _ = _random_problem(7)
    assert O.alg1_step(idx, U, L, 3, 1e-6, K_max=0)["fallback"]
    r = O.alg1_step(idx, U, L, 3, 1e-6, K_max=idx.V)
    assert not r["fallback"] and r["n_rows"] <= idx.V


def test_theorem1_certified_topk_is_global_topk():
    hits = 0
    for seed in range(60):
        idx, U, L, _ = _random_problem(100 + seed, V=80, C=8, spread=2.0)
        for k in (1, 3, 7):
            r = O.alg1_step(idx, U, L, k, -1.0, K_max=idx.V)              # top-k test alone
            assert r["topk_cert"]
            S = np.concatenate([idx.rows(c) for c in r["clusters"]])
            ids_S, _ = O.topk_bruteforce(L[S], k, S)
            ids_V, vals_V = O.topk_bruteforce(L, k)
            assert np.array_equal(ids_S, ids_V)
            # minimal prefix = every cluster whose bound reaches the true k-th logit
            want = {int(c) for c in range(idx.C) if idx.n[c] > 0 and U[c] >= vals_V[-1]}
            assert set(int(c) for c in r["clusters"]) == want
            hits += len(want) < idx.C
    assert hits > 20                                                       # the certificate really prunes


def test_singleton_clusters_open_exactly_the_topk():
    rng = np.random.default_rng(9)
    V, d, k = 40, 6, 5
    Wb = synth.f32_to_bf16_bits(rng.standard_normal((V, d)).astype(np.float32))
    b = rng.standard_normal(V).astype(np.float32)
    idx = O.build_index(Wb, b, np.arange(V), V, radius_slack=0.0)
    h64 = O.bf16_to_f64(synth.f32_to_bf16_bits(rng.standard_normal((1, d)).astype(np.float32)))
    L = O.full_logits(O.bf16_to_f64(Wb), b, h64)[0]
    U, _ = O.cluster_bounds(idx, h64)
    r = O.alg1_step(idx, U[0], L, k, -1.0, K_max=V)
    assert r["opened"] == k and set(r["clusters"].tolist()) == set(O.topk_bruteforce(L, k)[0].tolist())


def test_theorem2_tv_identity_and_tail_ordering():
    for seed in range(30):
        idx, U, L, _ = _random_problem(200 + seed, spread=1.5)
        order = O.cluster_order(U)
        T = O.tail_log_mass(idx, U, order)
        p = np.exp(L - O.logsumexp(L))
        for m in range(1, idx.C):
            S = np.concatenate([idx.rows(c) for c in order[:m]])
            if S.size == 0:
                continue
            inS = np.zeros(idx.V, bool); inS[S] = True
            pt = np.where(inS, np.exp(L - O.logsumexp(L[S])), 0.0)
            tv = 0.5 * np.abs(p - pt).sum()                                # total variation by definition
            ZS, R = np.exp(L[inS]).sum(), np.exp(L[~inS]).sum()
            assert math.isclose(tv, R / (ZS + R), rel_tol=1e-10, abs_tol=1e-15)
            assert math.isclose(tv, p[~inS].sum(), rel_tol=1e-10, abs_tol=1e-15)
            rest = [c for c in order[m:] if idx.n[c] > 0]
            Rhat = sum(int(idx.n[c]) * math.exp(U[c]) for c in rest)
            loose = (~inS).sum() * math.exp(max(U[c] for c in rest)) if rest else 0.0
            assert R <= Rhat * (1 + 1e-12) <= loose * (1 + 1e-12)
            if rest:
                assert math.isclose(T[m], math.log(Rhat), rel_tol=1e-12, abs_tol=1e-12)
        assert T[idx.C] == -math.inf


def test_soft_certificate_implies_tv_within_eps():
    seen = 0
    for seed in range(40):
        idx, U, L, _ = _random_problem(300 + seed, spread=2.5)
        for eps in (0.2, 0.02, 1e-3):
            r = O.alg1_step(idx, U, L, 0, eps, K_max=idx.V)               # softmax test alone
            assert r["soft_cert"]
            S = np.concatenate([idx.rows(c) for c in r["clusters"]])
            p = np.exp(L - O.logsumexp(L))
            inS = np.zeros(idx.V, bool); inS[S] = True
            assert p[~inS].sum() <= eps
            seen += r["opened"] < np.count_nonzero(idx.n)
    assert seen > 10


def test_soft_certificate_extremes():
    idx, U, L, _ = _random_problem(11)
    # eps -> 1: certified as soon as anything is scored
    assert O.alg1_step(idx, U, L, 0, 1 - 1e-12, K_max=idx.V)["opened"] == 1
    # flat logits (h = 0, no bias): never certified before the last cluster is opened
    Uflat = np.where(idx.n > 0, 0.0, -math.inf)
    r = O.alg1_step(idx, Uflat, np.zeros(idx.V), 0, 1e-3, K_max=idx.V)
    assert r["opened"] == np.count_nonzero(idx.n)


# ------------------------------------------------------------------ two-round schedule
@pytest.mark.parametrize("combine", [O.COMBINE_ALL, O.COMBINE_ANY])
def test_csv2r_certificates_hold_by_definition_and_contain_alg1(combine):
    rounds = {0: 0, 1: 0, 2: 0}
    for seed in range(60):
        idx, U, L, _ = _random_problem(400 + seed, V=90, C=9, spread=1.0 + (seed % 5) * 0.5)
        for k, eps in [(3, 0.05), (6, 1e-3), (2, 0.3), (4, -1.0), (0, 0.1)]:
            r = O.csv2r_step(idx, U, L, k, eps, K_max=idx.V, combine=combine)
            a = O.alg1_step(idx, U, L, k, eps, K_max=idx.V, combine=combine)
            assert not r["fallback"] and not a["fallback"]
            rounds[r["rounds"]] += 1
            assert a["opened"] <= r["m1"]                                  # minimal prefix is contained
            tk, sm = _certs_by_definition(idx, U, L, r["clusters"], k, eps)
            assert bool(r["flags"] & O.FLAG_TOPK_CERT) == (tk and k >= 1)
            assert bool(r["flags"] & O.FLAG_SOFTMAX_CERT) == (sm and eps > 0)
            if r["flags"] & O.FLAG_TOPK_CERT:
                assert np.array_equal(r["ids"], O.topk_bruteforce(L, k)[0])
            S = np.concatenate([idx.rows(c) for c in r["clusters"]])
            assert r["n_rows"] == S.size and r["n_clusters"] == len(r["clusters"])
            assert math.isclose(r["lse"], O.logsumexp(L[S]), rel_tol=1e-13)
            # seed prefix is the shortest with >= max(k,1) rows
            P = np.cumsum(idx.n[r["order"]])
            assert P[r["m0"] - 1] >= max(k, 1) and (r["m0"] == 1 or P[r["m0"] - 2] < max(k, 1))
    assert rounds[1] > 20 and rounds[2] > 20


def test_csv2r_budget_and_fallback_outputs():
    idx, U, L, _ = _random_problem(12, V=90, C=9)
    k, eps = 4, 1e-3
    r0 = O.csv2r_step(idx, U, L, k, eps, K_max=0)
    assert r0["fallback"] and r0["rounds"] == 0
    assert r0["flags"] == O.FLAG_FALLBACK | O.FLAG_TOPK_CERT | O.FLAG_SOFTMAX_CERT
    assert r0["n_rows"] == idx.V and r0["n_clusters"] == idx.C
    assert np.array_equal(r0["ids"], O.topk_bruteforce(L, k)[0])
    assert math.isclose(r0["lse"], O.logsumexp(L), rel_tol=1e-14)
    rV = O.csv2r_step(idx, U, L, k, eps, K_max=idx.V)
    assert not rV["fallback"]
    # a budget between the seed and the round-1 plan: fallback is decided before round 1 is scored
    if rV["rounds"] == 2:
        rb = O.csv2r_step(idx, U, L, k, eps, K_max=rV["n_rows"] - 1)
        assert rb["fallback"] and rb["rounds"] == 1


def test_csv2r_on_planted_recipe_behaves_like_the_workload_model():
    # aligned h: one cluster holds the whole top-k and nearly all of the softmax mass
    r, head, h = _small(seed=13, V=4000, d=256, C=32, B=1, steps=8, k=10)
    idx = O.build_index(head["W_bits"], head["b"], head["labels"], r.C)
    W = O.bf16_to_f64(head["W_bits"])
    for t in range(h.shape[0]):
        out = O.decode_step(W, head["b"], idx, h[t], r.k, r.eps, r.K_max_rows)[0]
        assert out["flags"] == O.FLAG_TOPK_CERT | O.FLAG_SOFTMAX_CERT and out["rounds"] == 1
        assert out["n_clusters"] == 1 and out["n_rows"] == 125
        L = O.full_logits(W, head["b"], O.bf16_to_f64(h[t]))[0]
        assert np.array_equal(out["ids"], O.topk_bruteforce(L, r.k)[0])
    # non-finite hidden state is flagged, not scored
    bad = h[0].copy(); bad[0, 3] = 0x7FC0
    assert O.decode_step(W, head["b"], idx, bad, r.k, r.eps, r.K_max_rows)[0]["flags"] == O.FLAG_INVALID


# ------------------------------------------------------------------ strictness of the two tests
def _singletons(logit_values):
    """One cluster per token, zero radius, one-dimensional weights: the bound of a cluster is its logit."""
    w = np.array(logit_values, dtype=np.float32)[:, None]
    Wb = synth.f32_to_bf16_bits(w)
    idx = O.build_index(Wb, None, np.arange(len(w)), len(w), radius_slack=0.0)
    h64 = np.array([[1.0]])
    L = O.full_logits(O.bf16_to_f64(Wb), None, h64)[0]
    U, _ = O.cluster_bounds(idx, h64)
    assert np.array_equal(U[0], L)
    return idx, U[0], L


def test_topk_test_is_strict():
    # logits 5,3,3,1 and k=2: after opening {5,3} the next bound EQUALS the 2nd logit, so Definition 1
    # (strict inequality) is not met and the tied cluster must be opened as well.
    idx, U, L = _singletons([5.0, 3.0, 3.0, 1.0])
    assert O.alg1_step(idx, U, L, 2, -1.0, K_max=4)["opened"] == 3
    r = O.csv2r_step(idx, U, L, 2, -1.0, K_max=4)
    assert r["m0"] == 2 and r["m1"] == 3 and r["rounds"] == 2 and r["flags"] == O.FLAG_TOPK_CERT
    assert r["ids"].tolist() == [0, 1]                                     # equal logits: smaller id first


def test_softmax_test_is_non_strict():
    # two tokens with logit 0: with one open the tail ratio is exactly 1/2, which meets eps = 1/2
    idx, U, L = _singletons([0.0, 0.0])
    assert O.alg1_step(idx, U, L, 0, 0.5, K_max=2)["opened"] == 1
    assert O.alg1_step(idx, U, L, 0, 0.49, K_max=2)["opened"] == 2
    r = O.csv2r_step(idx, U, L, 0, 0.5, K_max=2)
    assert r["m1"] == 1 and r["flags"] == O.FLAG_SOFTMAX_CERT


# ----------------------------------------------------------------------------- fallback levels and adaptive budget
def _line_head(clusters):
    """d = 1 head whose logits for h = 1 are the listed values: one list per cluster (all bf16-exact)."""
    vals = np.array([v for c in clusters for v in c], dtype=np.float32)
    labels = np.array([i for i, c in enumerate(clusters) for _ in c], dtype=np.int64)
    W_bits = synth.f32_to_bf16_bits(vals.reshape(-1, 1))
    assert np.array_equal(synth.bf16_bits_to_f32(W_bits).ravel(), vals)
    b = np.zeros(vals.size, dtype=np.float32)
    idx = O.build_index(W_bits, b, labels, len(clusters))
    W64 = O.bf16_to_f64(W_bits)
    h_bits = synth.f32_to_bf16_bits(np.array([[1.0]], dtype=np.float32))
    return W64, b, idx, h_bits, vals


def test_partial_expansion_rescues_a_step_traced_by_hand():
    # k = 2.  Round 0 opens c0 = {10, 1}: theta0 = 1, next bound ~9 -> not certified; every cluster can still hold a
    # value >= 1, so the plan is all 10 rows > K_max = 6.  Opening one more cluster (Delta C = 1, c1 = {9, 8.5}) lifts
    # theta to 9 > the next bound ~8.6: certified with 4 rows in 2 rounds.  Without the level: full vocabulary.
    W64, b, idx, h_bits, vals = _line_head([[10, 1], [9, 8.5], [8.5625, 0], [2, 1.5], [1.25, 1.125]])
    plain = O.decode_step(W64, b, idx, h_bits, k=2, eps=0.0, K_max=6)[0]
    assert plain["flags"] & O.FLAG_FALLBACK and plain["rounds"] == 1
    lad = O.decode_step(W64, b, idx, h_bits, k=2, eps=0.0, K_max=6, max_rounds=4, delta_clusters=1)[0]
    assert lad["flags"] == O.FLAG_TOPK_CERT
    assert lad["rounds"] == 2 and lad["n_rows"] == 4 and lad["n_clusters"] == 2
    assert list(lad["ids"]) == [0, 2] and list(lad["logits"]) == [10.0, 9.0]
    # same answer as the full vocabulary gives
    assert list(plain["ids"]) == [0, 2]


def test_partial_expansion_stops_at_the_budget_and_at_max_rounds():
    W64, b, idx, h_bits, vals = _line_head([[10, 1], [9, 0.5], [8.5, 0.25], [8, 0.125], [7.5, 0]])
    # k = 2, theta0 = 1: the plan is everything (10 rows).  Budget 4 rows: one extra cluster fits, theta becomes 9,
    # next bound 8.5 < 9 -> certified.  Budget 3 rows: nothing fits -> full vocabulary after one round.
    ok = O.decode_step(W64, b, idx, h_bits, k=2, eps=0.0, K_max=4, max_rounds=3, delta_clusters=1)[0]
    assert ok["flags"] == O.FLAG_TOPK_CERT and ok["n_rows"] == 4 and ok["rounds"] == 2
    no = O.decode_step(W64, b, idx, h_bits, k=2, eps=0.0, K_max=3, max_rounds=3, delta_clusters=1)[0]
    assert no["flags"] & O.FLAG_FALLBACK and no["rounds"] == 1
    # k = 4 needs four clusters' heads: Delta C = 1 per round and only 2 rounds in total cannot get there
    few = O.decode_step(W64, b, idx, h_bits, k=4, eps=0.0, K_max=8, max_rounds=2, delta_clusters=1)[0]
    assert few["flags"] & O.FLAG_FALLBACK
    many = O.decode_step(W64, b, idx, h_bits, k=4, eps=0.0, K_max=8, max_rounds=5, delta_clusters=1)[0]
    assert many["flags"] == O.FLAG_TOPK_CERT and many["n_rows"] <= 8
    assert list(many["logits"]) == [10.0, 9.0, 8.5, 8.0]


def test_relaxed_tolerance_accepts_between_eps_and_two_eps():
    # softmax only.  S = {5, 5}, outside = {0, 0} with bound ~0: T - Z ~ -5, e^-5 = 0.00674.
    # eps = 0.005: eps/(1-eps) = 0.005025 < e^-5 < 0.010101 = 2eps/(1-2eps): fails at eps, holds at 2 eps.
    W64, b, idx, h_bits, vals = _line_head([[5, 5], [0, 0]])
    strict = O.decode_step(W64, b, idx, h_bits, k=0, eps=0.005, K_max=2)[0]
    assert strict["flags"] & O.FLAG_FALLBACK
    rel = O.decode_step(W64, b, idx, h_bits, k=0, eps=0.005, K_max=2, relax=True)[0]
    assert rel["flags"] == O.FLAG_SOFTMAX_RELAXED and rel["n_rows"] == 2 and rel["rounds"] == 1
    ZV = O.logsumexp(vals.astype(np.float64))
    outside = 1.0 - math.exp(rel["lse"] - ZV)           # probability mass outside S
    assert 0.005 < outside <= 0.01
    # with room in the budget the strict certificate is reached instead
    roomy = O.decode_step(W64, b, idx, h_bits, k=0, eps=0.005, K_max=4, relax=True)[0]
    assert roomy["flags"] == O.FLAG_SOFTMAX_CERT and roomy["n_rows"] == 4


def test_fallback_levels_never_break_the_certificates():
    # Theorem 1 / Theorem 2 against brute force over V, on steps that go through partial expansions and relaxation
    r = synth.small_recipe(V=1500, d=48, C=30, B=1, steps=40, k=8, eps=2e-3, h_mode="mix", sizes="zipf", iso_frac=0.2,
                           row_noise=0.3)
    head = synth.make_head(r)
    h = synth.make_hidden(r, head["centers"], steps=40)
    W64 = O.bf16_to_f64(head["W_bits"])
    idx = O.build_index(head["W_bits"], head["b"], head["labels"], r.C)
    seen = {"rescued": 0, "relaxed": 0, "fallback": 0, "cert": 0, "extra_rounds": 0}
    for s in range(40):
        L = O.full_logits(W64, head["b"], O.bf16_to_f64(np.atleast_2d(h[s])))[0]
        ids, top = O.topk_bruteforce(L, r.k)
        ZV = O.logsumexp(L)
        for eps in (r.eps, 0.0):
            for K_max in (150, 400, 900):
                base = O.decode_step(W64, head["b"], idx, h[s], r.k, eps, K_max, logits=L[None])[0]
                res = O.decode_step(W64, head["b"], idx, h[s], r.k, eps, K_max, logits=L[None], max_rounds=6,
                                    delta_clusters=2, relax=True)[0]
                assert res["rounds"] <= 6
                if res["flags"] & O.FLAG_FALLBACK:
                    seen["fallback"] += 1
                    assert base["flags"] & O.FLAG_FALLBACK          # the levels only ever remove fallbacks
                    continue
                assert res["n_rows"] <= K_max
                if res["flags"] & O.FLAG_TOPK_CERT:
                    assert np.array_equal(res["ids"], ids)
                out = 1.0 - math.exp(res["lse"] - ZV)
                if res["flags"] & O.FLAG_SOFTMAX_CERT:
                    assert out <= eps
                    seen["cert"] += 1
                if res["flags"] & O.FLAG_SOFTMAX_RELAXED:
                    assert eps > 0 and out <= 2 * eps
                    seen["relaxed"] += 1
                seen["extra_rounds"] += res["rounds"] > 2
                if base["flags"] & O.FLAG_FALLBACK and not res["flags"] & O.FLAG_SOFTMAX_RELAXED:
                    seen["rescued"] += 1
    assert all(v > 0 for v in seen.values()), seen


def test_kmax_controller_printed_formula_and_feedback_reading():
    # the printed update, evaluated by hand: 32064 * (1 + 0.01 * (0.02 - 0.10)) = 32064 * 0.9992 = 32038.3488
    assert O.kmax_update(32064, 0.10, literal=True) == pytest.approx(32038.3488, rel=1e-12)
    # the feedback reading moves the other way by the same amount
    assert O.kmax_update(32064, 0.10) == pytest.approx(32064 * 1.0008, rel=1e-12)
    # at the target nothing moves, in either reading
    assert O.kmax_update(5000.0, 0.02) == 5000.0 and O.kmax_update(5000.0, 0.02, literal=True) == 5000.0
    # constant rate: geometric closed form
    K = 1000.0
    for _ in range(50):
        K = O.kmax_update(K, 0.25, alpha=0.01, rho_target=0.02)
    assert K == pytest.approx(1000.0 * (1 + 0.01 * 0.23) ** 50, rel=1e-12)
    assert O.kmax_rows(123.9, 10, 1000) == 123 and O.kmax_rows(3.2, 10, 1000) == 10 and O.kmax_rows(5e3, 10, 1000) == 1000


def test_kmax_controller_closed_loop_needs_the_feedback_sign():
    # a fallback rate that falls as the budget grows (any such model will do): rho(K) = exp(-K / 2000)
    rho = lambda K: math.exp(-K / 2000.0)
    K_star = -2000.0 * math.log(0.02)                  # budget at which the rate equals the target
    for literal, toward in ((False, True), (True, False)):
        K = 0.5 * K_star
        d0 = abs(K - K_star)
        for _ in range(20000):
            K = O.kmax_update(K, rho(K), alpha=0.01, rho_target=0.02, literal=literal)
        assert (abs(K - K_star) < 0.01 * d0) == toward, (literal, K, K_star)


def test_nucleus_certificate_is_the_softmax_test_in_delta_form():
    # Section III, top-p certification: the delta-form on the final open set agrees with the step's softmax flag at
    # eps = delta / (1 + delta), and a certified step leaves at most that mass outside S (brute force over V)
    r = synth.small_recipe(V=1500, d=48, C=30, B=1, steps=30, k=0, eps=1e-3, h_mode="mix", row_noise=0.3)
    head = synth.make_head(r)
    h = synth.make_hidden(r, head["centers"], steps=30)
    W64 = O.bf16_to_f64(head["W_bits"])
    idx = O.build_index(head["W_bits"], head["b"], head["labels"], r.C)
    assert O.nucleus_eps(0.25) == 0.2 and math.isclose(math.log(0.25), math.log(0.2 / 0.8), rel_tol=1e-15)
    seen = 0
    for delta in (1e-3, 1e-2, 0.2):
        eps = O.nucleus_eps(delta)
        for s in range(30):
            L = O.full_logits(W64, head["b"], O.bf16_to_f64(np.atleast_2d(h[s])))
            res = O.decode_step(W64, head["b"], idx, h[s], 0, eps, r.K_max_rows, logits=L)[0]
            if res["flags"] & O.FLAG_FALLBACK:
                continue
            seen += 1
            assert res["flags"] == O.FLAG_SOFTMAX_CERT
            assert O.nucleus_holds(idx, res["U"], res["clusters"], res["lse"], delta)
            outside = 1.0 - math.exp(res["lse"] - O.logsumexp(L[0]))
            assert outside <= delta / (1.0 + delta)
    assert seen > 40


def test_bf16_centroids_keep_the_bound_sound_and_cost_little():
    # the radius is measured to the stored (rounded) centroid, so Eq. "cluster_bound" still dominates every logit
    r = synth.small_recipe(V=3000, d=96, C=24, B=4, steps=6, h_mode="mix", iso_frac=0.3)
    head = synth.make_head(r)
    h = synth.make_hidden(r, head["centers"], steps=6)
    W64 = O.bf16_to_f64(head["W_bits"])
    i32 = O.build_index(head["W_bits"], head["b"], head["labels"], r.C)
    i16 = O.build_index(head["W_bits"], head["b"], head["labels"], r.C, centroid_bf16=True)
    # stored values are bfloat16-exact and within half a bf16 ulp (at most 2^-8 relative) of the float32 centroid
    bits = i16.mu.view(np.uint32)
    assert np.all(bits & 0xFFFF == 0)
    assert np.all(np.abs(i16.mu - i32.mu) <= 2.0 ** -8 * np.abs(i32.mu) + 1e-45)
    assert np.array_equal(i16.perm, i32.perm) and np.array_equal(i16.bmax, i32.bmax)
    # triangle inequality: the radius moves by at most the distance between the two stored centroids
    shift = np.sqrt(((i16.mu.astype(np.float64) - i32.mu.astype(np.float64)) ** 2).sum(axis=1))
    assert np.all(np.abs(i16.R.astype(np.float64) - i32.R.astype(np.float64)) <= 1.001 * shift * (1 + 2.0 ** -14) + 1e-6)
    for s in range(6):
        h64 = O.bf16_to_f64(h[s])
        L = O.full_logits(W64, head["b"], h64)
        for idx in (i16, i32):
            U, hn = O.cluster_bounds(idx, h64)
            for c in range(r.C):
                rows = idx.rows(c)
                assert np.all(L[:, rows].max(axis=1) <= U[:, c])
        # steps stay certified-correct with the looser bounds
        for b_, res in enumerate(O.decode_step(W64, head["b"], i16, h[s], 5, 1e-3, r.K_max_rows, logits=L)):
            if res["flags"] & O.FLAG_TOPK_CERT:
                ids, _ = O.topk_bruteforce(L[b_], 5)
                assert np.array_equal(res["ids"], ids)
    assert O.metadata_bytes_bf16(1024, 4096) == 1024 * (8192 + 12)


# ------------------------------------------------------------------ the softmax prefix s, the order's tie-break, the margins
def _flat_clusters(values, sizes):
    """d = 1 head, h = 1: cluster c holds sizes[c] rows that all have the logit values[c] (bf16-exact), no bias, no
    radius slack: the radius is 0 and the bound of a cluster IS its logit."""
    vals = np.repeat(np.array(values, dtype=np.float32), sizes)
    labels = np.repeat(np.arange(len(values)), sizes)
    W_bits = synth.f32_to_bf16_bits(vals.reshape(-1, 1))
    idx = O.build_index(W_bits, None, labels, len(values), radius_slack=0.0)
    L = O.full_logits(O.bf16_to_f64(W_bits), None, np.array([[1.0]]))[0]
    U, _ = O.cluster_bounds(idx, np.array([[1.0]]))
    assert np.all(idx.R == 0) and np.array_equal(U[0], np.array(values, dtype=np.float64))
    return idx, U[0], L


def test_softmax_prefix_is_the_shortest_that_meets_theorem2_traced_by_hand():
    # Four clusters of two rows with logits 10, 8, 6, 0; eps = 0.01, ln(eps/(1-eps)) = ln(1/99) = -4.59512.
    # Round 0 opens {10,10}: Z0 = 10 + ln 2.  Tail masses (the ln 2 of "two rows each" cancels against Z0):
    #   one cluster open   ln(e^8 + e^6 + 1) - 10 = -1.87278   > -4.59512   fails
    #   two clusters open  ln(e^6 + 1)       - 10 = -3.99752   > -4.59512   fails
    #   three open         ln(1)             - 10 = -10        <= -4.59512  holds      -> s = 3, not 2 and not 4
    # Even against the larger Z of two open clusters the second prefix fails (-3.99752 - ln(1 + e^-2) = -4.12445), so
    # three clusters is also the minimal certifying prefix of Algorithm 1.
    idx, U, L = _flat_clusters([10.0, 8.0, 6.0, 0.0], [2, 2, 2, 2])
    eps = 0.01
    lam = math.log(1.0 / 99.0)
    t1, t2, t3 = math.log(math.exp(8) + math.exp(6) + 1) - 10, math.log(math.exp(6) + 1) - 10, -10.0
    assert t1 > lam and t2 > lam and t3 <= lam and t2 - math.log(1 + math.exp(-2)) > lam
    soft = O.csv2r_step(idx, U, L, 0, eps, K_max=8)                       # softmax test alone: m0 = 1 row suffices
    assert soft["m0"] == 1 and soft["m1"] == 3 and soft["rounds"] == 2 and soft["flags"] == O.FLAG_SOFTMAX_CERT
    assert soft["n_rows"] == 6 and soft["clusters"].tolist() == [0, 1, 2]
    assert O.alg1_step(idx, U, L, 0, eps, K_max=8)["opened"] == 3
    # both certificates, k = 2: theta0 = 10 > next bound 8, so a = m0 = 1 and the softmax prefix alone sets m1 = max(1, 3)
    both = O.csv2r_step(idx, U, L, 2, eps, K_max=8, combine=O.COMBINE_ALL)
    assert both["m0"] == 1 and both["m1"] == 3 and both["rounds"] == 2
    assert both["flags"] == O.FLAG_TOPK_CERT | O.FLAG_SOFTMAX_CERT and both["ids"].tolist() == [0, 1]
    # either certificate: the top-k test already holds after round 0
    either = O.csv2r_step(idx, U, L, 2, eps, K_max=8, combine=O.COMBINE_ANY)
    assert either["m1"] == 1 and either["rounds"] == 1 and either["flags"] == O.FLAG_TOPK_CERT
    # the budget is tested on the planned prefix (6 rows): 5 rows are not enough, 6 are
    assert O.csv2r_step(idx, U, L, 0, eps, K_max=5)["fallback"] and not O.csv2r_step(idx, U, L, 0, eps, K_max=6)["fallback"]
    # the margins the parity tests use as tie bands are the distances of exactly these comparisons
    mg = soft["margins"]
    assert mg["sm0"][0] == pytest.approx(t1 - lam, rel=1e-12) and mg["sm0"][1] == pytest.approx(10 + math.log(2), rel=1e-12)
    assert mg["s_lo"][0] == pytest.approx(t2 - lam, rel=1e-12)          # the prefix one shorter: how far it is from passing
    assert mg["s_hi"][0] == pytest.approx(lam - t3, rel=1e-12)          # the chosen prefix: how far it is from failing
    assert mg["seed"] == (2.0, 10.0) and mg["s_order"] == (6.0, 6.0)     # |10 - 8| at the seed boundary, |6 - 0| after s
    mb = both["margins"]
    assert mb["tk0"] == (2.0, 10.0)                                       # next bound 8 against theta0 = 10
    assert mb["tk1"] == (10.0, 10.0)                                      # after round 1: next bound 0 against theta1 = 10
    assert mb["id_gap"] == (2.0, 10.0)                                    # 2nd logit 10 against the 3rd, 8


def test_equal_bounds_open_the_smaller_cluster_id_first():
    # Two clusters tie for the largest bound and the seed prefix has room for one of them only (softmax test alone,
    # eps = 0.6: with one of the two equal clusters open the tail ratio is 1/2 + a negligible rest <= 0.6).
    for values, first in (([4.0, 4.0, -20.0], 0), ([1.0, 4.0, 4.0], 1), ([4.0, -3.0, 4.0], 0)):
        idx, U, L = _flat_clusters(values, [1, 1, 1])
        order = O.cluster_order(U)
        assert order[0] == first and order[1] == max(i for i, v in enumerate(values) if v == 4.0)
        r = O.csv2r_step(idx, U, L, 0, 0.6, K_max=3)
        assert r["rounds"] == 1 and r["clusters"].tolist() == [first] and r["flags"] == O.FLAG_SOFTMAX_CERT
        assert O.alg1_step(idx, U, L, 0, 0.6, K_max=3)["clusters"].tolist() == [first]
        # k = 1, either certificate: Definition 1 fails (the tied bound is not strictly below theta0), Theorem 2 holds
        r = O.csv2r_step(idx, U, L, 1, 0.6, K_max=3, combine=O.COMBINE_ANY)
        assert r["clusters"].tolist() == [first] and r["ids"].tolist() == [first] and r["flags"] == O.FLAG_SOFTMAX_CERT
        assert r["margins"]["seed"][0] == 0.0 and r["margins"]["tk0"][0] == 0.0      # both comparisons are exact ties


# ------------------------------------------------------------------ top-m bias table (Section III, bias binning)
def test_bias_table_hand_computed_cluster():
    # one cluster, d = 1: rows 5, 3, 1 -> centroid 3, radius 2; the row AT the centroid carries the outlying bias 4.
    # h = 1: logits 5, 7, 1.  Eq. "cluster_bound": 3 + 2 + 4 = 9.  With m = 2 the outlier is bounded on its own,
    # 3 + 0*1 + 4 = 7, and the others by 3 + 2*1 + 0 = 5: the bound is 7, the largest logit itself.
    Wb = synth.f32_to_bf16_bits(np.array([[5.0], [3.0], [1.0]], dtype=np.float32))
    b = np.array([0.0, 4.0, 0.0], dtype=np.float32)
    h = np.array([[1.0]])
    plain = O.build_index(Wb, b, np.zeros(3, dtype=int), 1, radius_slack=0.0)
    tab = O.build_index(Wb, b, np.zeros(3, dtype=int), 1, radius_slack=0.0, bias_table_m=2)
    assert O.cluster_bounds(plain, h)[0][0, 0] == 9.0
    assert tab.bias_table.tolist() == [[[0.0, 4.0], [2.0, 0.0]]]
    assert O.cluster_bounds(tab, h)[0][0, 0] == 7.0
    # which term wins depends on ||h||: at ||h|| = 3 the shared radius takes over: 9 + max(0 + 4, 6 + 0) = 15 (logits 15, 13, 3)
    assert O.cluster_bounds(tab, 3.0 * h)[0][0, 0] == 15.0 and O.cluster_bounds(plain, 3.0 * h)[0][0, 0] == 19.0
    # m = 3: two tokens on their own (bias 4, then bias 0 with the smaller id: row 5, distance 2), the rest {row 1}: radius 2
    t3 = O.build_index(Wb, b, np.zeros(3, dtype=int), 1, radius_slack=0.0, bias_table_m=3).bias_table
    assert t3.tolist() == [[[0.0, 4.0], [2.0, 0.0], [2.0, 0.0]]]
    # more table entries than tokens: the unused ones never win
    t5 = O.build_index(Wb, b, np.zeros(3, dtype=int), 1, radius_slack=0.0, bias_table_m=5)
    assert np.isneginf(t5.bias_table[0, 3:, 1]).all() and O.cluster_bounds(t5, h)[0][0, 0] == 7.0


def test_bias_table_keeps_the_bound_sound_and_never_loosens_it():
    rng = np.random.default_rng(77)
    tighter = total = 0
    for seed in range(6):
        r, head, h = _small(seed=20 + seed, V=1500, d=48, C=20, steps=5, sizes="zipf" if seed % 2 else "equal")
        b = head["b"].copy()
        b[rng.integers(0, r.V, 40)] += rng.normal(0, 1.0, 40).astype(np.float32)      # a few outlying biases
        W = O.bf16_to_f64(head["W_bits"])
        plain = O.build_index(head["W_bits"], b, head["labels"], r.C)
        one = O.build_index(head["W_bits"], b, head["labels"], r.C, bias_table_m=1)
        assert one.bias_table is None                                               # m = 1 is Eq. "cluster_bound" itself
        for m in (2, 3, 8):
            tab = O.build_index(head["W_bits"], b, head["labels"], r.C, bias_table_m=m)
            assert tab.bias_table.shape == (r.C, m, 2)
            # the first entry carries the largest bias, the shared entry's radius never exceeds the cluster radius
            assert np.array_equal(tab.bias_table[:, 0, 1], plain.bmax)
            assert np.all(tab.bias_table[:, :, 0] <= plain.R[:, None])
            for t in range(h.shape[0]):
                h64 = O.bf16_to_f64(h[t])
                L = O.full_logits(W, b, h64)
                Up, _ = O.cluster_bounds(plain, h64)
                Ut, _ = O.cluster_bounds(tab, h64)
                assert np.all(L <= Ut[:, head["labels"]] + 1e-12)                    # Cauchy-Schwarz invariant still holds
                assert np.all(Ut <= Up + 1e-12)                                      # never looser
                tighter += int((Ut < Up - 1e-9).sum())
                total += Ut.size
    assert tighter > 0.2 * total
    # a table with a single shared entry per cluster (every token "rest") is the plain bound
    r, head, h = _small(seed=31)
    plain = O.build_index(head["W_bits"], head["b"], head["labels"], r.C)
    fake = O.OracleIndex(plain.mu, plain.R, plain.bmax, plain.n, plain.perm,
                         np.stack([plain.R, plain.bmax], axis=1)[:, None, :])
    h64 = O.bf16_to_f64(h[0])
    assert np.allclose(O.cluster_bounds(fake, h64)[0], O.cluster_bounds(plain, h64)[0], rtol=1e-14, atol=0)
    # certified steps stay exact with the tighter bounds, and never open more rows
    W = O.bf16_to_f64(head["W_bits"])
    tab = O.build_index(head["W_bits"], head["b"], head["labels"], r.C, bias_table_m=3)
    for t in range(h.shape[0]):
        L = O.full_logits(W, head["b"], O.bf16_to_f64(h[t]))
        for b_, (rp, rt) in enumerate(zip(O.decode_step(W, head["b"], plain, h[t], 5, 1e-3, r.V, logits=L),
                                          O.decode_step(W, head["b"], tab, h[t], 5, 1e-3, r.V, logits=L))):
            assert rt["flags"] & O.FLAG_TOPK_CERT and np.array_equal(rt["ids"], O.topk_bruteforce(L[b_], 5)[0])
            assert O.alg1_step(tab, rt["U"], L[b_], 5, 1e-3, r.V)["n_rows"] <= O.alg1_step(plain, rp["U"], L[b_], 5, 1e-3, r.V)["n_rows"]


def test_certified_distribution_brackets_the_true_probabilities():
    # p~ over all of S sums to one; the true probabilities lie in [(1 - eps) p~, p~] for a certified step; the nucleus is
    # the shortest prefix reaching top_p (checked by enumeration) and covers (1 - eps) top_p of the true mass
    r = synth.small_recipe(V=1500, d=48, C=30, B=1, steps=20, k=40, eps=5e-3, h_mode="mix", row_noise=0.3)
    head = synth.make_head(r)
    h = synth.make_hidden(r, head["centers"], steps=20)
    W64 = O.bf16_to_f64(head["W_bits"])
    idx = O.build_index(head["W_bits"], head["b"], head["labels"], r.C)
    p1, c1, n1 = O.certified_distribution(np.log(np.array([0.5, 0.25, 0.125, 0.125])), 0.0, 0.8)
    assert np.allclose(p1, [0.5, 0.25, 0.125, 0.125], rtol=1e-15) and np.allclose(c1, [0.5, 0.75, 0.875, 1.0], rtol=1e-15) and n1 == 3
    assert O.certified_distribution(np.log(np.array([0.5, 0.25])), 0.0, 0.8)[2] == 0          # the list ends first
    assert O.certified_distribution(np.log(np.array([0.5, 0.5])), 0.0, 0.0)[2] == 0           # no nucleus asked for
    seen = 0
    for s in range(20):
        L = O.full_logits(W64, head["b"], O.bf16_to_f64(np.atleast_2d(h[s])))
        res = O.decode_step(W64, head["b"], idx, h[s], r.k, r.eps, r.K_max_rows, logits=L)[0]
        if res["flags"] & O.FLAG_FALLBACK or not res["flags"] & O.FLAG_SOFTMAX_CERT:
            continue
        seen += 1
        p, cum, nuc = O.certified_distribution(res["logits"], res["lse"], 0.9)
        true = np.exp(L[0][res["ids"]] - O.logsumexp(L[0]))
        assert np.all(true <= p * (1 + 1e-12)) and np.all(true >= (1 - r.eps) * p * (1 - 1e-12))
        assert np.all(np.diff(cum) >= 0) and cum[-1] <= 1 + 1e-12
        want = next((j + 1 for j in range(len(p)) if sum(p[:j + 1]) >= 0.9), 0)
        assert nuc == want
        if nuc:
            assert true[:nuc].sum() >= (1 - r.eps) * 0.9
        S = np.concatenate([idx.rows(c) for c in res["clusters"]])
        allp, _, _ = O.certified_distribution(L[0][S], res["lse"])
        assert math.isclose(allp.sum(), 1.0, rel_tol=1e-12)
    assert seen > 10


# ------------------------------------------------------------------ spherical clustering and the angular bound (Section III)
def _planar(angles_deg, norms):
    a = np.radians(np.array(angles_deg, dtype=np.float64))
    W = (np.array(norms)[:, None] * np.stack([np.cos(a), np.sin(a)], 1)).astype(np.float32)
    return np.pad(W, ((0, 0), (0, 6)))                               # d = 8


def test_angular_bound_hand_computed_in_the_plane():
    # unit rows at -10 and +10 degrees: direction (1,0), angular radius 10 degrees.  h of norm 2 at 40 degrees:
    # phi - theta = 30 degrees, bound 2 cos 30 = sqrt 3, attained by the row at +10 degrees.
    W = _planar([-10, 10], [1, 1])
    Wb = synth.f32_to_bf16_bits(W)
    idx = O.build_index_angular(Wb, None, np.zeros(2, dtype=int), 1, slack=0.0, angle_slack=0.0)
    W64 = O.bf16_to_f64(Wb)
    theta = math.acos(float(W64[0] @ idx.mu[0].astype(np.float64) / np.linalg.norm(W64[0]) / np.linalg.norm(idx.mu[0])))
    assert abs(math.degrees(theta) - 10) < 0.3                        # bf16 rounding of the rows moves it a little
    def hvec(deg, norm):
        v = np.zeros((1, 8)); v[0, 0] = norm * math.cos(math.radians(deg)); v[0, 1] = norm * math.sin(math.radians(deg))
        return v
    for deg in (40.0, 95.0, 170.0, -60.0):
        h = hvec(deg, 2.0)
        L = O.full_logits(W64, None, h)[0]
        U = O.cluster_bounds(idx, h)[0][0, 0]
        rho = np.linalg.norm(W64, axis=1)
        phi = math.radians(abs(deg))
        g = math.cos(phi - theta)
        want = 2.0 * (rho.max() if g >= 0 else rho.min()) * g
        assert U >= L.max() - 1e-6 and abs(U - want) < 2e-3 * max(1.0, abs(want))   # float32 storage of cos/sin/norms
        assert abs(U - L.max()) < 2e-2                                 # and tight: the row on the near edge attains it
    # h inside the cone: nothing better than ||w|| ||h|| can be said
    U = O.cluster_bounds(idx, hvec(5.0, 3.0))[0][0, 0]
    assert abs(U - 3.0 * np.linalg.norm(W64, axis=1).max()) < 1e-6
    # rows of different length: the longest decides a positive bound, the shortest a negative one
    W2 = _planar([-10, 10], [1, 3])
    idx2 = O.build_index_angular(synth.f32_to_bf16_bits(W2), None, np.zeros(2, dtype=int), 1, slack=0.0, angle_slack=0.0)
    assert abs(idx2.ang[0, 2] - 3.0) < 1e-2 and abs(idx2.ang[0, 3] - 1.0) < 1e-2     # bf16 rows: lengths 3 and 1 up to rounding
    L = O.full_logits(O.bf16_to_f64(synth.f32_to_bf16_bits(W2)), None, hvec(170.0, 2.0))[0]
    U = O.cluster_bounds(idx2, hvec(170.0, 2.0))[0][0, 0]
    assert U < 0 and U >= L.max() - 1e-6


def test_angular_bound_dominates_every_logit():
    rng = np.random.default_rng(91)
    for seed in range(5):
        r, head, h = _small(seed=40 + seed, V=1500, d=48, C=20, steps=6, iso_frac=0.4, h_mode="mix", row_noise=0.5 + seed)
        Wf = synth.bf16_bits_to_f32(head["W_bits"]) * rng.uniform(0.3, 2.0, (r.V, 1)).astype(np.float32)     # scattered row norms
        Wb = synth.f32_to_bf16_bits(Wf)
        W = O.bf16_to_f64(Wb)
        for slack in (0.0, 2.0 ** -14):
            idx = O.build_index_angular(Wb, head["b"], head["labels"], r.C, slack=slack, angle_slack=0.0 if slack == 0 else 2.0 ** -12)
            assert np.all(np.abs(np.linalg.norm(idx.mu.astype(np.float64), axis=1) - 1) < 1e-6)
            for t in range(h.shape[0]):
                h64 = np.concatenate([O.bf16_to_f64(h[t]), -O.bf16_to_f64(h[t]), W[rng.integers(0, r.V, 2)] * 5.0])   # also opposite and in-cone directions
                L = O.full_logits(W, head["b"], h64)
                U, hn = O.cluster_bounds(idx, h64)
                assert np.all(L <= U[:, head["labels"]] + 1e-9)
    # certified steps on an angular index return the full-vocabulary top-k
    r, head, h = _small(seed=46, V=2000, d=64, C=16, steps=6)
    idx = O.build_index_angular(head["W_bits"], head["b"], head["labels"], r.C)
    W = O.bf16_to_f64(head["W_bits"])
    for t in range(h.shape[0]):
        L = O.full_logits(W, head["b"], O.bf16_to_f64(h[t]))
        for b_, res in enumerate(O.decode_step(W, head["b"], idx, h[t], 5, 1e-3, r.V, logits=L)):
            assert res["flags"] & O.FLAG_TOPK_CERT and np.array_equal(res["ids"], O.topk_bruteforce(L[b_], 5)[0])


def test_spherical_kmeans_recovers_planted_directions():
    rng = np.random.default_rng(92)
    C, per, d = 6, 60, 32
    dirs = rng.standard_normal((C, d)); dirs /= np.linalg.norm(dirs, axis=1, keepdims=True)
    lab = np.repeat(np.arange(C), per)
    W = dirs[lab] + 0.05 * rng.standard_normal((C * per, d))
    W *= rng.uniform(0.2, 5.0, (C * per, 1))                           # lengths carry no information
    Wb = synth.f32_to_bf16_bits(W.astype(np.float32))
    first = np.array([c * per for c in range(C)])
    labels, got = O.spherical_kmeans(Wb, first, iters=3)
    assert np.array_equal(labels, lab)
    assert np.all(np.abs(np.linalg.norm(got.astype(np.float64), axis=1) - 1) < 1e-6)
    assert np.all(np.einsum("ij,ij->i", got.astype(np.float64), dirs) > 0.99)
    # Euclidean Lloyd from the same start is misled by the lengths
    assert not np.array_equal(O.lloyd_kmeans(Wb, first, iters=3)[0], lab)
    # assignment: largest cosine, ties to the smaller id, length of the row irrelevant
    Wt = np.array([[2.0, 0.0], [0.0, 0.1], [3.0, 3.0], [-1.0, 0.0]])
    D = np.array([[1.0, 0.0], [0.0, 1.0], [1.0, 0.0]])
    assert O.spherical_assign(Wt, D).tolist() == [0, 1, 0, 1]
