"""Pins for the CPU oracle: each checks oracle/ against something the paper or
the mathematics fixes, never against the oracle's own formula or the GPU path."""
import itertools
import json
import math
import os

import numpy as np
import pytest

import oracle
from synth import workloads as wl

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "hand_cases.json")
ROUTERS = [("binary32", oracle.route, np.float32), ("literal", oracle.route_literal, np.float64)]


def _cases():
    with open(GOLDEN) as f:
        return json.load(f)["cases"]


# ---------------------------------------------------------------- hand cases --

@pytest.mark.parametrize("case", _cases(), ids=lambda c: c["name"])
@pytest.mark.parametrize("router", ROUTERS, ids=lambda r: r[0])
def test_hand_cases(case, router):
    _, fn, dt = router
    logits = np.log(np.array(case["p"], dtype=np.float64)).astype(dt)
    out = fn(logits, case["k"], case["c"], case["eps_high"], case["t_fix"],
             np.array(case["loads_in"], dtype=np.int32))
    assert out["expert_ids"].tolist() == case["expert_ids"]
    assert out["loads"].tolist() == case["loads_out"]
    assert out["expanded"].tolist() == case["expanded"]
    assert out["cstar"].tolist() == case["cstar"]
    np.testing.assert_allclose(out["weights"], np.array(case["weights"]), atol=1e-6)


# ------------------------------------------------------ reductions to top-k --

def _numpy_topk(logits, k):
    order = np.argsort(-logits.astype(np.float64), axis=1, kind="stable")
    return order[:, :k].astype(np.int32)


@pytest.mark.parametrize("E,k", [(8, 2), (64, 6), (5, 1), (16, 16), (256, 8)])
@pytest.mark.parametrize("how", ["c_equals_k", "eps_small", "t_fix_one"])
@pytest.mark.parametrize("router", ROUTERS, ids=lambda r: r[0])
def test_reduces_to_library_topk(E, k, how, router):
    """c = k, a small eps_high, or t_fix = 1 (distinct scores) all give vanilla
    top-k routing whatever the loads are (Method, Final assignment; Evaluation:
    'when c = k the curves coincide')."""
    _, fn, dt = router
    T = 300
    logits = wl.random_logits(11 + E + k, T, E, scale=1.5).astype(dt)
    loads_in = np.random.default_rng(5).integers(0, 1000, size=E).astype(np.int32)
    c, eps, tfix = min(E, k + 3), 0.9999, 0.3
    if how == "c_equals_k":
        c = k
    elif how == "eps_small":
        eps = 1e-6
    else:
        tfix = 1.0
    out = fn(logits, k, c, eps, tfix, loads_in)
    want = _numpy_topk(logits, k)
    assert np.array_equal(out["expert_ids"], want)
    assert np.array_equal(out["loads"], loads_in + np.bincount(want.ravel(), minlength=E))
    z = logits.astype(np.float64)
    sm = np.exp(z - z.max(1, keepdims=True))
    w = np.take_along_axis(sm, want.astype(np.int64), 1)
    np.testing.assert_allclose(out["weights"], w / w.sum(1, keepdims=True), atol=1e-12)


def test_peaked_tokens_keep_topk_whatever_the_loads():
    """A token whose top-k mass clears eps_high is routed to its top-k even if those
    experts are the most loaded (Method, Expansion rule)."""
    E, k, T = 16, 2, 200
    rng = np.random.default_rng(3)
    logits = (rng.standard_normal((T, E)) * 0.1).astype(np.float32)
    hot = rng.integers(0, E, size=(T, 2))
    hot[:, 1] = (hot[:, 0] + 1 + rng.integers(0, E - 1, size=T)) % E
    logits[np.arange(T), hot[:, 0]] += 9.0
    logits[np.arange(T), hot[:, 1]] += 8.0
    loads_in = np.full(E, 10_000, dtype=np.int32)
    for _, fn, dt in ROUTERS:
        out = fn(logits.astype(dt), k, E, 0.9, 0.01, loads_in)
        assert not out["expanded"].any()
        assert np.array_equal(out["expert_ids"], hot)


# ------------------------------------------------------------- brute force --

def _brute_force_route(z, k, c, eps, tfix, loads_in):
    """Independent restatement for tiny inputs: softmax with numpy, the pool from
    the printed set definition, and the final assignment by enumerating every
    k-subset of the working set and keeping the one whose sorted (load, -score,
    index) keys are lexicographically least."""
    T, E = z.shape
    L = loads_in.astype(np.int64).copy()
    ids = np.zeros((T, k), dtype=np.int32)
    for t in range(T):
        s = np.exp(z[t] - z[t].max())
        s = s / s.sum()
        ranked = sorted(range(E), key=lambda i: (-z[t, i], i))
        topk = ranked[:k]
        if sum(s[i] for i in topk) >= eps:
            A = topk
        else:
            cut = tfix * s[ranked[0]]
            pool = sorted(set(i for i in range(E) if s[i] >= cut) | set(topk),
                          key=lambda i: (-z[t, i], i))
            work = pool[: min(c, len(pool))]
            best = None
            for sub in itertools.combinations(work, k):
                keys = sorted((L[i], -z[t, i], i) for i in sub)
                if best is None or keys < best[0]:
                    best = (keys, sub)
            A = sorted(best[1], key=lambda i: (-z[t, i], i))
        ids[t] = A
        for i in A:
            L[i] += 1
    return ids, L


def _margin_safe(z, k, eps, tfix, margin=1e-4):
    """Tokens whose decisions do not hinge on rounding: distinct logits, top-k mass
    and pool cut both away from their thresholds."""
    z = z.astype(np.float64)
    s = np.exp(z - z.max(1, keepdims=True))
    s /= s.sum(1, keepdims=True)
    srt = -np.sort(-s, axis=1)
    ok = np.abs(srt[:, :k].sum(1) - eps) > margin
    ok &= np.all(np.abs(s / srt[:, :1] - tfix) > margin, axis=1)
    zs = np.sort(z, axis=1)
    ok &= np.all(np.diff(zs, axis=1) > 1e-6, axis=1)
    return ok


@pytest.mark.parametrize("seed", range(12))
def test_brute_force_tiny(seed):
    rng = np.random.default_rng(100 + seed)
    E = int(rng.integers(2, 9))
    k = int(rng.integers(1, E + 1))
    c = int(rng.integers(k, E + 1))
    eps = float(rng.uniform(0.3, 1.05))
    tfix = float(rng.uniform(0.05, 1.0))
    T = 60
    z = (rng.standard_normal((T, E)) * rng.uniform(0.05, 2.0)).astype(np.float32)
    z = z[_margin_safe(z, k, eps, tfix)]
    loads_in = rng.integers(0, 4, size=E).astype(np.int32)
    want_ids, want_L = _brute_force_route(z.astype(np.float64), k, c, eps, tfix, loads_in)
    for _, fn, dt in ROUTERS:
        out = fn(z.astype(dt), k, c, eps, tfix, loads_in)
        assert np.array_equal(out["expert_ids"], want_ids)
        assert np.array_equal(out["loads"], want_L)


@pytest.mark.parametrize("seed", range(4))
def test_brute_force_with_exact_ties(seed):
    """Equal logits: the lower expert index ranks first everywhere (top-k membership,
    trimming, and the score tie-break of the load sort)."""
    rng = np.random.default_rng(200 + seed)
    E, k, c = 6, 2, 4
    z = wl.random_logits(300 + seed, 80, E, kind="ties", tie_levels=3, scale=0.5)
    eps, tfix = 0.999, 0.37
    loads_in = rng.integers(0, 3, size=E).astype(np.int32)
    keep = np.ones(len(z), dtype=bool)          # ties are the point: only guard the thresholds
    s = np.exp(z.astype(np.float64) - z.max(1, keepdims=True))
    keep &= np.all(np.abs(s / s.max(1, keepdims=True) - tfix) > 1e-4, axis=1)
    z = z[keep]
    want_ids, want_L = _brute_force_route(z.astype(np.float64), k, c, eps, tfix, loads_in)
    for _, fn, dt in ROUTERS:
        out = fn(z.astype(dt), k, c, eps, tfix, loads_in)
        assert np.array_equal(out["expert_ids"], want_ids)
        assert np.array_equal(out["loads"], want_L)


# ------------------------------------------------------ load-only closed form --

@pytest.mark.parametrize("E,k,T", [(8, 2, 400), (64, 6, 640), (5, 3, 100)])
def test_load_only_is_perfectly_balanced(E, k, T):
    """Ignoring scores (every expert a candidate) gives imbalance 1 / max violation 0
    (Evaluation, Baselines: 'load-only ... perfect balance')."""
    logits = wl.random_logits(7, T, E, scale=2.0)
    for _, fn, dt in ROUTERS:
        for t_stop in (T, T // 3):
            out = fn(logits[:t_stop].astype(dt), k, E, 2.0, 1e-30, np.zeros(E, np.int32))
            assert out["expanded"].all()
            assert out["loads"].max() - out["loads"].min() <= 1
            if (t_stop * k) % E == 0:
                assert np.all(out["loads"] == t_stop * k // E)


# -------------------------------------------------------------- invariants ---

@pytest.mark.parametrize("seed", range(6))
def test_invariants(seed):
    rng = np.random.default_rng(400 + seed)
    E = int(rng.choice([4, 8, 16, 64, 100]))
    k = int(rng.integers(1, min(E, 8) + 1))
    c = int(rng.integers(k, min(E, 16) + 1))
    T = 500
    z = wl.random_logits(500 + seed, T, E, scale=float(rng.uniform(0.2, 3)))
    loads_in = rng.integers(0, 50, size=E).astype(np.int32)
    eps, tfix = float(rng.uniform(0.2, 1.0)), float(rng.uniform(0.1, 1.0))
    out = oracle.route(z, k, c, eps, tfix, loads_in)
    ids = out["expert_ids"]
    assert ids.min() >= 0 and ids.max() < E
    assert all(len(set(r)) == k for r in ids.tolist())                 # |A| = k distinct
    np.testing.assert_allclose(out["weights"].sum(1), 1.0, atol=1e-12)  # renormalised
    assert out["loads"].sum() - loads_in.sum() == T * k                 # loads sum to T*k
    assert np.array_equal(out["loads"] - loads_in, np.bincount(ids.ravel(), minlength=E))
    assert np.all(out["cstar"] >= k) and np.all(out["cstar"] <= c)
    # ids listed by descending score; top-k branch rows equal the library top-k
    zz = np.take_along_axis(z, ids.astype(np.int64), 1)
    assert np.all(np.diff(zz, axis=1) <= 0)
    fixed = out["expanded"] == 0
    assert np.array_equal(ids[fixed], _numpy_topk(z, k)[fixed])
    # every chosen expert is among the c highest-scoring ones
    rank = np.argsort(np.argsort(-z.astype(np.float64), axis=1, kind="stable"), axis=1)
    assert np.all(np.take_along_axis(rank, ids.astype(np.int64), 1) < out["cstar"][:, None])
    # non-renormalised weights are the plain softmax scores
    raw = oracle.route(z, k, c, eps, tfix, loads_in, renormalize=False)
    sm = np.exp(z.astype(np.float64) - z.max(1, keepdims=True).astype(np.float64))
    sm /= sm.sum(1, keepdims=True)
    np.testing.assert_allclose(raw["weights"], np.take_along_axis(sm, ids.astype(np.int64), 1),
                               atol=1e-12)
    assert np.array_equal(raw["expert_ids"], ids)


def test_separation_chosen_before_unchosen():
    """Inside the working set every chosen expert sorts before every unchosen one
    under (load at that moment, score rank)."""
    E, k, c, T = 8, 2, 5, 300
    z = wl.random_logits(77, T, E, scale=0.3)
    out = oracle.route(z, k, c, 2.0, 0.2, np.zeros(E, np.int32))
    L = np.zeros(E, dtype=np.int64)
    for t in range(T):
        ranked = sorted(range(E), key=lambda i: (-float(z[t, i]), i))
        work = ranked[: out["cstar"][t]]
        chosen = set(out["expert_ids"][t].tolist())
        key = {e: (L[e], work.index(e)) for e in work}
        assert chosen <= set(work)
        assert max(key[e] for e in chosen) < min([key[e] for e in work if e not in chosen],
                                                 default=(math.inf, 0))
        for e in chosen:
            L[e] += 1


def test_split_call_equals_one_call():
    """Routing tokens [0,a) then [a,T) with the counters carried over equals one call."""
    E, k, c, T = 64, 6, 8, 700
    z = wl.random_logits(9, T, E, scale=0.8)
    L0 = np.arange(E, dtype=np.int32) % 5
    whole = oracle.route(z, k, c, 0.6, 0.5, L0)
    a = 233
    first = oracle.route(z[:a], k, c, 0.6, 0.5, L0)
    second = oracle.route(z[a:], k, c, 0.6, 0.5, first["loads"])
    assert np.array_equal(np.vstack([first["expert_ids"], second["expert_ids"]]), whole["expert_ids"])
    assert np.array_equal(second["loads"], whole["loads"])


def test_adjacent_tokens_with_disjoint_working_sets_commute():
    E, k, c = 8, 2, 3
    za = np.array([[5, 4.9, 4.8, 0, 0, 0, 0, 0]], dtype=np.float32)
    zb = np.array([[0, 0, 0, 0, 0, 4.8, 4.9, 5]], dtype=np.float32)
    L0 = np.array([2, 0, 1, 0, 0, 1, 0, 2], dtype=np.int32)
    ab = oracle.route(np.vstack([za, zb]), k, c, 0.99, 0.5, L0)
    ba = oracle.route(np.vstack([zb, za]), k, c, 0.99, 0.5, L0)
    assert np.array_equal(ab["loads"], ba["loads"])
    assert np.array_equal(ab["expert_ids"][0], ba["expert_ids"][1])
    assert ab["expert_ids"][0].tolist() == [1, 2]      # lighter experts of {0,1,2}


# ----------------------------------------------------------------- dispatch --

@pytest.mark.parametrize("E,k,T", [(8, 2, 1000), (64, 6, 777), (3, 1, 1), (4, 2, 0)])
def test_dispatch_is_the_stable_counting_sort(E, k, T):
    z = wl.random_logits(21, T, E)
    out = oracle.route(z, k, min(E, k + 2), 0.7, 0.5, np.zeros(E, np.int32))
    flat = out["expert_ids"].ravel()
    assert np.array_equal(out["permutation"], np.argsort(flat, kind="stable").astype(np.int32))
    counts = np.bincount(flat, minlength=E)
    assert np.array_equal(out["expert_offsets"], np.concatenate([[0], np.cumsum(counts)]))
    assert out["expert_offsets"][E] == T * k


# --------------------------------------------------------------------- gate --

@pytest.mark.parametrize("dtype", [wl.DTYPE_F32, wl.DTYPE_BF16])
def test_gate_matches_numpy_fp64_matmul(dtype):
    rng = np.random.default_rng(31)
    hidden, w = wl.make_gate(rng, 37, 200, 11, dtype, bias=np.linspace(-2, 2, 11))
    z = oracle.gate(hidden, w, dtype)
    if dtype == wl.DTYPE_BF16:
        h64, w64 = wl.bf16_bits_to_f32(hidden).astype(np.float64), wl.bf16_bits_to_f32(w).astype(np.float64)
    else:
        h64, w64 = hidden.astype(np.float64), w.astype(np.float64)
    np.testing.assert_allclose(z, h64 @ w64.T, rtol=0, atol=1e-12)
    # orientation: expert e uses row e of W (a transposed operand would fail here)
    assert abs(z[3, 5] - float(h64[3] @ w64[5])) < 1e-12


def test_gate_bias_recipe_places_the_bias():
    """The generator's pinv construction really lands the requested bias on the logits."""
    rng = np.random.default_rng(32)
    bias = np.array([3.0, 0, 0, -2.0, 0, 0, 0, 0])
    hidden, w = wl.make_gate(rng, 4000, 256, 8, wl.DTYPE_F32, bias=bias)
    z = oracle.gate(hidden, w, wl.DTYPE_F32)
    np.testing.assert_allclose(z.mean(0), bias, atol=0.03)


# ------------------------------------------------- binary32 building blocks --

def test_exp_canon_against_libm():
    xs = np.concatenate([np.linspace(-80, 0, 4001), -np.logspace(-8, 1.9, 500)]).astype(np.float32)
    got = np.array([oracle.exp_canon(x) for x in xs], dtype=np.float64)
    want = np.exp(xs.astype(np.float64))
    assert np.max(np.abs(got / want - 1.0)) < 2.5e-7
    assert oracle.exp_canon(0.0) == 1.0
    assert oracle.exp_canon(-80.0) > 0.0
    # monotone on a fine grid near 0 (ordering of scores follows ordering of logits)
    fine = -np.arange(0, 2000, dtype=np.float32) * np.float32(1e-4)
    vals = [oracle.exp_canon(x) for x in fine]
    assert all(a >= b for a, b in zip(vals, vals[1:]))


def test_tree_sum_shape():
    # integers: any order gives the exact sum
    v = np.arange(1, 12, dtype=np.float32)
    assert oracle.tree_sum(v) == 66.0
    # the stated tree for 4 values is (v0+v2)+(v1+v3); these values tell it apart
    # from left-to-right and from (v0+v1)+(v2+v3)
    v = np.array([1.0, 2.0 ** -24, 2.0 ** -24, 2.0 ** -24], dtype=np.float32)
    f = np.float32
    assert oracle.tree_sum(v) == float((f(v[0]) + f(v[2])) + (f(v[1]) + f(v[3])))
    w = np.array([2.0 ** 24, 1.0, -(2.0 ** 24), 1.0], dtype=np.float32)
    assert oracle.tree_sum(w) == 2.0          # (w0+w2)+(w1+w3); left-to-right gives 1
    # padding with zeros does not change the result
    assert oracle.tree_sum(np.concatenate([w, np.zeros(3, np.float32)])) == oracle.tree_sum(
        np.concatenate([w, np.zeros(4, np.float32)]))


@pytest.mark.parametrize("shape", ["mixtral", "deepseek"])
def test_binary32_reading_agrees_with_literal_fp64(shape):
    """On tokens whose thresholds are not within rounding distance, the binary32
    decision arithmetic and the paper's formulas in fp64 route identically."""
    s = wl.SHAPES[shape]
    z = wl.random_logits(55, 3000, s.E, scale=0.9)
    for layer in (0, s.layers // 2):
        eps, tfix = wl.thresholds(shape, layer)
        ok = _margin_safe(z, s.k, eps, tfix, margin=1e-5)
        a = oracle.route(z[ok], s.k, s.c, eps, tfix, np.zeros(s.E, np.int32))
        b = oracle.route_literal(z[ok].astype(np.float64), s.k, s.c, eps, tfix, np.zeros(s.E, np.int32))
        for key in ("expert_ids", "loads", "expanded", "cstar", "permutation", "expert_offsets"):
            assert np.array_equal(a[key], b[key]), key
        np.testing.assert_allclose(a["weights"], b["weights"], atol=1e-12)
        assert 0 < a["expanded"].mean() < 1          # both branches exercised


def test_argument_errors():
    z = np.zeros((2, 4), dtype=np.float32)
    L = np.zeros(4, np.int32)
    for k, c, eps, tfix in [(0, 2, .5, .5), (3, 2, .5, .5), (2, 5, .5, .5), (2, 3, 0.0, .5),
                            (2, 3, .5, 0.0), (2, 3, .5, 1.5)]:
        with pytest.raises(ValueError):
            oracle.route(z, k, c, eps, tfix, L)


# ---------------------------------------------------- per-token gate statistics ----

def test_token_stats_closed_forms():
    """Uniform scores: M_k = k/E, H = ln E, every expert in the pool.  Two experts:
    the binary entropy of the logistic function.  One dominant expert: H -> 0."""
    E, k = 8, 2
    r = oracle.token_stats(np.zeros((1, E), np.float32), k, 0.5)
    assert abs(r["topk_mass"][0] - k / E) < 1e-15
    assert abs(r["entropy"][0] - math.log(E)) < 1e-14
    assert r["pool_size"][0] == E
    a = 0.7
    r = oracle.token_stats(np.array([[a, 0.0]], np.float32), 1, 1.0)
    s = 1.0 / (1.0 + math.exp(-float(np.float32(a))))
    assert abs(r["topk_mass"][0] - s) < 1e-15
    assert abs(r["entropy"][0] - (-s * math.log(s) - (1 - s) * math.log(1 - s))) < 1e-14
    assert r["pool_size"][0] == 1          # only the best score reaches 1.0 * s_(1)
    z = np.zeros((1, 16), np.float32)
    z[0, 3] = 60.0
    r = oracle.token_stats(z, 2, 0.5)
    assert r["entropy"][0] < 1e-20 and abs(r["topk_mass"][0] - 1.0) < 1e-15
    assert r["pool_size"][0] == 2          # pool of one, united with the top-2


def test_token_stats_against_scipy():
    from scipy.special import softmax
    from scipy.stats import entropy
    z = wl.random_logits(77, 500, 24, scale=1.7)
    k, tfix = 3, 0.35
    r = oracle.token_stats(z, k, tfix)
    s = softmax(z.astype(np.float64), axis=1)
    np.testing.assert_allclose(r["entropy"], entropy(s, axis=1), rtol=0, atol=1e-12)
    np.testing.assert_allclose(r["topk_mass"], np.sort(s, axis=1)[:, -k:].sum(1), rtol=0, atol=1e-13)
    # pool size by the printed definition, on tokens with no score within 1e-6 of the cut
    cut = tfix * s.max(1, keepdims=True)
    safe = (np.abs(s - cut) > 1e-6 * cut).all(1)
    assert safe.mean() > 0.9
    m = np.maximum((s >= cut).sum(1), k)
    assert np.array_equal(r["pool_size"][safe], m[safe])
    # invariant under a common shift of the logits (exact: 0.5 steps are representable)
    r2 = oracle.token_stats(z + np.float32(4.0), k, tfix)
    np.testing.assert_allclose(r2["entropy"], r["entropy"], atol=1e-6)
    # bounds
    assert (r["entropy"] >= 0).all() and (r["entropy"] <= math.log(24) + 1e-12).all()
    assert (r["topk_mass"] >= k / 24 - 1e-12).all() and (r["topk_mass"] <= 1 + 1e-12).all()


def test_pool_size_is_the_routers_working_set_bound():
    """min(c, m) is the working-set size the router reports for expanded tokens."""
    z = wl.random_logits(78, 2000, 64, scale=0.6)
    k, c, eps, tfix = 6, 10, 0.7, 0.4
    r = oracle.token_stats(z, k, tfix)
    ref = oracle.route(z, k, c, eps, tfix, np.zeros(64, np.int32))
    ex = ref["expanded"].astype(bool)
    assert ex.sum() > 100
    assert np.array_equal(ref["cstar"][ex], np.minimum(c, r["pool_size"][ex]))


# ------------------------------------------------------------ imbalance metrics ----

def test_imbalance_closed_forms():
    """Equal counts: I = 1, MV = 0.  All tokens on one expert: I = E.  One GPU per
    expert: the GPU-level figure is the expert-level one.  Everything on one GPU of
    G: I_gpu = G.  Two experts per GPU with their counts paired up evenly: I_gpu = 1."""
    E = 8
    r = oracle.imbalance(np.full((1, E), 5, np.int32))
    assert r["I"][0] == 1.0 and r["MV"][0] == 0.0 and r["agg"][0] == 1.0
    hot = np.zeros((1, E), np.int32)
    hot[0, 3] = 40
    assert oracle.imbalance(hot)["I"][0] == E
    n = np.array([[7, 1, 4, 4, 2, 6, 8, 0]], np.int32)
    r = oracle.imbalance(n, placement=np.eye(E))
    assert abs(r["I_gpu"][0] - r["I"][0]) < 1e-15 and abs(r["I"][0] - 8 / 4.0) < 1e-15
    one = np.zeros((4, E))
    one[2] = 1.0
    assert abs(oracle.imbalance(n, placement=one)["I_gpu"][0] - 4.0) < 1e-15
    pairs = np.zeros((4, E))
    for g, (a, b) in enumerate([(0, 1), (2, 3), (4, 5), (6, 7)]):
        pairs[g, a] = pairs[g, b] = 1.0
    assert abs(oracle.imbalance(n, placement=pairs)["I_gpu"][0] - 1.0) < 1e-15
    # replication: every expert split evenly over all GPUs balances any counts
    assert abs(oracle.imbalance(n, placement=np.full((4, E), 0.25))["I_gpu"][0] - 1.0) < 1e-15
    # an empty layer counts as balanced
    assert oracle.imbalance(np.zeros((1, E), np.int32))["I"][0] == 1.0


def test_imbalance_against_numpy_and_weights():
    rng = np.random.default_rng(5)
    L, E, G = 6, 16, 4
    n = rng.integers(0, 500, size=(L, E)).astype(np.int32)
    A = rng.random((G, E))
    A /= A.sum(0, keepdims=True)
    w = rng.random(L)
    w /= w.sum()
    r = oracle.imbalance(n, placement=A, weights=w)
    I = n.max(1) / n.mean(1)
    ng = n.astype(np.float64) @ A.T
    Ig = ng.max(1) / ng.mean(1)
    np.testing.assert_allclose(r["I"], I, rtol=1e-14)
    np.testing.assert_allclose(r["MV"], I - 1, rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(r["I_gpu"], Ig, rtol=1e-13)
    np.testing.assert_allclose(r["agg"], [w @ I, w @ Ig], rtol=1e-13)
    # default weights: the plain mean over layers
    np.testing.assert_allclose(oracle.imbalance(n)["agg"][0], I.mean(), rtol=1e-14)
    # bounds with rho = E / G experts per GPU under a pure placement of equal sizes:
    # I / rho... the most loaded GPU holds at least the most loaded expert
    pure = np.zeros((G, E))
    pure[np.arange(E) % G, np.arange(E)] = 1.0
    rp = oracle.imbalance(n, placement=pure)
    assert (rp["I_gpu"] >= rp["I"] / (E // G) - 1e-12).all() and (rp["I_gpu"] <= rp["I"] + 1e-12).all()


def test_percentiles_hand_values_and_library():
    """Worked by hand: five values, positions h = 4q/100.  P50 is the middle value,
    P95 sits 0.8 of the way from the 4th to the 5th, P25 is the 2nd, P0/P100 the ends.
    Then against the numerical library's default percentile on random data, and the
    properties that pin the definition: monotone in q, invariant under permutation, a
    constant list gives the constant, two values interpolate linearly."""
    v = [3.0, 1.0, 10.0, 2.0, 4.0]                       # sorted: 1 2 3 4 10
    got = oracle.percentiles(v, [0, 25, 50, 95, 100, 10])
    np.testing.assert_allclose(got, [1.0, 2.0, 3.0, 4.0 + 0.8 * 6.0, 10.0, 1.4], rtol=0, atol=1e-14)
    rng = np.random.default_rng(11)
    for n in (1, 2, 7, 100, 1001):
        x = rng.random(n) * 9 + 1
        q = np.array([0, 1, 33.3, 50, 95, 99.9, 100])
        np.testing.assert_allclose(oracle.percentiles(x, q), np.percentile(x, q), rtol=1e-14)
        np.testing.assert_allclose(oracle.percentiles(x[::-1], q), oracle.percentiles(x, q), rtol=0)
        assert np.all(np.diff(oracle.percentiles(x, np.linspace(0, 100, 41))) >= 0)
    assert np.all(oracle.percentiles([2.5] * 9, [0, 50, 95]) == 2.5)
    np.testing.assert_allclose(oracle.percentiles([1.0, 3.0], [50, 95]), [2.0, 2.9], atol=1e-15)
    with pytest.raises(ValueError):
        oracle.percentiles([1.0], [101])
    with pytest.raises(ValueError):
        oracle.percentiles([], [50])


# ----------------------------------------------------------- RANDOM trimming ----

def test_philox_known_answers():
    with open(os.path.join(os.path.dirname(__file__), "golden", "philox4x32_10_kat.json")) as f:
        kat = json.load(f)["vectors"]
    for v in kat:
        out = oracle.philox4x32([int(x, 16) for x in v["ctr"]], [int(x, 16) for x in v["key"]])
        assert [f"{int(x):08x}" for x in out] == v["out"]


def test_sample_ranks_by_hand_and_properties():
    # seed 0, stream 0, token 0: the stream starts 6627e8d5, e169c58d (first vector
    # above).  m = 3, c = 2: draw 0 swaps position 0 with 0 + floor(0.3990 * 3) = 1,
    # draw 1 swaps position 1 with 1 + floor(0.8805 * 2) = 2: [0,1,2] -> [1,0,2] -> [1,2,0]
    assert oracle.sample_ranks(3, 2, 0, 0, 0).tolist() == [1, 2]
    # fifth draw comes from the second block (counter word 3 = 1)
    blk1 = oracle.philox4x32([7, 0, 3, 1], [11, 0])
    r = oracle.sample_ranks(200, 5, 11, 3, 7)
    assert len(set(r.tolist())) == 5 and (np.diff(r) > 0).all() and r.min() >= 0 and r.max() < 200
    arr = list(range(200))
    blk0 = oracle.philox4x32([7, 0, 3, 0], [11, 0])
    for i, w in enumerate(list(blk0) + [blk1[0]]):
        j = i + ((int(w) * (200 - i)) >> 32)
        arr[i], arr[j] = arr[j], arr[i]
    assert sorted(arr[:5]) == r.tolist()
    # token index and seed are 64-bit: the high halves reach the generator
    assert oracle.sample_ranks(50, 4, 1 << 40, 0, 5).tolist() != oracle.sample_ranks(50, 4, 0, 0, 5).tolist()
    assert oracle.sample_ranks(50, 4, 9, 0, 1 << 33).tolist() != oracle.sample_ranks(50, 4, 9, 0, 0).tolist()


def test_sample_ranks_uniform():
    """Every position is drawn with probability c/m and every pair equally often
    (chi-square against the uniform law, fixed seed)."""
    m, c, n = 10, 3, 30000
    single = np.zeros(m)
    pair = np.zeros((m, m))
    for t in range(n):
        r = oracle.sample_ranks(m, c, 2025, 1, t)
        single[r] += 1
        for a, b in itertools.combinations(r.tolist(), 2):
            pair[a, b] += 1
    exp1 = n * c / m
    chi1 = ((single - exp1) ** 2 / exp1).sum()
    assert chi1 < 27.9                      # 9 degrees of freedom, p = 0.001
    iu = np.triu_indices(m, 1)
    exp2 = n * 3 / 45.0                     # 3 pairs per sample, 45 possible pairs
    chi2 = ((pair[iu] - exp2) ** 2 / exp2).sum()
    assert chi2 < 78.8                      # 44 degrees of freedom, p = 0.001


def test_random_trimming_reduces_to_top_when_nothing_is_trimmed():
    z = wl.random_logits(91, 1500, 16, scale=1.2)
    L0 = np.arange(16, dtype=np.int32) % 4
    # pool never larger than c = E; and a threshold that no token fails
    for k, c, eps, tfix in [(2, 16, 2.0, 0.05), (3, 16, 0.8, 0.3), (2, 5, 1e-6, 0.01)]:
        a = oracle.route(z, k, c, eps, tfix, L0)
        b = oracle.route_random(z, k, c, eps, tfix, L0, seed=77)
        for key in ("expert_ids", "loads", "permutation", "expert_offsets", "expanded", "cstar"):
            assert np.array_equal(a[key], b[key]), key
        np.testing.assert_allclose(a["weights"], b["weights"], atol=0)


def test_random_trimming_against_brute_force():
    """Tiny shapes: Algorithm 1 re-enacted in Python on top of three separately pinned
    pieces (branch flag, pool size, sampled positions); the k least-loaded candidates by
    sorting (load, score rank) tuples."""
    rng = np.random.default_rng(3)
    sampled_tokens = 0
    top_missing = 0
    both_branches = [0, 0]
    for trial in range(60):
        E = int(rng.integers(4, 10))
        k = int(rng.integers(1, 4))
        c = int(rng.integers(k, min(E, k + 3) + 1))
        T = 40
        z = wl.random_logits(1000 + trial, T, E, scale=0.4)
        eps, tfix = (0.95, 0.2) if trial % 2 else (0.6, 0.5)
        # tokens whose thresholds are not within rounding: the branch flag and the pool
        # size then follow from a plain numpy softmax, not from the code under test
        z = z[_margin_safe(z, k, eps, tfix)]
        T = len(z)
        L = rng.integers(0, 3, E).astype(np.int64)
        seed, stream, off = 1234 + trial, trial % 3, 10 ** 10 * trial
        ref = oracle.route_random(z, k, c, eps, tfix, L.astype(np.int32), seed, stream, off)
        s_all = np.exp(z.astype(np.float64) - z.astype(np.float64).max(1, keepdims=True))
        s_all /= s_all.sum(1, keepdims=True)
        for t in range(T):
            order = np.argsort(-z[t], kind="stable")
            mass = s_all[t, order[:k]].sum()
            expanded = not mass >= eps
            both_branches[int(expanded)] += 1
            if not expanded:
                A = order[:k].tolist()
            else:
                m = max(k, int((s_all[t] >= tfix * s_all[t].max()).sum()))
                if m > c:
                    ranks = oracle.sample_ranks(m, c, seed, stream, off + t).tolist()
                    sampled_tokens += 1
                    top_missing += 0 not in ranks
                else:
                    ranks = list(range(m))
                keyed = sorted((int(L[order[r]]), r) for r in ranks)[:k]
                A = [int(order[r]) for r in sorted(r for _, r in keyed)]
            assert ref["expert_ids"][t].tolist() == A, (trial, t)
            L[A] += 1
        assert np.array_equal(ref["loads"], L)
    assert sampled_tokens > 200 and top_missing > 20     # the best expert is not protected
    assert min(both_branches) > 200


def test_random_trimming_threshold_equalities():
    """The two non-strict comparisons of the expansion rule under RANDOM trimming.
    (a) Top-k mass exactly at eps_high with a pool larger than c: the token keeps its
    top-k whatever the seed (a strict test would sample and send it to the idle experts).
    (b) A score exactly at the cut-off belongs to the pool: with k = c = 1 the pool of two
    is sampled, and for a seed whose (separately pinned) draw takes position 1 the token
    goes to the second expert; a strict cut would leave a pool of one and expert 0."""
    z = np.zeros((1, 4), np.float32)                       # four equal scores of 0.25
    for seed in range(20):
        out = oracle.route_random(z, 2, 3, 0.5, 0.5, np.array([7, 7, 0, 0], np.int32), seed)
        assert out["expert_ids"].tolist() == [[0, 1]] and not out["expanded"][0]
    zb = np.log(np.array([[1.0, 1.0, 0.5, 0.5]])).astype(np.float32)
    picks = set()
    for seed in range(40):
        pos = int(oracle.sample_ranks(2, 1, seed, 0, 0)[0])
        out = oracle.route_random(zb, 1, 1, 0.99, 1.0, np.zeros(4, np.int32), seed)
        assert out["expert_ids"].tolist() == [[pos]], seed
        picks.add(pos)
    assert picks == {0, 1}


@pytest.mark.parametrize("case", [c for c in _cases() if c["c"] >= c["E"] or
                                  c["name"] in ("mass_equal_to_threshold", "score_equal_to_cutoff")],
                         ids=lambda c: c["name"])
def test_hand_cases_under_random_trimming(case):
    """Where the pool cannot exceed c nothing is sampled, so the hand-worked results hold
    for RANDOM trimming as they stand (Algorithm 1: both modes keep a pool of at most c)."""
    logits = np.log(np.array(case["p"], dtype=np.float64)).astype(np.float32)
    out = oracle.route_random(logits, case["k"], case["c"], case["eps_high"], case["t_fix"],
                              np.array(case["loads_in"], np.int32), seed=99)
    assert out["expert_ids"].tolist() == case["expert_ids"]
    assert out["loads"].tolist() == case["loads_out"]
    assert out["expanded"].tolist() == case["expanded"]


def test_random_trimming_split_call():
    z = wl.random_logits(92, 600, 12, scale=0.3)
    L0 = np.zeros(12, np.int32)
    whole = oracle.route_random(z, 2, 4, 2.0, 0.01, L0, seed=5, stream=2, token_offset=1000)
    a = oracle.route_random(z[:250], 2, 4, 2.0, 0.01, L0, seed=5, stream=2, token_offset=1000)
    b = oracle.route_random(z[250:], 2, 4, 2.0, 0.01, a["loads"], seed=5, stream=2, token_offset=1250)
    assert np.array_equal(np.vstack([a["expert_ids"], b["expert_ids"]]), whole["expert_ids"])
    assert np.array_equal(b["loads"], whole["loads"])
    other = oracle.route_random(z, 2, 4, 2.0, 0.01, L0, seed=6, stream=2, token_offset=1000)
    assert not np.array_equal(other["expert_ids"], whole["expert_ids"])


def test_oracle_runs_clean_under_sanitizers(tmp_path):
    """The oracle compiled with -fsanitize=address,undefined, driven over the hand-worked
    cases and over shapes at the limits of its arguments (one expert, k = E = 256, no
    tokens): no out-of-bounds access, no undefined operation, and the hand cases still
    come out as worked."""
    import shutil
    import subprocess
    if shutil.which("gcc") is None:
        pytest.skip("no gcc")
    here = os.path.dirname(os.path.abspath(__file__))
    root = os.path.dirname(here)
    lines = []
    for c in _cases():
        p = np.array(c["p"], dtype=np.float64)
        ids = np.array(c["expert_ids"], dtype=np.int64)
        lines.append(" ".join(map(str, [c["E"], c["k"], c["c"], c["eps_high"], c["t_fix"], p.shape[0]]
                                   + list(c["loads_in"]) + [repr(float(x)) for x in p.ravel()]
                                   + list(ids.ravel()))))
    cases = tmp_path / "cases.txt"
    cases.write_text("\n".join(lines) + "\n")
    exe = tmp_path / "oracle_san"
    cmd = ["gcc", "-O1", "-g", "-std=c11", "-ffp-contract=off", "-fno-fast-math",
           "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-static-libasan",
           "-o", str(exe), os.path.join(here, "oracle_sanitize_driver.c"),
           os.path.join(root, "oracle", "laser_oracle.c"), "-lm"]
    built = subprocess.run(cmd, capture_output=True, text=True)
    if built.returncode != 0 and "asan" in built.stderr.lower():
        pytest.skip("no sanitizer runtime for this gcc: " + built.stderr[-200:])
    assert built.returncode == 0, built.stderr
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:verify_asan_link_order=0",
               UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1")
    run = subprocess.run([str(exe), str(cases)], capture_output=True, text=True, env=env, timeout=300)
    assert run.returncode == 0, run.stdout[-2000:] + run.stderr[-4000:]
    assert run.stdout.strip().endswith("clean")
