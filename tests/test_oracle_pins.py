"""Pins of the fp64 CPU oracle against things it did not compute itself.

Paper-printed parameter counts, hand-worked examples (tests/golden), closed
forms, numpy's matmul on merged weights, and the invariants the method fixes.
Each pin is chosen so that one plausible mistake in the oracle (a dropped
term, a transposed operand, a wrong gather index, a wrong mask) fails it.
"""
import math
import os

import numpy as np
import pytest

import oracle
from oracle import Adapters

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def read_golden(name):
    rec = {}
    with open(os.path.join(GOLD, name)) as f:
        for line in f:
            line = line.split("#", 1)[0].strip()
            if not line:
                continue
            key, vals = line.split(":", 1)
            rec[key.strip()] = np.array([float(v) for v in vals.split()], dtype=np.float64)
    return rec


def f32_to_bf16_bits(x):
    """Round-to-nearest-even bf16 bit patterns of an fp32 array (test-side helper)."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    return (((u + 0x7FFF + ((u >> 16) & 1)) >> 16) & 0xFFFF).astype(np.uint16)


def bf16_bits_to_f64(b):
    return (b.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def single_tenant(A, B, site, d1s=None):
    """Adapters with one tenant whose (A, B) sit at `site`; the other sites get rank-matching zeros."""
    r = A.shape[1]
    As, Bs = [], []
    for m in range(7):
        if m == site:
            As.append(np.ascontiguousarray(A))
            Bs.append(np.ascontiguousarray(B))
        else:
            As.append(np.zeros((1, r), dtype=A.dtype))
            Bs.append(np.zeros((r, 1), dtype=A.dtype))
    return Adapters([As], [Bs], [r])


def random_adapters(rng, T, ranks, d, F, dtype=np.float64, scale=1.0):
    A, B = [], []
    for t in range(T):
        At, Bt = [], []
        for m in range(7):
            d1, d2 = oracle.site_dims(m, d, F)
            At.append((rng.standard_normal((d1, ranks[t])) * scale).astype(dtype))
            Bt.append((rng.standard_normal((ranks[t], d2)) * scale).astype(dtype))
        A.append(At)
        B.append(Bt)
    return Adapters(A, B, list(ranks))


# --------------------------------------------------------------------------- paper-printed values
def test_param_counts_match_the_paper():
    g = read_golden("param_counts.txt")
    d, F, L, r = (int(v) for v in g["shape_7b"])
    lora, router, max_act = oracle.param_counts(d, F, L, r)
    assert round(lora / 1e6, 1) == g["lora_millions"][0]
    assert round((lora + router) / 1e6, 1) == g["tunable_millions"][0]
    assert round(max_act / 1e6, 1) == g["max_activated_millions"][0]
    # closed forms: 4 attention sites of (d+d) and 3 FFN sites of (d+F), router d x 7 without bias
    assert lora == L * r * (4 * 2 * d + 3 * (d + F))
    assert router == L * d * 7
    # a second active expert per layer, or a router bias, would no longer print as 16.4M / 80.9M
    assert round((max_act + L * r * (d + F)) / 1e6, 1) != g["max_activated_millions"][0]
    assert round((lora + router + L * d) / 1e6, 1) != g["tunable_millions"][0]


def test_site_dims():
    assert [oracle.site_dims(m, 4096, 11008) for m in range(7)] == [
        (4096, 4096)] * 4 + [(4096, 11008), (4096, 11008), (11008, 4096)]


# --------------------------------------------------------------------------- hand-worked Eq. 1
@pytest.mark.parametrize("site", [0, 3, 6])
def test_worked_linear_example(site):
    g = read_golden("worked_examples.txt")
    W_math = g["lin_W_math"].reshape(2, 3)
    W = np.ascontiguousarray(W_math.T)  # storage [d2, d1]
    ad = single_tenant(g["lin_A"].reshape(2, 1), g["lin_B"].reshape(1, 3), site)
    X = np.stack([g["lin_x0"], g["lin_x1"]])
    tid = [0, 0]
    y = oracle.routed_linear(X, W, ad, site, tid, [site, (site + 1) % 7])
    np.testing.assert_array_equal(y[0], g["lin_y0_routed"])
    np.testing.assert_array_equal(y[1], g["lin_y1_base"])
    y = oracle.routed_linear(X, W, ad, site, tid, [(site + 2) % 7, site], bias=g["lin_bias"])
    np.testing.assert_array_equal(y[0], g["lin_y0_base"] + g["lin_bias"])
    np.testing.assert_array_equal(y[1], g["lin_y1_routed"] + g["lin_bias"])
    y = oracle.routed_linear(X[:1], W, ad, site, [0], [site], bias=g["lin_bias"])
    np.testing.assert_array_equal(y[0], g["lin_y0_routed_bias"])


def test_unit_vectors_read_rows_of_W_and_A():
    """x = e_i returns row i of the paper's W (and of A through B = I): pins every index order."""
    d1, d2, r = 5, 4, 3
    W_math = np.arange(d1 * d2, dtype=np.float64).reshape(d1, d2) * 10 + 1
    A = np.arange(d1 * r, dtype=np.float64).reshape(d1, r) + 100
    B = np.zeros((r, d2))
    B[0, 1], B[1, 3], B[2, 0] = 1.0, 2.0, -1.0  # t0 -> y1, 2*t1 -> y3, -t2 -> y0
    ad = single_tenant(A, B, 2)
    y = oracle.routed_linear(np.eye(d1), np.ascontiguousarray(W_math.T), ad, 2, [0] * d1, [2] * d1)
    for i in range(d1):
        expect = W_math[i].copy()
        expect[1] += A[i, 0]
        expect[3] += 2 * A[i, 1]
        expect[0] -= A[i, 2]
        np.testing.assert_array_equal(y[i], expect)


# --------------------------------------------------------------------------- library second opinion
@pytest.mark.parametrize("storage", ["f64", "f32", "bf16"])
def test_merged_weights_identity_with_numpy(storage):
    """Eq. 1 equals x (W + A B): numpy's matmul on the merged matrix is the second opinion."""
    rng = np.random.default_rng(7)
    M, d1, d2, r = 6, 48, 40, 5
    X, Wm = rng.standard_normal((M, d1)), rng.standard_normal((d1, d2))
    A, B = rng.standard_normal((d1, r)), rng.standard_normal((r, d2))
    if storage == "f32":
        X, Wm, A, B = (a.astype(np.float32) for a in (X, Wm, A, B))
        wide = lambda a: a.astype(np.float64)
    elif storage == "bf16":
        X, Wm, A, B = (f32_to_bf16_bits(a) for a in (X, Wm, A, B))
        wide = bf16_bits_to_f64
    else:
        wide = lambda a: a
    ad = single_tenant(A, B, 4)
    y = oracle.routed_linear(X, np.ascontiguousarray(Wm.T), ad, 4, [0] * M, [4] * M)
    ref = wide(X) @ (wide(Wm) + wide(A) @ wide(B))
    np.testing.assert_allclose(y, ref, rtol=0, atol=1e-12 * np.abs(ref).max())


def test_bf16_widening_known_patterns():
    bits = np.array([[0x3F80, 0xC000, 0x0000, 0x3DCD]], dtype=np.uint16)  # 1, -2, 0, 0.10009765625
    W = np.array([[0x3F80, 0, 0, 0], [0, 0x3F80, 0, 0], [0, 0, 0x3F80, 0], [0, 0, 0, 0x3F80]], dtype=np.uint16)
    ad = single_tenant(np.zeros((4, 1), np.uint16), np.zeros((1, 4), np.uint16), 0)
    y = oracle.routed_linear(bits, W, ad, 0, [0], [1])
    np.testing.assert_array_equal(y[0], [1.0, -2.0, 0.0, 0.10009765625])


# --------------------------------------------------------------------------- invariants of the routed linear
def _random_problem(seed, M=5, T=3, d=12, F=20, ranks=(2, 4, 3)):
    rng = np.random.default_rng(seed)
    ad = random_adapters(rng, T, ranks, d, F)
    W = [rng.standard_normal(oracle.site_dims(m, d, F)[::-1]) for m in range(7)]
    tid = rng.integers(0, T, M)
    route = rng.integers(0, 7, M)
    return rng, ad, W, tid, route, d, F


def test_zero_B_reproduces_the_base_linear_exactly():
    rng, ad, W, tid, route, d, F = _random_problem(1)
    for t in range(3):
        for m in range(7):
            ad.B[t][m][...] = 0.0
    for site in range(7):
        d1, d2 = oracle.site_dims(site, d, F)
        X = rng.standard_normal((5, d1))
        y = oracle.routed_linear(X, W[site], ad, site, tid, [site] * 5)
        base = oracle.routed_linear(X, W[site], ad, site, tid, [(site + 1) % 7] * 5)
        np.testing.assert_array_equal(y, base)
        np.testing.assert_allclose(base, X @ W[site].T, rtol=0, atol=1e-12)


def test_sparse_top1_equals_dense_one_hot_mixture():
    rng, ad, W, tid, route, d, F = _random_problem(2)
    gate = np.zeros((5, 7))
    gate[np.arange(5), route] = 1.0
    for site in range(7):
        d1, _ = oracle.site_dims(site, d, F)
        X = rng.standard_normal((5, d1))
        sparse = oracle.routed_linear(X, W[site], ad, site, tid, route)
        dense = oracle.routed_linear_dense(X, W[site], ad, site, tid, gate)
        np.testing.assert_allclose(sparse, dense, rtol=0, atol=1e-13 * np.abs(dense).max())
    # summed over the sites, each request receives exactly one LoRA delta
    hits = sum(int(route[b] == s) for b in range(5) for s in range(7))
    assert hits == 5


def test_top_k_selection_against_a_stable_sort_and_its_special_cases():
    rng = np.random.default_rng(12)
    logits = rng.standard_normal((200, 7))
    logits[:40] = np.round(logits[:40] * 2) / 2  # many exact ties
    for k in range(1, 7):
        route, gap = oracle.select_topk(logits, k)
        for b in range(200):
            order = np.argsort(-logits[b], kind="stable")  # ties keep the lower index first
            chosen = {int(j) for j in order[:k]}
            got = {m for m in range(7) if oracle.route_has(route[b], m)}
            assert got == chosen
            assert gap[b] == logits[b][order[k - 1]] - logits[b][order[k]]
            assert (route[b] < 7) == (k == 1)
    r1, g1 = oracle.select_topk(logits, 1)
    r0, g0 = oracle.select(logits)
    np.testing.assert_array_equal(r1, r0)
    np.testing.assert_array_equal(g1, g0)
    assert not any(oracle.route_has(255, m) for m in range(7))  # "no route" selects nothing


def test_set_valued_routes_equal_the_dense_mixture_with_a_multi_hot_gate():
    """k > 1 (the experiments' text): the chosen sites' LoRA terms are added unweighted."""
    rng, ad, W, tid, _, d, F = _random_problem(4)
    logits = rng.standard_normal((5, 7))
    for k in (2, 3, 6):
        route, _ = oracle.select_topk(logits, k)
        gate = np.array([[1.0 if oracle.route_has(route[b], m) else 0.0 for m in range(7)] for b in range(5)])
        assert (gate.sum(axis=1) == k).all()
        for site in range(7):
            d1, _ = oracle.site_dims(site, d, F)
            X = rng.standard_normal((5, d1))
            sparse = oracle.routed_linear(X, W[site], ad, site, tid, route)
            dense = oracle.routed_linear_dense(X, W[site], ad, site, tid, gate)
            np.testing.assert_allclose(sparse, dense, rtol=0, atol=1e-13 * np.abs(dense).max())
            # and a request's term at this site is the same as with the single-site route
            single = oracle.routed_linear(X, W[site], ad, site, tid, np.full(5, site, dtype=np.uint8))
            base = oracle.routed_linear(X, W[site], ad, site, tid, np.full(5, 255, dtype=np.uint8))
            for b in range(5):
                np.testing.assert_array_equal(sparse[b], single[b] if gate[b, site] else base[b])


def test_gate_only_at_routed_site_and_own_tenant():
    """Tenant t's B is the constant t+1 and A sums x: the delta reveals which tenant and which rows were used."""
    T, d, F, M = 4, 6, 6, 8
    A = [[np.ones((oracle.site_dims(m, d, F)[0], 1)) for m in range(7)] for _ in range(T)]
    B = [[np.full((1, oracle.site_dims(m, d, F)[1]), float(t + 1)) for m in range(7)] for t in range(T)]
    ad = Adapters(A, B, [1] * T)
    rng = np.random.default_rng(3)
    X = rng.integers(-3, 4, (M, d)).astype(np.float64)
    W = np.zeros((d, d))
    tid = np.array([3, 1, 0, 2, 2, 0, 1, 3])
    route = np.array([2, 2, 5, 2, 0, 2, 6, 2])
    y = oracle.routed_linear(X, W, ad, 2, tid, route)
    for b in range(M):
        expect = (tid[b] + 1) * X[b].sum() if route[b] == 2 else 0.0
        np.testing.assert_array_equal(y[b], np.full(d, expect))


def test_delta_is_linear_in_B_and_has_rank_at_most_r():
    rng = np.random.default_rng(4)
    d1, d2, r = 16, 14, 3
    A, B1, B2 = rng.standard_normal((d1, r)), rng.standard_normal((r, d2)), rng.standard_normal((r, d2))
    W = rng.standard_normal((d2, d1))
    I = np.eye(d1)
    base = oracle.routed_linear(I, W, single_tenant(A, B1, 0), 0, [0] * d1, [1] * d1)
    f = lambda Bm: oracle.routed_linear(I, W, single_tenant(A, Bm, 0), 0, [0] * d1, [0] * d1) - base
    np.testing.assert_allclose(f(2 * B1 - 3 * B2), 2 * f(B1) - 3 * f(B2), atol=1e-12)
    s = np.linalg.svd(f(B1), compute_uv=False)
    assert (s > 1e-10 * s[0]).sum() == r


def test_rows_are_independent_and_row_to_req_maps_rows_to_requests():
    rng, ad, W, tid, route, d, F = _random_problem(5)
    X = rng.standard_normal((5, d))
    y = oracle.routed_linear(X, W[1], ad, 1, tid, route)
    perm = rng.permutation(5)
    yp = oracle.routed_linear(X[perm], W[1], ad, 1, tid[perm], route[perm])
    np.testing.assert_array_equal(yp, y[perm])
    # several rows per request (prefill tokens, beams): every row uses its request's tenant and route
    r2r = np.array([4, 4, 0, 2, 2, 2, 1])
    Xm = rng.standard_normal((7, d))
    ym = oracle.routed_linear(Xm, W[1], ad, 1, tid, route, row_to_req=r2r)
    for m in range(7):
        one = oracle.routed_linear(Xm[m:m + 1], W[1], ad, 1, tid[r2r[m]:r2r[m] + 1], route[r2r[m]:r2r[m] + 1])
        np.testing.assert_array_equal(ym[m], one[0])
    # sampled rows equal the same rows of the full result
    sub = oracle.routed_linear(Xm, W[1], ad, 1, tid, route, row_to_req=r2r, rows=[5, 0, 3])
    np.testing.assert_array_equal(sub, ym[[5, 0, 3]])


def test_bad_indices_are_reported():
    rng, ad, W, tid, route, d, F = _random_problem(6)
    X = rng.standard_normal((5, d))
    with pytest.raises(ValueError):
        oracle.routed_linear(X, W[0], ad, 0, [0, 1, 2, 3, 0], [0] * 5)  # tenant 3 of 3
    with pytest.raises(ValueError):
        oracle.routed_linear(X, W[0], ad, 0, tid, route, row_to_req=[0, 1, 2, 3, 5])
    with pytest.raises(ValueError):
        oracle.routed_linear(X, W[0], ad, 7, tid, route)


# --------------------------------------------------------------------------- pooler, activation, router
def test_worked_router_example():
    g = read_golden("worked_examples.txt")
    H = g["rt_H"].reshape(3, 2)
    Wr = np.ascontiguousarray(g["rt_Wr_cols"].reshape(1, 7, 2))
    for kind, name in [(oracle.POOL_MEAN, "mean"), (oracle.POOL_LAST, "last"), (oracle.POOL_MAX, "max")]:
        np.testing.assert_array_equal(oracle.pool(H, [0], [3], kind)[0], g[f"rt_{name}"])
        res = oracle.route(H, [0], [3], [0], Wr, kind, oracle.ACT_IDENTITY)
        np.testing.assert_array_equal(res.logits[0], g[f"rt_logits_{name}"])
        assert res.route[0] == int(g[f"rt_route_{name}"][0])
        if f"rt_gap_{name}" in g:
            assert res.gap[0] == g[f"rt_gap_{name}"][0]
    res = oracle.route(H, [0], [3], [0], Wr, oracle.POOL_MEAN, oracle.ACT_RELU)
    np.testing.assert_array_equal(res.logits[0], g["rt_logits_mean_relu"])
    assert res.route[0] == int(g["rt_route_mean_relu"][0]) and res.gap[0] == 0.0  # exact tie: lowest index
    res = oracle.route(H, [0], [3], [0], Wr, oracle.POOL_MEAN, oracle.ACT_TANH)
    t3, t2 = math.tanh(3.0), math.tanh(-2.0)
    np.testing.assert_allclose(res.logits[0], [t3, t2, t3 + t2, -t3, -t2, 0.5 * (t3 + t2), -2 * t3 - t2], atol=1e-15)
    assert res.route[0] == 0


def test_activation_closed_forms():
    x = np.array([-3.0, -1.0, -0.0, 0.5, 2.0])
    np.testing.assert_array_equal(oracle.activation(x, oracle.ACT_IDENTITY), x)
    np.testing.assert_array_equal(oracle.activation(x, oracle.ACT_RELU), [0, 0, 0, 0.5, 2.0])
    np.testing.assert_allclose(oracle.activation(x, oracle.ACT_TANH), [math.tanh(v) for v in x], atol=1e-16)
    gelu = oracle.activation(x, oracle.ACT_GELU)
    np.testing.assert_allclose(gelu, [v * 0.5 * math.erfc(-v / math.sqrt(2)) for v in x], atol=1e-15)
    # x Phi(x) - (-x) Phi(-x) = x, and GELU(1) = Phi(1) = 0.841344746...
    np.testing.assert_allclose(gelu - oracle.activation(-x, oracle.ACT_GELU), x, atol=1e-15)
    assert abs(oracle.activation([1.0], oracle.ACT_GELU)[0] - 0.8413447460685429) < 1e-15


def test_rational_activation_special_cases():
    x = np.linspace(-2, 2, 9)
    ident = np.zeros(12)
    ident[1] = 1.0  # a_1 = 1, every b = 0  ->  Ra(x) = x
    np.testing.assert_allclose(oracle.activation(x, oracle.ACT_RATIONAL, ident), x, atol=1e-15)
    c = np.zeros(12)
    c[0], c[2], c[6] = 1.0, -2.0, 0.5  # 1 - 2x^2 + 0.5x^6
    c[7], c[9] = 3.0, -1.0  # 3x - x^3 inside the absolute value
    expect = (1 - 2 * x ** 2 + 0.5 * x ** 6) / (1 + np.abs(3 * x - x ** 3))
    np.testing.assert_allclose(oracle.activation(x, oracle.ACT_RATIONAL, c), expect, rtol=1e-14)
    assert (oracle.activation(x, oracle.ACT_RATIONAL, c) != (1 - 2 * x ** 2 + 0.5 * x ** 6) / (1 + 3 * x - x ** 3))[x < 0].any()


def test_pooler_special_cases():
    rng = np.random.default_rng(8)
    d = 10
    H = rng.standard_normal((40, d))
    starts, lens = [3, 20, 39], [9, 1, 1]
    mean, last = oracle.pool(H, starts, lens, oracle.POOL_MEAN), oracle.pool(H, starts, lens, oracle.POOL_LAST)
    np.testing.assert_array_equal(mean[1], H[20])  # n_p = 1: mean = last = the row
    np.testing.assert_array_equal(last[1], H[20])
    np.testing.assert_array_equal(last[0], H[11])  # last valid row, not the last row of H
    np.testing.assert_array_equal(last[2], H[39])
    np.testing.assert_allclose(mean[0], H[3:12].mean(0), atol=1e-15)
    # rows t = 0..n-1 holding the value t: mean (n-1)/2, last n-1, max n-1
    n = 17
    ramp = np.repeat(np.arange(n, dtype=np.float64)[:, None], d, 1)
    Hr = np.concatenate([np.full((5, d), 1e6), ramp, np.full((4, d), -1e6)])
    assert (oracle.pool(Hr, [5], [n], oracle.POOL_MEAN) == (n - 1) / 2).all()
    assert (oracle.pool(Hr, [5], [n], oracle.POOL_LAST) == n - 1).all()
    assert (oracle.pool(Hr, [5], [n], oracle.POOL_MAX) == n - 1).all()
    # constant rows pool to the row
    Hc = np.repeat(rng.standard_normal((1, d)), 6, 0)
    for kind in (oracle.POOL_MEAN, oracle.POOL_LAST, oracle.POOL_MAX):
        np.testing.assert_allclose(oracle.pool(Hc, [0], [6], kind)[0], Hc[0], atol=1e-15)
    with pytest.raises(ValueError):
        oracle.pool(H, [35], [6], oracle.POOL_MEAN)
    with pytest.raises(ValueError):
        oracle.pool(H, [0], [0], oracle.POOL_MEAN)


def test_route_ignores_padding_and_token_order():
    rng = np.random.default_rng(9)
    d, T = 16, 3
    H = rng.standard_normal((50, d))
    Wr = rng.standard_normal((T, 7, d))
    starts, lens, tid = [2, 20, 33], [11, 7, 13], [2, 0, 1]
    ref = oracle.route(H, starts, lens, tid, Wr, oracle.POOL_MEAN, oracle.ACT_GELU)
    H2 = H.copy()
    valid = np.zeros(50, bool)
    for s, n in zip(starts, lens):
        valid[s:s + n] = True
    H2[~valid] = 1e9  # padded rows never enter
    H2[2:13] = H2[2:13][rng.permutation(11)]  # mean pooling does not see token order
    got = oracle.route(H2, starts, lens, tid, Wr, oracle.POOL_MEAN, oracle.ACT_GELU)
    np.testing.assert_array_equal(got.route, ref.route)
    np.testing.assert_allclose(got.logits, ref.logits, atol=1e-12)
    # a valid token does matter
    H3 = H.copy()
    H3[12] += 100.0
    assert not np.allclose(oracle.route(H3, starts, lens, tid, Wr).logits[0], oracle.route(H, starts, lens, tid, Wr).logits[0])


def test_router_uses_the_requests_own_tenant_and_column_layout():
    """Tenant t's column j is e_{(j+t) mod d}: logits read z at shifted coordinates."""
    d, T = 9, 4
    Wr = np.zeros((T, 7, d))
    for t in range(T):
        for j in range(7):
            Wr[t, j, (j + t) % d] = 1.0
    z = np.arange(1.0, d + 1)[None].repeat(T, 0)
    logits = oracle.router_logits(z, Wr, [0, 1, 2, 3])
    for t in range(T):
        np.testing.assert_array_equal(logits[t], [z[0, (j + t) % d] for j in range(7)])
    route, gap = oracle.select(logits)
    np.testing.assert_array_equal(route, [6, 6, 6, 5])  # z grows with the index; tenant 3 wraps: (5+3)%9 = 8 is largest
    np.testing.assert_array_equal(gap, [1, 1, 1, 1])


def test_top1_of_softmax_is_argmax_of_logits_and_scale_invariant():
    rng = np.random.default_rng(10)
    logits = rng.standard_normal((200, 7)) * 3
    route, gap = oracle.select(logits)
    for b in range(200):
        p = oracle.softmax7(logits[b])
        assert abs(p.sum() - 1) < 1e-14 and (p > 0).all()
        assert int(np.argmax(p)) == route[b] == int(np.argmax(logits[b]))
        np.testing.assert_allclose(p, np.exp(logits[b]) / np.exp(logits[b]).sum(), rtol=1e-13)
        srt = np.sort(logits[b])
        assert gap[b] == srt[-1] - srt[-2]
    np.testing.assert_array_equal(oracle.select(logits * 7.5)[0], route)
    tie = np.array([[1.0, 5.0, 5.0, 0.0, 5.0, -1.0, 2.0]])
    assert oracle.select(tie)[0][0] == 1 and oracle.select(tie)[1][0] == 0.0


def test_selfattn_pooler_special_cases():
    rng = np.random.default_rng(11)
    d = 8
    H = rng.standard_normal((12, d))
    zero = np.zeros((1, d))
    np.testing.assert_allclose(oracle.pool(H, [2], [7], oracle.POOL_SELFATTN, zero, [0])[0],
                               H[2:9].mean(0), atol=1e-15)  # uniform attention = average pooling
    # a sharp query picks the token with the largest score
    w = rng.standard_normal((1, d)) * 200
    best = 2 + int(np.argmax(H[2:9] @ w[0]))
    np.testing.assert_allclose(oracle.pool(H, [2], [7], oracle.POOL_SELFATTN, w, [0])[0], H[best], atol=1e-9)
    # generic query against numpy
    w = rng.standard_normal((2, d))
    u = H[2:9] @ w[1]
    a = np.exp(u - u.max())
    a /= a.sum()
    np.testing.assert_allclose(oracle.pool(H, [2], [7], oracle.POOL_SELFATTN, w, [1])[0], a @ H[2:9], atol=1e-14)


# --------------------------------------------------------------------------- layer chain
def _pad_identity(d2, d1):
    W = np.zeros((d2, d1))
    n = min(d1, d2)
    W[np.arange(n), np.arange(n)] = 1.0
    return W


def test_layer_decode_closed_form_with_identity_weights():
    """Identity-like weights and no LoRA: q=k=v=x, h=2x, m=silu(2x)*2x on the first d lanes, y=h+m."""
    d, F, B = 6, 9, 3
    rng = np.random.default_rng(12)
    x = rng.standard_normal((B, d))
    W = [_pad_identity(*oracle.site_dims(m, d, F)[::-1]) for m in range(7)]
    ad = random_adapters(rng, 1, [2], d, F)
    y, qkv = oracle.layer_decode(x, W, ad, [0] * B, [7] * B, F)  # route 7 = no site
    np.testing.assert_array_equal(qkv, np.concatenate([x, x, x], 1))
    h = 2 * x
    np.testing.assert_allclose(y, h + h / (1 + np.exp(-h)) * h, atol=1e-14)
    # supplied attention output replaces a = v
    att = rng.standard_normal((B, d))
    y2, _ = oracle.layer_decode(x, W, ad, [0] * B, [7] * B, F, attn_out=att)
    h2 = x + att
    np.testing.assert_allclose(y2, h2 + h2 / (1 + np.exp(-h2)) * h2, atol=1e-14)
    # weightless RMS normalisation in front of q/k/v and gate/up; the residual stream stays un-normed
    y3, qkv3 = oracle.layer_decode(x, W, ad, [0] * B, [7] * B, F, flags=oracle.FLAG_RMSNORM)
    xn = x / np.sqrt((x ** 2).mean(1, keepdims=True) + 1e-5)
    np.testing.assert_allclose(qkv3[:, :d], xn, atol=1e-15)
    h3 = x + xn
    hn = h3 / np.sqrt((h3 ** 2).mean(1, keepdims=True) + 1e-5)
    np.testing.assert_allclose(y3, h3 + hn / (1 + np.exp(-hn)) * hn, atol=1e-14)


def test_layer_decode_matches_numpy_chain_and_routes_one_site_per_request():
    rng, ad, W, tid, route, d, F = _random_problem(13, M=7)
    route = np.arange(7)  # request b routed to site b
    x = rng.standard_normal((7, d))
    y, qkv = oracle.layer_decode(x, W, ad, tid, route, F)

    def lin(inp, site, b):
        out = inp @ W[site].T
        if route[b] == site:
            out = out + (inp @ ad.A[tid[b]][site]) @ ad.B[tid[b]][site]
        return out

    for b in range(7):
        q, k, v = (lin(x[b], s, b) for s in range(3))
        h = x[b] + lin(v, 3, b)
        m = lin(h, 4, b)
        m = m / (1 + np.exp(-m)) * lin(h, 5, b)
        np.testing.assert_allclose(qkv[b], np.concatenate([q, k, v]), atol=1e-12)
        np.testing.assert_allclose(y[b], h + lin(m, 6, b), atol=1e-10)
    # with every B zeroed the same call is the plain layer
    for t in range(3):
        for m_ in range(7):
            ad.B[t][m_][...] = 0
    y0, _ = oracle.layer_decode(x, W, ad, tid, route, F)
    yb, _ = oracle.layer_decode(x, W, ad, tid, [7] * 7, F)
    np.testing.assert_array_equal(y0, yb)


def test_routes_are_a_pure_function_of_the_prompt():
    """The route table depends on (prompt, tenant router) only: recomputing gives the same bytes,
    and decode consumes it read-only."""
    rng = np.random.default_rng(14)
    d, T, B = 16, 3, 5
    H = rng.standard_normal((60, d)).astype(np.float32)
    Wr = rng.standard_normal((T, 7, d)).astype(np.float32)
    starts, lens, tid = [0, 10, 25, 40, 52], [10, 15, 15, 12, 8], [0, 1, 2, 1, 0]
    a = oracle.route(H, starts, lens, tid, Wr, oracle.POOL_LAST, oracle.ACT_TANH)
    b = oracle.route(H, starts, lens, tid, Wr, oracle.POOL_LAST, oracle.ACT_TANH)
    assert a.route.tobytes() == b.route.tobytes()
    F = 24
    ad = random_adapters(rng, T, [2, 2, 2], d, F, dtype=np.float32)
    W = [rng.standard_normal(oracle.site_dims(m, d, F)[::-1]).astype(np.float32) for m in range(7)]
    table = a.route.copy()
    for step in range(3):
        x = rng.standard_normal((B, d)).astype(np.float32)
        oracle.layer_decode(x, W, ad, tid, table, F)
        assert table.tobytes() == a.route.tobytes()
