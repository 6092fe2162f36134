"""Pins for the CPU oracle: every check here compares the oracle with something that is
NOT the oracle -- a closed form, a library routine on a special case, brute-force loops,
a construction whose answer is known in advance, or a figure the paper prints."""
import itertools
import os

import numpy as np
import pytest

import synth_inputs as si
from oracle import parse_oracle as po

GOLD = os.path.join(os.path.dirname(__file__), "golden")


@pytest.fixture(scope="module")
def lay():
    # n != m on purpose so a transposed operand cannot go unnoticed
    return si.small_layer(11, n=96, m=80, R=48, G=6, dtype="f32")


# ----------------------------------------------------------------- forward pins
def test_full_selection_is_truncated_svd_product(lay):
    """S = all groups  =>  W_S = U0 diag(sigma) V  and numpy's SVD recovers sigma (Eq. 1)."""
    W = po.reconstruct(lay.U0, lay.sigma, lay.V, range(lay.G), lay.gs)
    assert np.allclose(W, lay.U0 @ np.diag(lay.sigma) @ lay.V, atol=1e-13)
    sv = np.linalg.svd(W, compute_uv=False)
    assert np.allclose(sv[:lay.R], (np.arange(lay.R) + 1.0) ** -0.5, atol=1e-12)
    assert np.all(sv[lay.R:] < 1e-12)


def test_brute_force_rank_one_sum(lay):
    """Eq. 4 literally: sum over selected rank-1 experts sigma_i u_i (v_i . x), scalar loops."""
    rng = np.random.default_rng(5)
    n, m, R, G, gs = 12, 10, 8, 4, 2
    small = si.small_layer(3, n, m, R, G, "f32")
    X = rng.standard_normal((3, n))
    S = [2, 0]
    ref = np.zeros((3, m))
    for t in range(3):
        for g in S:
            for i in range(g * gs, (g + 1) * gs):
                dot = 0.0
                for c in range(n):
                    dot += small.V[i, c] * X[t, c]
                for j in range(m):
                    ref[t, j] += small.sigma[i] * small.U0[j, i] * dot
    Y = po.forward(small.U0, small.sigma, small.V, gs, X, [0, 3], [S])
    assert np.allclose(Y, ref, atol=1e-13)


def test_group_order_does_not_matter(lay):
    rng = np.random.default_rng(6)
    X = rng.standard_normal((5, lay.n))
    S = [4, 1, 3]
    Y0 = po.forward(lay.U0, lay.sigma, lay.V, lay.gs, X, [0, 5], [S])
    for perm in itertools.permutations(S):
        Y = po.forward(lay.U0, lay.sigma, lay.V, lay.gs, X, [0, 5], [list(perm)])
        assert np.allclose(Y, Y0, atol=1e-13)


def test_left_out_group_contributes_its_own_term_only(lay):
    """Y_S - Y_{S minus g} = X (U_g Sigma_g V_g)^T ; the hard-mask form of Sec. 4.2 says an
    unselected expert contributes exactly zero."""
    rng = np.random.default_rng(7)
    X = rng.standard_normal((4, lay.n))
    S, g, gs = [0, 2, 5], 2, lay.gs
    YS = po.forward(lay.U0, lay.sigma, lay.V, gs, X, [0, 4], [S])
    Yminus = po.forward(lay.U0, lay.sigma, lay.V, gs, X, [0, 4], [[0, 5]])
    r = slice(g * gs, (g + 1) * gs)
    own = X @ ((lay.U0[:, r] * lay.sigma[r]) @ lay.V[r]).T
    assert np.allclose(YS - Yminus, own, atol=1e-13)
    # zeroing the factors of a group outside S changes nothing
    U2 = lay.U0.copy(); U2[:, 1 * gs:2 * gs] = 123.0
    assert np.array_equal(po.forward(U2, lay.sigma, lay.V, gs, X, [0, 4], [S]), YS)


def test_orthonormal_closed_forms(lay):
    """||W_S x||^2 = sum_{i in S} sigma_i^2 (v_i.x)^2 ; ||W_full - W_S||_F^2 = sum_{i notin S} sigma_i^2
    (Eckart-Young residual, Sec. 2)."""
    rng = np.random.default_rng(8)
    x = rng.standard_normal((1, lay.n))
    S = [1, 2, 4]
    rows = po.group_rows(S, lay.gs)
    y = po.forward(lay.U0, lay.sigma, lay.V, lay.gs, x, [0, 1], [S])
    energy = np.sum(lay.sigma[rows] ** 2 * (lay.V[rows] @ x[0]) ** 2)
    assert np.isclose(np.sum(y ** 2), energy, rtol=1e-12)
    Wf = po.reconstruct(lay.U0, lay.sigma, lay.V, range(lay.G), lay.gs)
    WS = po.reconstruct(lay.U0, lay.sigma, lay.V, S, lay.gs)
    rest = np.setdiff1d(np.arange(lay.R), rows)
    assert np.isclose(np.linalg.norm(Wf - WS) ** 2, np.sum(lay.sigma[rest] ** 2), rtol=1e-12)


def test_two_matmul_form_equals_dense_form(lay):
    """Eq. 10: W x = A (B^T x) with A = U Sigma, B^T = V, restricted to the selected columns."""
    rng = np.random.default_rng(9)
    X = rng.standard_normal((6, lay.n))
    S = [0, 3]
    rows = po.group_rows(S, lay.gs)
    A = lay.U0 * lay.sigma
    Z = X @ lay.V[rows].T
    assert np.allclose(Z @ A[:, rows].T,
                       po.forward(lay.U0, lay.sigma, lay.V, lay.gs, X, [0, 6], [S]), atol=1e-13)


def test_per_prompt_subsets_and_ragged_offsets(lay):
    """Each prompt's rows use that prompt's subset only; checked with dense numpy per prompt."""
    rng = np.random.default_rng(10)
    off = [0, 3, 4, 9]
    X = rng.standard_normal((9, lay.n))
    subs = [[0, 1], [5, 2], [3, 4]]
    Y = po.forward(lay.U0, lay.sigma, lay.V, lay.gs, X, off, subs)
    A = lay.U0 * lay.sigma
    for p in range(3):
        rows = po.group_rows(subs[p], lay.gs)
        ref = X[off[p]:off[p + 1]] @ (A[:, rows] @ lay.V[rows]).T
        assert np.allclose(Y[off[p]:off[p + 1]], ref, atol=1e-13)


def test_decode_equals_prefill_on_single_rows(lay):
    """Sec. 4.3 rank reuse: the step output is the same product with the prefill subset."""
    rng = np.random.default_rng(12)
    x = rng.standard_normal((3, lay.n))
    subs = [[0, 1], [2, 3], [0, 1]]
    yd = po.decode_step(lay.U0, lay.sigma, lay.V, lay.gs, x, subs)
    for b in range(3):
        yp = po.forward(lay.U0, lay.sigma, lay.V, lay.gs, x[b:b + 1], [0, 1], [subs[b]])
        assert np.array_equal(yd[b:b + 1], yp)


# ----------------------------------------------------------------- route pins
def test_pool_is_the_token_mean():
    X = np.arange(24, dtype=float).reshape(6, 4)
    E = po.pool(X, [0, 2, 6])
    assert np.allclose(E[0], [2, 3, 4, 5]) and np.allclose(E[1], [14, 15, 16, 17])


def test_route_known_by_construction():
    """W_r rows = scaled unit vectors: score_g = c_g * e[g], so the top-k is known in advance."""
    G, d, k = 6, 8, 3
    Wr = np.zeros((G, d)); scale = [1, 5, 2, 9, 3, 7]
    for g in range(G):
        Wr[g, g] = scale[g]
    e = np.ones((1, d))
    sub, margin = po.route(e, Wr, k)
    assert sub.tolist() == [[1, 3, 5]] and np.isclose(margin[0], 2.0)
    # permuting router rows permutes the chosen ids
    perm = [3, 0, 5, 1, 4, 2]
    sub2, _ = po.route(e, Wr[perm], k)
    assert sorted(perm[i] for i in sub2[0]) == [1, 3, 5]


def test_route_against_brute_force_subsets():
    """Top-k maximises the sum of selected scores over all k-subsets (tiny G)."""
    rng = np.random.default_rng(13)
    G, d, k = 7, 5, 3
    Wr = rng.standard_normal((G, d)); E = rng.standard_normal((9, d))
    subs, _ = po.route(E, Wr, k)
    for p in range(9):
        s = [sum(Wr[g, c] * E[p, c] for c in range(d)) for g in range(G)]
        best = max(itertools.combinations(range(G), k), key=lambda c: sum(s[g] for g in c))
        assert subs[p].tolist() == list(best)


def test_route_ties_prefer_lower_id_and_output_is_ascending():
    sub, margin = po.topk_ascending([1.0, 3.0, 3.0, 3.0, 0.0], 2)
    assert sub.tolist() == [1, 2] and margin == 0.0
    sub, margin = po.topk_ascending([0.5, 0.1, 0.9], 3)
    assert sub.tolist() == [0, 1, 2] and margin == float("inf")


def test_router_is_one_bias_free_matrix_per_projection():
    """The printed router size equals sum over projections of d_in * r_max with no bias."""
    vals = {}
    for line in open(os.path.join(GOLD, "router_param_count.txt")):
        if line.strip() and not line.startswith("#"):
            key, v = line.split(); vals[key] = float(v)
    L, h, f = int(vals["llama7b_layers"]), int(vals["llama7b_hidden"]), int(vals["llama7b_intermediate"])
    shapes = [(h, h)] * 4 + [(f, h)] * 2 + [(h, f)]          # (d_out, d_in) of q,k,v,o,gate,up,down
    params = L * sum(n * min(m, n) for m, n in shapes)
    assert round(params / 1e6, 2) == vals["router_params_millions"]
    with_bias = params + L * sum(min(m, n) for m, n in shapes)
    assert round(with_bias / 1e6, 2) != vals["router_params_millions"]
    # and the oracle's router is that map: linear and bias-free
    rng = np.random.default_rng(1)
    Wr = rng.standard_normal((4, 6)); a = rng.standard_normal((1, 6)); b = rng.standard_normal((1, 6))
    assert np.allclose(po.route_scores(2 * a + 3 * b, Wr), 2 * po.route_scores(a, Wr) + 3 * po.route_scores(b, Wr))
    assert np.array_equal(po.route_scores(np.zeros((1, 6)), Wr), np.zeros((1, 4)))


# ----------------------------------------------------------------- cache pins
def _wr(L=2, G=6, d=16, seed=3):
    return np.random.default_rng(seed).standard_normal((L, G, d))


def test_cache_special_cases():
    d, L, k = 16, 2, 3
    Wr = _wr(L, 6, d)
    c = po.PatternCache(8, d, L, k)
    e = np.zeros(d); e[0] = 1.0
    ent, sim = c.lookup(e[None], 0.9)
    assert ent.tolist() == [-1]                                   # empty cache => miss
    entry, hit, subs = c.lookup_or_route(e[None], 0.9, Wr)
    assert entry.tolist() == [0] and hit.tolist() == [0] and c.count == 1
    for l in range(L):                                            # stored value == route(key)
        assert subs[0, l].tolist() == po.route(e[None], Wr[l], k)[0][0].tolist()
    ent, sim = c.lookup(np.stack([e, 7.5 * e]), 0.9)              # identical / positively scaled
    assert ent.tolist() == [0, 0] and np.allclose(sim, 1.0)
    o = np.zeros(d); o[1] = 1.0                                   # orthogonal => cos 0 => miss
    ent, sim = c.lookup(o[None], 0.9)
    assert ent.tolist() == [-1] and abs(sim[0]) < 1e-15
    # threshold is inclusive, decided on the cosine: cos = 0.8 exactly representable case
    v = np.zeros(d); v[0], v[1] = 4.0, 3.0                        # cos(e, v) = 4/5
    assert c.lookup(v[None], 0.8 - 1e-12)[0].tolist() == [0]
    assert c.lookup(v[None], 0.8 + 1e-12)[0].tolist() == [-1]


def test_cache_known_cosines_and_first_max_wins():
    d = 4
    c = po.PatternCache(8, d, 1, 1)
    keys = np.array([[1, 0, 0, 0], [0, 2, 0, 0], [3, 0, 0, 0], [1, 1, 0, 0]], float)
    for j, kk in enumerate(keys):
        c.insert(kk, [[j]])
    assert np.allclose(po.cosine(np.array([1., 1, 0, 0]), keys), [2 ** -0.5, 2 ** -0.5, 2 ** -0.5, 1.0])
    ent, sim = c.lookup(np.array([[5., 0, 0, 0]]), 0.5)           # keys 0 and 2 tie at cos 1
    assert ent.tolist() == [0]
    ent, _ = c.lookup(np.array([[1., 1, 0, 0]]), 0.5)
    assert ent.tolist() == [3]


def test_cache_sequential_semantics_and_capacity():
    """A miss inserted for prompt i is visible to prompt i+1 of the same batch; a full cache
    still answers but stops growing."""
    d, L, k = 16, 1, 2
    Wr = _wr(L, 5, d)
    rng = np.random.default_rng(4)
    a = rng.standard_normal(d); b = rng.standard_normal(d)
    E = np.stack([a, a * 2, b, a + 1e-3 * b, b])
    c = po.PatternCache(2, d, L, k)
    entry, hit, subs = c.lookup_or_route(E, 0.9, Wr)
    assert entry.tolist() == [0, 0, 1, 0, 1] and hit.tolist() == [0, 1, 0, 1, 1] and c.count == 2
    assert np.array_equal(subs[1], subs[0]) and np.array_equal(subs[4], subs[2])
    z = rng.standard_normal(d)
    entry, hit, subs = c.lookup_or_route(z[None], 0.9, Wr)        # full: routed, not inserted
    assert entry.tolist() == [-1] and hit.tolist() == [0] and c.count == 2
    assert subs[0, 0].tolist() == po.route(z[None], Wr[0], k)[0][0].tolist()


def test_cache_hit_returns_route_of_the_key():
    d, L, k = 32, 3, 4
    Wr = _wr(L, 9, d, seed=8)
    E, cid = si.clustered_embeddings(np.random.default_rng(2), 40, d, 5, 0.05)
    c = po.PatternCache(64, d, L, k)
    entry, hit, subs = c.lookup_or_route(E, 0.9, Wr)
    for p in range(40):
        key = c.keys[entry[p]]
        for l in range(L):
            assert subs[p, l].tolist() == po.route(key[None], Wr[l], k)[0][0].tolist()
    # one entry per cluster present, every later member of a cluster hits
    assert c.count == len(set(cid.tolist()))
    assert int(hit.sum()) == 40 - c.count


def test_clustered_workload_hit_rate_closed_form():
    """16 clusters, 256 prompts, spread 0.1, tau 0.9: exactly one miss per cluster present
    => hit rate (256-16)/256 = 93.75 % and 16 cached entries."""
    E, cid, off, Wr = si.config4_embeddings(d=512)       # geometry is the same at reduced d
    assert len(set(cid.tolist())) == 16
    c = po.PatternCache(1024, 512, 3, 10)
    entry, hit, subs, sims, rm = c.lookup_or_route(E, 0.9, Wr, return_detail=True)
    assert c.count == 16 and hit.mean() == 240 / 256
    first = {}
    for p in range(256):
        first.setdefault(int(cid[p]), p)
        assert entry[p] == sorted(first.values()).index(first[int(cid[p])])


# ----------------------------------------------------------------- pack / bucket pins
def test_pack_is_slab_concatenation(lay):
    Vt, Ut = lay.Vt_store, lay.Ut_store
    gs = lay.gs
    Vs, Us = po.pack(Vt, Ut, [4, 0, 2], gs)
    assert Vs.tobytes() == b"".join(Vt[g * gs:(g + 1) * gs].tobytes() for g in (0, 2, 4))
    assert Us.tobytes() == b"".join(Ut[g * gs:(g + 1) * gs].tobytes() for g in (0, 2, 4))
    Va, Ua = po.pack(Vt, Ut, range(lay.G), gs)
    assert Va.tobytes() == Vt.tobytes() and Ua.tobytes() == Ut.tobytes()
    bits = si.f32_to_bf16_bits(Vt)                       # dtype-agnostic: bf16 bit patterns too
    assert po.pack(bits, bits, [1], gs)[0].tobytes() == bits[gs:2 * gs].tobytes()


def test_packed_factors_give_the_same_forward(lay):
    """Aggregation leaves the forward computation unchanged (Sec. 4.4)."""
    rng = np.random.default_rng(14)
    X = rng.standard_normal((4, lay.n))
    S = [1, 3, 4]
    Vt, Ut = lay.stored_values()
    Vs, Us = po.pack(Vt, Ut, S, lay.gs)
    Y = po.forward(lay.U0, lay.sigma, lay.V, lay.gs, X, [0, 4], [S])
    assert np.allclose((X @ Vs.T) @ Us, Y, rtol=0, atol=1e-5)    # stored factors are float32


def test_bucket_properties():
    subs = np.array([[1, 2], [0, 3], [1, 2], [2, 3], [0, 3], [1, 2]])
    pid, perm, off, npat, rep = po.bucket(subs)
    assert pid.tolist() == [0, 1, 0, 2, 1, 0] and npat == 3
    assert perm.tolist() == [0, 2, 5, 1, 4, 3] and off.tolist() == [0, 3, 5, 6]
    assert rep.tolist() == [0, 1, 3]
    # decode workload: sequence i uses pattern i mod 4 => 4 buckets of 8, stable
    pats = np.array([[0, 1], [2, 3], [4, 5], [6, 7]])
    pid, perm, off, npat, rep = po.bucket(pats[np.arange(32) % 4])
    assert npat == 4 and off.tolist() == [0, 8, 16, 24, 32]
    assert sorted(perm.tolist()) == list(range(32))
    for j in range(4):
        assert perm[off[j]:off[j + 1]].tolist() == list(range(j, 32, 4))


# ----------------------------------------------------------------- planted mistakes
def _forward_pins_hold(lay) -> bool:
    """The closed-form pins above, folded into one predicate."""
    rng = np.random.default_rng(15)
    X = rng.standard_normal((3, lay.n))
    S = [1, 4]
    rows = po.group_rows(S, lay.gs)
    y = po.forward(lay.U0, lay.sigma, lay.V, lay.gs, X, [0, 3], [S])
    energy = np.sum(lay.sigma[rows][None, :] ** 2 * (X @ lay.V[rows].T) ** 2, axis=1)
    ok = np.allclose(np.sum(y ** 2, axis=1), energy, rtol=1e-10)
    Wf = po.reconstruct(lay.U0, lay.sigma, lay.V, range(lay.G), lay.gs)
    sv = np.linalg.svd(Wf, compute_uv=False)[:lay.R]
    ok = ok and np.allclose(sv, (np.arange(lay.R) + 1.0) ** -0.5, atol=1e-10)
    A = lay.U0 * lay.sigma
    ok = ok and np.allclose(y, (X @ lay.V[rows].T) @ A[:, rows].T, atol=1e-12)
    return bool(ok)


def test_pins_catch_planted_mistakes(lay, monkeypatch):
    """Plant plausible bugs in the oracle (on the CPU) and check that the pins notice."""
    assert _forward_pins_hold(lay)
    orig = po.reconstruct

    def dropped_sigma(U0, sigma, V, subset, gs):
        return orig(U0, np.ones_like(sigma), V, subset, gs)

    def wrong_sign(U0, sigma, V, subset, gs):
        return -orig(U0, sigma, V, subset, gs)

    def off_by_one_group(U0, sigma, V, subset, gs):
        return orig(U0, sigma, V, [(int(g) + 1) % (len(sigma) // gs) for g in subset], gs)

    def sigma_squared(U0, sigma, V, subset, gs):
        return orig(U0, sigma ** 2, V, subset, gs)

    for bad in (dropped_sigma, wrong_sign, off_by_one_group, sigma_squared):
        monkeypatch.setattr(po, "reconstruct", bad)
        assert not _forward_pins_hold(lay), bad.__name__
    monkeypatch.setattr(po, "reconstruct", orig)

    # a transposed operand in the apply step
    def transposed_apply(U0, sigma, V, gs, X, off, subsets):
        W = orig(U0, sigma, V, subsets[0], gs)
        return np.asarray(X) @ W[:, :W.shape[0]] if W.shape[0] <= W.shape[1] else None

    sq = si.small_layer(21, n=40, m=40, R=16, G=4, dtype="f32")
    X = np.random.default_rng(2).standard_normal((2, 40))
    good = po.forward(sq.U0, sq.sigma, sq.V, sq.gs, X, [0, 2], [[0, 2]])
    assert not np.allclose(transposed_apply(sq.U0, sq.sigma, sq.V, sq.gs, X, [0, 2], [[0, 2]]), good)
    # routing mistakes: descending-vs-ascending score order, and a bias term
    e = np.ones((1, 8)); Wr = np.diag([1., 5, 2, 9, 3, 7, 4, 6])
    assert po.route(e, Wr, 3)[0].tolist() == [[3, 5, 7]]
    assert po.route(e, -Wr, 3)[0].tolist() == [[0, 2, 4]]


# ----------------------------------------------------------------- generator sanity
def test_generator_recipe(lay):
    assert np.allclose(lay.U0.T @ lay.U0, np.eye(lay.R), atol=1e-12)
    assert np.allclose(lay.V @ lay.V.T, np.eye(lay.R), atol=1e-12)
    assert np.allclose(lay.sigma, (np.arange(lay.R) + 1.0) ** -0.5)
    assert np.allclose(lay.Ut_store, (lay.U0 * lay.sigma).T.astype(np.float32))
    x = np.array([1.0, 1.00390625, 1.01171875, -3.0e-5, 65504.0], np.float32)
    bits = si.f32_to_bf16_bits(x)
    back = si.bf16_bits_to_f32(bits)
    assert back[0] == 1.0 and back[1] == 1.0 and back[2] == 1.015625   # ties to even, then up
    assert np.all(np.abs(back - x) <= np.abs(x) * 2.0 ** -8)


def test_route_with_shared_head_is_the_best_superset_of_the_shared_groups():
    """Shared experts (Sec. 4.4): the routed subset is the k-subset of largest total score among those that
    contain groups 0..n_shared-1 (brute force over all subsets), and n_shared = 0 is the plain top-k."""
    import itertools
    rng = np.random.default_rng(31)
    G, d, k = 7, 12, 4
    Wr = rng.standard_normal((G, d))
    E = rng.standard_normal((5, d))
    S = E @ Wr.T
    plain, _ = po.route(E, Wr, k)
    same, _ = po.route(E, Wr, k, n_shared=0)
    assert np.array_equal(plain, same)
    for n_shared in (1, 2, 3, 4):
        subs, _ = po.route(E, Wr, k, n_shared=n_shared)
        for p in range(E.shape[0]):
            best = max((c for c in itertools.combinations(range(G), k) if set(range(n_shared)) <= set(c)),
                       key=lambda c: sum(S[p][g] for g in c))
            assert tuple(subs[p]) == tuple(sorted(best))
            assert list(subs[p]) == sorted(subs[p]) and len(set(subs[p])) == k


def test_zero_padded_groups_change_nothing():
    """Padding every rank group with zero ranks (what the operand-order layout needs when a group is not a whole
    number of 32-rank blocks) leaves the routed product unchanged; the full-stack workload's ranks come out as
    the ratio says (4096x4096: 16 groups of 80; 4096<->11008: 16 groups of 112)."""
    assert si.config3_ranks(4096, 4096) == (1280, 80)
    assert si.config3_ranks(4096, 11008) == (1792, 112) and si.config3_ranks(11008, 4096) == (1792, 112)
    lay = si.small_layer(41, 96, 64, 40, 4, "f32")            # groups of 10 ranks
    pad = si.pad_groups(lay, 16)
    assert pad.R == 64 and pad.gs == 16 and pad.G == 4
    rng = np.random.default_rng(42)
    X = rng.standard_normal((9, 96))
    off = np.array([0, 4, 9], np.int32)
    subs = np.array([[0, 2], [1, 3]], np.int32)
    Y0 = po.forward(lay.U0, lay.sigma, lay.V, lay.gs, X, off, subs)
    Y1 = po.forward(pad.U0, pad.sigma, pad.V, pad.gs, X, off, subs)
    assert np.allclose(Y0, Y1, rtol=0, atol=1e-13)
    V0, U0p = po.pack(lay.Vt_store, lay.Ut_store, subs[0], lay.gs)
    V1, U1p = po.pack(pad.Vt_store, pad.Ut_store, subs[0], pad.gs)
    assert np.array_equal(V1.reshape(2, 16, -1)[:, :10].reshape(20, -1), V0) and np.all(V1.reshape(2, 16, -1)[:, 10:] == 0)


def test_router_training_step_against_finite_differences():
    """Sec. 4.2: dL/dm is checked by perturbing the mask of the (quadratic) loss, d m_soft / d Wr by perturbing
    the router matrix in the soft-mask formula; their composition is the straight-through gradient.  The soft
    mask sums to K (up to eps) as the K-normalisation promises."""
    rng = np.random.default_rng(51)
    n, m, R, G, k, tau, eps = 24, 20, 12, 4, 2, 0.7, 1e-6
    lay = si.small_layer(52, n, m, R, G, "f32")
    gs = lay.gs
    off = np.array([0, 5, 9], np.int32)
    X = rng.standard_normal((9, n))
    Wd = rng.standard_normal((m, n)) * 0.3
    Yd = X @ Wd.T
    Wr = rng.standard_normal((G, n)) * 0.5
    loss, grad, dm = po.router_grad(lay.U0, lay.sigma, lay.V, gs, X, off, Yd, Wr, k, tau, eps)
    E = po.pool(X, off)
    Wg = [po.reconstruct(lay.U0, lay.sigma, lay.V, [g], gs) for g in range(G)]

    def loss_of_mask(p, mvec):
        a, b = off[p], off[p + 1]
        Yh = sum(mvec[g] * (X[a:b] @ Wg[g].T) for g in range(G))
        return float(((Yh - Yd[a:b]) ** 2).sum())

    h = 1e-6
    grad_fd = np.zeros_like(Wr)
    for p in range(2):
        s = Wr @ E[p]
        hard = np.zeros(G); hard[po.topk_ascending(s, k)[0]] = 1.0
        assert abs(loss_of_mask(p, hard) - loss[p]) < 1e-9 * max(1.0, loss[p])
        dm_fd = np.array([(loss_of_mask(p, hard + h * np.eye(G)[g]) - loss_of_mask(p, hard - h * np.eye(G)[g])) / (2 * h)
                          for g in range(G)])
        assert np.allclose(dm_fd, dm[p], rtol=1e-5, atol=1e-6)
        assert abs(po.soft_mask(s, k, tau, eps).sum() - k) < 1e-4
        for j in range(G):
            for c in range(n):
                Wp = Wr.copy(); Wp[j, c] += h
                Wm = Wr.copy(); Wm[j, c] -= h
                dmsoft = (po.soft_mask(Wp @ E[p], k, tau, eps) - po.soft_mask(Wm @ E[p], k, tau, eps)) / (2 * h)
                grad_fd[j, c] += float(dm[p] @ dmsoft)
    assert np.allclose(grad_fd, grad, rtol=1e-4, atol=1e-7)


# ----------------------------------------------------------------- error metric and soft mask pins
def _rel_errors_pins_hold(fn) -> bool:
    """Hand-computed cases of the two error figures.  Y = [[3, 4]], Yref = [[0, 5]]: difference (3, -1), Frobenius
    sqrt(10) over 5, max-abs 3 over 5.  Second case: 99 exact entries of value 1 and one entry off by 1, so the two
    figures differ tenfold (0.1 against 1) and neither can stand in for the other.  Third case: the result is twice
    the reference, so both errors are 1 relative to the REFERENCE (they would be 0.5 relative to the result)."""
    ok = True
    fro, mx = fn([[3.0, 4.0]], [[0.0, 5.0]])
    ok &= abs(fro - np.sqrt(10.0) / 5.0) < 1e-15 and abs(mx - 3.0 / 5.0) < 1e-15
    Yref = np.ones((10, 10)); Y = Yref.copy(); Y[3, 7] = 2.0
    fro, mx = fn(Y, Yref)
    ok &= abs(fro - 0.1) < 1e-15 and abs(mx - 1.0) < 1e-15
    fro, mx = fn([[2.0, -4.0, 6.0]], [[1.0, -2.0, 3.0]])
    ok &= abs(fro - 1.0) < 1e-15 and abs(mx - 1.0) < 1e-15
    fro, mx = fn([[1.0, -1.0]], [[1.0, 2.0]])          # the only error is negative: (0, -3)
    ok &= abs(fro - 3.0 / np.sqrt(5.0)) < 1e-15 and abs(mx - 1.5) < 1e-15
    fro, mx = fn([[1.5, -2.0]], [[1.5, -2.0]])
    ok &= fro == 0.0 and mx == 0.0
    return bool(ok)


def test_rel_errors_on_hand_computed_arrays():
    """The helper every float tolerance goes through gives the hand-computed figures, does not divide by zero on a
    zero reference, and the same cases reject the plausible wrong forms: dividing by the result's norm, by the
    wrong kind of norm, or a signed maximum."""
    assert _rel_errors_pins_hold(po.rel_errors)
    assert np.isfinite(po.rel_errors([[0.0]], [[0.0]])).all()
    d = lambda Y, Yr: np.asarray(Y, float) - np.asarray(Yr, float)
    by_result = lambda Y, Yr: (np.linalg.norm(d(Y, Yr)) / np.linalg.norm(Y), np.max(np.abs(d(Y, Yr))) / np.max(np.abs(Y)))
    max_over_fro = lambda Y, Yr: (np.linalg.norm(d(Y, Yr)) / np.linalg.norm(Yr), np.max(np.abs(d(Y, Yr))) / np.linalg.norm(Yr))
    signed_max = lambda Y, Yr: (np.linalg.norm(d(Y, Yr)) / np.linalg.norm(Yr), np.max(d(Y, Yr)) / np.max(Yr))
    mean_not_norm = lambda Y, Yr: (np.abs(d(Y, Yr)).mean() / np.abs(Yr).mean(), np.max(np.abs(d(Y, Yr))) / np.max(np.abs(Yr)))
    for bad in (by_result, max_over_fro, signed_max, mean_not_norm):
        assert not _rel_errors_pins_hold(bad)


def test_soft_mask_values_fixed_by_the_formula():
    """Eq. 9 on inputs whose value is known without the oracle: equal scores give K/G each (times 1/(1+eps G/..));
    two scores have their sigmoids written out by hand; a lower temperature sharpens the mask (the score is DIVIDED
    by it), a higher one flattens it towards K/G."""
    G, K = 5, 2
    m = po.soft_mask(np.full(G, 0.3), K, 0.7, 0.0)
    assert np.allclose(m, K / G, atol=1e-15)
    # eps enters the denominator only: sum of sigmoids A = G*a, m = K a / (G a + eps)
    a = 1.0 / (1.0 + np.exp(-0.3 / 0.7)); eps = 1e-3
    assert np.allclose(po.soft_mask(np.full(G, 0.3), K, 0.7, eps), K * a / (G * a + eps), atol=1e-15)
    # two scores, temperature 2: sigmoid(ln3) = 3/4, sigmoid(-ln3) = 1/4 -> mask = K * (3/4, 1/4) / 1
    s = np.array([2.0 * np.log(3.0), -2.0 * np.log(3.0)])
    assert np.allclose(po.soft_mask(s, 1, 2.0, 0.0), [0.75, 0.25], atol=1e-15)
    assert np.allclose(po.soft_mask(s, 2, 2.0, 0.0), [1.5, 0.5], atol=1e-15)
    # temperature 1 on the same scores: sigmoid(2 ln 3) = 9/10, sigmoid(-2 ln 3) = 1/10 -> sharper
    assert np.allclose(po.soft_mask(s, 1, 1.0, 0.0), [0.9, 0.1], atol=1e-15)
    # multiplying by the temperature instead of dividing would give (0.9, 0.1) at temperature 2 and fail the line above
    s3 = np.array([1.0, 0.0, -1.0])
    sharp, flat = po.soft_mask(s3, 1, 0.1, 0.0), po.soft_mask(s3, 1, 10.0, 0.0)
    assert sharp[0] > 0.6 and sharp[2] < 1e-4 and np.all(np.abs(flat - 1.0 / 3.0) < 0.02)
    # the largest score always gets the largest mask entry; the entries sum to K when eps = 0
    assert np.argmax(sharp) == 0 and abs(po.soft_mask(s3, 2, 0.5, 0.0).sum() - 2.0) < 1e-15


def test_plan_rows_hand_case_and_properties():
    """Row-level grouping: a hand case (tile of 4 rows), then properties on random input: every real row appears exactly
    once, rows of a tile share the tile's pattern, prompts of a pattern keep arrival order, padding only at the end of a
    pattern's run and shorter than a tile."""
    off = np.array([0, 3, 5, 6, 11], np.int32)          # lengths 3, 2, 1, 5
    pid = np.array([2, 0, 7, 2], np.int32)               # 7 is out of range for n_patterns = 3
    rowmap, tpat = po.plan_rows(off, pid, 3, tile=4)
    assert rowmap.tolist() == [3, 4, -1, -1,   0, 1, 2, 6, 7, 8, 9, 10,   5, -1, -1, -1]
    assert tpat.tolist() == [0, 2, 2, -1]
    rng = np.random.default_rng(77)
    lengths = rng.integers(1, 40, size=23)
    off = si.offsets_from_lengths(lengths)
    pid = rng.integers(-1, 6, size=23).astype(np.int32)  # -1 and 5 are invalid for n_patterns = 5
    rowmap, tpat = po.plan_rows(off, pid, 5, tile=16)
    real = rowmap[rowmap >= 0]
    assert sorted(real.tolist()) == list(range(int(off[-1])))
    prompt_of = np.searchsorted(off, np.arange(off[-1]), side="right") - 1
    for t, b in enumerate(tpat):
        rows = rowmap[t * 16:(t + 1) * 16]
        for r in rows[rows >= 0]:
            q = pid[prompt_of[r]]
            assert (q if 0 <= q < 5 else -1) == b
    for b in set(tpat.tolist()):
        run = rowmap[np.repeat(tpat == b, 16)]
        n_real = int((run >= 0).sum())
        assert np.all(run[:n_real] >= 0) and np.all(run[n_real:] == -1) and len(run) - n_real < 16
        assert np.all(np.diff(run[:n_real]) > 0)          # arrival order = ascending rows within a pattern


def test_decode_groups_hand_case_and_consistency_with_decode_step():
    # hand case: 3 patterns over 6 groups, 5 sequences, one with an invalid pattern id
    subsets = np.array([[0, 2], [2, 5], [1, 2]], np.int32)
    used, masks = po.decode_groups(subsets, [0, 1, 1, 7, 2], 6)
    assert used == [0, 1, 2, 5]
    assert masks == [0b00001, 0b10000, 0b10111, 0, 0, 0b00110]
    # a group outside the used list changes no sequence's decode output; a group inside changes exactly the sequences
    # of its mask (left-out group contributes exactly zero: Sec. 4.1)
    rng = np.random.default_rng(5)
    n, m, R, G = 24, 20, 12, 6
    gs = R // G
    U0, _ = np.linalg.qr(rng.standard_normal((m, R)))
    V = np.linalg.qr(rng.standard_normal((n, R)))[0].T
    sigma = (np.arange(R) + 1.0) ** -0.5
    seq_pat = np.array([0, 1, 1, 2])
    x = rng.standard_normal((4, n))
    y = po.decode_step(U0, sigma, V, gs, x, subsets[seq_pat])
    used, masks = po.decode_groups(subsets, seq_pat, G)
    for g in range(G):
        s2 = sigma.copy()
        s2[g * gs:(g + 1) * gs] *= 3.0                       # disturb one group
        y2 = po.decode_step(U0, s2, V, gs, x, subsets[seq_pat])
        changed = sum(1 << b for b in range(4) if not np.allclose(y[b], y2[b], rtol=0, atol=1e-12))
        assert changed == masks[g], g
        assert (g in used) == (masks[g] != 0)
