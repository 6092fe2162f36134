"""CPU oracle for the prompt-routed low-rank linear layer (PARSE inference path).

TEST INFRASTRUCTURE ONLY.  Plain numpy in float64 plus Python loops; slow on
purpose.  It imports nothing from the GPU package and shares no code with it.
Only the test-suite, the smoke check and the benchmark's CPU-baseline leg may
call it; the product path never does.

What each function follows:
  reconstruct / forward   Sec. 4.1 Eq. 3-4: W_hat x = sum_{i in R(x)} sigma_i u_i v_i^T x,
                          with the expert set a union of rank groups; the routed result
                          is exactly the dense product with the reconstructed W_S.
  pool / route            Sec. 4.1 Eq. 5: R(x) = TopK(f_theta(x)), f_theta one bias-free
                          linear map; the router input is one embedding per prompt
                          (Sec. 4.1 last paragraph), here the mean of the prompt's tokens.
  PatternCache            Sec. 4.3 "Rank Retrieval for Prefilling": embedding -> subset
                          map answered by nearest neighbour (cosine); a similarity
                          threshold and insert-on-miss are this build's reading.
  pack                    Sec. 4.4 "Expert Memory Aggregation": selected components moved
                          into one contiguous block, forward unchanged.
  bucket / plan_rows      grouping of prompts (and of their token rows) that share a subset
                          (Sec. 4.3: patterns are shared across prompts), so one launch or
                          tile serves one pattern.
  decode                  Sec. 4.3 "Rank Reuse for Decoding": the prefill subset is fixed
                          for every later step; same product with one row per sequence.
  decode_groups           what a decode step over a batch needs from the fixed subsets:
                          which groups some sequence selected, and which sequences hold each.
  soft_mask / router_grad Sec. 4.2 Eq. 6-9: reconstruction loss against the dense output,
                          hard top-k mask forward, K-normalised sigmoid mask backward
                          (straight-through), gradient with respect to the router matrix.

Pins (tests/test_oracle_pins.py): full selection == truncated-SVD product and
numpy.linalg.svd recovers sigma; Eckart-Young residual closed form; orthonormal
energy identity; brute-force rank-1 loops; group-order invariance; left-out group
contributes exactly its own term; hand-built routers with known top-k; cache
special cases and the clustered-workload hit-rate closed form; pack/bucket
identities; `rel_errors` and `soft_mask` on hand-computed values.  The FORM of the
error metric (`rel_errors`: Frobenius and max-abs, both relative to the reference) is
this build's choice: the paper states none; what the helper computes is pinned.
"""
from __future__ import annotations

import numpy as np

F64 = np.float64


# ------------------------------------------------------------------ forward
def group_rows(subset, gs: int) -> np.ndarray:
    """Rank indices covered by the groups of `subset`, in the order given."""
    subset = np.asarray(subset, dtype=np.int64).reshape(-1)
    return (subset[:, None] * gs + np.arange(gs, dtype=np.int64)[None, :]).reshape(-1)


def reconstruct(U0, sigma, V, subset, gs: int) -> np.ndarray:
    """W_S = sum_{g in S} U0[:, g] diag(sigma_g) V[g, :], formed densely (m x n, float64)."""
    U0 = np.asarray(U0, F64); sigma = np.asarray(sigma, F64); V = np.asarray(V, F64)
    W = np.zeros((U0.shape[0], V.shape[1]), F64)
    for g in np.asarray(subset, dtype=np.int64).reshape(-1):
        r = slice(int(g) * gs, (int(g) + 1) * gs)
        W += (U0[:, r] * sigma[r][None, :]) @ V[r, :]
    return W


def forward(U0, sigma, V, gs: int, X, tok_offsets, subsets) -> np.ndarray:
    """Y[t] = W_{S_p} x_t for every token t of prompt p (Eq. 4); subsets is [P][k]."""
    X = np.asarray(X, F64)
    tok_offsets = np.asarray(tok_offsets, dtype=np.int64)
    Y = np.zeros((X.shape[0], np.asarray(U0).shape[0]), F64)
    for p in range(len(tok_offsets) - 1):
        a, b = int(tok_offsets[p]), int(tok_offsets[p + 1])
        W = reconstruct(U0, sigma, V, subsets[p], gs)
        Y[a:b] = X[a:b] @ W.T
    return Y


def decode_step(U0, sigma, V, gs: int, x, seq_subsets) -> np.ndarray:
    """One decode step: row b uses the subset fixed for sequence b at prefill."""
    B = np.asarray(x).shape[0]
    return forward(U0, sigma, V, gs, x, np.arange(B + 1), seq_subsets)


# ------------------------------------------------------------------ route
def pool(X, tok_offsets) -> np.ndarray:
    """e_p = mean over the prompt's token rows (float64)."""
    X = np.asarray(X, F64)
    tok_offsets = np.asarray(tok_offsets, dtype=np.int64)
    E = np.zeros((len(tok_offsets) - 1, X.shape[1]), F64)
    for p in range(E.shape[0]):
        a, b = int(tok_offsets[p]), int(tok_offsets[p + 1])
        E[p] = X[a:b].sum(axis=0) / float(b - a)
    return E


def route_scores(E, Wr) -> np.ndarray:
    """s_p = W_r e_p  (Eq. 5 scores), E [P][d], Wr [G][d] -> [P][G]."""
    return np.asarray(E, F64) @ np.asarray(Wr, F64).T


def topk_ascending(scores, k: int):
    """Top-k groups of one score vector; ties go to the lower group id; the set is
    returned ascending.  Also returns the margin s_(k) - s_(k+1) (inf when k == G)."""
    s = np.asarray(scores, F64).reshape(-1)
    order = sorted(range(len(s)), key=lambda g: (-s[g], g))
    chosen = sorted(order[:k])
    margin = float(s[order[k - 1]] - s[order[k]]) if k < len(s) else float("inf")
    return np.asarray(chosen, dtype=np.int32), margin


def topk_with_shared(scores, k: int, n_shared: int = 0):
    """Subset of one score vector when groups 0..n_shared-1 are always active (Sec. 4.4, shared experts at
    the head of memory): those, plus the k - n_shared best of the other groups; ascending ids and the margin
    of the routed part."""
    if n_shared <= 0:
        return topk_ascending(scores, k)
    if n_shared >= k:
        return np.arange(k, dtype=np.int32), float("inf")
    s = np.asarray(scores, F64).reshape(-1)
    rest, mg = topk_ascending(s[n_shared:], k - n_shared)
    return np.concatenate([np.arange(n_shared, dtype=np.int32), rest + n_shared]).astype(np.int32), mg


def route(E, Wr, k: int, n_shared: int = 0):
    """subset[P][k] (ascending ids) and per-prompt margins for embeddings E.

    n_shared > 0 (Sec. 4.4, expert memory aggregation: the components with the largest singular values are
    shared by all prompts and sit at the head of memory): groups 0..n_shared-1 are always active, the router
    chooses the k - n_shared best of the remaining groups; the margin is that of the routed part."""
    S = route_scores(E, Wr)
    subs, margins = [], []
    for p in range(S.shape[0]):
        c, mg = topk_with_shared(S[p], k, n_shared)
        subs.append(c); margins.append(mg)
    return np.asarray(subs, dtype=np.int32).reshape(S.shape[0], k), np.asarray(margins, F64)


# ------------------------------------------------------------------ cache
def cosine(e, K) -> np.ndarray:
    """cosine similarity of e [d] with every row of K [C][d]."""
    e = np.asarray(e, F64); K = np.asarray(K, F64)
    return (K @ e) / (np.linalg.norm(K, axis=1) * np.linalg.norm(e))


class PatternCache:
    """Embedding -> per-layer subsets; sequential semantics in arrival order.

    lookup: nearest neighbour by cosine; the smallest index attaining the maximum wins;
    a hit needs similarity >= tau.  lookup_or_route: a miss routes every layer's
    subset, and appends (embedding, subsets) while there is room (no eviction)."""

    def __init__(self, capacity: int, d: int, L: int, k: int, n_shared: int = 0):
        self.capacity, self.d, self.L, self.k, self.n_shared = capacity, d, L, k, n_shared
        self.keys = np.zeros((0, d), F64)
        self.values = np.zeros((0, L, k), np.int32)

    @property
    def count(self) -> int:
        return self.keys.shape[0]

    def insert(self, e, subsets) -> bool:
        if self.count >= self.capacity:
            return False
        self.keys = np.vstack([self.keys, np.asarray(e, F64).reshape(1, self.d)])
        self.values = np.concatenate(
            [self.values, np.asarray(subsets, np.int32).reshape(1, self.L, self.k)], axis=0)
        return True

    def lookup_one(self, e, tau: float):
        """-> (entry or -1, best similarity or -inf, best entry index or -1)."""
        if self.count == 0:
            return -1, float("-inf"), -1
        c = cosine(e, self.keys)
        j = int(np.argmax(c))           # numpy returns the first maximum
        return (j if c[j] >= tau else -1), float(c[j]), j

    def lookup(self, E, tau: float):
        ent, sim = [], []
        for e in np.asarray(E, F64):
            j, s, _ = self.lookup_one(e, tau)
            ent.append(j); sim.append(s)
        return np.asarray(ent, np.int32), np.asarray(sim, F64)

    def lookup_or_route(self, E, tau: float, Wr, return_detail: bool = False):
        """Wr [L][G][d].  Returns entry[P] (entry that answered: the hit entry, or the new
        entry's index on an inserted miss, or -1 on a miss with a full cache), hit[P] (0/1),
        subsets[P][L][k]."""
        E = np.asarray(E, F64)
        Wr = np.asarray(Wr, F64)
        P = E.shape[0]
        entry = np.zeros(P, np.int32); hit = np.zeros(P, np.uint8)
        subs = np.zeros((P, self.L, self.k), np.int32)
        sims = np.full(P, -np.inf); route_margin = np.full(P, np.inf)
        for p in range(P):
            j, s, _ = self.lookup_one(E[p], tau)
            sims[p] = s
            if j >= 0:
                entry[p], hit[p], subs[p] = j, 1, self.values[j]
                continue
            S = np.zeros((self.L, self.k), np.int32)
            for l in range(self.L):
                c, mg = topk_with_shared(Wr[l] @ E[p], self.k, self.n_shared)
                S[l] = c
                route_margin[p] = min(route_margin[p], mg)
            subs[p] = S
            new_index = self.count
            entry[p] = new_index if self.insert(E[p], S) else -1
        if return_detail:
            return entry, hit, subs, sims, route_margin
        return entry, hit, subs


# ------------------------------------------------------------------ router training step
def soft_mask(scores, k: int, temperature: float, eps: float) -> np.ndarray:
    """Sec. 4.2 Eq. 9: m_i = K sigmoid(s_i / tau) / (sum_j sigmoid(s_j / tau) + eps)."""
    a = 1.0 / (1.0 + np.exp(-np.asarray(scores, F64) / temperature))
    return k * a / (a.sum() + eps)


def router_grad(U0, sigma, V, gs: int, X, tok_offsets, Y_dense, Wr, k: int, temperature: float, eps: float):
    """One training step of the router (Sec. 4.2), groups as experts, one embedding per prompt.

    Forward (Eq. 7): y_hat = sum_g m_g^hard W_g x with m^hard the top-k indicator of s = Wr e_p.
    Loss (Eq. 6): sum over the prompt's tokens of ||y_hat - y_dense||^2.
    Backward (Eq. 8-9): the mask's value is the hard one, its derivative the soft one's:
      dL/dm_g = sum_t 2 (y_hat_t - y_t)^T W_g x_t,   dL/ds = J^T dL/dm with J = d m^soft / d s,
      dL/dWr = sum_p dL/ds(p) e_p^T.
    Returns (loss[P], grad_Wr[G][d], dL/dm[P][G])."""
    X = np.asarray(X, F64); Yd = np.asarray(Y_dense, F64); Wr = np.asarray(Wr, F64)
    G = Wr.shape[0]
    P = len(tok_offsets) - 1
    E = pool(X, tok_offsets)
    Wg = [reconstruct(U0, sigma, V, [g], gs) for g in range(G)]          # m x n each
    loss = np.zeros(P, F64); grad = np.zeros_like(Wr); dm_all = np.zeros((P, G), F64)
    for p in range(P):
        a, b = int(tok_offsets[p]), int(tok_offsets[p + 1])
        s = Wr @ E[p]
        hard, _ = topk_ascending(s, k)
        Yh = sum(X[a:b] @ Wg[g].T for g in hard)
        res = Yh - Yd[a:b]
        loss[p] = float((res ** 2).sum())
        dm = np.array([2.0 * float((res * (X[a:b] @ Wg[g].T)).sum()) for g in range(G)])
        sg = 1.0 / (1.0 + np.exp(-s / temperature))
        A = sg.sum() + eps
        dsg = sg * (1.0 - sg) / temperature
        # J[g][j] = d m_g / d s_j = k (delta_gj dsg_j / A - sg_g dsg_j / A^2)
        J = k * (np.diag(dsg) / A - np.outer(sg, dsg) / A ** 2)
        ds = J.T @ dm
        grad += np.outer(ds, E[p])
        dm_all[p] = dm
    return loss, grad, dm_all


# ------------------------------------------------------------------ pack / bucket
def pack(Vt, Ut, subset, gs: int):
    """Selected group slabs, ascending group id, concatenated: Vt_S [k*gs][n], Ut_S [k*gs][m].
    Works on any dtype (pure data movement)."""
    rows = group_rows(sorted(int(g) for g in np.asarray(subset).reshape(-1)), gs)
    return np.ascontiguousarray(np.asarray(Vt)[rows]), np.ascontiguousarray(np.asarray(Ut)[rows])


def bucket(subsets):
    """Patterns numbered by first appearance; perm = stable order of prompts by pattern id;
    bucket_off = prefix counts.  -> pattern_id[P], perm[P], bucket_off[n_pat+1], n_pat,
    rep[n_pat] (first prompt showing each pattern)."""
    subsets = np.asarray(subsets)
    P = subsets.shape[0]
    seen, rep = {}, []
    pid = np.zeros(P, np.int32)
    for p in range(P):
        key = tuple(int(v) for v in subsets[p].reshape(-1))
        if key not in seen:
            seen[key] = len(seen); rep.append(p)
        pid[p] = seen[key]
    perm = np.asarray(sorted(range(P), key=lambda p: (pid[p], p)), np.int32)
    off = np.zeros(len(seen) + 1, np.int32)
    for p in range(P):
        off[pid[p] + 1] += 1
    off = np.cumsum(off).astype(np.int32)
    return pid, perm, off, len(seen), np.asarray(rep, np.int32)


def plan_rows(tok_offsets, pattern_id, n_patterns: int, tile: int = 256):
    """Execution grouping at row granularity (Sec. 4.3: prompts that share a pattern run together): the token rows of
    all prompts with pattern 0 (arrival order), padded with -1 to a multiple of `tile`, then pattern 1, ... and last the
    prompts whose id is outside [0, n_patterns).  -> (rowmap [n_tiles * tile], tile_pattern [n_tiles] with -1 for the
    last bucket)."""
    tok_offsets = np.asarray(tok_offsets, dtype=np.int64)
    pattern_id = np.asarray(pattern_id, dtype=np.int64)
    rowmap, tile_pat = [], []
    for b in list(range(n_patterns)) + [-1]:
        rows = []
        for p in range(len(pattern_id)):
            pid = int(pattern_id[p]) if 0 <= pattern_id[p] < n_patterns else -1
            if pid == b:
                rows.extend(range(int(tok_offsets[p]), int(tok_offsets[p + 1])))
        if not rows:
            continue
        pad = (-len(rows)) % tile
        rowmap.extend(rows + [-1] * pad)
        tile_pat.extend([b] * ((len(rows) + pad) // tile))
    return np.asarray(rowmap, np.int32), np.asarray(tile_pat, np.int32)


# ------------------------------------------------------------------ error metric
def decode_groups(subsets, seq_pattern, G: int):
    """For a decode batch whose sequence b keeps subset subsets[seq_pattern[b]] (Sec. 4.3, rank reuse): the ascending
    list of groups that at least one sequence selected, and for every group the set of sequences that hold it as a
    bit mask (bit b = sequence b).  A sequence whose pattern id is out of range selects nothing."""
    subsets = np.asarray(subsets)
    masks = [0] * G
    for b, p in enumerate(np.asarray(seq_pattern).tolist()):
        if 0 <= p < len(subsets):
            for g in subsets[p].tolist():
                if 0 <= g < G:
                    masks[g] |= 1 << b
    used = [g for g in range(G) if masks[g]]
    return used, masks


def rel_errors(Y, Yref):
    """(Frobenius relative error, max-abs error over max-abs reference)."""
    Y = np.asarray(Y, F64); Yref = np.asarray(Yref, F64)
    fro = float(np.linalg.norm(Y - Yref) / max(np.linalg.norm(Yref), 1e-300))
    mx = float(np.max(np.abs(Y - Yref)) / max(np.max(np.abs(Yref)), 1e-300))
    return fro, mx
