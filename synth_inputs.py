"""Seeded synthetic inputs for the routed low-rank linear layer.

This module only draws random numbers and lays them out; it holds none of the
method's arithmetic (no routing, no cache logic, no products of factors with
activations).  Both the CPU oracle's tests and the GPU path's tests are fed
from here, so the two sides see byte-identical inputs.

Workload recipe (LLaMA-7B-shaped, values Gaussian):
  * factors: U0 (m x R) and V (R x n) have orthonormal columns / rows, taken
    from the QR factorisation of an N(0,1) matrix; singular values are
    sigma_i = (i+1)^-0.5; the stored left factor has sigma folded in
    (Sec. 4.4, Eq. 10: A = U Sigma, B^T = V with whitening absorbed).
  * router: W_r ~ N(0, 1/d), one bias-free linear map per matrix (Sec. 4.1,
    Eq. 5; Sec. 5.1 "single linear gating layer").
  * activations: N(0,1) tokens, `tok_offsets` gives the ragged prompt layout.
  * clustered prompt embeddings for the pattern-cache workload: Gaussian
    centroids plus isotropic noise.
Storage layout handed to both sides: rank-major `Vt[R][n]` (= B^T) and
`Ut[R][m]` (= A^T), each rank expert's vectors contiguous, a rank group one
contiguous slab of gs = R/G rows.
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np

SEED_BASE = 8568 * 10


# --------------------------------------------------------------------------
# bfloat16 storage helpers (bit patterns only; rounding is round-to-nearest-even,
# the format's standard conversion from binary32)
# --------------------------------------------------------------------------
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """binary32 -> bfloat16 bit patterns (uint16), round to nearest even."""
    b = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    lsb = (b >> np.uint32(16)) & np.uint32(1)
    r = b + np.uint32(0x7FFF) + lsb
    return (r >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    """bfloat16 bit patterns (uint16) -> the exact binary32 values."""
    return (np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


# --------------------------------------------------------------------------
# containers
# --------------------------------------------------------------------------
@dataclass
class Layer:
    """One routed low-rank linear: W = sum_i sigma_i u_i v_i^T, split in G groups."""
    n: int                  # d_in
    m: int                  # d_out
    R: int                  # stored rank
    G: int                  # rank groups
    dtype: str              # "f32" | "bf16"
    U0: np.ndarray          # [m][R] float64, orthonormal columns
    sigma: np.ndarray       # [R]    float64
    V: np.ndarray           # [R][n] float64, orthonormal rows
    Vt_store: np.ndarray    # [R][n] float32, or uint16 bf16 bits: what the device holds
    Ut_store: np.ndarray    # [R][m] same, sigma folded in

    @property
    def gs(self) -> int:
        return self.R // self.G

    def stored_values(self):
        """(Vt, Ut) as float64 arrays holding exactly the stored (rounded) values."""
        if self.dtype == "bf16":
            return (bf16_bits_to_f32(self.Vt_store).astype(np.float64),
                    bf16_bits_to_f32(self.Ut_store).astype(np.float64))
        return self.Vt_store.astype(np.float64), self.Ut_store.astype(np.float64)


@dataclass
class Workload:
    name: str
    layers: list
    Wr: np.ndarray              # [L][G][d] float32
    k: int
    d: int
    dtype: str
    tok_offsets: np.ndarray     # [P+1] int32
    X: np.ndarray               # [T_total][n] float32 or bf16 bits (layer 0's input width)
    extra: dict = field(default_factory=dict)

    @property
    def P(self) -> int:
        return len(self.tok_offsets) - 1

    def X_values(self) -> np.ndarray:
        if self.dtype == "bf16":
            return bf16_bits_to_f32(self.X).astype(np.float64)
        return self.X.astype(np.float64)


# --------------------------------------------------------------------------
# generators
# --------------------------------------------------------------------------
def orthonormal_columns(rng: np.random.Generator, rows: int, cols: int) -> np.ndarray:
    """rows x cols matrix with orthonormal columns (QR of an N(0,1) matrix)."""
    q, _ = np.linalg.qr(rng.standard_normal((rows, cols)))
    return q


def make_layer(rng, n: int, m: int, R: int, G: int, dtype: str, fast: bool = False) -> Layer:
    """fast=True replaces QR by column-normalised Gaussians (timing-only workloads)."""
    assert R % G == 0 and R <= min(m, n)
    if fast:
        U0 = rng.standard_normal((m, R))
        U0 /= np.linalg.norm(U0, axis=0, keepdims=True)
        V = rng.standard_normal((n, R))
        V = (V / np.linalg.norm(V, axis=0, keepdims=True)).T.copy()
    else:
        U0 = orthonormal_columns(rng, m, R)
        V = orthonormal_columns(rng, n, R).T.copy()
    sigma = (np.arange(R, dtype=np.float64) + 1.0) ** -0.5
    Ut32 = np.ascontiguousarray((U0 * sigma[None, :]).T, dtype=np.float32)
    Vt32 = np.ascontiguousarray(V, dtype=np.float32)
    if dtype == "bf16":
        Ut_store, Vt_store = f32_to_bf16_bits(Ut32), f32_to_bf16_bits(Vt32)
    else:
        Ut_store, Vt_store = Ut32, Vt32
    return Layer(n, m, R, G, dtype, U0, sigma, V, Vt_store, Ut_store)


def make_tokens(rng, rows: int, width: int, dtype: str) -> np.ndarray:
    x = rng.standard_normal((rows, width)).astype(np.float32)
    return f32_to_bf16_bits(x) if dtype == "bf16" else x


def make_router(rng, L: int, G: int, d: int) -> np.ndarray:
    return (rng.standard_normal((L, G, d)) / np.sqrt(d)).astype(np.float32)


def offsets_from_lengths(lengths) -> np.ndarray:
    off = np.zeros(len(lengths) + 1, dtype=np.int32)
    off[1:] = np.cumsum(np.asarray(lengths, dtype=np.int64))
    return off


def clustered_embeddings(rng, P: int, d: int, n_clusters: int, spread: float):
    """Embeddings e_p = centroid[c_p] + spread * N(0, I); returns (E float32, cluster ids)."""
    cent = rng.standard_normal((n_clusters, d))
    cid = rng.integers(0, n_clusters, size=P)
    E = cent[cid] + spread * rng.standard_normal((P, d))
    return E.astype(np.float32), cid.astype(np.int32)


# --------------------------------------------------------------------------
# named workloads
# --------------------------------------------------------------------------
def config0(seed: int = SEED_BASE + 0) -> Workload:
    """Tiny fp32 layer: n=m=1024, R=256 in 8 groups of 32, top-4, 4 prompts x 64 tokens."""
    rng = np.random.default_rng(seed)
    lay = make_layer(rng, 1024, 1024, 256, 8, "f32")
    Wr = make_router(rng, 1, 8, 1024)
    off = offsets_from_lengths([64] * 4)
    X = make_tokens(rng, int(off[-1]), 1024, "f32")
    return Workload("config0", [lay], Wr, 4, 1024, "f32", off, X)


def config1(seed: int = SEED_BASE + 1, P: int = 8, T: int = 512, fast: bool = False) -> Workload:
    """q_proj-shaped bf16 prefill: 4096x4096, R=2048 in 16 groups of 128, top-8."""
    rng = np.random.default_rng(seed)
    lay = make_layer(rng, 4096, 4096, 2048, 16, "bf16", fast=fast)
    Wr = make_router(rng, 1, 16, 4096)
    off = offsets_from_lengths([T] * P)
    X = make_tokens(rng, int(off[-1]), 4096, "bf16")
    return Workload("config1", [lay], Wr, 8, 4096, "bf16", off, X)


def config2(seed: int = SEED_BASE + 2, B: int = 32, n_patterns: int = 4, fast: bool = False,
            hidden: int = 4096, inter: int = 11008, R: int = 2560, G: int = 20, k: int = 10) -> Workload:
    """MLP-shaped bf16 decode: gate/up hidden->inter, down inter->hidden; R=2560 in 20 groups, top-10.

    `extra["pattern_emb"]` holds n_patterns random embeddings whose routes define the
    patterns; sequence i uses pattern i mod n_patterns for every step."""
    rng = np.random.default_rng(seed)
    layers = [make_layer(rng, hidden, inter, R, G, "bf16", fast=fast),
              make_layer(rng, hidden, inter, R, G, "bf16", fast=fast),
              make_layer(rng, inter, hidden, R, G, "bf16", fast=fast)]
    Wr = make_router(rng, 3, G, hidden)
    pe = rng.standard_normal((n_patterns, hidden)).astype(np.float32)
    off = offsets_from_lengths([1] * B)
    X = make_tokens(rng, B, hidden, "bf16")
    Xd = make_tokens(rng, B, inter, "bf16")
    return Workload("config2", layers, Wr, k, hidden, "bf16", off, X,
                    {"pattern_emb": pe, "seq_pattern": (np.arange(B) % n_patterns).astype(np.int32),
                     "X_down": Xd})


def config4_embeddings(seed: int = SEED_BASE + 4, P: int = 256, d: int = 4096,
                       n_clusters: int = 16, spread: float = 0.1, G: int = 20, L: int = 3):
    """Cache stress inputs: clustered embeddings, prompt lengths U{32..2048}, router [L][G][d]."""
    rng = np.random.default_rng(seed)
    E, cid = clustered_embeddings(rng, P, d, n_clusters, spread)
    lengths = rng.integers(32, 2049, size=P)
    Wr = make_router(rng, L, G, d)
    return E, cid, offsets_from_lengths(lengths), Wr


def pad_groups(lay: Layer, multiple: int = 32) -> Layer:
    """The same layer with every rank group padded with zero ranks to a multiple of `multiple` ranks (the
    operand-order layout wants groups of whole 32-rank blocks; a zero rank contributes nothing).  Pure data
    movement: stored rows are copied, padding rows are zero; U0 / sigma / V are padded alike."""
    gs, G = lay.gs, lay.G
    gp = (gs + multiple - 1) // multiple * multiple
    if gp == gs:
        return lay
    def pad_rows(a):      # [R][w] -> [G*gp][w]
        out = np.zeros((G, gp) + a.shape[1:], dtype=a.dtype)
        out[:, :gs] = a.reshape((G, gs) + a.shape[1:])
        return out.reshape((G * gp,) + a.shape[1:])
    U0 = None if lay.U0 is None else pad_rows(np.ascontiguousarray(lay.U0.T)).T.copy()
    sigma = None if lay.sigma is None else pad_rows(lay.sigma.reshape(-1, 1)).reshape(-1)
    V = None if lay.V is None else pad_rows(lay.V)
    return Layer(lay.n, lay.m, G * gp, G, lay.dtype, U0, sigma, V, pad_rows(lay.Vt_store), pad_rows(lay.Ut_store))


def config3_ranks(n: int, m: int, G: int = 16, kept: float = 0.6):
    """Stored rank of one projection of the full-stack workload: the factors keep `kept` of the dense parameter
    count, R = kept*m*n/(m+n), rounded so that a group holds a multiple of 16 ranks.  Returns (R, gs)."""
    R = kept * m * n / (m + n)
    gs = 16 * int(round(R / G / 16))
    return gs * G, gs


def small_layer(seed: int, n: int, m: int, R: int, G: int, dtype: str) -> Layer:
    return make_layer(np.random.default_rng(seed), n, m, R, G, dtype)
