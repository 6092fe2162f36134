// a6, two-launch form of the bf16 prefill product for batches that give the fused kernel too few token tiles to
// occupy the chip:  launch 1  Z = X Vt_S^T  (bf16, into the caller's workspace),  launch 2  Y = Z Ut_S.
// Both launches run ONE kernel, `gemm_tokens`: out^T[M-block, tokens] = sum_k F[M-block, k] * Tk[token, k], where F
// is a factor matrix in operand order (fetched straight from global memory, 1 KiB per wavefront instruction) and
// Tk the row-major token operand (X, then Z) staged through LDS.  A workgroup owns BT token rows x 4*NB*32
// factor rows; wavefront w owns NB consecutive 32-row factor blocks and all BT tokens, so each factor operand is
// fetched by exactly one wavefront and each staged token operand feeds NB matrix instructions.
// The intermediate costs 2*T*r_S*2 bytes of extra traffic (it stays in the last-level cache at these sizes) and
// buys a grid of (T/BT) x (M/(128 NB)) workgroups instead of T/64.
// Horizontal fusion (Sec. 4.4, Eq. 11-12): layers that read the same token rows share the two launches -- the
// first is the stacked product over the ranks of all layers, the second the batched product of every layer's own
// intermediate with its own left factor; a launch's grid is the layers' chunk lists laid end to end.
#include "prefill_common.hpp"

namespace parse {

constexpr int GT_MAX_LAYERS = 4;

// One product of one layer.  A launch covers up to GT_MAX_LAYERS of them (layers that share their token rows:
// the stacked first product and the batched second product of Sec. 4.4, Eq. 11-12): the factor-row chunks of the
// layers are numbered through, chunk_first is a layer's first.
struct GtLayer {
  const uint16_t *T;        // token operand [rows][K]
  const uint16_t *F;        // factor operands of all patterns
  uint16_t *O;              // output [rows][M]
  size_t pattern_stride;    // elements of F per pattern
  int mb_stride, kb_stride; // operand (mb, kb) starts at (mb*mb_stride + kb*kb_stride) * 512 elements
  int K, M, n_patterns;
  int chunk_first;
  const uint16_t *Fsh;      // shared head: operands of the first sh_blocks factor-row blocks (SH == 1) or
  int sh_blocks;            // reduction blocks (SH == 2) come from here, the rest from F, renumbered from 0
};
struct GtArgs {
  GtLayer L[GT_MAX_LAYERS];
  int n_layers;
  const int32_t *tok_offsets, *pattern_id;
  int rows, P;
  int ntiles, nchunks, GT;  // token tiles, factor-row chunks (all layers), token tiles per locality group
  int ngroups;              // locality groups: virtual ids run over ngroups * GT * nchunks
};

// KG = 1: four wavefronts, the whole reduction.  KG = 2: eight wavefronts, two groups of four that each run the
// same loop over one half of the reduction range with their own staged tiles and add their accumulators through
// LDS at the end.  The tile and the bytes fetched per workgroup are the same; what the second group buys is a
// second, independent instruction stream on every SIMD, so a wait of one wavefront is covered by the other.
// SH = 0: all factor operands from the pattern's block.  SH = 1: the leading factor-row blocks, SH = 2: the
// leading reduction blocks come from the layer's shared block (Sec. 4.4: shared experts at the head of memory,
// stored once) -- "two contiguous reads" per prompt instead of one.
// A workgroup walks a list of work items -- (token tile, chunk of factor rows, prompt segment of the tile) --
// one after the other; with a grid of one workgroup per compute unit and several items each, the operand
// requests of the next item are in flight while the finished item's tile is converted and written out, so neither
// the start-up round trips nor the output stores of an item sit between two reduction loops.
template <int BT, int NB, int DEPTH, int KG, int SH>
__global__ __launch_bounds__(PF_THREADS * KG) void gemm_tokens(GtArgs a) {
  constexpr int TPI = DEPTH / 4;   // staged tiles per unrolled loop iteration = ring depth in tiles
  constexpr int NT = BT / 32;
  constexpr int XP = BT * PF_BK / 8 / PF_THREADS;
  constexpr int xld = PF_BK + PF_XPAD;
  constexpr int XS_ELEMS = 2 * KG * BT * xld;
  constexpr int RED_ELEMS = KG > 1 ? PF_THREADS * 16 * NB * 2 : 0;   // one token block of accumulators, as bf16 units
  constexpr int OC = 4 * NB * 32, OLD = OC + 8;                      // output columns of the tile, padded LDS row
  constexpr int EPT = OC > 256 ? 1 : 2;                              // token blocks written out per pass
  static_assert(NT % EPT == 0, "token tiles are written out EPT blocks at a time");
  constexpr int OUT_ELEMS = EPT * 32 * OLD;
  constexpr int LDS_ELEMS = XS_ELEMS > RED_ELEMS ? (XS_ELEMS > OUT_ELEMS ? XS_ELEMS : OUT_ELEMS)
                                                 : (RED_ELEMS > OUT_ELEMS ? RED_ELEMS : OUT_ELEMS);
  __shared__ __attribute__((aligned(16))) uint16_t lds_raw[LDS_ELEMS];
  const int tid = threadIdx.x & (PF_THREADS - 1);
  const int kg = __builtin_amdgcn_readfirstlane((int)threadIdx.x / PF_THREADS);
  uint16_t *Xs = lds_raw + kg * 2 * BT * xld;
  const int lane = tid & 63, wave = tid >> 6, l32 = lane & 31, q = lane >> 5;
  // consecutive virtual ids share an XCD; a group of GT token tiles x all chunks is consecutive, so the tiles
  // of one prompt find their pattern's factors (and each other's token rows) in that die's L2.  A workgroup
  // takes `items` consecutive virtual ids.
  const int per_group = a.nchunks * a.GT;
  const int total = a.ngroups * per_group;
  const int items = (total + (int)gridDim.x - 1) / (int)gridDim.x;
  const int v_first = xcd_tile(blockIdx.x, gridDim.x) * items;
  int v_next = v_first;                       // next virtual id to look at
  const int v_end = min(v_first + items, total);

  int xdst[XP];
#pragma unroll
  for (int i = 0; i < XP; ++i) {
    const int piece = i * PF_THREADS + tid;
    xdst[i] = (piece / (PF_BK / 8)) * xld + (piece % (PF_BK / 8)) * 8;
  }
  const int xoff = l32 * xld + q * 8;

  // ---- state of the item whose reduction loop runs (set by advance()) ----
  const uint16_t *xsrc[XP];
  const uint16_t *fbase[NB], *fshared[NB];
  const uint16_t *lyT = nullptr, *lyF = nullptr, *lyFsh = nullptr;
  uint16_t *lyO = nullptr;
  size_t pattern_stride = 0, kstride = 0;
  int mb_stride = 0, K = 0, M = 0, n_patterns = 0, sh_blocks = 0, shb = 0;
  int nkb = 0, nkt = 0, nmb = 0, kbeg = 0, chunk = 0, mb0 = 0, row0 = 0, row_end = 0, seg_lo = 0, seg_hi = 0;
  bool valid = false, in_tile = false;        // in_tile: the current tile has another prompt segment to do
  u32x4 xr[2][XP];
  u32x4 fr[DEPTH][NB];

  auto fptr = [&](int i, int kb) -> const uint16_t * {
    if (SH == 2) return (kb < shb ? fshared[i] : fbase[i]) + (size_t)kb * kstride;
    return fbase[i] + (size_t)kb * kstride;
  };

  // Moves to the next item (the next prompt segment of the tile, else the next tile/chunk of this workgroup's
  // list), works out its operands and requests the first of them.  Returns false at the end of the list.
  auto advance = [&]() -> bool {
    if (in_tile) {
      seg_lo = seg_hi;
    } else {
      int tile = 0, gchunk = 0;
      for (;;) {
        if (v_next >= v_end) return false;
        const int v = v_next++;
        const int grp = v / per_group, rem = v % per_group;
        gchunk = rem / a.GT;
        tile = grp * a.GT + rem % a.GT;
        if (tile < a.ntiles) break;           // ids past the last token tile pad the last locality group
      }
      int li = 0;
#pragma unroll
      for (int i = 1; i < GT_MAX_LAYERS; ++i) li += (i < a.n_layers && gchunk >= a.L[i].chunk_first) ? 1 : 0;
      const GtLayer &ly = a.L[li];
      lyT = ly.T; lyF = ly.F; lyO = ly.O; lyFsh = ly.Fsh;
      pattern_stride = ly.pattern_stride; mb_stride = ly.mb_stride; kstride = (size_t)ly.kb_stride * 512;
      K = ly.K; M = ly.M; n_patterns = ly.n_patterns; sh_blocks = ly.sh_blocks;
      chunk = gchunk - ly.chunk_first;
      row0 = tile * BT;
      row_end = min(row0 + BT, a.rows);
      const int Kg = K / KG;
      nkb = Kg / 16; nkt = Kg / PF_BK; nmb = M / 32;
      kbeg = kg * Kg;                         // this wavefront group's part of the reduction range
      mb0 = chunk * 4 * NB + wave * NB;
      shb = SH == 2 ? sh_blocks : 0;
#pragma unroll
      for (int i = 0; i < XP; ++i) {
        const int piece = i * PF_THREADS + tid;
        const int r = piece / (PF_BK / 8), c = (piece % (PF_BK / 8)) * 8;
        xsrc[i] = lyT + (size_t)min(row0 + r, a.rows - 1) * K + kbeg + c;
      }
      seg_lo = row0;
    }
    // the first two token tiles do not depend on the prompt's pattern: requested before the prompt is looked up
#pragma unroll
    for (int i = 0; i < XP; ++i) xr[0][i] = *reinterpret_cast<const u32x4 *>(xsrc[i]);
#pragma unroll
    for (int i = 0; i < XP; ++i) xr[1][i] = *reinterpret_cast<const u32x4 *>(xsrc[i] + PF_BK);
    const int p = prompt_of_row_wave(a.tok_offsets, a.P, seg_lo);
    int hi = (p + 1 < a.P) ? a.tok_offsets[p + 1] : a.rows;
    seg_hi = min(max(hi, seg_lo + 1), row_end);
    in_tile = seg_hi < row_end;
    const int pid = a.pattern_id[p];
    valid = pid >= 0 && pid < n_patterns;
    const uint16_t *Fp = lyF + (valid ? (size_t)pid * pattern_stride : 0);
#pragma unroll
    for (int i = 0; i < NB; ++i) {
      const int mb = min(mb0 + i, nmb - 1);
      if (SH == 1) {
        const bool in_head = mb < sh_blocks;
        fbase[i] = (in_head ? lyFsh : Fp) + ((size_t)(in_head ? mb : mb - sh_blocks) * mb_stride * 64 + lane) * 8 +
                   (size_t)(kbeg / 16) * kstride;
      } else {
        fbase[i] = Fp + ((size_t)mb * mb_stride * 64 + lane) * 8 + (size_t)(kbeg / 16) * kstride;
      }
      // SH == 2: reduction block kb < shb is operand kb of the shared block, else operand kb - shb of the pattern's
      fshared[i] = SH == 2 ? lyFsh + ((size_t)mb * mb_stride * 64 + lane) * 8 : nullptr;
      if (SH == 2) fbase[i] -= (size_t)shb * kstride;
    }
#pragma unroll
    for (int d = 0; d < DEPTH; ++d)
#pragma unroll
      for (int i = 0; i < NB; ++i) fr[d][i] = *reinterpret_cast<const u32x4 *>(fptr(i, d));
    return true;
  };

  bool have = advance();
  while (have) {
    f32x16 acc[NT][NB];
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
      for (int i = 0; i < NB; ++i)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[t][i][e] = 0.f;
    __syncthreads();     // the previous item's output passes are done with the LDS
#pragma unroll
    for (int i = 0; i < XP; ++i) *reinterpret_cast<u32x4 *>(Xs + xdst[i]) = xr[0][i];
    __syncthreads();
    for (int kt0 = 0; kt0 < nkt; kt0 += TPI) {
#pragma unroll
      for (int u = 0; u < TPI; ++u) {
        const int kt = kt0 + u;   // LDS buffer = u & 1 (TPI is even)
        const int ktn = min(kt + 2, nkt - 1);
#pragma unroll
        for (int i = 0; i < XP; ++i) xr[u & 1][i] = *reinterpret_cast<const u32x4 *>(xsrc[i] + (size_t)ktn * PF_BK);
        bf16x8 xb[2][NT];
#pragma unroll
        for (int t = 0; t < NT; ++t)
          xb[0][t] = as_bf16x8(*reinterpret_cast<const u32x4 *>(Xs + (u & 1) * BT * xld + t * 32 * xld + xoff));
#pragma unroll
        for (int s = 0; s < 4; ++s) {
          if (s < 3) {
#pragma unroll
            for (int t = 0; t < NT; ++t)
              xb[(s + 1) & 1][t] =
                  as_bf16x8(*reinterpret_cast<const u32x4 *>(Xs + (u & 1) * BT * xld + t * 32 * xld + xoff + (s + 1) * 16));
          }
          __builtin_amdgcn_sched_barrier(0);
#pragma unroll
          for (int i = 0; i < NB; ++i)
#pragma unroll
            for (int t = 0; t < NT; ++t)
              acc[t][i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(fr[u * 4 + s][i]), xb[s & 1][t], acc[t][i], 0, 0, 0);
          const int kbn = min(kt * 4 + s + DEPTH, nkb - 1);
#pragma unroll
          for (int i = 0; i < NB; ++i) fr[u * 4 + s][i] = *reinterpret_cast<const u32x4 *>(fptr(i, kbn));
          __builtin_amdgcn_sched_barrier(0);
        }
#pragma unroll
        for (int i = 0; i < XP; ++i) *reinterpret_cast<u32x4 *>(Xs + ((u & 1) ^ 1) * BT * xld + xdst[i]) = xr[(u & 1) ^ 1][i];
        __syncthreads();
      }
    }
    if constexpr (KG > 1) {
      // the second group hands its accumulators over, one token block at a time (the staged tiles are dead)
      float *red = reinterpret_cast<float *>(lds_raw);
#pragma unroll
      for (int t = 0; t < NT; ++t) {
        if (kg == 1) {
#pragma unroll
          for (int i = 0; i < NB; ++i)
#pragma unroll
            for (int e = 0; e < 16; ++e) red[(i * 16 + e) * PF_THREADS + tid] = acc[t][i][e];
        }
        __syncthreads();
        if (kg == 0) {
#pragma unroll
          for (int i = 0; i < NB; ++i)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[t][i][e] += red[(i * 16 + e) * PF_THREADS + tid];
        }
        __syncthreads();
      }
    }
    // what the output passes of THIS item need, before advance() moves the state on to the next one
    uint16_t *const oO = lyO;
    const int oM = M, o_row0 = row0, o_lo = seg_lo, o_hi = seg_hi, o_chunk = chunk;
    const bool o_valid = valid;
    have = advance();    // the next item's first operands are in flight from here on
    // Output: lane holds token t*32 + l32, factor rows (mb0+i)*32 + 8*blk + 4*q + (0..3).  Tiles go through LDS,
    // EPT*32 tokens at a time, so that every store instruction writes whole output rows (OC*2 contiguous bytes
    // per token) instead of 8-byte pieces of 32 different rows.
    uint16_t *Ot = lds_raw;
#pragma unroll
    for (int tp = 0; tp < NT; tp += EPT) {
      if (tp > 0) __syncthreads();   // the previous pass has been read out
      if (kg == 0) {
#pragma unroll
        for (int t = tp; t < tp + EPT; ++t)
#pragma unroll
          for (int i = 0; i < NB; ++i)
#pragma unroll
            for (int blk = 0; blk < 4; ++blk) {
              u32x2 w;
              w[0] = o_valid ? cvt_pk_bf16(acc[t][i][blk * 4 + 0], acc[t][i][blk * 4 + 1]) : 0u;
              w[1] = o_valid ? cvt_pk_bf16(acc[t][i][blk * 4 + 2], acc[t][i][blk * 4 + 3]) : 0u;
              *reinterpret_cast<u32x2 *>(Ot + ((t - tp) * 32 + l32) * OLD + (wave * NB + i) * 32 + blk * 8 + q * 4) = w;
            }
      }
      __syncthreads();
      if (kg == 0) {
        constexpr int PPR = OC / 8;                 // 16-byte pieces per token row of the tile
        constexpr int ROWS = EPT * 32;
#pragma unroll
        for (int it = 0; it < ROWS * PPR / PF_THREADS; ++it) {
          const int piece = it * PF_THREADS + tid;
          const int r = piece / PPR, c = (piece % PPR) * 8;
          const int grow = o_row0 + tp * 32 + r, gcol = o_chunk * OC + c;
          if (grow >= o_lo && grow < o_hi && gcol < oM)
            *reinterpret_cast<u32x4 *>(oO + (size_t)grow * oM + gcol) = *reinterpret_cast<const u32x4 *>(Ot + r * OLD + c);
        }
      }
    }
  }
}

static int compute_units() {
  static int n_cu_of[64] = {0};
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 256;
  if (n_cu_of[dev] == 0) {
    hipDeviceProp_t prop;
    n_cu_of[dev] = (hipGetDeviceProperties(&prop, dev) == hipSuccess && prop.multiProcessorCount > 0) ? prop.multiProcessorCount : 256;
  }
  return n_cu_of[dev];
}

template <int BT, int NB, int DEPTH, int KG, int SH>
static int launch_gemm_tokens(GtArgs a, int GT, hipStream_t s) {
  a.ntiles = (a.rows + BT - 1) / BT;
  int chunks = 0;
  for (int l = 0; l < a.n_layers; ++l) {
    a.L[l].chunk_first = chunks;
    chunks += (a.L[l].M / 32 + 4 * NB - 1) / (4 * NB);
  }
  a.nchunks = chunks;
  a.GT = GT;
  a.ngroups = (a.ntiles + GT - 1) / GT;
  const int total = a.ngroups * GT * a.nchunks;
  // From two rounds of workgroups on, a fixed grid of one workgroup per compute unit walks the list (the next
  // item's operands are requested while the finished one is written out); below that, one item per workgroup.
  const int n_cu = compute_units();
  const int grid = total >= 2 * n_cu ? n_cu : total;
  hipLaunchKernelGGL((gemm_tokens<BT, NB, DEPTH, KG, SH>), dim3(grid), dim3(PF_THREADS * KG), 0, s, a);
  PARSE_LAUNCH_CHECK();
  return PARSE_OK;
}

// Z workspace: rows x rS bf16
size_t prefill_split_workspace_bytes(int rows, int rS) { return round_up((size_t)rows * rS * sizeof(uint16_t), 256); }

bool prefill_split_supported(int n, int rS) {
  return n % (2 * PF_BK) == 0 && rS % (2 * PF_BK) == 0 && n / 16 >= PF_DEPTH && rS / 16 >= PF_DEPTH;
}

// n_layers layers that share X (same n); p[l].X is the same pointer for all; Z[l] = layer l's part of the workspace.
int forward_prefill_split_multi_bf16(const PfArgs *p, int n_layers, uint16_t *const *Z, int avg_prompt_rows, hipStream_t s) {
  if (n_layers < 1 || n_layers > GT_MAX_LAYERS) return PARSE_ESHAPE;
  // launch 1 (stacked): factor rows = ranks of every layer (operand (rb, kb) at rb*(n/16) + kb), tokens = X
  GtArgs g1{};
  g1.n_layers = n_layers;
  g1.tok_offsets = p[0].tok_offsets; g1.pattern_id = p[0].pattern_id; g1.rows = p[0].rows; g1.P = p[0].P;
  GtArgs g2 = g1;
  bool deep2 = true, shared = false;
  for (int l = 0; l < n_layers; ++l) {
    const int rp = p[l].rS - p[l].sh_ranks;   // ranks in the per-pattern blocks
    g1.L[l] = GtLayer{p[l].X, p[l].Vt_S, Z[l], (size_t)rp * p[l].n, p[l].n / 16, 1, p[l].n, p[l].rS, p[l].n_patterns, 0,
                      p[l].Vt_sh, p[l].sh_ranks / 32};
    // launch 2 (batched): factor rows = output columns (operand (cb, kb) at kb*(m/32) + cb), tokens = Z of the layer
    g2.L[l] = GtLayer{Z[l], p[l].Ut_S, p[l].Y, (size_t)rp * p[l].m, 1, p[l].m / 32, p[l].rS, p[l].m, p[l].n_patterns, 0,
                      p[l].Ut_sh, p[l].sh_ranks / 16};
    deep2 = deep2 && (p[l].rS % (PF_BK * 4) == 0);
    shared = shared || p[l].sh_ranks > 0;
  }
  int gt64 = avg_prompt_rows / 64;  gt64 = gt64 < 1 ? 1 : (gt64 > 8 ? 8 : gt64);
  // a long reduction over few output tiles: eight wavefronts per workgroup (two reduction halves) when each
  // half is a whole number of ring periods, else four wavefronts
  const bool halves = p[0].n % (PF_BK * 4) == 0;
  int gt128 = avg_prompt_rows / 128;  gt128 = gt128 < 1 ? 1 : (gt128 > 8 ? 8 : gt128);
  // a batch with at least two rounds of 128-token tiles takes those for the first product too: a 128 x 256 tile
  // moves 40 % fewer bytes per flop through a compute unit than a 64 x 256 one
  int chunks1 = 0;
  for (int l = 0; l < n_layers; ++l) chunks1 += (p[l].rS / 32 + 7) / 8;
  const bool big = halves && (long long)((p[0].rows + 127) / 128) * chunks1 >= 512;
  int st;
  if (big) st = shared ? launch_gemm_tokens<128, 2, 16, 1, 1>(g1, gt128, s) : launch_gemm_tokens<128, 2, 16, 1, 0>(g1, gt128, s);
  else st = shared ? (halves ? launch_gemm_tokens<64, 2, 8, 2, 1>(g1, gt64, s) : launch_gemm_tokens<64, 2, 8, 1, 1>(g1, gt64, s))
                   : (halves ? launch_gemm_tokens<64, 2, 8, 2, 0>(g1, gt64, s) : launch_gemm_tokens<64, 2, 8, 1, 0>(g1, gt64, s));
  if (st != PARSE_OK) return st;
  // a deeper operand ring when every reduction length is a whole number of ring periods
  if (shared) return deep2 ? launch_gemm_tokens<128, 2, 16, 1, 2>(g2, gt128, s) : launch_gemm_tokens<128, 2, 8, 1, 2>(g2, gt128, s);
  return deep2 ? launch_gemm_tokens<128, 2, 16, 1, 0>(g2, gt128, s) : launch_gemm_tokens<128, 2, 8, 1, 0>(g2, gt128, s);
}

// O[rows][M] = Tk[rows][K] . F^T for ONE factor matrix F of M rows in the right factor's operand order (operand
// (rb, kb) at rb*(K/16) + kb), the same for every row: the first-product kernel with a single "pattern" that
// starts at F.  one_offsets = device {0, rows}, zero_id = device {0}.  K % 128 == 0, M % 32 == 0, K >= 128.
int tokens_times_factor_bf16(const uint16_t *Tk, const uint16_t *F, uint16_t *O, int rows, int K, int M,
                             const int32_t *one_offsets, const int32_t *zero_id, hipStream_t s) {
  if (K % (2 * PF_BK) != 0 || M % 32 != 0 || K / 16 < PF_DEPTH) return PARSE_ESHAPE;
  GtArgs g{};
  g.n_layers = 1;
  g.tok_offsets = one_offsets; g.pattern_id = zero_id; g.rows = rows; g.P = 1;
  g.L[0] = GtLayer{Tk, F, O, 0, K / 16, 1, K, M, 1, 0, nullptr, 0};
  return (K % (PF_BK * 4) == 0) ? launch_gemm_tokens<64, 2, 8, 2, 0>(g, 8, s) : launch_gemm_tokens<64, 2, 8, 1, 0>(g, 8, s);
}

int forward_prefill_split_bf16(const PfArgs &p, uint16_t *Z, int avg_prompt_rows, hipStream_t s) {
  uint16_t *Zs[1] = {Z};
  return forward_prefill_split_multi_bf16(&p, 1, Zs, avg_prompt_rows, s);
}

}  // namespace parse
