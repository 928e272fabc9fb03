// Step 2 of the A^3 fusion path: question-relevance score, Eq. 3 first line.
//
//   s_i = sum_{hq} sum_j softmax_i( q_{j,hq} . k'_{i, hq/G} * scale )      softmax over the context keys
//
// A column sum of row softmaxes needs every row's (max, sum exp) before any column can be
// summed, so the logits are formed twice:
//   pass A   per (run of keys, row): partial (max, sum exp)       -> workspace
//   pass B   per run of keys: the partials of a row are merged (in the prologue; the fp32 path has a small
//            kernel for it), then sum over all rows of exp(l - max)/sum -> per KV head column sums
//   head sum per token: the KV heads in order                      -> scores
// Rows, then heads, are reduced in a fixed order, so the result is deterministic (no atomics).
//
// bf16: logits on the matrix cores (32x32x16 bf16 MFMA), two kernels.  Up to 256 rows per KV head (a question of
// 64 tokens at 4 query heads per KV head): keys and the rows' Q tile stream through LDS by direct-to-LDS loads,
// one workgroup per CU with its whole run of keys in flight (scores_bf16_kernel).  More rows: a 256-key tile
// stays in LDS and the waves walk the rows, two workgroups per CU (scores_rows_bf16_kernel).  exp2 with log2(e)
// folded into the scale.
// fp32: plain FMA kernels (correctness configuration).
#include <mutex>

#include "a3_internal.h"

namespace {

constexpr float kLog2e = 1.4426950408889634f;

// largest i in [0, n) with a[i] <= x (a ascending, a[0] <= x)
__device__ __forceinline__ int find_segment(const int *__restrict__ a, int n, int x) {
  int lo = 0, hi = n;
  while (lo < hi) {
    int mid = (lo + hi) >> 1;
    if (a[mid] <= x) lo = mid + 1; else hi = mid;
  }
  return lo - 1;
}

struct scores_args {
  const void *q;            // [sum q_len, Hq, d]
  const void *k;            // [T, Hkv, d]
  const int *seg_start, *ctx_len, *q_len, *q_start;
  float2 *part;             // [n_tiles, total_rows] partial (max, sum) in the exp2 domain
  float2 *stats;            // [total_rows] (max + log2(sum), unused): written by the combine kernel
  int merged;               // bf16 path: the combine kernel has run (more than 32 runs of keys, rows in chunks, or
                            // question keys in the denominator); otherwise the second pass merges the partials itself
  float *scores;            // [T]
  float *part_scores;       // [Hkv, T] bf16 path: per KV head partial scores
  int n_req, Hq, Hkv, d, T, total_rows, n_tiles, tile_keys;
  uint32_t inv_G;           // ceil(2^32 / G) for G > 1: m / G = umulhi(m, inv_G) for every m < 2^32 / G
  float scale2;             // sm_scale * log2(e)
  float inv_scale2;
  int one_ctx_len, one_q_len;   // a single request whose segment starts at row 0: its lengths; otherwise -1
  // fused position recovery (first pass of the bf16 path only): stale keys in, realigned keys out
  const void *k_cat;        // [T, Hkv, d] keys at chunk-local positions
  void *k_out;              // [T, Hkv, d] realigned keys (may be k_cat itself)
  const int *tok_chunk;     // [T] chunk of a context row, -1 for question rows
  const float2 *chunk_cs;   // [n_chunks, d/2] (cos, sin) of chunk offset x theta_i
  int rope_layout;
  // the softmax of a question token also runs over the question keys up to itself (their (max, sum) sits
  // in the extra partial slot n_tiles): the literal denominator of Eq. 3 and the window votes of the
  // eviction extension
  int causal_q;
};

// ---------------------------------------------------------------------------------------
// (max, sum exp) of a question row over the question keys it sees (itself and the earlier ones of its
// request): one wave per (question token, query head), lanes over keys.  A few hundred short dot products.
// ---------------------------------------------------------------------------------------
template <typename T>
__global__ void __launch_bounds__(256)
scores_question_stats_kernel(scores_args a) {
  const int lane = threadIdx.x & 63, row = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= a.total_rows) return;
  const int jq = row / a.Hq, hq = row % a.Hq;
  const int r = find_segment(a.q_start, a.n_req, jq);
  const int j = jq - a.q_start[r];
  if (j >= a.q_len[r]) return;                                 // rows past the last request's question
  const int g = hq / (a.Hq / a.Hkv);
  const T *__restrict__ Q = (const T *)a.q + (size_t)row * a.d;
  const T *__restrict__ K = (const T *)a.k;
  const int key0 = a.seg_start[r] + a.ctx_len[r];
  float m = -INFINITY, z = 0.f;
  for (int u = lane; u <= j; u += 64) {
    const T *kp = K + ((size_t)(key0 + u) * a.Hkv + g) * a.d;
    float dot = 0.f;
    for (int c = 0; c < a.d; ++c) dot = fmaf((float)Q[c], (float)kp[c], dot);
    const float l = dot * a.scale2;
    const float mn = fmaxf(m, l);
    z = z * exp2f(m - mn) + exp2f(l - mn);                     // m = -inf, z = 0 on the first key: 0 * 0
    m = mn;
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) {
    const float pm = __shfl_xor(m, off), pz = __shfl_xor(z, off);
    const float mn = fmaxf(m, pm);
    const float za = z > 0.f ? z * exp2f(m - mn) : 0.f, zb = pz > 0.f ? pz * exp2f(pm - mn) : 0.f;
    z = (lane & off) ? zb + za : za + zb;
    m = mn;
  }
  if (lane == 0) a.part[(size_t)a.n_tiles * a.total_rows + row] = make_float2(m, z);
}

// ---------------------------------------------------------------------------------------
// combine partial row statistics (shared by both element types)
// ---------------------------------------------------------------------------------------
constexpr int kTileKeys = 64;      // fp32 kernels

__global__ void __launch_bounds__(256)
scores_combine_kernel(scores_args a) {
  // one row per 16 lanes: the lanes split the row's tiles, then merge pairwise (fixed tree)
  const int row = blockIdx.x * 16 + (threadIdx.x >> 4);
  const int slice = threadIdx.x & 15;
  float m = -INFINITY, z = 0.f;
  if (row < a.total_rows) {
    const int jq = row / a.Hq;
    const int r = find_segment(a.q_start, a.n_req, jq);
    const int tiles = (a.ctx_len[r] + a.tile_keys - 1) / a.tile_keys;
    for (int t = slice; t < tiles; t += 16) {
      float2 p = a.part[(size_t)t * a.total_rows + row];
      float mn = fmaxf(m, p.x);
      z = z * exp2f(m - mn) + p.y * exp2f(p.x - mn);
      m = mn;
    }
    if (a.causal_q && slice == 15) {                           // the question keys' share (slice 15 has the fewest tiles)
      float2 p = a.part[(size_t)a.n_tiles * a.total_rows + row];
      float mn = fmaxf(m, p.x);
      z = (z > 0.f ? z * exp2f(m - mn) : 0.f) + p.y * exp2f(p.x - mn);
      m = mn;
    }
  }
#pragma unroll
  for (int off = 8; off > 0; off >>= 1) {
    const float pm = __shfl_xor(m, off, 16), pz = __shfl_xor(z, off, 16);
    const float mn = fmaxf(m, pm);
    // a side that saw no tile has (m, z) = (-inf, 0): its factor must not become exp2(nan)
    const float za = z > 0.f ? z * exp2f(m - mn) : 0.f, zb = pz > 0.f ? pz * exp2f(pm - mn) : 0.f;
    z = (slice & off) ? zb + za : za + zb;                     // same operand order in both lanes of a pair
    m = mn;
  }
  // exp2(l - m) / z = exp2(l - (m + log2 z)): pass B subtracts one number per row
  if (slice == 0 && row < a.total_rows) a.stats[row] = make_float2(z > 0.f ? m + log2f(z) : INFINITY, 0.f);
}

// ---------------------------------------------------------------------------------------
// bf16 MFMA kernels, head_dim 128.  PASS 0 = partial row statistics, PASS 1 = column sums.
//
// Workgroup (8 waves) = up to 256 (question token, head) rows of one KV head against one run of
// `tile_keys` context keys of one request.  The keys stream through a ring of eight 64-key slots in LDS
// (direct-to-LDS loads by waves 0-3: four slots and the rows' Q tile are requested first thing, whole 256-byte
// rows, coalesced; the Q tile is read into registers once and its place then serves as slots 4-7, so a run of
// up to 512 keys is in flight in full).  Wave (rg, kh) owns rows 64 rg .. 64 rg + 63 and the keys
// 32 kh .. 32 kh + 31 of every slot; the two waves of a row group share a SIMD and run their matrix phase (the
// logits of a block: 16 MFMAs) and their vector phase (the exponentials of a block) in opposite order.
//   PASS 0  C[key][row]: a lane owns a row; per-row (max, sum exp) over the run -> one partial per (run, row)
//   PASS 1  C[row][key]: a lane owns a key; the partials of all runs are merged per row (fixed order, the
//           same in every workgroup), then sum over rows of exp2(l - stat) -> per (KV head, row chunk) column
//           sums; a last small kernel adds them in fixed order.
// ---------------------------------------------------------------------------------------
constexpr int kD = 128;
constexpr int kKRowBytes = kD * 2;                 // LDS rows are unpadded; their 16-byte pieces are XOR-swizzled
constexpr int kSlotKeys = 64;
constexpr int kSlots = 8;                          // the Q tile first occupies the place of slots 4 .. 7
constexpr int kSlotBytes = kSlotKeys * kKRowBytes; // 16 KB
constexpr int kChunkRows = 256;                    // rows of the score matrix per workgroup
constexpr int kScoreThreads = 512;
constexpr int kMinTileKeys = 256, kMaxTileKeys = 1024;
constexpr int kLdsQ = 4 * kSlotBytes;                            // Q tile [256][128] bf16, swizzled: read into registers
static_assert(kChunkRows * kKRowBytes == 4 * kSlotBytes, "the Q tile takes the place of four slots");   // before slot 4 is filled
constexpr int kLdsSt = kSlots * kSlotBytes;                       // [256] float: max + log2(sum) per row (PASS 1)
constexpr int kLdsRed = kLdsSt + kChunkRows * 4;                  // [4 rg][tile_keys] float column sums (PASS 1)
constexpr size_t kScoresLds = kLdsRed + 4 * kMaxTileKeys * 4;

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ __forceinline__ float halves_max(float x) {
  const uint32_t u = __float_as_uint(x);
  auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);   // low-half values / high-half values in all lanes
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float halves_sum(float x) {
  const uint32_t u = __float_as_uint(x);
  auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}
// Workgroup barrier that orders LDS traffic only: this wave's LDS accesses are complete before it, none of the
// later ones starts ahead of it.  (__syncthreads() would also wait for every global access in flight, i.e. for
// the whole ring of keys.)
#define A3_LDS_BARRIER()                                        \
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local"); \
  __builtin_amdgcn_s_barrier();                                 \
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local")
// vmcnt(n) alone (the other counters open): n = 0 .. 63
#define A3_VMCNT(n) __builtin_amdgcn_s_waitcnt(((n) & 15) | (((n) >> 4) << 14) | (7 << 4) | (15 << 8))

// row m = j * G + hh of a KV head's row space -> row of the [sum q_len, Hq] query tensor
struct row_map {
  int G, Hq, g, qrow0;
  uint32_t inv_G;
  __device__ __forceinline__ int operator()(int m) const {
    const int j = G > 1 ? (int)__umulhi((uint32_t)m, inv_G) : m;
    return (qrow0 + j) * Hq + g * G + (m - j * G);
  }
};

// At most 256 rows per KV head (longer questions and wide groups go to scores_rows_bf16_kernel below).
template <int PASS, bool REALIGN>
__global__ void __launch_bounds__(kScoreThreads, 2)
scores_bf16_kernel(scores_args a) {
  extern __shared__ __align__(16) unsigned char lds_raw[];
  // ---- which part of the problem: blockIdx % Hkv = KV head (with 8 heads: one head per XCD, whose L2 then
  // holds that head's Q rows and partial statistics) ----------------------------------------------------
  const int g = blockIdx.x % a.Hkv;
  int rest = blockIdx.x / a.Hkv;
  const int t = rest % a.n_tiles, r = rest / a.n_tiles;
  // (a batch of one request: its lengths are the layout's maxima, known on the host; no loads before the first keys
  // are requested)
  const int N = a.one_ctx_len >= 0 ? a.one_ctx_len : a.ctx_len[r];
  const int i0 = t * a.tile_keys;
  if (i0 >= N) return;
  const int G = a.Hq / a.Hkv;
  const int Mg = (a.one_ctx_len >= 0 ? a.one_q_len : a.q_len[r]) * G;   // rows of this KV head: m = j * G + hh
  if (Mg <= 0) return;
  const int s = a.one_ctx_len >= 0 ? 0 : a.seg_start[r], qrow0 = a.one_ctx_len >= 0 ? 0 : a.q_start[r];
  const row_map row_of{G, a.Hq, g, qrow0, a.inv_G};
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, lhi = lane >> 5;
  const int n_keys = min(a.tile_keys, N - i0);
  const int nQ = (n_keys + kSlotKeys - 1) / kSlotKeys;         // slots of this run, >= 1
  const bf16_t *__restrict__ Q = (const bf16_t *)a.q;
  const bf16_t *__restrict__ K = (const bf16_t *)a.k;
  const uint32_t lds_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char *)lds_raw;
  float *St = reinterpret_cast<float *>(lds_raw + kLdsSt);
  float *red = reinterpret_cast<float *>(lds_raw + kLdsRed);

  // Wave (rg, kh) owns the rows 64 rg .. 64 rg + 63 and the keys 32 kh .. 32 kh + 31 of every slot; the waves
  // (rg, 0) and (rg, 1) share a SIMD.  Between two barriers each wave forms the logits of one block (16 MFMAs
  // back to back: the matrix pipe) and folds one block into the row statistics / column sums (exponentials: the
  // vector ALU).  The kh = 0 waves do that in the order "logits of slot i + 1, fold slot i + 1", the kh = 1 waves
  // in the order "fold slot i, logits of slot i + 1": at any time one wave of a SIMD is in its matrix phase and
  // the other in its vector phase, each a plain stream of one kind of instruction.
  const int rg = wave & 3, kh = wave >> 2;

  // ---- direct-to-LDS loads (16 bytes per lane, lane i lands at base + 16 i), waves 0-3 only.  One wave
  // instruction brings 4 rows x 256 B; instruction j of wave w covers rows 4 (4 j + w) .. + 3 of a 64-row
  // group.  The lane fetches piece (slot ^ row % 16) of its row, so LDS slot s of row x holds piece
  // s ^ (x % 16) and the 16 rows a quarter wave reads at one piece index touch all 64 banks once.  Inline
  // assembly: the compiler then does not track these as LDS writes (it would wait for all of them before
  // every LDS read); the explicit vmcnt waits below cover them, and waves 0-3 issue no other vector memory
  // access until the ring has drained, so the counts are exact.  Waves 4-7 issue none: the compiler's own
  // counting is exact there (PASS 1 merges the partial statistics in those waves meanwhile).
  const bool loads = wave < 4;
  const int drow = 4 * (wave & 3) + (lane >> 4);               // row of the lane in instruction 0
  const int dpiece = (lane & 15) ^ (drow & 15);                // (drow + 16 j) % 16 does not depend on j
#define A3_KDMA(I)                                                                                             \
  _Pragma("unroll") for (int j = 0; j < 4; ++j) {                                                              \
    const int row_ = min(s + i0k + (I) * kSlotKeys + drow + 16 * j, a.T - 1);  /* past the run: loaded, masked */ \
    const bf16_t *gp_ = K + ((size_t)row_ * a.Hkv + g) * kD + dpiece * 8;                                      \
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off"                                         \
                 :: "s"(__builtin_amdgcn_readfirstlane(lds_base + ((I) & (kSlots - 1)) * kSlotBytes +           \
                                                       4 * (4 * j + (wave & 3)) * kKRowBytes)), "v"(gp_) : "memory"); \
  }
  // the Q tile: rows MBASE .. + 255 of this head (rows past Mg: a copy of the last row, ignored later)
#define A3_QDMA(MBASE)                                                                                         \
  _Pragma("unroll") for (int j = 0; j < 16; ++j) {                                                             \
    const int m_ = min((MBASE) + drow + 16 * j, Mg - 1);                                                       \
    const bf16_t *gp_ = Q + (size_t)row_of(m_) * kD + dpiece * 8;                                              \
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off"                                         \
                 :: "s"(__builtin_amdgcn_readfirstlane(lds_base + kLdsQ + 4 * (4 * j + wave) * kKRowBytes)), "v"(gp_) \
                 : "memory");                                                                                  \
  }
  const int i0k = i0, total_rows = a.total_rows;
  constexpr int m_base = 0;
  if (loads) {
    if (!REALIGN) { A3_KDMA(0) }
    A3_QDMA(0)
    if (!REALIGN) {
      if (nQ > 1) { A3_KDMA(1) }
      if (nQ > 2) { A3_KDMA(2) }
      if (nQ > 3) { A3_KDMA(3) }
    }
  }
  // ---- PASS 1, waves 4-7: max + log2(sum exp) of the 256 rows from the partials of all runs (every workgroup
  // of the row chunk forms the same numbers in the same order) --------------------------------------------
  if (PASS == 1 && wave >= 4) {
    const int ml = tid - 256, m = m_base + ml;
    float st = INFINITY;                                       // rows past Mg add nothing (see acc0 below)
    if (m < Mg) {
      const int row_id = row_of(m);
      const int runs = (N + a.tile_keys - 1) / a.tile_keys;
      if (a.merged) {
        st = a.stats[row_id].x;                                // many runs: a small kernel has merged them already
      } else {
        // first the maximum over the runs, then the sums rescaled to it, added in run order (at most 32 runs)
        float mx = -INFINITY, z = 0.f;
        float2 p[32];
#pragma unroll
        for (int u = 0; u < 32; ++u)
          p[u] = u < runs ? a.part[(size_t)u * total_rows + row_id] : make_float2(-INFINITY, 0.f);
#pragma unroll
        for (int u = 0; u < 32; ++u) mx = fmaxf(mx, p[u].x);
        // a run that saw no key has (max, sum) = (-inf, 0): its factor must not become exp2(nan)
#pragma unroll
        for (int u = 0; u < 32; ++u) z += p[u].y > 0.f ? p[u].y * fast_exp2(p[u].x - mx) : 0.f;
        // exp2(l - m) / z = exp2(l - (m + log2 z)): one number per row
        st = z > 0.f ? mx + log2f(z) : INFINITY;
      }
    }
    St[ml] = st;
  }

  // fragment reads: row / key 32 b + l32 of a 64-row group, piece 2 ks + lhi -> slot (2 ks + lhi) ^ (l32 % 16)
  const int kswz = (lhi ^ (l32 & 15)) * 16;
  const unsigned char *kt = lds_raw + (kh * 32 + l32) * kKRowBytes;      // + slot * kSlotBytes
  const unsigned char *qt = lds_raw + kLdsQ + (rg * 64 + l32) * kKRowBytes;

  // REALIGN: the stale keys come through registers, every pair is turned by its chunk's offset (Eq. 2), and
  // the rounded result goes both to the realigned cache and, in the swizzled layout, to the ring.  A lane owns
  // the 16-byte pieces c and c + 8 of one key per slot: in either pairing (adjacent coordinates, or i with
  // i + 64) it then holds whole pairs.  Three slots are in flight in registers.
  const bf16_t *Kc = (const bf16_t *)a.k_cat;                  // may be the same buffer as k_out
  bf16_t *Ko = (bf16_t *)a.k_out;
  const int rc = tid & 7, rkey = tid >> 3;
  constexpr int kPF = 3;
  bf16x8 plo[kPF], phi[kPF];
  int pchunk[kPF];
  float2 csr[8];
  int cs_cur = -1;
  const bool inter = a.rope_layout == A3_ROPE_INTERLEAVED;
#define A3_RLOAD(I, P)                                                                                         \
  {                                                                                                            \
    const int key_ = (I) * kSlotKeys + rkey;                                                                   \
    const int row_ = min(s + i0k + key_, a.T - 1);               /* past the run: loaded, never stored */      \
    const size_t off_ = ((size_t)row_ * a.Hkv + g) * kD;                                                       \
    plo[P] = *reinterpret_cast<const bf16x8 *>(Kc + off_ + 8 * rc);                                            \
    phi[P] = *reinterpret_cast<const bf16x8 *>(Kc + off_ + 64 + 8 * rc);                                       \
    pchunk[P] = key_ < n_keys ? a.tok_chunk[row_] : -1;                                                        \
  }
  // turns the registers of slot I and stores them
#define A3_RSTORE(I, P)                                                                                        \
  {                                                                                                            \
    const int key_ = (I) * kSlotKeys + rkey;                                                                   \
    const int row_ = min(s + i0k + key_, a.T - 1);                                                             \
    const size_t off_ = ((size_t)row_ * a.Hkv + g) * kD;                                                       \
    bf16x8 rlo = plo[P], rhi = phi[P];                                                                         \
    if (pchunk[P] >= 0) {                                                                                      \
      if (pchunk[P] != cs_cur) {                                                                               \
        const float2 *cs = a.chunk_cs + (size_t)pchunk[P] * (kD / 2);                                          \
        _Pragma("unroll") for (int e = 0; e < 8; ++e)   /* interleaved: pairs 4c..4c+3 and 32+4c..; half: 8c..8c+7 */ \
          csr[e] = inter ? cs[(e < 4 ? 4 * rc : 28 + 4 * rc) + e] : cs[8 * rc + e];                            \
        cs_cur = pchunk[P];                                                                                    \
      }                                                                                                        \
      if (inter) {                                                                                             \
        _Pragma("unroll") for (int p2 = 0; p2 < 4; ++p2) {                                                     \
          float y0, y1;                                                                                        \
          a3_rotate_pair(a3_bf2f(plo[P][2 * p2]), a3_bf2f(plo[P][2 * p2 + 1]), csr[p2], y0, y1);               \
          rlo[2 * p2] = a3_f2bf(y0); rlo[2 * p2 + 1] = a3_f2bf(y1);                                            \
          a3_rotate_pair(a3_bf2f(phi[P][2 * p2]), a3_bf2f(phi[P][2 * p2 + 1]), csr[4 + p2], y0, y1);           \
          rhi[2 * p2] = a3_f2bf(y0); rhi[2 * p2 + 1] = a3_f2bf(y1);                                            \
        }                                                                                                      \
      } else {                                                                                                 \
        _Pragma("unroll") for (int e = 0; e < 8; ++e) {          /* coordinate 8c+e pairs with 64+8c+e */      \
          float y0, y1;                                                                                        \
          a3_rotate_pair(a3_bf2f(plo[P][e]), a3_bf2f(phi[P][e]), csr[e], y0, y1);                              \
          rlo[e] = a3_f2bf(y0); rhi[e] = a3_f2bf(y1);                                                          \
        }                                                                                                      \
      }                                                                                                        \
    }                                                                                                          \
    if (key_ < n_keys) {                                                                                       \
      *reinterpret_cast<bf16x8 *>(Ko + off_ + 8 * rc) = rlo;                                                   \
      *reinterpret_cast<bf16x8 *>(Ko + off_ + 64 + 8 * rc) = rhi;                                              \
    }                                                                                                          \
    unsigned char *ld_ = lds_raw + ((I) & (kSlots - 1)) * kSlotBytes + rkey * kKRowBytes;                      \
    *reinterpret_cast<bf16x8 *>(ld_ + ((rc ^ (rkey & 15)) * 16)) = rlo;                                        \
    *reinterpret_cast<bf16x8 *>(ld_ + (((rc + 8) ^ (rkey & 15)) * 16)) = rhi;                                  \
  }
  // slot I + 1 goes from this lane's registers to the ring, then the registers take slot I + 1 + kPF
#define A3_RSTEP_STORE(I)                                                                                      \
  if (((I) + 1) % kPF == 0) { A3_RSTORE((I) + 1, 0) } else if (((I) + 1) % kPF == 1) { A3_RSTORE((I) + 1, 1) }  \
  else { A3_RSTORE((I) + 1, 2) }
#define A3_RSTEP_LOAD(I)                                                                                       \
  if ((I) + 1 + kPF < nQ) {                                                                                    \
    if (((I) + 1) % kPF == 0) { A3_RLOAD((I) + 1 + kPF, 0) } else if (((I) + 1) % kPF == 1) { A3_RLOAD((I) + 1 + kPF, 1) } \
    else { A3_RLOAD((I) + 1 + kPF, 2) }                                                                        \
  }
  // waves 0-3: slot I + 1 has landed when at most the (up to six) slots requested after it are in flight
#define A3_WAIT_SLOT(I)                                                                                        \
  {                                                                                                            \
    const int younger_ = nQ - (I) - 2;                                                                         \
    if (younger_ >= 6) A3_VMCNT(24); else if (younger_ == 5) A3_VMCNT(20); else if (younger_ == 4) A3_VMCNT(16); \
    else if (younger_ == 3) A3_VMCNT(12); else if (younger_ == 2) A3_VMCNT(8); else if (younger_ == 1) A3_VMCNT(4); \
    else A3_VMCNT(0);                                                                                          \
  }

  // ---- slot 0 and the Q tile have landed -------------------------------------------------------------
  if (REALIGN) {
    // (in waves 0-3 the Q tile's loads are older than these: the compiler's wait for the keys of slot 0 covers them)
    A3_RLOAD(0, 0)
    if (nQ > 1) { A3_RLOAD(1, 1) }
    if (nQ > 2) { A3_RLOAD(2, 2) }
    A3_RSTORE(0, 0)
    if (nQ > 3) { A3_RLOAD(3, 0) }
  } else if (loads) {                                          // younger than slot 0 and the Q tile: slots 1 .. 3
    if (nQ > 3) A3_VMCNT(12); else if (nQ == 3) A3_VMCNT(8); else if (nQ == 2) A3_VMCNT(4); else A3_VMCNT(0);
  }
  A3_LDS_BARRIER();                                            // (also publishes St)
  bf16x8 qf[2][kD / 16];
#pragma unroll
  for (int b = 0; b < 2; ++b)
#pragma unroll
    for (int ks = 0; ks < kD / 16; ++ks)
      qf[b][ks] = *reinterpret_cast<const bf16x8 *>(qt + b * 32 * kKRowBytes + ((32 * ks) ^ kswz));
  // what the accumulators start from: zero, or in PASS 1 the row's -(max + log2 sum) / scale, so that the
  // finished accumulator times the scale is the exponent of the softmax weight (+inf for a row past Mg:
  // its weights come out as exp2(-inf) = 0)
  f32x16 acc0[2];
#pragma unroll
  for (int b = 0; b < 2; ++b)
#pragma unroll
    for (int x = 0; x < 16; ++x)     // PASS 1 lane: key; registers: rows 8 (x / 4) + 4 lhi + x % 4 of row block b
      acc0[b][x] = PASS == 1 ? -St[rg * 64 + b * 32 + 8 * (x >> 2) + 4 * lhi + (x & 3)] * a.inv_scale2 : 0.f;
  if (nQ > 4) {
    A3_LDS_BARRIER();                                          // everybody has its Q fragments: their place is free
    if (!REALIGN && loads) {                                   // ... and joins the ring
      A3_KDMA(4)
      if (nQ > 5) { A3_KDMA(5) }
      if (nQ > 6) { A3_KDMA(6) }
      if (nQ > 7) { A3_KDMA(7) }
    }
  }

  f32x16 acc[2];
  bf16x8 kfr[kD / 16];
  float run_max[2] = {-INFINITY, -INFINITY}, run_sum[2] = {0.f, 0.f};
  // the eight K fragments of this wave's block of slot I, requested together
#define A3_KFRAGS(I)                                                                                           \
  _Pragma("unroll") for (int ks_ = 0; ks_ < kD / 16; ++ks_)                                                    \
    kfr[ks_] = *reinterpret_cast<const bf16x8 *>(kt + ((I) & (kSlots - 1)) * kSlotBytes + ((32 * ks_) ^ kswz));
  // matrix phase: the logits of the wave's 64 rows against its 32 keys (fragments in kfr).  The first slab starts
  // from acc0, so the accumulators never have to be cleared.
#define A3_LOGITS()                                                                                            \
  _Pragma("unroll") for (int ks = 0; ks < kD / 16; ++ks) _Pragma("unroll") for (int b = 0; b < 2; ++b) { \
    if (PASS == 0) acc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kfr[ks], qf[b][ks], ks == 0 ? acc0[b] : acc[b], 0, 0, 0); /* C[key][row] */ \
    else           acc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qf[b][ks], kfr[ks], ks == 0 ? acc0[b] : acc[b], 0, 0, 0); /* C[row][key] */ \
  }
  // vector phase: the logits in acc (block of slot I) go into the row statistics (PASS 0) or the column sums (PASS 1)
#define A3_FOLD(I)                                                                                             \
  {                                                                                          \
    const int key0_ = i0 + (I) * kSlotKeys + kh * 32;            /* first key of the block */                   \
    if (PASS == 0) {                                                                                           \
      /* lane: row (column l32 of block b); registers: keys key0 + 8 (x / 4) + 4 lhi + x % 4 */                \
      if (key0_ < N) {                                           /* the block holds a real key */              \
        if (key0_ + 31 >= N) {                                                                                 \
          int n_real = N - key0_ - 4 * lhi;                                                                    \
          asm volatile("" : "+v"(n_real));                                                                     \
          _Pragma("unroll") for (int b = 0; b < 2; ++b) _Pragma("unroll") for (int x = 0; x < 16; ++x)         \
            if (8 * (x >> 2) + (x & 3) >= n_real) acc[b][x] = -INFINITY;                                       \
        }                                                                                                      \
        _Pragma("unroll") for (int b = 0; b < 2; ++b) {                                                        \
          float mx = fmaxf(acc[b][0], acc[b][1]);                                                              \
          _Pragma("unroll") for (int x = 2; x < 16; x += 2) mx = fmaxf(fmaxf(mx, acc[b][x]), acc[b][x + 1]);   \
          mx = halves_max(mx) * a.scale2;                                                                      \
          const float new_max = fmaxf(run_max[b], mx);                                                         \
          float sum0 = 0.f, sum1 = 0.f;                                                                        \
          _Pragma("unroll") for (int x = 0; x < 16; x += 2) {                                                  \
            sum0 += fast_exp2(fmaf(acc[b][x], a.scale2, -new_max));                                            \
            sum1 += fast_exp2(fmaf(acc[b][x + 1], a.scale2, -new_max));                                        \
          }                                                                                                    \
          run_sum[b] = run_sum[b] * fast_exp2(run_max[b] - new_max) + (sum0 + sum1);   /* first block: 0 * 0 */ \
          run_max[b] = new_max;                                                                                \
        }                                                                                                      \
      }                                                                                                        \
    } else {                                                                                                   \
      /* lane: key l32 of the block; registers: rows 8 (x / 4) + 4 lhi + x % 4 of row block b */               \
      float p0 = 0.f, p1 = 0.f;                                                                                \
      _Pragma("unroll") for (int b = 0; b < 2; ++b) _Pragma("unroll") for (int x = 0; x < 16; x += 2) {        \
        p0 += fast_exp2(acc[b][x] * a.scale2);                                                                 \
        p1 += fast_exp2(acc[b][x + 1] * a.scale2);                                                             \
      }                                                                                                        \
      const float part_ = halves_sum(p0 + p1);                                                                 \
      if (lhi == 0) red[rg * a.tile_keys + (I) * kSlotKeys + kh * 32 + l32] = part_;                           \
    }                                                                                                          \
  }

  A3_KFRAGS(0)
  A3_LOGITS()
  if (kh == 0) { A3_FOLD(0) }
  for (int i = 0; i + 1 < nQ; ++i) {
    if (REALIGN) { A3_RSTEP_STORE(i) } else if (loads) { A3_WAIT_SLOT(i) }
    A3_LDS_BARRIER();                                          // slot i + 1 is in the ring
    if (REALIGN) { A3_RSTEP_LOAD(i) }
    // every wave has read slot i (its MFMAs were issued before the barrier): refill its place
    else if (loads && i + kSlots < nQ) { A3_KDMA(i + kSlots) }
    A3_KFRAGS(i + 1)
    if (kh == 0) {
      A3_LOGITS()
      A3_FOLD(i + 1)
    } else {
      A3_FOLD(i)
      A3_LOGITS()
    }
  }
  if (kh == 1) { A3_FOLD(nQ - 1) }
#undef A3_FOLD
#undef A3_LOGITS
#undef A3_KFRAGS

  if (PASS == 0) {
    // (max, sum) of this wave's rows over its half of the keys; the two halves of a row group merge in LDS
    float2 *pair = reinterpret_cast<float2 *>(lds_raw + kLdsRed);
    float z[2];
#pragma unroll
    for (int b = 0; b < 2; ++b) z[b] = halves_sum(run_sum[b]);
    if (kh == 1 && lhi == 0) {
#pragma unroll
      for (int b = 0; b < 2; ++b) pair[rg * 64 + b * 32 + l32] = make_float2(run_max[b], z[b]);
    }
    __syncthreads();
    if (kh == 0 && lhi == 0) {
#pragma unroll
      for (int b = 0; b < 2; ++b) {
        const int m = m_base + rg * 64 + b * 32 + l32;
        if (m < Mg) {
          const float2 o = pair[rg * 64 + b * 32 + l32];
          const float mn = fmaxf(run_max[b], o.x);             // keys 0 .. 31 of slot 0 are real: run_max is finite
          const float zz = z[b] * fast_exp2(run_max[b] - mn) + (o.y > 0.f ? o.y * fast_exp2(o.x - mn) : 0.f);
          a.part[(size_t)t * a.total_rows + row_of(m)] = make_float2(mn, zz);
        }
      }
    }
  }
#undef A3_QDMA
#undef A3_WAIT_SLOT
#undef A3_RSTEP_LOAD
#undef A3_RSTEP_STORE
#undef A3_RSTORE
#undef A3_RLOAD
#undef A3_KDMA

  if (PASS == 1) {
    __syncthreads();
    // column sums of this (KV head, row chunk): the four row groups in a fixed order
    float *mine = a.part_scores + (size_t)g * a.T + s + i0;
    for (int key = tid; key < n_keys; key += kScoreThreads)
      mine[key] = (red[key] + red[a.tile_keys + key]) + (red[2 * a.tile_keys + key] + red[3 * a.tile_keys + key]);
  }
}
#undef A3_VMCNT
#undef A3_LDS_BARRIER

// ---------------------------------------------------------------------------------------
// bf16 MFMA kernel for more than 256 rows per KV head (long questions, wide query groups, batches of them).
// Workgroup (4 waves) = all rows of one KV head of one request against a tile of 256 keys, which stays in LDS
// (64 KB, so two workgroups share a CU and one loads while the other multiplies) while the waves walk the rows
// in groups of 64 with their Q fragments straight from global memory (L2).  The tile arrives in four quarters
// of 64 keys, all requested up front; the logits of a wave's first 64 rows against a quarter are formed as soon
// as it has landed.  PASS 0 leaves (max, sum exp) per (tile, row), a small kernel merges them per row, PASS 1
// forms the column sums of exp2(l - stat).  Same results layout as the kernel above.
// ---------------------------------------------------------------------------------------
constexpr int kRowsTileKeys = 256;
constexpr size_t kScoresRowsLds = (size_t)kRowsTileKeys * kKRowBytes + 4 * 64 * sizeof(float) +
                                  4 * kRowsTileKeys * sizeof(float);

template <int PASS, bool REALIGN>
__global__ void __launch_bounds__(256, 2)
scores_rows_bf16_kernel(scores_args a) {
  extern __shared__ __align__(16) unsigned char lds_raw[];
  float *St = reinterpret_cast<float *>(lds_raw + kRowsTileKeys * kKRowBytes);      // after the K tile; [4 waves][64 rows]
  float *red = reinterpret_cast<float *>(St + 4 * 64);                                // [4 waves][256 keys]

  const int r = blockIdx.z, g = blockIdx.y;
  const int N = a.ctx_len[r];
  const int i0 = blockIdx.x * kRowsTileKeys;
  if (i0 >= N) return;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, lhi = lane >> 5;
  const int s = a.seg_start[r];
  const int nq = a.q_len[r];
  const int G = a.Hq / a.Hkv;
  const int Mg = nq * G;                // rows of this KV head: m = j*G + hh
  const int qrow0 = a.q_start[r];
  const bf16_t *__restrict__ Q = (const bf16_t *)a.q;
  const bf16_t *__restrict__ K = (const bf16_t *)a.k;

  // Q fragments of this wave's first 64 rows: requested before the K tile so that both latencies overlap
  // (rows past Mg are clamped and ignored later)
  bf16x8 qf[2][kD / 16];
  int row_id[2];
#define A3_LOAD_Q(RB0)                                                                                 \
  _Pragma("unroll") for (int b = 0; b < 2; ++b) {                                                      \
    const int m_ = min((RB0) + b * 32 + l32, Mg - 1);                                                  \
    row_id[b] = (qrow0 + m_ / G) * a.Hq + g * G + m_ % G;      /* row of the [sum q_len * Hq] row space */ \
    const bf16_t *qp_ = Q + (size_t)row_id[b] * kD + lhi * 8;                                          \
    _Pragma("unroll") for (int ks = 0; ks < kD / 16; ++ks) qf[b][ks] = *reinterpret_cast<const bf16x8 *>(qp_ + ks * 16); \
  }
  if (Mg > 0) { A3_LOAD_Q(min(wave * 64, Mg - 1)) }
  const bool have_rows = wave * 64 < Mg;                       // this wave has a first group of rows
  if (PASS == 1) {
    // max + log2(sum) of this wave's 64 rows, read back as broadcasts below; rows past Mg contribute 0
    const int m = wave * 64 + lane;
    float st = INFINITY;                                       // exp2(x - inf) = 0
    if (m < Mg) st = a.stats[(qrow0 + m / G) * a.Hq + g * G + m % G].x;
    St[wave * 64 + lane] = st;                                 // same-wave write/read: no barrier needed
  }

  // The K tile arrives in four quarters of 64 keys.  Every load of the tile is issued up front; the logits
  // of the wave's first 64 rows against quarter q are formed as soon as that quarter is in LDS, while the
  // later quarters are still on their way, so the arithmetic runs under the memory time instead of after it.
  constexpr int kQuarters = 4;
  constexpr int kKB = kRowsTileKeys / 32;                      // 32-key blocks per tile
  const int n_kb = min(kKB, (N - i0 + 31) / 32);               // key blocks with at least one real key
  // fragment read: key 32 kb + l32, piece 2 ks + lhi -> slot (2 ks + lhi) ^ (l32 % 16)
  const unsigned char *kt = lds_raw + l32 * kKRowBytes;
  const int kswz = (lhi ^ (l32 & 15)) * 16;
  float colsum[kKB];
#pragma unroll
  for (int kb = 0; kb < kKB; ++kb) colsum[kb] = 0.f;
  float run_max[2] = {-INFINITY, -INFINITY}, run_sum[2] = {0.f, 0.f};

  // logits of the current 64 rows (fragments in qf) against key block KB, folded into the running row
  // statistics (pass A) or into the column sums (pass B)
#define A3_KEY_BLOCK(KB)                                                                                       \
  {                                                                                                            \
    f32x16 acc[2];                                                                                             \
    _Pragma("unroll") for (int b = 0; b < 2; ++b)                                                              \
      _Pragma("unroll") for (int x = 0; x < 16; ++x) acc[b][x] = 0.f;                                          \
    _Pragma("unroll") for (int ks = 0; ks < kD / 16; ++ks) {                                                   \
      const bf16x8 kf = *reinterpret_cast<const bf16x8 *>(kt + (KB) * 32 * kKRowBytes + ((32 * ks) ^ kswz));   \
      _Pragma("unroll") for (int b = 0; b < 2; ++b) {                                                          \
        if (PASS == 0) acc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[b][ks], acc[b], 0, 0, 0); /* C[key][row] */ \
        else           acc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qf[b][ks], kf, acc[b], 0, 0, 0); /* C[row][key] */ \
      }                                                                                                        \
    }                                                                                                          \
    if (PASS == 0) {                                                                                           \
      /* lane: row (column l32 of block b); registers: keys i0 + 32 kb + 8(x/4) + 4 lhi + x%4 */               \
      const bool tail = i0 + 32 * (KB) + 31 >= N;                                                              \
      _Pragma("unroll") for (int b = 0; b < 2; ++b) {                                                          \
        if (tail) {                                                                                            \
          /* (the empty statement keeps the 16 comparisons of each of the unrolled blocks here: gathered at */ \
          /* the top of the kernel their lane masks do not fit the scalar registers)                        */ \
          int n_real = N - i0 - 32 * (KB) - 4 * lhi;                                                           \
          asm volatile("" : "+v"(n_real));                                                                     \
          _Pragma("unroll") for (int x = 0; x < 16; ++x)                                                       \
            if (8 * (x >> 2) + (x & 3) >= n_real) acc[b][x] = -INFINITY;                                       \
        }                                                                                                      \
        float mx = acc[b][0];                                                                                  \
        _Pragma("unroll") for (int x = 1; x < 16; ++x) mx = fmaxf(mx, acc[b][x]);                              \
        mx = halves_max(mx) * a.scale2;                        /* block 0 of a tile always has a real key */   \
        const float new_max = fmaxf(run_max[b], mx);                                                           \
        float sum = 0.f;                                                                                       \
        _Pragma("unroll") for (int x = 0; x < 16; ++x) sum += fast_exp2(fmaf(acc[b][x], a.scale2, -new_max));  \
        run_sum[b] = run_sum[b] * fast_exp2(run_max[b] - new_max) + sum;   /* per lane half */                 \
        run_max[b] = new_max;                                                                                  \
      }                                                                                                        \
    } else {                                                                                                   \
      /* lane: key l32 of block kb; registers: rows 8(x/4) + 4 lhi + x%4 of row block b */                     \
      float part = 0.f;                                                                                        \
      _Pragma("unroll") for (int b = 0; b < 2; ++b)                                                            \
        _Pragma("unroll") for (int x = 0; x < 16; ++x) {                                                       \
          const float st = St[wave * 64 + b * 32 + 8 * (x >> 2) + 4 * lhi + (x & 3)];                          \
          part += fast_exp2(fmaf(acc[b][x], a.scale2, -st));                                                   \
        }                                                                                                      \
      colsum[KB] += part;                                                                                      \
    }                                                                                                          \
  }
  // the 64 rows are done: pass A leaves their (max, sum) over this tile
#define A3_ROWS_DONE(RB0)                                                                                      \
  if (PASS == 0) {                                                                                             \
    _Pragma("unroll") for (int b = 0; b < 2; ++b) {                                                            \
      const float z = halves_sum(run_sum[b]);                                                                  \
      if (lhi == 0 && (RB0) + b * 32 + l32 < Mg)                                                               \
        a.part[(size_t)blockIdx.x * a.total_rows + row_id[b]] = make_float2(run_max[b], z);                    \
    }                                                                                                          \
  }

  // ---- K tile: 256 keys x 128 dims of head g, global memory -> LDS directly (16 bytes per lane, lane i
  // lands at base + 16 i).  One wave instruction brings 4 keys x 256 B; instruction j of wave w covers
  // keys 4 (4 j + w) .. +3, so the instructions 4 q .. 4 q + 3 of the four waves bring quarter q.  The lane
  // fetches piece (slot ^ key % 16) of its key, so LDS slot s of key r holds piece s ^ (r % 16) and the 16
  // keys a quarter wave reads at one piece index touch all 64 banks once.  Inline assembly: the compiler
  // then does not track these as LDS writes (it would wait for all of them before every LDS read); the
  // explicit waits below cover them.
  if (!REALIGN) {
    // The compiler's own wait for the Q fragments and the row statistics would, counted by the hardware, also
    // wait for everything issued before them; they are therefore awaited first, then the tile is requested.
    __builtin_amdgcn_s_waitcnt(0);
    const int drow = 4 * wave + (lane >> 4);                   // key of the lane in instruction 0
    const int dpiece = (lane & 15) ^ (drow & 15);              // (4 (4 j + w) + lane/16) % 16 does not depend on j
    const uint32_t lds_k = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char *)lds_raw;
#pragma unroll
    for (int j = 0; j < kRowsTileKeys / 16; ++j) {
      const int row = min(s + i0 + drow + 16 * j, a.T - 1);    // tail rows: loaded, masked below
      const bf16_t *gp = K + ((size_t)row * a.Hkv + g) * kD + dpiece * 8;
      asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off"
                   :: "s"(__builtin_amdgcn_readfirstlane(lds_k + 4 * (4 * j + wave) * kKRowBytes)), "v"(gp) : "memory");
    }
    // at most the 4 (3 - QT) younger instructions of this wave are still in flight: its part of quarter QT
    // has landed; after the barrier everybody's has.  (vmcnt in bits 3:0 and 15:14, the other counters open.)
#define A3_QUARTER(QT)                                                                                         \
    __builtin_amdgcn_s_waitcnt((4 * (kQuarters - 1 - (QT))) | (7 << 4) | (15 << 8));                           \
    __builtin_amdgcn_s_barrier();                                                                              \
    if (have_rows) {                                                                                           \
      if (2 * (QT) < n_kb) A3_KEY_BLOCK(2 * (QT))                                                              \
      if (2 * (QT) + 1 < n_kb) A3_KEY_BLOCK(2 * (QT) + 1)                                                      \
    }
    A3_QUARTER(0)
    A3_QUARTER(1)
    A3_QUARTER(2)
    A3_QUARTER(3)
#undef A3_QUARTER
  } else {
    // Position recovery (Eq. 2) on the way in: the tile comes from the stale cache through registers,
    // every pair is turned by its chunk's offset, and the rounded result goes both to the realigned cache
    // and, in the same swizzled layout as above, to LDS.  A lane owns the 16-byte pieces c and c + 8 of
    // a key: in either pairing (adjacent coordinates, or i with i + 64) it then holds whole pairs.
    const bf16_t *Kc = (const bf16_t *)a.k_cat;               // may be the same buffer as k_out
    bf16_t *Ko = (bf16_t *)a.k_out;
    const int c = tid & 7, kr0 = tid >> 3;                     // 32 keys per round, 8 rounds: 2 per quarter
    constexpr int kRounds = kRowsTileKeys / 32;
    // all loads of the stale keys and of their chunk numbers are issued before the first rotation
    bf16x8 lo[kRounds], hi[kRounds];
    int chunk[kRounds];
#pragma unroll
    for (int j = 0; j < kRounds; ++j) {
      const int key = kr0 + 32 * j;
      const int row = min(s + i0 + key, a.T - 1);              // tail rows: loaded, never stored to the cache
      const size_t off = ((size_t)row * a.Hkv + g) * kD;
      lo[j] = *reinterpret_cast<const bf16x8 *>(Kc + off + 8 * c);
      hi[j] = *reinterpret_cast<const bf16x8 *>(Kc + off + 64 + 8 * c);
      chunk[j] = i0 + key < N ? a.tok_chunk[row] : -1;
    }
    // the eight (cos, sin) pairs of this lane's coordinates are reloaded only when the chunk changes
    // from one of its keys to the next (rarely: a tile spans few chunks)
    const bool inter = a.rope_layout == A3_ROPE_INTERLEAVED;
    float2 csr[8];
    int cur = -1;
#pragma unroll
    for (int j = 0; j < kRounds; ++j) {
      const int key = kr0 + 32 * j;
      const bool real = i0 + key < N;
      const int row = min(s + i0 + key, a.T - 1);
      const size_t off = ((size_t)row * a.Hkv + g) * kD;
      bf16x8 rlo = lo[j], rhi = hi[j];
      if (chunk[j] >= 0) {
        if (chunk[j] != cur) {
          const float2 *cs = a.chunk_cs + (size_t)chunk[j] * (kD / 2);
#pragma unroll
          for (int e = 0; e < 8; ++e)                          // interleaved: pairs 4c..4c+3 and 32+4c..; half: 8c..8c+7
            csr[e] = inter ? cs[(e < 4 ? 4 * c : 28 + 4 * c) + e] : cs[8 * c + e];
          cur = chunk[j];
        }
        if (inter) {
#pragma unroll
          for (int p2 = 0; p2 < 4; ++p2) {
            float y0, y1;
            a3_rotate_pair(a3_bf2f(lo[j][2 * p2]), a3_bf2f(lo[j][2 * p2 + 1]), csr[p2], y0, y1);
            rlo[2 * p2] = a3_f2bf(y0); rlo[2 * p2 + 1] = a3_f2bf(y1);
            a3_rotate_pair(a3_bf2f(hi[j][2 * p2]), a3_bf2f(hi[j][2 * p2 + 1]), csr[4 + p2], y0, y1);
            rhi[2 * p2] = a3_f2bf(y0); rhi[2 * p2 + 1] = a3_f2bf(y1);
          }
        } else {
#pragma unroll
          for (int e = 0; e < 8; ++e) {                        // coordinate 8c+e pairs with 64+8c+e
            float y0, y1;
            a3_rotate_pair(a3_bf2f(lo[j][e]), a3_bf2f(hi[j][e]), csr[e], y0, y1);
            rlo[e] = a3_f2bf(y0); rhi[e] = a3_f2bf(y1);
          }
        }
      }
      if (real) {
        *reinterpret_cast<bf16x8 *>(Ko + off + 8 * c) = rlo;
        *reinterpret_cast<bf16x8 *>(Ko + off + 64 + 8 * c) = rhi;
      }
      unsigned char *ld = lds_raw + key * kKRowBytes;
      *reinterpret_cast<bf16x8 *>(ld + ((c ^ (key & 15)) * 16)) = rlo;
      *reinterpret_cast<bf16x8 *>(ld + (((c + 8) ^ (key & 15)) * 16)) = rhi;
      if (j & 1) {
        // quarter j / 2 is in LDS once everybody's two rounds are written (this wave's writes first: the
        // LDS counter only; a full fence would also wait for the keys still on their way)
        __builtin_amdgcn_s_waitcnt(15 | (3 << 14) | (7 << 4) | (0 << 8));
        __builtin_amdgcn_s_barrier();
        if (have_rows) {
          if (j - 1 < n_kb) A3_KEY_BLOCK(j - 1)
          if (j < n_kb) A3_KEY_BLOCK(j)
        }
      }
    }
  }
  if (have_rows) { A3_ROWS_DONE(wave * 64) }

  // ---- the wave's further rows (more than 256 rows per KV head): the whole tile is in LDS by now --------------
  for (int rb0 = wave * 64 + 256; rb0 < Mg; rb0 += 256) {      // this wave's rows rb0 .. rb0+63
    A3_LOAD_Q(rb0)
    if (PASS == 1) {
      const int m = rb0 + lane;
      float st = INFINITY;
      if (m < Mg) st = a.stats[(qrow0 + m / G) * a.Hq + g * G + m % G].x;
      St[wave * 64 + lane] = st;
    }
    run_max[0] = run_max[1] = -INFINITY;
    run_sum[0] = run_sum[1] = 0.f;
    for (int kb = 0; kb < n_kb; ++kb) A3_KEY_BLOCK(kb)
    A3_ROWS_DONE(rb0)
  }
#undef A3_KEY_BLOCK
#undef A3_ROWS_DONE
#undef A3_LOAD_Q
  if (PASS == 1) {
#pragma unroll
    for (int kb = 0; kb < kKB; ++kb) {
      const float v = halves_sum(colsum[kb]);
      if (lhi == 0) red[wave * kRowsTileKeys + kb * 32 + l32] = v;
    }
    __syncthreads();
    const int key = i0 + tid;
    if (tid < kRowsTileKeys && key < N)
      a.part_scores[(size_t)g * a.T + s + key] = (red[tid] + red[kRowsTileKeys + tid]) +
                                                 (red[2 * kRowsTileKeys + tid] + red[3 * kRowsTileKeys + tid]);
  }
}

// scores[t] = sum over KV heads of their column sums, in head order; question rows get -inf
__global__ void __launch_bounds__(256)
scores_head_sum_kernel(scores_args a, const int *__restrict__ tok_chunk) {
  const int t = blockIdx.x * 256 + threadIdx.x;
  if (t >= a.T) return;
  float v = -INFINITY;
  if (tok_chunk[t] >= 0) {
    v = 0.f;
    for (int g = 0; g < a.Hkv; ++g) v += a.part_scores[(size_t)g * a.T + t];
  }
  a.scores[t] = v;
}

// ---------------------------------------------------------------------------------------
// fp32 kernels (any head_dim <= 128)
// ---------------------------------------------------------------------------------------
template <int PASS>
__global__ void __launch_bounds__(256)
scores_f32_kernel(scores_args a) {
  __shared__ float Ks[kTileKeys][128 + 1];
  __shared__ float Qs[4][128];
  __shared__ float red[4][kTileKeys];

  const int r = blockIdx.y;
  const int N = a.ctx_len[r];
  const int i0 = blockIdx.x * kTileKeys;
  const int tid = threadIdx.x;
  const int key = tid & 63, slice = tid >> 6;
  const int s = a.seg_start[r];
  const int nq = a.q_len[r];
  if (PASS == 1 && blockIdx.x == 0 && a.scores)
    for (int j = tid; j < nq; j += 256) a.scores[s + N + j] = -INFINITY;
  if (i0 >= N) return;
  const int d = a.d, G = a.Hq / a.Hkv, Mg = nq * G, qrow0 = a.q_start[r];
  const float *__restrict__ Q = (const float *)a.q;
  const float *__restrict__ K = (const float *)a.k;
  float total = 0.f;                     // PASS 1, tid < kTileKeys: the key's score over all heads so far

  for (int g = 0; g < a.Hkv; ++g) {
    float colsum = 0.f;
    __syncthreads();
    for (int i = tid; i < kTileKeys * d; i += 256) {
      int kr = i / d, c = i % d;
      int row = min(s + i0 + kr, a.T - 1);
      Ks[kr][c] = K[((size_t)row * a.Hkv + g) * d + c];
    }
    for (int mb = 0; mb < Mg; mb += 4) {
      const int m = mb + slice;
      const int mc = m < Mg ? m : Mg - 1;
      const int row_id = (qrow0 + mc / G) * a.Hq + g * G + mc % G;
      __syncthreads();
      for (int c = key; c < d; c += 64) Qs[slice][c] = Q[(size_t)row_id * d + c];
      __syncthreads();
      float dot = 0.f;
      for (int c = 0; c < d; ++c) dot = fmaf(Qs[slice][c], Ks[key][c], dot);
      float l = (i0 + key < N) ? dot * a.scale2 : -INFINITY;
      if (PASS == 0) {
        // (max, sum) over the 64 keys of this tile for row m: wave-wide reduction (one wave per slice)
        float mx = l;
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off, 64));
        float e = exp2f(l - mx);
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) e += __shfl_xor(e, off, 64);
        if (key == 0 && m < Mg) a.part[(size_t)blockIdx.x * a.total_rows + row_id] = make_float2(mx, e);
      } else if (m < Mg) {
        colsum += exp2f(l - a.stats[row_id].x);
      }
    }
    if (PASS == 1) {
      // this head's column sums: the four row slices in a fixed order, then the heads in order
      __syncthreads();
      red[slice][key] = colsum;
      __syncthreads();
      if (tid < kTileKeys && i0 + tid < N) {
        const float v = (red[0][tid] + red[1][tid]) + (red[2][tid] + red[3][tid]);
        if (a.part_scores) a.part_scores[(size_t)g * a.T + s + i0 + tid] = v;
        total += v;
      }
    }
  }
  if (PASS == 1 && a.scores && tid < kTileKeys && i0 + tid < N) a.scores[s + i0 + tid] = total;
}

}  // namespace

// bf16 path: rows of the score matrix per KV head, in chunks of 256 (one chunk: the ring kernel)
static int scores_row_chunks(const a3_layout *L) {
  const int G = L->n_q_heads / L->n_kv_heads;
  const int c = (int)(((long long)L->max_q_len * G + kChunkRows - 1) / kChunkRows);
  return c < 1 ? 1 : c;
}

// bf16 path: keys per workgroup.  A multiple of the 64-key ring slot in [256, 1024], chosen so that the
// workgroups (one per CU at a time: 150 KB of LDS) fill the 256 CUs in as few, as full rounds as possible; a
// workgroup's fixed cost (its Q tile, the merge of the partials, the start-up of the ring) is worth about 192 keys.
static int scores_tile_keys_bf16(const a3_layout *L) {
  // more than 256 rows per KV head: the kernel that keeps a 256-key tile in LDS and walks the rows
  if (scores_row_chunks(L) > 1) return kRowsTileKeys;
  const long long per_tile = (long long)L->n_req * L->n_kv_heads;
  long long best_cost = -1;
  int best = kMinTileKeys;
  for (int tk = kMinTileKeys; tk <= kMaxTileKeys; tk += kSlotKeys) {
    const long long wgs = per_tile * ((L->max_ctx_len + tk - 1) / tk);
    const long long cost = ((wgs + 255) / 256) * (tk + 192);
    if (best_cost < 0 || cost < best_cost) { best_cost = cost; best = tk; }
  }
  return best;
}

size_t a3_scores_ws_bytes(const a3_layout *L) {
  // rows of the score matrix over the whole batch are bounded by n_req * max_q_len * Hq
  const size_t total_rows = (size_t)L->n_req * L->max_q_len * L->n_q_heads;
  const int tk = L->dtype == A3_BF16 ? kMinTileKeys : kTileKeys;         // the most runs of keys either path can have
  const size_t n_tiles = (size_t)(L->max_ctx_len + tk - 1) / tk;
  return a3_align_up((n_tiles + 1) * total_rows * sizeof(float2), 256) + a3_align_up(total_rows * sizeof(float2), 256) +
         a3_align_up((size_t)L->n_kv_heads * L->total_tokens * sizeof(float), 256) + 256;
}

// k_cat != nullptr: the first pass of the bf16 path also realigns (k_cat -> k_fused); the fp32 path runs the
// realign kernel first.
// causal_q: the question keys a question token sees join its softmax denominator.  votes != nullptr: the per
// KV head column sums [Hkv, T] go there; scores may then be NULL (no sum over heads).
static a3_status scores_launch(const a3_layout *L, const void *q_question, const void *k_cat, void *k_fused,
                               float *scores, void *ws, size_t ws_bytes, void *stream, int causal_q = 0,
                               float *votes = nullptr) {
  a3_status s = a3_check_layout(L, "a3_question_scores", true);
  if (s != A3_OK) return s;
  A3_REQUIRE(q_question && k_fused && (scores || votes), A3_ERR_INVALID_ARG, "a3_question_scores: NULL tensor");
  A3_REQUIRE(a3_aligned16(q_question) && a3_aligned16(k_fused), A3_ERR_INVALID_ARG,
             "a3_question_scores: tensors must be 16-byte aligned");
  A3_REQUIRE(ws != nullptr, A3_ERR_WORKSPACE, "a3_question_scores: workspace is NULL");
  A3_REQUIRE(ws_bytes >= a3_scores_ws_bytes(L), A3_ERR_WORKSPACE,
             "a3_question_scores: workspace %zu bytes, need %zu", ws_bytes, a3_scores_ws_bytes(L));
  A3_REQUIRE(L->max_ctx_len > 0 && L->max_q_len > 0, A3_ERR_UNSUPPORTED,
             "a3_question_scores: needs max_ctx_len > 0 and max_q_len > 0");
  hipStream_t st = (hipStream_t)stream;
  const bool bf16 = L->dtype == A3_BF16;
  const size_t total_rows = (size_t)L->n_req * L->max_q_len * L->n_q_heads;   // upper bound, used as row pitch
  const int tk = bf16 ? scores_tile_keys_bf16(L) : kTileKeys;
  const int n_tiles = (L->max_ctx_len + tk - 1) / tk;
  const int tk_min = bf16 ? kMinTileKeys : kTileKeys;
  const int max_tiles = (L->max_ctx_len + tk_min - 1) / tk_min;               // what the workspace is sized for
  a3_ws_cursor cur(ws, ws_bytes);
  scores_args a;
  a.q = q_question; a.k = k_fused;
  a.seg_start = L->seg_start; a.ctx_len = L->ctx_len; a.q_len = L->q_len; a.q_start = L->q_start;
  a.part = (float2 *)cur.take((size_t)(max_tiles + 1) * total_rows * sizeof(float2));
  a.stats = (float2 *)cur.take(total_rows * sizeof(float2));
  a.part_scores = (float *)cur.take((size_t)L->n_kv_heads * L->total_tokens * sizeof(float));
  if (votes) a.part_scores = votes;                            // a KV head's column sums are its votes
  else if (!bf16) a.part_scores = nullptr;                     // fp32 path adds the heads itself
  const int G = L->n_q_heads / L->n_kv_heads;
  a.inv_G = G > 1 ? (uint32_t)(((1ull << 32) + G - 1) / G) : 0u;
  a.causal_q = causal_q;
  a.merged = 0;
  a.scores = scores;
  a.n_req = L->n_req; a.Hq = L->n_q_heads; a.Hkv = L->n_kv_heads; a.d = L->head_dim; a.T = L->total_tokens;
  a.total_rows = (int)total_rows; a.n_tiles = n_tiles; a.tile_keys = tk;
  a.scale2 = a3_scale_of(L) * kLog2e;
  a.inv_scale2 = 1.0f / a.scale2;
  const bool one = L->n_req == 1 && L->max_ctx_len + L->max_q_len == L->total_tokens;
  a.one_ctx_len = one ? L->max_ctx_len : -1;
  a.one_q_len = one ? L->max_q_len : -1;
  a.k_cat = k_cat; a.k_out = k_fused; a.tok_chunk = L->tok_chunk; a.chunk_cs = (const float2 *)L->rope_chunk_cs;
  a.rope_layout = L->rope_layout;
  const bool fuse = k_cat != nullptr && bf16 && L->n_chunks > 0;
  if (k_cat != nullptr && !fuse) {
    s = a3_rope_realign(L, k_cat, k_fused, stream);
    if (s != A3_OK) return s;
  }
  if (causal_q) {
    const dim3 qgrid((unsigned)((total_rows + 3) / 4));
    if (bf16) hipLaunchKernelGGL(scores_question_stats_kernel<bf16_t>, qgrid, dim3(256), 0, st, a);
    else hipLaunchKernelGGL(scores_question_stats_kernel<float>, qgrid, dim3(256), 0, st, a);
  }
  if (bf16) {
    static a3_once_per_device lds_once;
    const hipError_t e = a3_once(lds_once, []() {
      const void *fns[] = {(const void *)scores_bf16_kernel<0, false>, (const void *)scores_bf16_kernel<1, false>,
                           (const void *)scores_bf16_kernel<0, true>};
      for (const void *fn : fns) {
        const hipError_t e_ = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)kScoresLds);
        if (e_ != hipSuccess) return e_;
      }
      const void *rows_fns[] = {(const void *)scores_rows_bf16_kernel<0, false>, (const void *)scores_rows_bf16_kernel<1, false>,
                                (const void *)scores_rows_bf16_kernel<0, true>};
      for (const void *fn : rows_fns) {
        const hipError_t e_ = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)kScoresRowsLds);
        if (e_ != hipSuccess) return e_;
      }
      return hipSuccess;
    });
    if (e != hipSuccess) return a3_fail(A3_ERR_HIP, "a3_question_scores: cannot raise the dynamic LDS limit: %s", hipGetErrorString(e));
    a.merged = (n_tiles > 32 || scores_row_chunks(L) > 1 || causal_q) ? 1 : 0;
    const long long wgs = (long long)L->n_req * n_tiles * L->n_kv_heads;
    A3_REQUIRE(wgs < (1LL << 31), A3_ERR_UNSUPPORTED, "a3_question_scores: batch too large");
    const dim3 grid((unsigned)wgs);
    if (scores_row_chunks(L) > 1) {
      // (tile_keys is kRowsTileKeys here; every row of a KV head in one workgroup)
      const dim3 rgrid((unsigned)n_tiles, (unsigned)L->n_kv_heads, (unsigned)L->n_req);
      if (fuse) hipLaunchKernelGGL((scores_rows_bf16_kernel<0, true>), rgrid, dim3(256), kScoresRowsLds, st, a);
      else hipLaunchKernelGGL((scores_rows_bf16_kernel<0, false>), rgrid, dim3(256), kScoresRowsLds, st, a);
      hipLaunchKernelGGL(scores_combine_kernel, dim3((unsigned)((total_rows + 15) / 16)), dim3(256), 0, st, a);
      hipLaunchKernelGGL((scores_rows_bf16_kernel<1, false>), rgrid, dim3(256), kScoresRowsLds, st, a);
    } else {
      if (fuse) hipLaunchKernelGGL((scores_bf16_kernel<0, true>), grid, dim3(kScoreThreads), kScoresLds, st, a);
      else hipLaunchKernelGGL((scores_bf16_kernel<0, false>), grid, dim3(kScoreThreads), kScoresLds, st, a);
      if (a.merged) hipLaunchKernelGGL(scores_combine_kernel, dim3((unsigned)((total_rows + 15) / 16)), dim3(256), 0, st, a);
      hipLaunchKernelGGL((scores_bf16_kernel<1, false>), grid, dim3(kScoreThreads), kScoresLds, st, a);
    }
    if (scores)
      hipLaunchKernelGGL(scores_head_sum_kernel, dim3((L->total_tokens + 255) / 256), dim3(256), 0, st, a, L->tok_chunk);
  } else {
    const dim3 grid(n_tiles, L->n_req), cgrid((unsigned)((total_rows + 15) / 16));
    hipLaunchKernelGGL(scores_f32_kernel<0>, grid, dim3(256), 0, st, a);
    hipLaunchKernelGGL(scores_combine_kernel, cgrid, dim3(256), 0, st, a);
    hipLaunchKernelGGL(scores_f32_kernel<1>, grid, dim3(256), 0, st, a);
  }
  A3_CHECK_LAUNCH("a3_question_scores");
  return A3_OK;
}


extern "C" a3_status a3_question_scores(const a3_layout *L, const void *q_question, const void *k_fused, float *scores,
                                        void *ws, size_t ws_bytes, void *stream) {
  return scores_launch(L, q_question, nullptr, const_cast<void *>(k_fused), scores, ws, ws_bytes, stream);
}

extern "C" a3_status a3_realign_scores(const a3_layout *L, const void *q_question, const void *k_cat, void *k_fused,
                                       float *scores, void *ws, size_t ws_bytes, void *stream) {
  if (k_cat == nullptr) return a3_fail(A3_ERR_INVALID_ARG, "a3_realign_scores: k_cat is NULL");
  if (!a3_aligned16(k_cat)) return a3_fail(A3_ERR_INVALID_ARG, "a3_realign_scores: tensors must be 16-byte aligned");
  return scores_launch(L, q_question, k_cat, k_fused, scores, ws, ws_bytes, stream);
}

// ---------------------------------------------------------------------------------------
// a3_question_scores for callers that cannot allocate (code under graph capture, serving loops that forbid
// it): the partial row statistics and per-head partial scores that a3_question_scores keeps in the caller's
// workspace live in a fixed array of the library's own device image instead.  One array per GPU, shared by
// every call on that GPU and holding the last call's contents; every word a call reads it has written itself
// before, so nothing has to be cleared between calls.
// ---------------------------------------------------------------------------------------
constexpr size_t kScratchBytes = (size_t)A3_SCORES_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

namespace {
constexpr int kMaxDevices = 64;
std::once_flag scratch_once[kMaxDevices];
void *scratch_ptr[kMaxDevices];          // device address of `scratch` on each GPU (the symbol itself is a host stand-in)
hipError_t scratch_err[kMaxDevices];
}  // namespace

extern "C" a3_status a3_question_scores_noalloc(const a3_layout *L, const void *q_question, const void *k_fused,
                                                float *scores, void *stream) {
  a3_status s = a3_check_layout(L, "a3_question_scores_noalloc", true);
  if (s != A3_OK) return s;
  A3_REQUIRE(q_question && k_fused && scores, A3_ERR_INVALID_ARG, "a3_question_scores_noalloc: NULL tensor");
  const size_t need = a3_scores_ws_bytes(L);
  A3_REQUIRE(need <= kScratchBytes, A3_ERR_WORKSPACE,
             "a3_question_scores_noalloc: this batch needs %zu bytes of scratch, the built-in array holds %zu "
             "(use a3_question_scores with a workspace)", need, kScratchBytes);
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return a3_fail(A3_ERR_HIP, "a3_question_scores_noalloc: hipGetDevice: %s", hipGetErrorString(e));
  A3_REQUIRE(dev >= 0 && dev < kMaxDevices, A3_ERR_UNSUPPORTED, "a3_question_scores_noalloc: device %d", dev);
  // once per device, with that device current: each GPU holds its own copy of the array at its own address
  std::call_once(scratch_once[dev], [dev]() {
    void *p = nullptr;
    scratch_err[dev] = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    scratch_ptr[dev] = scratch_err[dev] == hipSuccess ? p : nullptr;
  });
  if (scratch_err[dev] != hipSuccess || scratch_ptr[dev] == nullptr)
    return a3_fail(A3_ERR_HIP, "a3_question_scores_noalloc: hipGetSymbolAddress: %s", hipGetErrorString(scratch_err[dev]));
  return scores_launch(L, q_question, nullptr, const_cast<void *>(k_fused), scores, scratch_ptr[dev], kScratchBytes, stream);
}

// Eq. 3, first line, with the softmax of a question token taken over every key it sees: the context keys
// and the question keys up to itself (the literal reading of the equation's denominator).
extern "C" a3_status a3_question_scores_causal(const a3_layout *L, const void *q_question, const void *k_fused,
                                               float *scores, void *ws, size_t ws_bytes, void *stream) {
  A3_REQUIRE(scores != nullptr, A3_ERR_INVALID_ARG, "a3_question_scores_causal: scores is NULL");
  return scores_launch(L, q_question, nullptr, const_cast<void *>(k_fused), scores, ws, ws_bytes, stream, 1);
}

// Eviction extension: votes of the question window per KV head (same normalisation, no sum over KV heads).
extern "C" a3_status a3_window_votes(const a3_layout *L, const void *q_question, const void *k_fused, float *votes,
                                     void *ws, size_t ws_bytes, void *stream) {
  A3_REQUIRE(votes != nullptr, A3_ERR_INVALID_ARG, "a3_window_votes: votes is NULL");
  return scores_launch(L, q_question, nullptr, const_cast<void *>(k_fused), nullptr, ws, ws_bytes, stream, 1, votes);
}
