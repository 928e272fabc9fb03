// Step 2 of the A^3 fusion path: question-relevance score, Eq. 3 first line.
//
//   s_i = sum_{hq} sum_j softmax_i( q_{j,hq} . k'_{i, hq/G} * scale )      softmax over the context keys
//
// A column sum of row softmaxes needs every row's (max, sum exp) before any column can be
// summed, so the logits are formed twice:
//   pass A   per (key tile, row): partial (max, sum exp)          -> workspace
//   combine  per row: merge the partials                          -> max + log2(sum) per row
//   pass B   per key tile: sum over all rows of exp(l - max)/sum  -> scores
// Rows, then heads, are reduced in a fixed order, so the result is deterministic (no atomics).
//
// bf16: logits on the matrix cores (32x32x16 bf16 MFMA).  A workgroup owns 256 keys of one KV
// head: the K tile (64 KB) sits in LDS (loaded there directly, swizzled) and every Q fragment a wave loads
// (straight from global memory, Q is L2 resident) meets all 8 key blocks, so both K and Q cross
// the L2 once per pass.  Pass B leaves one partial score per KV head; a last small kernel adds the
// heads in order.  exp2 with log2(e) folded into the scale.
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
  float2 *stats;            // [total_rows] (max + log2(sum), unused)
  float *scores;            // [T]
  float *part_scores;       // [Hkv, T] bf16 path: per KV head partial scores
  int n_req, Hq, Hkv, d, T, total_rows, n_tiles, tile_keys;
  float scale2;             // sm_scale * log2(e)
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
constexpr int kTileKeysMfma = 256; // bf16 kernels

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
// Workgroup = 256 keys of one request and one KV head; each wave walks the (question token, head)
// rows of the group 64 at a time.
// ---------------------------------------------------------------------------------------
constexpr int kD = 128;
constexpr int kKRowBytes = kD * 2;    // LDS rows are unpadded; their 16-byte pieces are XOR-swizzled
constexpr size_t kScoresLds = (size_t)kTileKeysMfma * kKRowBytes + 4 * 64 * sizeof(float) +
                              4 * kTileKeysMfma * sizeof(float);

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

template <int PASS, bool REALIGN>
__global__ void __launch_bounds__(256, 2)
scores_bf16_kernel(scores_args a) {
  extern __shared__ __align__(16) unsigned char lds_raw[];
  float *St = reinterpret_cast<float *>(lds_raw + kTileKeysMfma * kKRowBytes);      // after the K tile; [4 waves][64 rows]
  float *red = reinterpret_cast<float *>(St + 4 * 64);                                // [4 waves][256 keys]

  const int r = blockIdx.z, g = blockIdx.y;
  const int N = a.ctx_len[r];
  const int i0 = blockIdx.x * kTileKeysMfma;
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
  constexpr int kKB = kTileKeysMfma / 32;                      // 32-key blocks per tile
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
    for (int j = 0; j < kTileKeysMfma / 16; ++j) {
      const int row = min(s + i0 + drow + 16 * j, a.T - 1);    // tail rows: loaded, masked below
      const bf16_t *gp = K + ((size_t)row * a.Hkv + g) * kD + dpiece * 8;
      asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, off"
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
    constexpr int kRounds = kTileKeysMfma / 32;
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
      if (lhi == 0) red[wave * kTileKeysMfma + kb * 32 + l32] = v;
    }
    __syncthreads();
    const int key = i0 + tid;
    if (tid < kTileKeysMfma && key < N)
      a.part_scores[(size_t)g * a.T + s + key] = (red[tid] + red[kTileKeysMfma + tid]) +
                                                 (red[2 * kTileKeysMfma + tid] + red[3 * kTileKeysMfma + tid]);
  }
}

// scores[t] = sum over KV heads of the partial scores, in head order; question rows get -inf
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

static int scores_tile_keys(const a3_layout *L) { return L->dtype == A3_BF16 ? kTileKeysMfma : kTileKeys; }

size_t a3_scores_ws_bytes(const a3_layout *L) {
  // rows of the score matrix over the whole batch are bounded by n_req * max_q_len * Hq
  const size_t total_rows = (size_t)L->n_req * L->max_q_len * L->n_q_heads;
  const int tk = scores_tile_keys(L);
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
  const size_t total_rows = (size_t)L->n_req * L->max_q_len * L->n_q_heads;   // upper bound, used as row pitch
  const int tk = scores_tile_keys(L);
  const int n_tiles = (L->max_ctx_len + tk - 1) / tk;
  a3_ws_cursor cur(ws, ws_bytes);
  scores_args a;
  a.q = q_question; a.k = k_fused;
  a.seg_start = L->seg_start; a.ctx_len = L->ctx_len; a.q_len = L->q_len; a.q_start = L->q_start;
  a.part = (float2 *)cur.take((size_t)(n_tiles + 1) * total_rows * sizeof(float2));
  a.stats = (float2 *)cur.take(total_rows * sizeof(float2));
  a.part_scores = (float *)cur.take((size_t)L->n_kv_heads * L->total_tokens * sizeof(float));
  if (votes) a.part_scores = votes;
  else if (L->dtype != A3_BF16) a.part_scores = nullptr;       // fp32 path adds the heads itself
  a.causal_q = causal_q;
  a.scores = scores;
  a.n_req = L->n_req; a.Hq = L->n_q_heads; a.Hkv = L->n_kv_heads; a.d = L->head_dim; a.T = L->total_tokens;
  a.total_rows = (int)total_rows; a.n_tiles = n_tiles; a.tile_keys = tk;
  a.scale2 = a3_scale_of(L) * kLog2e;
  a.k_cat = k_cat; a.k_out = k_fused; a.tok_chunk = L->tok_chunk; a.chunk_cs = (const float2 *)L->rope_chunk_cs;
  a.rope_layout = L->rope_layout;
  const bool fuse = k_cat != nullptr && L->dtype == A3_BF16 && L->n_chunks > 0;
  if (k_cat != nullptr && !fuse) {
    s = a3_rope_realign(L, k_cat, k_fused, stream);
    if (s != A3_OK) return s;
  }
  dim3 cgrid((unsigned)((total_rows + 15) / 16));
  if (causal_q) {
    const dim3 qgrid((unsigned)((total_rows + 3) / 4));
    if (L->dtype == A3_BF16) hipLaunchKernelGGL(scores_question_stats_kernel<bf16_t>, qgrid, dim3(256), 0, st, a);
    else hipLaunchKernelGGL(scores_question_stats_kernel<float>, qgrid, dim3(256), 0, st, a);
  }
  if (L->dtype == A3_BF16) {
    static bool attr_done = false;
    if (!attr_done) {
      hipError_t e0 = hipFuncSetAttribute((const void *)scores_bf16_kernel<0, false>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                          (int)kScoresLds);
      hipError_t e1 = hipFuncSetAttribute((const void *)scores_bf16_kernel<1, false>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                          (int)kScoresLds);
      hipError_t e2 = hipFuncSetAttribute((const void *)scores_bf16_kernel<0, true>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                          (int)kScoresLds);
      if (e2 != hipSuccess) e0 = e2;
      if (e0 != hipSuccess || e1 != hipSuccess)
        return a3_fail(A3_ERR_HIP, "a3_question_scores: cannot raise the dynamic LDS limit");
      attr_done = true;
    }
    dim3 grid(n_tiles, L->n_kv_heads, L->n_req);
    if (fuse) hipLaunchKernelGGL((scores_bf16_kernel<0, true>), grid, dim3(256), kScoresLds, st, a);
    else hipLaunchKernelGGL((scores_bf16_kernel<0, false>), grid, dim3(256), kScoresLds, st, a);
    hipLaunchKernelGGL(scores_combine_kernel, cgrid, dim3(256), 0, st, a);
    hipLaunchKernelGGL((scores_bf16_kernel<1, false>), grid, dim3(256), kScoresLds, st, a);
    if (scores)
      hipLaunchKernelGGL(scores_head_sum_kernel, dim3((L->total_tokens + 255) / 256), dim3(256), 0, st, a, L->tok_chunk);
  } else {
    dim3 grid(n_tiles, L->n_req);
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
