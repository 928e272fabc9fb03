// Step 2 of the A^3 fusion path: question-relevance score, Eq. 3 first line.
//
//   s_i = sum_{hq} sum_j softmax_i( q_{j,hq} . k'_{i, hq/G} * scale )      softmax over the context keys
//
// A column sum of row softmaxes needs every row's (max, sum exp) before any column can be
// summed, so the logits are formed twice:
//   pass A   per (key tile, row): partial (max, sum exp)          -> workspace
//   combine  per row: merge the partials                          -> (max, 1/sum) per row
//   pass B   per key tile: sum over all rows of exp(l - max)/sum  -> scores
// Heads and rows are reduced in a fixed order inside the workgroup that owns a key tile, so
// the result is deterministic (no atomics).
//
// bf16: logits on the matrix cores (32x32x16 bf16 MFMA), K tile staged in LDS with a padded
// stride, Q fragments read straight from global memory (they are L2 resident), exp2 with
// log2(e) folded into the scale.  fp32: plain FMA kernels (correctness configuration).
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
  float2 *stats;            // [total_rows] (max, 1/sum)
  float *scores;            // [T]
  int n_req, Hq, Hkv, d, T, total_rows, n_tiles;
  float scale2;             // sm_scale * log2(e)
};

// ---------------------------------------------------------------------------------------
// combine partial row statistics (shared by both element types)
// ---------------------------------------------------------------------------------------
constexpr int kTileKeys = 64;

__global__ void __launch_bounds__(256)
scores_combine_kernel(scores_args a) {
  // 32 rows x 8 tile slices per workgroup
  __shared__ float2 red[8][32];
  const int row = blockIdx.x * 32 + (threadIdx.x & 31);
  const int slice = threadIdx.x >> 5;
  float m = -INFINITY, z = 0.f;
  if (row < a.total_rows) {
    const int jq = row / a.Hq;
    const int r = find_segment(a.q_start, a.n_req, jq);
    const int tiles = (a.ctx_len[r] + kTileKeys - 1) / kTileKeys;
    for (int t = slice; t < tiles; t += 8) {
      float2 p = a.part[(size_t)t * a.total_rows + row];
      float mn = fmaxf(m, p.x);
      z = z * exp2f(m - mn) + p.y * exp2f(p.x - mn);
      m = mn;
    }
  }
  red[slice][threadIdx.x & 31] = make_float2(m, z);
  __syncthreads();
  if (slice == 0 && row < a.total_rows) {
    for (int s = 1; s < 8; ++s) {
      float2 p = red[s][threadIdx.x & 31];
      if (p.y > 0.f) {
        float mn = fmaxf(m, p.x);
        z = z * exp2f(m - mn) + p.y * exp2f(p.x - mn);
        m = mn;
      }
    }
    a.stats[row] = make_float2(m, z > 0.f ? 1.0f / z : 0.f);
  }
}

// ---------------------------------------------------------------------------------------
// bf16 MFMA kernel, head_dim 128.  PASS 0 = partial row statistics, PASS 1 = column sums.
// Workgroup = one 64-key tile of one request; loops over KV heads and 128-row blocks.
// ---------------------------------------------------------------------------------------
constexpr int kD = 128;
constexpr int kKStride = kD + 8;      // LDS row stride (elements): 272 B

template <int PASS>
__global__ void __launch_bounds__(256)
scores_bf16_kernel(scores_args a) {
  __shared__ __align__(16) bf16_t Ks[kTileKeys * kKStride];
  __shared__ float2 St[128];           // PASS 1: (max, 1/sum) of the current 128-row block
  __shared__ float red[4][kTileKeys];

  const int r = blockIdx.y;
  const int N = a.ctx_len[r];
  const int i0 = blockIdx.x * kTileKeys;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int s = a.seg_start[r];
  const int nq = a.q_len[r];
  if (PASS == 1 && blockIdx.x == 0) {
    for (int j = tid; j < nq; j += 256) a.scores[s + N + j] = -INFINITY;   // question rows are not candidates
  }
  if (i0 >= N) return;
  const int G = a.Hq / a.Hkv;
  const int Mg = nq * G;                // rows per KV head: m = j*G + hh
  const int qrow0 = a.q_start[r];
  const bf16_t *__restrict__ Q = (const bf16_t *)a.q;
  const bf16_t *__restrict__ K = (const bf16_t *)a.k;
  const int l32 = lane & 31, lhi = lane >> 5;

  float colsum[2] = {0.f, 0.f};        // PASS 1: this lane's keys (block 0 / 1), partial over its rows

  for (int g = 0; g < a.Hkv; ++g) {
    __syncthreads();                    // previous K tile fully consumed
    // stage K tile: 64 keys x 128 dims; 16 lanes cover one 256-byte row
    for (int i = tid; i < kTileKeys * 16; i += 256) {
      int kr = i >> 4, c = i & 15;
      int row = s + i0 + kr;
      if (row > a.T - 1) row = a.T - 1;  // tail of the last tile: loaded, masked below
      uint4 v = *reinterpret_cast<const uint4 *>(K + ((size_t)row * a.Hkv + g) * kD + c * 8);
      *reinterpret_cast<uint4 *>(Ks + kr * kKStride + c * 8) = v;
    }
    __syncthreads();

    for (int mb = 0; mb < Mg; mb += 128) {
      // this wave's 32 rows; the lane's row for fragment loads
      int m = mb + wave * 32 + l32;
      int mc = m < Mg ? m : Mg - 1;
      const int row_id = (qrow0 + mc / G) * a.Hq + g * G + mc % G;   // row of the [sum q_len * Hq] row space
      const bf16_t *qp = Q + (size_t)row_id * kD + lhi * 8;
      if (PASS == 1) {
        __syncthreads();                // St of the previous block consumed
        if (tid < 128) {
          int m2 = mb + tid;
          float2 st = make_float2(0.f, 0.f);
          if (m2 < Mg) st = a.stats[(qrow0 + m2 / G) * a.Hq + g * G + m2 % G];
          St[tid] = st;
        }
        __syncthreads();
      }
      f32x16 acc[2];
#pragma unroll
      for (int b = 0; b < 2; ++b)
#pragma unroll
        for (int x = 0; x < 16; ++x) acc[b][x] = 0.f;
#pragma unroll
      for (int ks = 0; ks < kD / 16; ++ks) {
        bf16x8 qf = *reinterpret_cast<const bf16x8 *>(qp + ks * 16);
#pragma unroll
        for (int b = 0; b < 2; ++b) {
          bf16x8 kf = *reinterpret_cast<const bf16x8 *>(Ks + (b * 32 + l32) * kKStride + ks * 16 + lhi * 8);
          if (PASS == 0) acc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf, acc[b], 0, 0, 0);   // C[key][row]
          else           acc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qf, kf, acc[b], 0, 0, 0);   // C[row][key]
        }
      }
      if (PASS == 0) {
        // lane: row m (column l32); registers: keys b*32 + 8(x/4) + 4 lhi + x%4
        float mx = -INFINITY;
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
          for (int x = 0; x < 16; ++x) {
            int key = i0 + b * 32 + 8 * (x >> 2) + 4 * lhi + (x & 3);
            float l = key < N ? acc[b][x] * a.scale2 : -INFINITY;
            acc[b][x] = l;
            mx = fmaxf(mx, l);
          }
        mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
        float sum = 0.f;
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
          for (int x = 0; x < 16; ++x) sum += exp2f(acc[b][x] - mx);
        sum += __shfl_xor(sum, 32, 64);
        if (lhi == 0 && m < Mg) a.part[(size_t)blockIdx.x * a.total_rows + row_id] = make_float2(mx, sum);
      } else {
        // lane: key l32 of block b (column); registers: rows 8(x/4) + 4 lhi + x%4 of this wave's block
#pragma unroll
        for (int b = 0; b < 2; ++b) {
          float part = 0.f;
#pragma unroll
          for (int x = 0; x < 16; ++x) {
            float2 st = St[wave * 32 + 8 * (x >> 2) + 4 * lhi + (x & 3)];
            part += exp2f(acc[b][x] * a.scale2 - st.x) * st.y;    // st.y = 0 for rows beyond Mg
          }
          colsum[b] += part;
        }
      }
    }
  }
  if (PASS == 1) {
#pragma unroll
    for (int b = 0; b < 2; ++b) {
      float v = colsum[b] + __shfl_xor(colsum[b], 32, 64);
      if (lhi == 0) red[wave][b * 32 + l32] = v;
    }
    __syncthreads();
    if (tid < kTileKeys && i0 + tid < N)
      a.scores[s + i0 + tid] = (red[0][tid] + red[1][tid]) + (red[2][tid] + red[3][tid]);
  }
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
  if (PASS == 1 && blockIdx.x == 0)
    for (int j = tid; j < nq; j += 256) a.scores[s + N + j] = -INFINITY;
  if (i0 >= N) return;
  const int d = a.d, G = a.Hq / a.Hkv, Mg = nq * G, qrow0 = a.q_start[r];
  const float *__restrict__ Q = (const float *)a.q;
  const float *__restrict__ K = (const float *)a.k;
  float colsum = 0.f;

  for (int g = 0; g < a.Hkv; ++g) {
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
        float2 st = a.stats[row_id];
        colsum += exp2f(l - st.x) * st.y;
      }
    }
  }
  if (PASS == 1) {
    red[slice][key] = colsum;
    __syncthreads();
    if (tid < kTileKeys && i0 + tid < N)
      a.scores[s + i0 + tid] = (red[0][tid] + red[1][tid]) + (red[2][tid] + red[3][tid]);
  }
}

}  // namespace

size_t a3_scores_ws_bytes(const a3_layout *L) {
  // rows of the score matrix over the whole batch are bounded by n_req * max_q_len * Hq
  size_t total_rows = (size_t)L->n_req * L->max_q_len * L->n_q_heads;
  size_t n_tiles = (size_t)(L->max_ctx_len + kTileKeys - 1) / kTileKeys;
  return a3_align_up(n_tiles * total_rows * sizeof(float2), 256) + a3_align_up(total_rows * sizeof(float2), 256) + 256;
}

extern "C" a3_status a3_question_scores(const a3_layout *L, const void *q_question, const void *k_fused, float *scores,
                                        void *ws, size_t ws_bytes, void *stream) {
  a3_status s = a3_check_layout(L, "a3_question_scores", true);
  if (s != A3_OK) return s;
  A3_REQUIRE(q_question && k_fused && scores, A3_ERR_INVALID_ARG, "a3_question_scores: NULL tensor");
  A3_REQUIRE(a3_aligned16(q_question) && a3_aligned16(k_fused), A3_ERR_INVALID_ARG,
             "a3_question_scores: tensors must be 16-byte aligned");
  A3_REQUIRE(ws != nullptr, A3_ERR_WORKSPACE, "a3_question_scores: workspace is NULL");
  A3_REQUIRE(ws_bytes >= a3_scores_ws_bytes(L), A3_ERR_WORKSPACE,
             "a3_question_scores: workspace %zu bytes, need %zu", ws_bytes, a3_scores_ws_bytes(L));
  hipStream_t st = (hipStream_t)stream;
  const size_t total_rows = (size_t)L->n_req * L->max_q_len * L->n_q_heads;   // upper bound, used as row pitch
  const int n_tiles = (L->max_ctx_len + kTileKeys - 1) / kTileKeys;
  a3_ws_cursor cur(ws, ws_bytes);
  scores_args a;
  a.q = q_question; a.k = k_fused;
  a.seg_start = L->seg_start; a.ctx_len = L->ctx_len; a.q_len = L->q_len; a.q_start = L->q_start;
  a.part = (float2 *)cur.take((size_t)n_tiles * total_rows * sizeof(float2));
  a.stats = (float2 *)cur.take(total_rows * sizeof(float2));
  a.scores = scores;
  a.n_req = L->n_req; a.Hq = L->n_q_heads; a.Hkv = L->n_kv_heads; a.d = L->head_dim; a.T = L->total_tokens;
  a.total_rows = (int)total_rows; a.n_tiles = n_tiles;
  a.scale2 = a3_scale_of(L) * kLog2e;
  if (n_tiles == 0 || L->max_q_len == 0) {
    // nothing to score with: every context row gets 0 through pass B's early exit; not supported
    return a3_fail(A3_ERR_UNSUPPORTED, "a3_question_scores: needs max_ctx_len > 0 and max_q_len > 0");
  }
  dim3 grid(n_tiles, L->n_req);
  dim3 cgrid((unsigned)((total_rows + 31) / 32));
  if (L->dtype == A3_BF16) {
    hipLaunchKernelGGL(scores_bf16_kernel<0>, grid, dim3(256), 0, st, a);
    hipLaunchKernelGGL(scores_combine_kernel, cgrid, dim3(256), 0, st, a);
    hipLaunchKernelGGL(scores_bf16_kernel<1>, grid, dim3(256), 0, st, a);
  } else {
    hipLaunchKernelGGL(scores_f32_kernel<0>, grid, dim3(256), 0, st, a);
    hipLaunchKernelGGL(scores_combine_kernel, cgrid, dim3(256), 0, st, a);
    hipLaunchKernelGGL(scores_f32_kernel<1>, grid, dim3(256), 0, st, a);
  }
  A3_CHECK_LAUNCH("a3_question_scores");
  return A3_OK;
}
