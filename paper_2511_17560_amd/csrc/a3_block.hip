// H(.) of Eq. 5: from the attention output of one layer to the input of the next, for the active rows.
//
//   r1 = r0 + O Wo^T                                   output projection, residual
//   r2 = r1 + (silu(n1 Wg^T) * (n1 Wu^T)) Wd^T         n1 = RMSNorm(r1; g_post): gated MLP, residual
//   x' = RMSNorm(r2; g_next)                           input norm of the next block (or the final norm)
//
// The paper names H in one clause (layer normalisation and feed-forward network applied to the attention
// output); this is the pre-norm block of the model families it evaluates.
//
// bf16: three launches of one row-tiled MFMA GEMM (weights [out, in], both operands reduction-contiguous)
// with two epilogues -- "add to the residual row" and "silu(gate) * up" -- and two launches of a
// one-wave-per-row RMSNorm.  The GEMM main loop is the one of the Q/K/V projection: 256 weight rows x
// 64*TB activation rows per workgroup, direct-to-LDS loads into a ring of 32-wide k-slabs, every
// fragment read and every load issued singly behind an MFMA.  For the gated pair a wave's 128 weight
// rows are 64 gate rows and the 64 up rows of the same features, so gate and up of one output meet in
// one lane and the activation is formed on the fp32 accumulators.
// fp32: plain LDS-tiled FMA kernels (correctness configuration, not tuned).
#include "a3_internal.h"
#include "a3_gemm_tile.h"

namespace {

enum { EPI_RESID = 0, EPI_SWIGLU = 1 };

// ---------------------------------------------------------------------------------------
// RMSNorm: one wave per row, two passes over the row (the second is served by the cache)
// ---------------------------------------------------------------------------------------
template <typename T>
__global__ void __launch_bounds__(256)
rms_norm_kernel(const T *x, const int *__restrict__ in_idx, const T *__restrict__ g, float eps, T *out,
                const int *__restrict__ out_idx, int n_rows, int h) {   // x and out may be the same buffer
  constexpr int V = a3_elem<T>::kVec;
  const int lane = threadIdx.x & 63, row = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= n_rows) return;
  const int src = in_idx ? in_idx[row] : row, dst = out_idx ? out_idx[row] : row;
  const T *xr = x + (size_t)src * h;
  T *orow = out + (size_t)dst * h;
  typedef T vec_t __attribute__((ext_vector_type(V)));
  float ss = 0.f;
  for (int v = lane; v < h / V; v += 64) {
    const vec_t t = *reinterpret_cast<const vec_t *>(xr + v * V);
#pragma unroll
    for (int e = 0; e < V; ++e) { const float f = (float)t[e]; ss = fmaf(f, f, ss); }
  }
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) ss += __shfl_xor(ss, o);
  const float inv = 1.0f / sqrtf(ss / (float)h + eps);
  for (int v = lane; v < h / V; v += 64) {
    const vec_t t = *reinterpret_cast<const vec_t *>(xr + v * V);
    const vec_t w = *reinterpret_cast<const vec_t *>(g + v * V);
    vec_t y;
#pragma unroll
    for (int e = 0; e < V; ++e) y[e] = (T)((float)t[e] * inv * (float)w[e]);
    *reinterpret_cast<vec_t *>(orow + v * V) = y;
  }
}

// ---------------------------------------------------------------------------------------
// bf16 MFMA GEMM with the two epilogues
// ---------------------------------------------------------------------------------------
struct gemm_args {
  const bf16_t *a;       // activation rows [*, K]
  const int *a_idx;      // row i of the product reads activation row a_idx[i] (NULL: row i)
  int n_rows;
  const bf16_t *w0;      // [N, K]; EPI_SWIGLU: the gate weights
  const bf16_t *w1;      // EPI_SWIGLU: the up weights [N, K]
  bf16_t *out;           // EPI_RESID: [*, N], row out_idx[i] += product row i; EPI_SWIGLU: [n_rows, N]
  const int *out_idx;
  int K, N;
  int n_ftiles, n_tok_tiles;
};

template <int TB, int EPI, bool K64>
__global__ void __launch_bounds__(256, (TB == 2 && !K64) ? 2 : 1)
gemm_bf16_kernel(gemm_args a) {
  constexpr int kTokTile = 64 * TB;
  constexpr int kFeat = EPI == EPI_RESID ? 256 : 128;        // output features per workgroup
  extern __shared__ __align__(16) unsigned char lds[];

  // consecutive workgroup ids go to different XCDs; all row tiles of one feature tile stay on one XCD
  const int xcd = blockIdx.x & 7, q = blockIdx.x >> 3;
  const int ft = xcd + 8 * (q / a.n_tok_tiles), tt = q % a.n_tok_tiles;
  if (ft >= a.n_ftiles) return;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, lhi = lane >> 5;
  const int fh = wave & 1, th = wave >> 1;

  const int tok0 = tt * kTokTile + th * 32 * TB;

  // ---- the product.  EPI_RESID: weight-tile row r is weight row kFeat ft + r.  EPI_SWIGLU: rows 0..63 of a
  // wave's half are the gate rows of its 64 features, rows 64..127 the up rows of the same features.
  f32x16 acc[4][TB];
  gemm_tile_mainloop<TB, K64>(
      acc, lds, a.K,
      [&](int row) -> const bf16_t * {
        if (EPI == EPI_RESID) return a.w0 + (size_t)min(kFeat * ft + row, a.N - 1) * a.K;
        const int r = row & 127;
        const int f = min(kFeat * ft + 64 * (row >> 7) + (r & 63), a.N - 1);
        return (r < 64 ? a.w0 : a.w1) + (size_t)f * a.K;
      },
      [&](int row) -> const bf16_t * {
        const int m = min(tt * kTokTile + row, a.n_rows - 1);    // clamp: computed but never stored
        return a.a + (size_t)(a.a_idx ? a.a_idx[m] : m) * a.K;
      });

  // ---- epilogue ----------------------------------------------------------------------------------------
  // Each wave turns its fp32 tile through its own piece of the now free LDS, one 32-row block at a time
  // ([32 rows][128 weight rows], row stride 528 bytes).  Read back, a lane holds weight rows 4c..4c+3 and
  // 64+4c..64+4c+3 of one activation row and 16 lanes cover that row: global accesses are whole runs.
  __syncthreads();
  const int fblock = EPI == EPI_RESID ? kFeat * ft + 128 * fh : kFeat * ft + 64 * fh;   // first output feature
  if (fblock >= a.N) return;
  constexpr int kEpiStride = 528;
  unsigned char *epi = lds + wave * (32 * kEpiStride);
  const int ec = lane & 15, er = lane >> 4;
  int orow[TB][8];
#pragma unroll
  for (int tb = 0; tb < TB; ++tb)
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const int tok = tok0 + tb * 32 + er + 4 * j;
      orow[tb][j] = tok < a.n_rows ? (a.out_idx ? a.out_idx[tok] : tok) : -1;
    }
#pragma unroll
  for (int tb = 0; tb < TB; ++tb) {
    // accumulator block (fb, tb), register r of this lane: weight row 32 fb + 8 (r/4) + 4 lhi + r%4, row l32
#pragma unroll
    for (int fb = 0; fb < 4; ++fb)
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        f32x4 v;
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] = acc[fb][tb][4 * q4 + e];
        *reinterpret_cast<f32x4 *>(epi + l32 * kEpiStride + (32 * fb + 8 * q4 + 4 * lhi) * 4) = v;
      }
    if (EPI == EPI_RESID) {
      bf16x4 rl[8], rh[8];
#pragma unroll
      for (int j = 0; j < 8; ++j)
        if (orow[tb][j] >= 0) {
          const bf16_t *p = a.out + (size_t)orow[tb][j] * a.N + fblock;
          rl[j] = *reinterpret_cast<const bf16x4 *>(p + 4 * ec);
          rh[j] = *reinterpret_cast<const bf16x4 *>(p + 64 + 4 * ec);
        }
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const int row = er + 4 * j;
        const f32x4 lo = *reinterpret_cast<const f32x4 *>(epi + row * kEpiStride + ec * 16);
        const f32x4 hi = *reinterpret_cast<const f32x4 *>(epi + row * kEpiStride + 256 + ec * 16);
        if (orow[tb][j] >= 0) {
          bf16_t *p = a.out + (size_t)orow[tb][j] * a.N + fblock;
          bf16x4 vlo, vhi;
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            vlo[e] = a3_f2bf(a3_bf2f(rl[j][e]) + lo[e]);
            vhi[e] = a3_f2bf(a3_bf2f(rh[j][e]) + hi[e]);
          }
          *reinterpret_cast<bf16x4 *>(p + 4 * ec) = vlo;
          *reinterpret_cast<bf16x4 *>(p + 64 + 4 * ec) = vhi;
        }
      }
    } else {
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const int row = er + 4 * j;
        const f32x4 gt = *reinterpret_cast<const f32x4 *>(epi + row * kEpiStride + ec * 16);         // gate
        const f32x4 up = *reinterpret_cast<const f32x4 *>(epi + row * kEpiStride + 256 + ec * 16);   // up
        if (orow[tb][j] >= 0) {
          bf16x4 v;
#pragma unroll
          for (int e = 0; e < 4; ++e) v[e] = a3_f2bf(gt[e] / (1.0f + __expf(-gt[e])) * up[e]);
          *reinterpret_cast<bf16x4 *>(a.out + (size_t)orow[tb][j] * a.N + fblock + 4 * ec) = v;
        }
      }
    }
  }
}

// ---------------------------------------------------------------------------------------
// fp32 GEMM with the same two epilogues (correctness configuration)
// ---------------------------------------------------------------------------------------
struct gemm_args_f32 {
  const float *a;
  const int *a_idx;
  int n_rows;
  const float *w0, *w1;
  float *out;
  const int *out_idx;
  int K, N;
};

template <int EPI>
__global__ void __launch_bounds__(256)
gemm_f32_kernel(gemm_args_f32 a) {
  constexpr int R = 16, F = 64, BK = 32;
  __shared__ float As[R][BK + 1];
  __shared__ float W0s[F][BK + 1];
  __shared__ float W1s[EPI == EPI_SWIGLU ? F : 1][BK + 1];
  const int f0 = blockIdx.x * F, m0 = blockIdx.y * R;
  const int tid = threadIdx.x, ty = tid >> 4, tx = tid & 15;
  float acc0[4] = {0.f, 0.f, 0.f, 0.f}, acc1[4] = {0.f, 0.f, 0.f, 0.f};
  for (int k0 = 0; k0 < a.K; k0 += BK) {
    for (int i = tid; i < R * BK; i += 256) {
      const int r = i / BK, c = i % BK, m = m0 + r;
      float v = 0.f;
      if (m < a.n_rows && k0 + c < a.K) v = a.a[(size_t)(a.a_idx ? a.a_idx[m] : m) * a.K + k0 + c];
      As[r][c] = v;
    }
    for (int i = tid; i < F * BK; i += 256) {
      const int r = i / BK, c = i % BK;
      const bool ok = f0 + r < a.N && k0 + c < a.K;
      W0s[r][c] = ok ? a.w0[(size_t)(f0 + r) * a.K + k0 + c] : 0.f;
      if (EPI == EPI_SWIGLU) W1s[r][c] = ok ? a.w1[(size_t)(f0 + r) * a.K + k0 + c] : 0.f;
    }
    __syncthreads();
    for (int c = 0; c < BK; ++c) {
      const float x = As[ty][c];
#pragma unroll
      for (int f = 0; f < 4; ++f) {
        acc0[f] = fmaf(x, W0s[tx + 16 * f][c], acc0[f]);
        if (EPI == EPI_SWIGLU) acc1[f] = fmaf(x, W1s[tx + 16 * f][c], acc1[f]);
      }
    }
    __syncthreads();
  }
  const int m = m0 + ty;
  if (m >= a.n_rows) return;
  const int orow = a.out_idx ? a.out_idx[m] : m;
#pragma unroll
  for (int f = 0; f < 4; ++f) {
    const int feat = f0 + tx + 16 * f;
    if (feat >= a.N) continue;
    float *p = a.out + (size_t)orow * a.N + feat;
    if (EPI == EPI_RESID) *p += acc0[f];
    else *p = acc0[f] / (1.0f + expf(-acc0[f])) * acc1[f];
  }
}

// rows per workgroup (64 TB): useful rows / padded rows x how evenly the workgroups fill 256 CUs (the
// busiest CU sets the time; two co-resident 128-row workgroups share their CU's matrix pipes) x a bonus
// for the lower cache traffic of larger tiles
int pick_tb(int n_rows, int n_ftiles) {
  int best_tb = 2;
  double best = -1.0;
  for (int c = 2; c <= 4; ++c) {
    const int tiles = (n_rows + 64 * c - 1) / (64 * c);
    const long wgs = (long)tiles * n_ftiles;
    const long rounds = (wgs + 255) / 256;
    const double fill = (double)wgs / (double)(rounds * 256L);
    const double pad = (double)n_rows / (double)(tiles * 64 * c);
    const double traffic = 256.0 * 64 * c / (256.0 + 64 * c) / 128.0;
    const double score = pad * fill * (0.5 + 0.5 * traffic);
    if (score > best) { best = score; best_tb = c; }
  }
  return best_tb;
}

template <int EPI>
a3_status gemm_bf16_launch(const gemm_args &a0, hipStream_t st, const char *who) {
  gemm_args a = a0;
  a.n_ftiles = EPI == EPI_RESID ? (a.N + 255) / 256 : (a.N + 127) / 128;
  int tb = pick_tb(a.n_rows, a.n_ftiles);
  { const int t = a3_knob(A3_KNOB_GEMM_TB); if (t >= 2 && t <= 4) tb = t; }   // tuning value "gemm_tb"
  a.n_tok_tiles = (a.n_rows + 64 * tb - 1) / (64 * tb);
  // 128-byte row pieces whenever K allows (tuning value "gemm_k64" = 0: the 64-byte loop)
  bool k64 = a.K % 64 == 0;
  if (a3_knob(A3_KNOB_GEMM_K64) == 0) k64 = false;
  static a3_once_per_device lds_once;
  const hipError_t once_err = a3_once(lds_once, []() {
    hipError_t e1 = hipFuncSetAttribute((const void *)gemm_bf16_kernel<2, EPI, false>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)gemm_tile_lds_bytes(2));
    hipError_t e2 = hipFuncSetAttribute((const void *)gemm_bf16_kernel<3, EPI, false>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)gemm_tile_lds_bytes(3));
    hipError_t e3 = hipFuncSetAttribute((const void *)gemm_bf16_kernel<4, EPI, false>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)gemm_tile_lds_bytes(4));
    hipError_t e4 = hipFuncSetAttribute((const void *)gemm_bf16_kernel<3, EPI, true>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)gemm_tile_lds_bytes_k64(3));
    hipError_t e5 = hipFuncSetAttribute((const void *)gemm_bf16_kernel<4, EPI, true>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)gemm_tile_lds_bytes_k64(4));
    hipError_t e6 = hipFuncSetAttribute((const void *)gemm_bf16_kernel<2, EPI, true>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)gemm_tile_lds_bytes_k64(2));
    for (hipError_t e : {e1, e2, e3, e4, e5, e6}) if (e != hipSuccess) return e;
    return hipSuccess;
  });
  if (once_err != hipSuccess) return a3_fail(A3_ERR_HIP, "%s: cannot raise the dynamic LDS limit", who);
  const unsigned grid = 8u * (unsigned)((a.n_ftiles + 7) / 8) * (unsigned)a.n_tok_tiles;
  if (tb == 2 && k64) hipLaunchKernelGGL((gemm_bf16_kernel<2, EPI, true>), dim3(grid), dim3(256), gemm_tile_lds_bytes_k64(2), st, a);
  else if (tb == 2) hipLaunchKernelGGL((gemm_bf16_kernel<2, EPI, false>), dim3(grid), dim3(256), gemm_tile_lds_bytes(2), st, a);
  else if (tb == 3 && k64) hipLaunchKernelGGL((gemm_bf16_kernel<3, EPI, true>), dim3(grid), dim3(256), gemm_tile_lds_bytes_k64(3), st, a);
  else if (tb == 3) hipLaunchKernelGGL((gemm_bf16_kernel<3, EPI, false>), dim3(grid), dim3(256), gemm_tile_lds_bytes(3), st, a);
  else if (k64) hipLaunchKernelGGL((gemm_bf16_kernel<4, EPI, true>), dim3(grid), dim3(256), gemm_tile_lds_bytes_k64(4), st, a);
  else hipLaunchKernelGGL((gemm_bf16_kernel<4, EPI, false>), dim3(grid), dim3(256), gemm_tile_lds_bytes(4), st, a);
  A3_CHECK_LAUNCH(who);
  return A3_OK;
}

template <int EPI>
a3_status gemm_f32_launch(const gemm_args_f32 &a, hipStream_t st, const char *who) {
  dim3 grid((a.N + 63) / 64, (a.n_rows + 15) / 16);
  hipLaunchKernelGGL(gemm_f32_kernel<EPI>, grid, dim3(256), 0, st, a);
  A3_CHECK_LAUNCH(who);
  return A3_OK;
}

a3_status rms_norm_launch(const a3_layout *L, const void *x, const int *in_idx, const void *g, float eps, void *out,
                          const int *out_idx, int n_rows, hipStream_t st, const char *who) {
  const dim3 grid((n_rows + 3) / 4);
  if (L->dtype == A3_BF16)
    hipLaunchKernelGGL(rms_norm_kernel<bf16_t>, grid, dim3(256), 0, st, (const bf16_t *)x, in_idx, (const bf16_t *)g, eps,
                       (bf16_t *)out, out_idx, n_rows, L->hidden);
  else
    hipLaunchKernelGGL(rms_norm_kernel<float>, grid, dim3(256), 0, st, (const float *)x, in_idx, (const float *)g, eps,
                       (float *)out, out_idx, n_rows, L->hidden);
  A3_CHECK_LAUNCH(who);
  return A3_OK;
}

size_t elem_bytes(const a3_layout *L) { return L->dtype == A3_BF16 ? 2 : 4; }

}  // namespace

extern "C" size_t a3_block_tail_ws_bytes(const a3_layout *L, int ffn, int n_rows) {
  if (L == nullptr || ffn <= 0 || n_rows < 0 || L->hidden <= 0) return 0;
  if (L->dtype != A3_BF16 && L->dtype != A3_F32) return 0;
  const size_t e = elem_bytes(L);
  return a3_align_up((size_t)n_rows * L->hidden * e, 256) + a3_align_up((size_t)n_rows * ffn * e, 256) + 256;
}

extern "C" a3_status a3_rms_norm(const a3_layout *L, const void *x, const int *row_idx, int n_rows, const void *g,
                                 float eps, void *out, void *stream) {
  a3_status s = a3_check_layout(L, "a3_rms_norm", false);
  if (s != A3_OK) return s;
  A3_REQUIRE(n_rows >= 0 && n_rows <= L->total_tokens, A3_ERR_INVALID_ARG, "a3_rms_norm: n_rows %d outside [0, %d]",
             n_rows, L->total_tokens);
  if (n_rows == 0) return A3_OK;
  A3_REQUIRE(x && g && out, A3_ERR_INVALID_ARG, "a3_rms_norm: NULL tensor");
  A3_REQUIRE(a3_aligned16(x) && a3_aligned16(g) && a3_aligned16(out), A3_ERR_INVALID_ARG,
             "a3_rms_norm: tensors must be 16-byte aligned");
  A3_REQUIRE(eps >= 0.f, A3_ERR_INVALID_ARG, "a3_rms_norm: eps %g is negative", (double)eps);
  A3_REQUIRE(L->hidden % 8 == 0, A3_ERR_UNSUPPORTED, "a3_rms_norm: needs hidden %% 8 == 0, got %d", L->hidden);
  return rms_norm_launch(L, x, row_idx, g, eps, out, row_idx, n_rows, (hipStream_t)stream, "a3_rms_norm");
}

extern "C" a3_status a3_block_tail(const a3_layout *L, const void *attn_out, const int *act_idx, int n_act,
                                   const a3_block_weights *w, void *resid, void *hidden_next, void *ws,
                                   size_t ws_bytes, void *stream) {
  a3_status s = a3_check_layout(L, "a3_block_tail", false);
  if (s != A3_OK) return s;
  A3_REQUIRE(n_act >= 0 && n_act <= L->total_tokens, A3_ERR_INVALID_ARG, "a3_block_tail: n_act %d outside [0, %d]",
             n_act, L->total_tokens);
  if (n_act == 0) return A3_OK;
  A3_REQUIRE(w != nullptr, A3_ERR_INVALID_ARG, "a3_block_tail: weights are NULL");
  A3_REQUIRE(attn_out && resid && hidden_next, A3_ERR_INVALID_ARG, "a3_block_tail: NULL tensor");
  A3_REQUIRE(w->wo && w->g_post && w->w_gate && w->w_up && w->w_down && w->g_next, A3_ERR_INVALID_ARG,
             "a3_block_tail: a weight is NULL");
  const void *ptrs[] = {attn_out, resid, hidden_next, w->wo, w->g_post, w->w_gate, w->w_up, w->w_down, w->g_next};
  for (const void *p : ptrs)
    A3_REQUIRE(a3_aligned16(p), A3_ERR_INVALID_ARG, "a3_block_tail: tensors must be 16-byte aligned");
  A3_REQUIRE(w->ffn > 0, A3_ERR_INVALID_ARG, "a3_block_tail: ffn %d", w->ffn);
  A3_REQUIRE(w->eps >= 0.f, A3_ERR_INVALID_ARG, "a3_block_tail: eps %g is negative", (double)w->eps);
  A3_REQUIRE(L->hidden % 8 == 0, A3_ERR_UNSUPPORTED, "a3_block_tail: needs hidden %% 8 == 0, got %d", L->hidden);
  const int h = L->hidden, f = w->ffn, qd = L->n_q_heads * L->head_dim;
  if (L->dtype == A3_BF16)
    A3_REQUIRE(h % 128 == 0 && f % 64 == 0 && qd % 32 == 0, A3_ERR_UNSUPPORTED,
               "a3_block_tail: bf16 needs hidden %% 128 == 0, ffn %% 64 == 0, heads x head_dim %% 32 == 0 (got %d, %d, %d)",
               h, f, qd);
  A3_REQUIRE(ws != nullptr, A3_ERR_WORKSPACE, "a3_block_tail: workspace is NULL");
  const size_t need = a3_block_tail_ws_bytes(L, f, n_act);
  A3_REQUIRE(ws_bytes >= need, A3_ERR_WORKSPACE, "a3_block_tail: workspace %zu bytes, need %zu", ws_bytes, need);
  hipStream_t st = (hipStream_t)stream;
  a3_ws_cursor cur(ws, ws_bytes);
  void *normed = cur.take((size_t)n_act * h * elem_bytes(L));
  void *act = cur.take((size_t)n_act * f * elem_bytes(L));

  // r1 = r0 + O Wo^T
  if (L->dtype == A3_BF16) {
    gemm_args a{(const bf16_t *)attn_out, nullptr, n_act, (const bf16_t *)w->wo, nullptr, (bf16_t *)resid, act_idx, qd, h, 0, 0};
    if ((s = gemm_bf16_launch<EPI_RESID>(a, st, "a3_block_tail")) != A3_OK) return s;
  } else {
    gemm_args_f32 a{(const float *)attn_out, nullptr, n_act, (const float *)w->wo, nullptr, (float *)resid, act_idx, qd, h};
    if ((s = gemm_f32_launch<EPI_RESID>(a, st, "a3_block_tail")) != A3_OK) return s;
  }
  // n1 = RMSNorm(r1; g_post), compact
  if ((s = rms_norm_launch(L, resid, act_idx, w->g_post, w->eps, normed, nullptr, n_act, st, "a3_block_tail")) != A3_OK)
    return s;
  // act = silu(n1 Wg^T) * (n1 Wu^T);  r2 = r1 + act Wd^T
  if (L->dtype == A3_BF16) {
    gemm_args a{(const bf16_t *)normed, nullptr, n_act, (const bf16_t *)w->w_gate, (const bf16_t *)w->w_up, (bf16_t *)act, nullptr, h, f, 0, 0};
    if ((s = gemm_bf16_launch<EPI_SWIGLU>(a, st, "a3_block_tail")) != A3_OK) return s;
    gemm_args b{(const bf16_t *)act, nullptr, n_act, (const bf16_t *)w->w_down, nullptr, (bf16_t *)resid, act_idx, f, h, 0, 0};
    if ((s = gemm_bf16_launch<EPI_RESID>(b, st, "a3_block_tail")) != A3_OK) return s;
  } else {
    gemm_args_f32 a{(const float *)normed, nullptr, n_act, (const float *)w->w_gate, (const float *)w->w_up, (float *)act, nullptr, h, f};
    if ((s = gemm_f32_launch<EPI_SWIGLU>(a, st, "a3_block_tail")) != A3_OK) return s;
    gemm_args_f32 b{(const float *)act, nullptr, n_act, (const float *)w->w_down, nullptr, (float *)resid, act_idx, f, h};
    if ((s = gemm_f32_launch<EPI_RESID>(b, st, "a3_block_tail")) != A3_OK) return s;
  }
  // x' = RMSNorm(r2; g_next) at the rows' own places
  return rms_norm_launch(L, resid, act_idx, w->g_next, w->eps, hidden_next, act_idx, n_act, st, "a3_block_tail");
}
