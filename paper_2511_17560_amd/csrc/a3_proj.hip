// Step 4 (projection part) of the A^3 fusion path: Q/K/V of the listed rows, Eq. 5 first lines.
//
//   Q = RoPE_p(x Wq^T + bq),  K = RoPE_p(x Wk^T + bk),  V = x Wv^T + bv        p = position of the row
//
// bf16: a row-gathering MFMA GEMM.  One workgroup computes one head (128 output features) for
// 128 listed rows.  The weight tile is the MFMA "row" operand and the gathered hidden rows
// the "column" operand, so a lane ends up holding, for ONE token, 4 consecutive features per
// accumulator quad and all 128 features of the head across its 4 accumulator blocks: both
// RoPE pairings (adjacent coordinates, or i with i+64) are lane-local and the rotation runs in
// the epilogue on the fp32 accumulators, before the single rounding to bf16.
// fp32: a plain LDS-tiled FMA kernel (correctness configuration, not tuned).
#include "a3_internal.h"

namespace {

// ---------------------------------------------------------------------------------------
// bf16 MFMA kernel
// ---------------------------------------------------------------------------------------
constexpr int kHeadDim = 128;        // features per tile = one head
constexpr int kTokTile = 128;        // listed rows per tile
constexpr int kBK = 64;              // reduction slab
constexpr int kStride = kBK + 8;     // LDS row stride in elements: 144 B, 16 rows cover all 64 banks once
constexpr int kThreads = 256;
constexpr int kTileElems = 128 * kStride;
constexpr size_t kProjLds = (size_t)4 * kTileElems * sizeof(bf16_t);   // W and X tiles, double buffered

struct proj_args {
  const bf16_t *hidden;
  const int *row_idx;
  int n_rows;
  const bf16_t *w[3];
  const bf16_t *bias[3];
  bf16_t *out[3];
  const int *tok_pos;
  const float2 *pos_cs;
  int K, Hq, Hkv, rope_layout;
};

__global__ void __launch_bounds__(kThreads)
proj_bf16_kernel(proj_args a) {
  extern __shared__ __align__(16) unsigned char lds_raw[];
  bf16_t *Ws = reinterpret_cast<bf16_t *>(lds_raw);          // [2][128][kStride]
  bf16_t *Xs = Ws + 2 * kTileElems;                          // [2][128][kStride]

  // which projection / head this tile belongs to
  int head = blockIdx.x, which = 0, heads_out = a.Hq;
  if (head >= a.Hq) { head -= a.Hq; which = 1; heads_out = a.Hkv; }
  if (which == 1 && head >= a.Hkv) { head -= a.Hkv; which = 2; }
  bf16_t *__restrict__ out = a.out[which];
  if (out == nullptr) return;
  const bf16_t *__restrict__ W = a.w[which] + (size_t)head * kHeadDim * a.K;
  const int m0 = blockIdx.y * kTokTile;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;

  // global -> LDS staging: thread moves 16 B of 4 rows of each tile per slab
  const int c16 = tid & 7, r0 = tid >> 3;
  const bf16_t *wsrc[4], *xsrc[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    int r = r0 + 32 * i;
    wsrc[i] = W + (size_t)r * a.K + c16 * 8;
    int m = m0 + r;
    if (m >= a.n_rows) m = a.n_rows - 1;            // clamp: computed but never stored
    int src_row = a.row_idx ? a.row_idx[m] : m;
    xsrc[i] = a.hidden + (size_t)src_row * a.K + c16 * 8;
  }
  uint4 wreg[4], xreg[4];
  auto gload = [&](int k0) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      wreg[i] = *reinterpret_cast<const uint4 *>(wsrc[i] + k0);
      xreg[i] = *reinterpret_cast<const uint4 *>(xsrc[i] + k0);
    }
  };
  auto lstore = [&](int buf) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      int off = buf * kTileElems + (r0 + 32 * i) * kStride + c16 * 8;
      *reinterpret_cast<uint4 *>(Ws + off) = wreg[i];
      *reinterpret_cast<uint4 *>(Xs + off) = xreg[i];
    }
  };

  f32x16 acc[4];
#pragma unroll
  for (int b = 0; b < 4; ++b)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[b][r] = 0.f;

  const int frag_row = lane & 31, frag_k = (lane >> 5) * 8;
  const int KT = a.K / kBK;
  gload(0);
  lstore(0);
  __syncthreads();
  for (int kt = 0; kt < KT; ++kt) {
    const int buf = kt & 1;
    if (kt + 1 < KT) gload((kt + 1) * kBK);
    const bf16_t *wb = Ws + buf * kTileElems + frag_row * kStride + frag_k;
    const bf16_t *xb = Xs + buf * kTileElems + (wave * 32 + frag_row) * kStride + frag_k;
#pragma unroll
    for (int ks = 0; ks < kBK / 16; ++ks) {
      bf16x8 xf = *reinterpret_cast<const bf16x8 *>(xb + ks * 16);
#pragma unroll
      for (int b = 0; b < 4; ++b) {
        bf16x8 wf = *reinterpret_cast<const bf16x8 *>(wb + b * 32 * kStride + ks * 16);
        acc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf, xf, acc[b], 0, 0, 0);
      }
    }
    if (kt + 1 < KT) lstore(buf ^ 1);
    __syncthreads();
  }

  // ---- epilogue: bias, RoPE, one rounding, store -------------------------------------------
  // accumulator block b, register r of this lane: feature f = 32 b + 8 (r/4) + 4 (lane/32) + r%4,
  // token = wave*32 + lane%32
  const int tok = m0 + wave * 32 + (lane & 31);
  if (tok >= a.n_rows) return;
  const int fq = (lane >> 5) * 4;
  const bf16_t *bias = a.bias[which];
  if (bias) {
#pragma unroll
    for (int b = 0; b < 4; ++b)
#pragma unroll
      for (int r = 0; r < 16; ++r)
        acc[b][r] += a3_bf2f(bias[head * kHeadDim + 32 * b + 8 * (r >> 2) + fq + (r & 3)]);
  }
  if (which != 2) {
    const int src_row = a.row_idx ? a.row_idx[tok] : tok;
    const float2 *cs = a.pos_cs + (size_t)a.tok_pos[src_row] * (kHeadDim / 2);
    if (a.rope_layout == A3_ROPE_INTERLEAVED) {
#pragma unroll
      for (int b = 0; b < 4; ++b)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int f = 32 * b + 8 * q + fq;                 // first of 4 consecutive features
          const float4 t = *reinterpret_cast<const float4 *>(cs + (f >> 1));   // pairs f/2 and f/2+1
          float x0 = acc[b][4 * q], x1 = acc[b][4 * q + 1], x2 = acc[b][4 * q + 2], x3 = acc[b][4 * q + 3];
          acc[b][4 * q] = x0 * t.x - x1 * t.y;
          acc[b][4 * q + 1] = x0 * t.y + x1 * t.x;
          acc[b][4 * q + 2] = x2 * t.z - x3 * t.w;
          acc[b][4 * q + 3] = x2 * t.w + x3 * t.z;
        }
    } else {
#pragma unroll
      for (int b = 0; b < 2; ++b)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int p = 32 * b + 8 * (r >> 2) + fq + (r & 3);   // pair index = feature in the first half
          const float2 t = cs[p];
          float xa = acc[b][r], xb2 = acc[b + 2][r];
          acc[b][r] = xa * t.x - xb2 * t.y;
          acc[b + 2][r] = xa * t.y + xb2 * t.x;
        }
    }
  }
  bf16_t *orow = out + ((size_t)tok * heads_out + head) * kHeadDim;
#pragma unroll
  for (int b = 0; b < 4; ++b)
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      bf16x4 v;
      v[0] = a3_f2bf(acc[b][4 * q]);
      v[1] = a3_f2bf(acc[b][4 * q + 1]);
      v[2] = a3_f2bf(acc[b][4 * q + 2]);
      v[3] = a3_f2bf(acc[b][4 * q + 3]);
      *reinterpret_cast<bf16x4 *>(orow + 32 * b + 8 * q + fq) = v;
    }
}

// ---------------------------------------------------------------------------------------
// fp32 kernel: 16 listed rows x one head per workgroup
// ---------------------------------------------------------------------------------------
constexpr int kF32Rows = 16;
constexpr int kF32BK = 32;

struct proj_args_f32 {
  const float *hidden;
  const int *row_idx;
  int n_rows;
  const float *w[3];
  const float *bias[3];
  float *out[3];
  const int *tok_pos;
  const float2 *pos_cs;
  int K, Hq, Hkv, d, rope_layout;
};

__global__ void __launch_bounds__(256)
proj_f32_kernel(proj_args_f32 a) {
  __shared__ float Xs[kF32Rows][kF32BK + 1];
  __shared__ float Wt[128][kF32BK + 1];
  __shared__ float Ys[kF32Rows][128];

  int head = blockIdx.x, which = 0, heads_out = a.Hq;
  if (head >= a.Hq) { head -= a.Hq; which = 1; heads_out = a.Hkv; }
  if (which == 1 && head >= a.Hkv) { head -= a.Hkv; which = 2; }
  float *__restrict__ out = a.out[which];
  if (out == nullptr) return;
  const int d = a.d;
  const float *__restrict__ W = a.w[which] + (size_t)head * d * a.K;
  const int m0 = blockIdx.y * kF32Rows;
  const int tid = threadIdx.x;
  const int ty = tid >> 4, tx = tid & 15;          // token ty, features tx + 16 f
  const int nf = d / 16;

  float acc[8];
#pragma unroll
  for (int f = 0; f < 8; ++f) acc[f] = 0.f;

  for (int k0 = 0; k0 < a.K; k0 += kF32BK) {
    for (int i = tid; i < kF32Rows * kF32BK; i += 256) {
      int r = i / kF32BK, c = i % kF32BK;
      int m = m0 + r;
      float v = 0.f;
      if (m < a.n_rows) {
        int src = a.row_idx ? a.row_idx[m] : m;
        v = a.hidden[(size_t)src * a.K + k0 + c];
      }
      Xs[r][c] = v;
    }
    for (int i = tid; i < d * kF32BK; i += 256) {
      int r = i / kF32BK, c = i % kF32BK;
      Wt[r][c] = W[(size_t)r * a.K + k0 + c];
    }
    __syncthreads();
    for (int c = 0; c < kF32BK; ++c) {
      float x = Xs[ty][c];
#pragma unroll
      for (int f = 0; f < 8; ++f)
        if (f < nf) acc[f] = fmaf(x, Wt[tx + 16 * f][c], acc[f]);
    }
    __syncthreads();
  }
  const float *bias = a.bias[which];
#pragma unroll
  for (int f = 0; f < 8; ++f)
    if (f < nf) Ys[ty][tx + 16 * f] = acc[f] + (bias ? bias[head * d + tx + 16 * f] : 0.f);
  __syncthreads();

  const int half = d / 2;
  for (int i = tid; i < kF32Rows * half; i += 256) {
    int r = i / half, p = i % half;
    int m = m0 + r;
    if (m >= a.n_rows) continue;
    int ia, ib;
    if (a.rope_layout == A3_ROPE_INTERLEAVED) { ia = 2 * p; ib = 2 * p + 1; } else { ia = p; ib = p + half; }
    float xa = Ys[r][ia], xb = Ys[r][ib];
    float ya = xa, yb = xb;
    if (which != 2) {
      int src = a.row_idx ? a.row_idx[m] : m;
      float2 t = a.pos_cs[(size_t)a.tok_pos[src] * half + p];
      ya = xa * t.x - xb * t.y;
      yb = xa * t.y + xb * t.x;
    }
    float *orow = out + ((size_t)m * heads_out + head) * d;
    orow[ia] = ya;
    orow[ib] = yb;
  }
}

}  // namespace

extern "C" a3_status a3_selected_qkv_proj(const a3_layout *L, const void *hidden, const int *row_idx, int n_rows,
                                          const void *wq, const void *wk, const void *wv, const void *bq,
                                          const void *bk, const void *bv, void *q_out, void *k_out, void *v_out,
                                          void *stream) {
  a3_status s = a3_check_layout(L, "a3_selected_qkv_proj", true);
  if (s != A3_OK) return s;
  A3_REQUIRE(n_rows >= 0 && n_rows <= L->total_tokens, A3_ERR_INVALID_ARG,
             "a3_selected_qkv_proj: n_rows %d outside [0, %d]", n_rows, L->total_tokens);
  if (n_rows == 0 || (!q_out && !k_out && !v_out)) return A3_OK;
  A3_REQUIRE(hidden, A3_ERR_INVALID_ARG, "a3_selected_qkv_proj: hidden is NULL");
  A3_REQUIRE((!q_out || wq) && (!k_out || wk) && (!v_out || wv), A3_ERR_INVALID_ARG,
             "a3_selected_qkv_proj: an output is requested without its weight");
  const void *ptrs[] = {hidden, wq, wk, wv, bq, bk, bv, q_out, k_out, v_out};
  for (const void *p : ptrs)
    A3_REQUIRE(a3_aligned16(p), A3_ERR_INVALID_ARG, "a3_selected_qkv_proj: tensors must be 16-byte aligned");
  hipStream_t st = (hipStream_t)stream;
  const int n_heads_total = L->n_q_heads + 2 * L->n_kv_heads;
  if (L->dtype == A3_BF16) {
    A3_REQUIRE(L->hidden % kBK == 0, A3_ERR_UNSUPPORTED, "a3_selected_qkv_proj: bf16 needs hidden %% 64 == 0, got %d",
               L->hidden);
    static bool attr_done = false;
    if (!attr_done) {
      hipError_t e = hipFuncSetAttribute((const void *)proj_bf16_kernel, hipFuncAttributeMaxDynamicSharedMemorySize,
                                         (int)kProjLds);
      if (e != hipSuccess) return a3_fail(A3_ERR_HIP, "a3_selected_qkv_proj: %s", hipGetErrorString(e));
      attr_done = true;
    }
    proj_args a;
    a.hidden = (const bf16_t *)hidden; a.row_idx = row_idx; a.n_rows = n_rows;
    a.w[0] = (const bf16_t *)wq; a.w[1] = (const bf16_t *)wk; a.w[2] = (const bf16_t *)wv;
    a.bias[0] = (const bf16_t *)bq; a.bias[1] = (const bf16_t *)bk; a.bias[2] = (const bf16_t *)bv;
    a.out[0] = (bf16_t *)q_out; a.out[1] = (bf16_t *)k_out; a.out[2] = (bf16_t *)v_out;
    a.tok_pos = L->tok_pos; a.pos_cs = (const float2 *)L->rope_pos_cs;
    a.K = L->hidden; a.Hq = L->n_q_heads; a.Hkv = L->n_kv_heads; a.rope_layout = L->rope_layout;
    dim3 grid(n_heads_total, (n_rows + kTokTile - 1) / kTokTile);
    hipLaunchKernelGGL(proj_bf16_kernel, grid, dim3(kThreads), kProjLds, st, a);
  } else {
    proj_args_f32 a;
    a.hidden = (const float *)hidden; a.row_idx = row_idx; a.n_rows = n_rows;
    a.w[0] = (const float *)wq; a.w[1] = (const float *)wk; a.w[2] = (const float *)wv;
    a.bias[0] = (const float *)bq; a.bias[1] = (const float *)bk; a.bias[2] = (const float *)bv;
    a.out[0] = (float *)q_out; a.out[1] = (float *)k_out; a.out[2] = (float *)v_out;
    a.tok_pos = L->tok_pos; a.pos_cs = (const float2 *)L->rope_pos_cs;
    a.K = L->hidden; a.Hq = L->n_q_heads; a.Hkv = L->n_kv_heads; a.d = L->head_dim; a.rope_layout = L->rope_layout;
    dim3 grid(n_heads_total, (n_rows + kF32Rows - 1) / kF32Rows);
    hipLaunchKernelGGL(proj_f32_kernel, grid, dim3(256), 0, st, a);
  }
  A3_CHECK_LAUNCH("a3_selected_qkv_proj");
  return A3_OK;
}
