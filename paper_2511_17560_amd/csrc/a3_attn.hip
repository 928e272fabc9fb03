// Step 4 (attention part) of the A^3 fusion path: Eq. 4 and the last line of Eq. 5.
//
//   O[i, hq] = softmax( q[i, hq] . K'[u, hq/G] * scale ) V[u, hq/G]   over rows u <= act_idx[i] of the request
//
// The query rows are a sparse, ascending subset of the prompt (the selected tokens and the
// question), each with its own causal length.  bf16 path:
//   plan kernel   one workgroup: counts active rows per request and writes tile descriptors
//                 (request, first row, number of visible keys of the tile's last row)
//   main kernel   flash attention on the matrix cores.  The G query heads that share a KV head
//                 are packed with the active rows into one row space m = row*G + head, so a K/V
//                 tile is loaded once per group.  Everything is computed transposed:
//                     S^T[key][m] = K Q^T          (A = K fragment from LDS, B = Q fragment in registers)
//                     O^T[d][m]  += V^T P^T        (A = V^T fragment from LDS, B = P^T from the S^T accumulators)
//                 In this orientation a lane owns ONE query row m: max, sum and rescale are lane-local,
//                 and 8 consecutive S^T accumulators are exactly one B operand of the second product.
//                 V is transposed on its way into LDS (4 keys x 8 dims per lane, register transpose)
//                 with key bits 2 and 3 swapped so that the A operand is a single 16-byte LDS read.
// fp32 path: one workgroup per (active row, head), plain FMA (correctness configuration).
#include "a3_internal.h"

namespace {

constexpr float kLog2e = 1.4426950408889634f;
constexpr int kD = 128;
constexpr int kTM = 128;            // packed (row, head) pairs per workgroup: 4 waves x 32
constexpr int kTK = 64;             // keys per tile
constexpr int kKStride = kD + 8;    // K tile  [key][d]   row stride in elements (272 B)
constexpr int kVStride = kTK + 8;   // V^T tile [d][key]  row stride in elements (144 B)

struct attn_plan {
  int *cnt;          // [n_req]   active rows per request
  int *a_lo;         // [n_req+1] first active row of each request
  int *tile_start;   // [n_req+1] first tile of each request
  int4 *desc;        // [max_tiles] (request, first m of the tile, visible keys of its last row, rows*G of the request)
  int *n_tiles;      // [1]
};

__global__ void __launch_bounds__(1024)
attn_plan_kernel(attn_plan p, const int *__restrict__ act_idx, int n_act, const int *__restrict__ tok_req,
                 const int *__restrict__ seg_start, int n_req, int G, int max_tiles) {
  const int tid = threadIdx.x;
  for (int r = tid; r < n_req; r += 1024) p.cnt[r] = 0;
  __syncthreads();
  for (int a = tid; a < n_act; a += 1024) atomicAdd(&p.cnt[tok_req[act_idx[a]]], 1);
  __syncthreads();
  if (tid == 0) {
    int a = 0, t = 0;
    for (int r = 0; r < n_req; ++r) {
      p.a_lo[r] = a;
      p.tile_start[r] = t;
      a += p.cnt[r];
      t += (p.cnt[r] * G + kTM - 1) / kTM;
    }
    p.a_lo[n_req] = a;
    p.tile_start[n_req] = t;
    *p.n_tiles = t < max_tiles ? t : max_tiles;
  }
  __syncthreads();
  for (int r = 0; r < n_req; ++r) {
    const int t0 = p.tile_start[r], nt = p.tile_start[r + 1] - t0;
    const int a0 = p.a_lo[r], nr = p.cnt[r];
    for (int j = tid; j < nt; j += 1024) {
      if (t0 + j >= max_tiles) break;
      int last = ((j + 1) * kTM - 1) / G;
      if (last > nr - 1) last = nr - 1;
      int kv = act_idx[a0 + last] - seg_start[r] + 1;
      p.desc[t0 + j] = make_int4(r, j * kTM, kv, nr * G);
    }
  }
}

struct attn_args {
  const void *q, *k, *v;
  void *out;
  const int *act_idx;
  const int *seg_start;
  const int *tok_req;
  attn_plan plan;
  int n_act, Hq, Hkv, d;
  float scale2;
};

__device__ __forceinline__ uint32_t pack_lo(uint32_t a, uint32_t b) { return (a & 0xffffu) | (b << 16); }
__device__ __forceinline__ uint32_t pack_hi(uint32_t a, uint32_t b) { return (a >> 16) | (b & 0xffff0000u); }

__global__ void __launch_bounds__(256)
attn_bf16_kernel(attn_args a) {
  __shared__ __align__(16) bf16_t Ks[kTK * kKStride];
  __shared__ __align__(16) bf16_t Vt[kD * kVStride];

  const int n_tiles = *a.plan.n_tiles;
  const int g = blockIdx.x % a.Hkv;
  const int rank = blockIdx.x / a.Hkv;
  if (rank >= n_tiles) return;
  const int4 desc = a.plan.desc[n_tiles - 1 - rank];      // later tiles see more keys: start them first
  const int r = desc.x, m0 = desc.y, kv_len = desc.z, m_end = desc.w;
  const int G = a.Hq / a.Hkv;
  const int a0 = a.plan.a_lo[r];
  const int base = a.seg_start[r];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, lhi = lane >> 5;

  const bf16_t *__restrict__ Q = (const bf16_t *)a.q;
  const bf16_t *__restrict__ K = (const bf16_t *)a.k;
  const bf16_t *__restrict__ V = (const bf16_t *)a.v;

  // this lane's query row
  const int m = m0 + wave * 32 + l32;
  const bool valid = m < m_end;
  const int mc = valid ? m : m_end - 1;
  const int arow = a0 + mc / G, hq = g * G + mc % G;
  const int limit = a.act_idx[arow] - base;              // last visible key (request-relative)

  bf16x8 qf[kD / 16];
  {
    const bf16_t *qp = Q + ((size_t)arow * a.Hq + hq) * kD + lhi * 8;
#pragma unroll
    for (int ks = 0; ks < kD / 16; ++ks) qf[ks] = *reinterpret_cast<const bf16x8 *>(qp + ks * 16);
  }

  f32x16 o[4];
#pragma unroll
  for (int b = 0; b < 4; ++b)
#pragma unroll
    for (int x = 0; x < 16; ++x) o[b][x] = 0.f;
  float row_max = -INFINITY, row_sum = 0.f;

  // staging roles: K tile: 16 lanes per 256-byte row; V tile: lane = (4 keys, 8 dims)
  const int vkg = tid >> 4, vc = tid & 15;                 // keys 4*vkg.., dims 8*vc..
  const int vpos = ((4 * vkg) & ~12) | (((4 * vkg) & 4) << 1) | (((4 * vkg) & 8) >> 1);   // swap key bits 2 and 3

  for (int k0 = 0; k0 < kv_len; k0 += kTK) {
    __syncthreads();                                       // previous tile consumed
    for (int i = tid; i < kTK * 16; i += 256) {
      int kr = i >> 4, c = i & 15;
      int row = k0 + kr;
      if (row > kv_len - 1) row = kv_len - 1;              // stay inside the visible range; masked below
      uint4 v = *reinterpret_cast<const uint4 *>(K + ((size_t)(base + row) * a.Hkv + g) * kD + c * 8);
      *reinterpret_cast<uint4 *>(Ks + kr * kKStride + c * 8) = v;
    }
    {
      uint4 rows[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        int row = k0 + 4 * vkg + i;
        if (row > kv_len - 1) row = kv_len - 1;
        rows[i] = *reinterpret_cast<const uint4 *>(V + ((size_t)(base + row) * a.Hkv + g) * kD + vc * 8);
      }
      const uint32_t *r0 = reinterpret_cast<const uint32_t *>(&rows[0]);
      const uint32_t *r1 = reinterpret_cast<const uint32_t *>(&rows[1]);
      const uint32_t *r2 = reinterpret_cast<const uint32_t *>(&rows[2]);
      const uint32_t *r3 = reinterpret_cast<const uint32_t *>(&rows[3]);
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        uint2 even = make_uint2(pack_lo(r0[w], r1[w]), pack_lo(r2[w], r3[w]));   // dim 8vc+2w,   keys 0..3
        uint2 odd = make_uint2(pack_hi(r0[w], r1[w]), pack_hi(r2[w], r3[w]));    // dim 8vc+2w+1, keys 0..3
        *reinterpret_cast<uint2 *>(Vt + (8 * vc + 2 * w) * kVStride + vpos) = even;
        *reinterpret_cast<uint2 *>(Vt + (8 * vc + 2 * w + 1) * kVStride + vpos) = odd;
      }
    }
    __syncthreads();

    // ---- S^T = K Q^T : two 32-key blocks ------------------------------------------------
    f32x16 st[2];
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int x = 0; x < 16; ++x) st[b][x] = 0.f;
#pragma unroll
    for (int ks = 0; ks < kD / 16; ++ks)
#pragma unroll
      for (int b = 0; b < 2; ++b) {
        bf16x8 kf = *reinterpret_cast<const bf16x8 *>(Ks + (b * 32 + l32) * kKStride + ks * 16 + lhi * 8);
        st[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[ks], st[b], 0, 0, 0);
      }

    // ---- online softmax for this lane's row ------------------------------------------------
    // accumulator x of block b: key k0 + 32 b + 8 (x/4) + 4 lhi + x%4
    float mx = -INFINITY;
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int x = 0; x < 16; ++x) {
        int key = k0 + 32 * b + 8 * (x >> 2) + 4 * lhi + (x & 3);
        float s = key <= limit ? st[b][x] * a.scale2 : -INFINITY;
        st[b][x] = s;
        mx = fmaxf(mx, s);
      }
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
    const float new_max = fmaxf(row_max, mx);              // finite: key 0 is visible to every row
    const float alpha = exp2f(row_max - new_max);
    row_max = new_max;
    float psum = 0.f;
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int x = 0; x < 16; ++x) {
        float p = exp2f(st[b][x] - new_max);
        st[b][x] = p;
        psum += p;
      }
    row_sum = row_sum * alpha + psum;                      // per lane half; halves are added at the end
#pragma unroll
    for (int b = 0; b < 4; ++b)
#pragma unroll
      for (int x = 0; x < 16; ++x) o[b][x] *= alpha;

    // ---- O^T += V^T P^T ------------------------------------------------------------------------
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int s2 = 0; s2 < 2; ++s2) {
        bf16x8 pf;
#pragma unroll
        for (int e = 0; e < 8; ++e) pf[e] = a3_f2bf(st[b][8 * s2 + e]);
#pragma unroll
        for (int db = 0; db < 4; ++db) {
          bf16x8 vf = *reinterpret_cast<const bf16x8 *>(Vt + (db * 32 + l32) * kVStride + 32 * b + 16 * s2 + 8 * lhi);
          o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf, o[db], 0, 0, 0);
        }
      }
  }

  row_sum += __shfl_xor(row_sum, 32, 64);
  if (!valid) return;
  const float inv = 1.0f / row_sum;
  bf16_t *orow = (bf16_t *)a.out + ((size_t)arow * a.Hq + hq) * kD;
  // accumulator x of block db: dim 32 db + 8 (x/4) + 4 lhi + x%4
#pragma unroll
  for (int db = 0; db < 4; ++db)
#pragma unroll
    for (int q4 = 0; q4 < 4; ++q4) {
      bf16x4 v;
#pragma unroll
      for (int e = 0; e < 4; ++e) v[e] = a3_f2bf(o[db][4 * q4 + e] * inv);
      *reinterpret_cast<bf16x4 *>(orow + 32 * db + 8 * q4 + 4 * lhi) = v;
    }
}

// ---------------------------------------------------------------------------------------
// fp32: one workgroup per (active row, query head)
// ---------------------------------------------------------------------------------------
__global__ void __launch_bounds__(256)
attn_f32_kernel(attn_args a) {
  __shared__ float qs[128];
  __shared__ float P[256];
  __shared__ float red[256];

  const int arow = blockIdx.x, hq = blockIdx.y;
  const int tid = threadIdx.x;
  const int d = a.d, G = a.Hq / a.Hkv, g = hq / G;
  const int t = a.act_idx[arow];
  const int base = a.seg_start[a.tok_req[t]];
  const int nk = t - base + 1;
  const float *__restrict__ Q = (const float *)a.q;
  const float *__restrict__ K = (const float *)a.k;
  const float *__restrict__ V = (const float *)a.v;
  for (int c = tid; c < d; c += 256) qs[c] = Q[((size_t)arow * a.Hq + hq) * d + c] * a.scale2;
  __syncthreads();

  const int col = tid % d, slice = tid / d, n_slices = 256 / d;   // d = 64: 4 key slices, d = 128: 2
  float o_acc = 0.f, row_max = -INFINITY, row_sum = 0.f;
  for (int k0 = 0; k0 < nk; k0 += 256) {
    const int key = k0 + tid;
    float l = -INFINITY;
    if (key < nk) {
      const float *kp = K + ((size_t)(base + key) * a.Hkv + g) * d;
      float dot = 0.f;
      for (int c = 0; c < d; ++c) dot = fmaf(qs[c], kp[c], dot);
      l = dot;
    }
    red[tid] = l;
    __syncthreads();
    for (int off = 128; off > 0; off >>= 1) {
      if (tid < off) red[tid] = fmaxf(red[tid], red[tid + off]);
      __syncthreads();
    }
    const float new_max = fmaxf(row_max, red[0]);
    __syncthreads();
    const float p = exp2f(l - new_max);
    P[tid] = p;
    red[tid] = p;
    __syncthreads();
    for (int off = 128; off > 0; off >>= 1) {
      if (tid < off) red[tid] += red[tid + off];
      __syncthreads();
    }
    const float alpha = exp2f(row_max - new_max);
    row_sum = row_sum * alpha + red[0];
    row_max = new_max;
    float part = 0.f;
    const int kend = min(256, nk - k0);
    for (int kk = slice; kk < kend; kk += n_slices)
      part = fmaf(P[kk], V[((size_t)(base + k0 + kk) * a.Hkv + g) * d + col], part);
    o_acc = o_acc * alpha + part;
    __syncthreads();
  }
  red[tid] = o_acc;
  __syncthreads();
  if (tid < d) {
    float sum = 0.f;
    for (int s = 0; s < n_slices; ++s) sum += red[s * d + tid];
    ((float *)a.out)[((size_t)arow * a.Hq + hq) * d + tid] = sum / row_sum;
  }
}

int attn_max_tiles(const a3_layout *L, int n_act) {
  const int G = L->n_q_heads / L->n_kv_heads;
  return (int)(((long long)n_act * G + kTM - 1) / kTM) + L->n_req;
}

}  // namespace

size_t a3_attn_ws_bytes(const a3_layout *L, int max_active_rows) {
  size_t per_req = a3_align_up((size_t)(L->n_req + 1) * sizeof(int), 256);
  return 3 * per_req + a3_align_up((size_t)attn_max_tiles(L, max_active_rows) * sizeof(int4), 256) + 512;
}

extern "C" a3_status a3_fused_attention(const a3_layout *L, const void *q_act, const int *act_idx, int n_act,
                                        const void *k_fused, const void *v_fused, void *out, void *ws,
                                        size_t ws_bytes, void *stream) {
  a3_status s = a3_check_layout(L, "a3_fused_attention", true);
  if (s != A3_OK) return s;
  A3_REQUIRE(n_act >= 0 && n_act <= L->total_tokens, A3_ERR_INVALID_ARG,
             "a3_fused_attention: n_act %d outside [0, %d]", n_act, L->total_tokens);
  if (n_act == 0) return A3_OK;
  A3_REQUIRE(q_act && act_idx && k_fused && v_fused && out, A3_ERR_INVALID_ARG, "a3_fused_attention: NULL argument");
  A3_REQUIRE(a3_aligned16(q_act) && a3_aligned16(k_fused) && a3_aligned16(v_fused) && a3_aligned16(out),
             A3_ERR_INVALID_ARG, "a3_fused_attention: tensors must be 16-byte aligned");
  hipStream_t st = (hipStream_t)stream;
  attn_args a;
  a.q = q_act; a.k = k_fused; a.v = v_fused; a.out = out;
  a.act_idx = act_idx; a.seg_start = L->seg_start; a.tok_req = L->tok_req;
  a.n_act = n_act; a.Hq = L->n_q_heads; a.Hkv = L->n_kv_heads; a.d = L->head_dim;
  a.scale2 = a3_scale_of(L) * kLog2e;
  a.plan = attn_plan{nullptr, nullptr, nullptr, nullptr, nullptr};
  if (L->dtype == A3_BF16) {
    A3_REQUIRE(ws != nullptr, A3_ERR_WORKSPACE, "a3_fused_attention: workspace is NULL");
    A3_REQUIRE(ws_bytes >= a3_attn_ws_bytes(L, n_act), A3_ERR_WORKSPACE,
               "a3_fused_attention: workspace %zu bytes, need %zu", ws_bytes, a3_attn_ws_bytes(L, n_act));
    const int max_tiles = attn_max_tiles(L, n_act);
    a3_ws_cursor cur(ws, ws_bytes);
    a.plan.cnt = (int *)cur.take((size_t)(L->n_req + 1) * sizeof(int));
    a.plan.a_lo = (int *)cur.take((size_t)(L->n_req + 1) * sizeof(int));
    a.plan.tile_start = (int *)cur.take((size_t)(L->n_req + 1) * sizeof(int));
    a.plan.desc = (int4 *)cur.take((size_t)max_tiles * sizeof(int4));
    a.plan.n_tiles = (int *)cur.take(sizeof(int));
    hipLaunchKernelGGL(attn_plan_kernel, dim3(1), dim3(1024), 0, st, a.plan, act_idx, n_act, L->tok_req, L->seg_start,
                       L->n_req, L->n_q_heads / L->n_kv_heads, max_tiles);
    hipLaunchKernelGGL(attn_bf16_kernel, dim3((unsigned)max_tiles * L->n_kv_heads), dim3(256), 0, st, a);
  } else {
    hipLaunchKernelGGL(attn_f32_kernel, dim3(n_act, L->n_q_heads), dim3(256), 0, st, a);
  }
  A3_CHECK_LAUNCH("a3_fused_attention");
  return A3_OK;
}
