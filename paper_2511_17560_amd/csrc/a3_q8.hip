// 8-bit form of the precomputed chunk caches (the paper fixes no format; it names loading the caches as the
// method's limitation and cache quantisation as orthogonal).  One packed row of one layer is one record
//     [ K codes: Hkv*d int8 | V codes: Hkv*d int8 | K scales: Hkv float32 | V scales: Hkv float32 ],
// x = code * scale per row and KV head, so that a chunk's rows of both caches are ONE contiguous block and
// reach the GPU in one copy.  Position recovery (Eq. 2) runs on the dequantised keys in the same kernel that
// expands the record: the 8-bit data are read once, the realigned keys and the values written once in the
// storage type.  HBM-bound: 1 byte + 4/d bytes in, 2 (or 4) bytes out per element.
#include "a3_internal.h"

namespace {

constexpr int kBlock = 256;

typedef signed char i8x8 __attribute__((ext_vector_type(8)));

__host__ __device__ inline size_t q8_row_bytes(int n_kv_heads, int head_dim) {
  return (size_t)n_kv_heads * (2 * head_dim + 8);
}

// One lane: 16 coordinates of one (row, head), of the key and of the value.  Interleaved pairing: 16
// consecutive coordinates (8 pairs); half pairing: coordinates 8c .. 8c+7 and the same + d/2 (8 pairs).
template <typename T>
__global__ void __launch_bounds__(kBlock)
expand_q8_kernel(const signed char *__restrict__ rows, T *__restrict__ k_out, T *__restrict__ v_out,
                 const int *__restrict__ tok_chunk, const float2 *__restrict__ chunk_cs, int n_rows, int n_heads,
                 int head_dim, int rope_layout, int rotate) {
  const int per_head = head_dim / 16;
  const long gid = (long)blockIdx.x * kBlock + threadIdx.x;
  if (gid >= (long)n_rows * n_heads * per_head) return;
  const int c = (int)(gid % per_head);
  const long th = gid / per_head;                              // row * n_heads + head
  const int t = (int)(th / n_heads), h = (int)(th % n_heads);
  const int half = head_dim / 2, kd = n_heads * head_dim;
  const bool inter = rope_layout == A3_ROPE_INTERLEAVED;
  const int e0 = inter ? 16 * c : 8 * c, e1 = inter ? 16 * c + 8 : half + 8 * c;   // the two runs of 8
  const signed char *rec = rows + (size_t)t * q8_row_bytes(n_heads, head_dim);
  const float *scales = reinterpret_cast<const float *>(rec + 2 * kd);
  const long obase = th * head_dim;
  typedef T vec8 __attribute__((ext_vector_type(8)));
  if (k_out) {
    const float s = scales[h];
    const i8x8 qa = *reinterpret_cast<const i8x8 *>(rec + h * head_dim + e0);
    const i8x8 qb = *reinterpret_cast<const i8x8 *>(rec + h * head_dim + e1);
    float xa[8], xb[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) { xa[e] = (float)qa[e] * s; xb[e] = (float)qb[e] * s; }
    const int chunk = rotate ? tok_chunk[t] : -1;
    if (chunk >= 0) {
      const float2 *cs = chunk_cs + (size_t)chunk * half;
      if (inter) {
        // pairs (e0 + 2p, e0 + 2p + 1) with pair index (e0 >> 1) + p, and the same for the second run
#pragma unroll
        for (int p = 0; p < 4; ++p) {
          float y0, y1;
          a3_rotate_pair(xa[2 * p], xa[2 * p + 1], cs[(e0 >> 1) + p], y0, y1);
          xa[2 * p] = y0; xa[2 * p + 1] = y1;
          a3_rotate_pair(xb[2 * p], xb[2 * p + 1], cs[(e1 >> 1) + p], y0, y1);
          xb[2 * p] = y0; xb[2 * p + 1] = y1;
        }
      } else {
#pragma unroll
        for (int e = 0; e < 8; ++e) {                          // coordinate e0 + e pairs with e0 + e + d/2
          float y0, y1;
          a3_rotate_pair(xa[e], xb[e], cs[e0 + e], y0, y1);
          xa[e] = y0; xb[e] = y1;
        }
      }
    }
    vec8 ya, yb;
#pragma unroll
    for (int e = 0; e < 8; ++e) { ya[e] = (T)xa[e]; yb[e] = (T)xb[e]; }
    *reinterpret_cast<vec8 *>(k_out + obase + e0) = ya;
    *reinterpret_cast<vec8 *>(k_out + obase + e1) = yb;
  }
  if (v_out) {
    const float s = scales[n_heads + h];
    const i8x8 qa = *reinterpret_cast<const i8x8 *>(rec + kd + h * head_dim + e0);
    const i8x8 qb = *reinterpret_cast<const i8x8 *>(rec + kd + h * head_dim + e1);
    vec8 ya, yb;
#pragma unroll
    for (int e = 0; e < 8; ++e) { ya[e] = (T)((float)qa[e] * s); yb[e] = (T)((float)qb[e] * s); }
    *reinterpret_cast<vec8 *>(v_out + obase + e0) = ya;
    *reinterpret_cast<vec8 *>(v_out + obase + e1) = yb;
  }
}

// The quantiser (run once, when a chunk's caches are produced).  One lane: 16 consecutive coordinates of the
// key and of the value; the head_dim / 16 lanes of a (row, head) are neighbours in a wave and share the maxima.
// The scale is the float32 rounding of max|x| / 127 taken in float64 and the code the float64 quotient rounded
// half to even, so that the integer decision is the same as in a float64 reference.
template <typename T>
__device__ inline void quantize_run(const T *__restrict__ src, signed char *__restrict__ dst, float *scale_out,
                                    int per_head, int c) {
  float v[16];
  typedef T vec8 __attribute__((ext_vector_type(8)));
#pragma unroll
  for (int half = 0; half < 2; ++half) {
    const vec8 in = *reinterpret_cast<const vec8 *>(src + 8 * half);
#pragma unroll
    for (int e = 0; e < 8; ++e) v[8 * half + e] = (float)in[e];
  }
  float amax = 0.f;
#pragma unroll
  for (int e = 0; e < 16; ++e) amax = fmaxf(amax, fabsf(v[e]));
  for (int m = 1; m < per_head; m <<= 1) amax = fmaxf(amax, __shfl_xor(amax, m));
  const float s = (float)((double)amax / 127.0);
  if (c == 0) *scale_out = s;
#pragma unroll
  for (int half = 0; half < 2; ++half) {
    i8x8 q;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      double r = s > 0.f ? rint((double)v[8 * half + e] / (double)s) : 0.0;
      r = fmin(fmax(r, -127.0), 127.0);
      q[e] = (signed char)(int)r;
    }
    *reinterpret_cast<i8x8 *>(dst + 8 * half) = q;
  }
}

template <typename T>
__global__ void __launch_bounds__(kBlock)
quantize_q8_kernel(const T *__restrict__ k, const T *__restrict__ v, signed char *__restrict__ rows, long total,
                   int n_heads, int head_dim) {
  const int per_head = head_dim / 16;
  const long gid = (long)blockIdx.x * kBlock + threadIdx.x;
  if (gid >= total) return;                                    // total is a multiple of per_head: whole groups leave
  const int c = (int)(gid % per_head);
  const long th = gid / per_head;
  const long t = th / n_heads;
  const int h = (int)(th % n_heads), kd = n_heads * head_dim;
  signed char *rec = rows + (size_t)t * q8_row_bytes(n_heads, head_dim);
  float *scales = reinterpret_cast<float *>(rec + 2 * kd);
  quantize_run(k + th * head_dim + 16 * c, rec + h * head_dim + 16 * c, scales + h, per_head, c);
  quantize_run(v + th * head_dim + 16 * c, rec + kd + h * head_dim + 16 * c, scales + n_heads + h, per_head, c);
}

}  // namespace

extern "C" size_t a3_q8_row_bytes(const a3_layout *L) {
  if (a3_check_layout(L, "a3_q8_row_bytes", false) != A3_OK) return 0;
  return q8_row_bytes(L->n_kv_heads, L->head_dim);
}

extern "C" a3_status a3_quantize_q8(const a3_layout *L, const void *k, const void *v, void *cache_q8, void *stream) {
  a3_status s = a3_check_layout(L, "a3_quantize_q8", false);
  if (s != A3_OK) return s;
  A3_REQUIRE(k && v && cache_q8, A3_ERR_INVALID_ARG, "a3_quantize_q8: NULL tensor");
  A3_REQUIRE(a3_aligned16(k) && a3_aligned16(v) && a3_aligned16(cache_q8), A3_ERR_INVALID_ARG,
             "a3_quantize_q8: tensors must be 16-byte aligned");
  const long total = (long)L->total_tokens * L->n_kv_heads * (L->head_dim / 16);
  const dim3 grid((unsigned)((total + kBlock - 1) / kBlock));
  hipStream_t st = (hipStream_t)stream;
  if (L->dtype == A3_BF16)
    hipLaunchKernelGGL(quantize_q8_kernel<bf16_t>, grid, dim3(kBlock), 0, st, (const bf16_t *)k, (const bf16_t *)v,
                       (signed char *)cache_q8, total, L->n_kv_heads, L->head_dim);
  else
    hipLaunchKernelGGL(quantize_q8_kernel<float>, grid, dim3(kBlock), 0, st, (const float *)k, (const float *)v,
                       (signed char *)cache_q8, total, L->n_kv_heads, L->head_dim);
  A3_CHECK_LAUNCH("a3_quantize_q8");
  return A3_OK;
}

extern "C" a3_status a3_rope_realign_q8(const a3_layout *L, const void *cache_q8, void *k_fused, void *v_fused,
                                        void *stream) {
  a3_status s = a3_check_layout(L, "a3_rope_realign_q8", true);
  if (s != A3_OK) return s;
  A3_REQUIRE(cache_q8 && (k_fused || v_fused), A3_ERR_INVALID_ARG, "a3_rope_realign_q8: NULL tensor");
  A3_REQUIRE(a3_aligned16(cache_q8) && a3_aligned16(k_fused) && a3_aligned16(v_fused), A3_ERR_INVALID_ARG,
             "a3_rope_realign_q8: tensors must be 16-byte aligned");
  const long total = (long)L->total_tokens * L->n_kv_heads * (L->head_dim / 16);
  const dim3 grid((unsigned)((total + kBlock - 1) / kBlock));
  hipStream_t st = (hipStream_t)stream;
  const float2 *cs = (const float2 *)L->rope_chunk_cs;
  const int rotate = L->n_chunks > 0;
  if (L->dtype == A3_BF16)
    hipLaunchKernelGGL(expand_q8_kernel<bf16_t>, grid, dim3(kBlock), 0, st, (const signed char *)cache_q8,
                       (bf16_t *)k_fused, (bf16_t *)v_fused, L->tok_chunk, cs, L->total_tokens, L->n_kv_heads,
                       L->head_dim, L->rope_layout, rotate);
  else
    hipLaunchKernelGGL(expand_q8_kernel<float>, grid, dim3(kBlock), 0, st, (const signed char *)cache_q8,
                       (float *)k_fused, (float *)v_fused, L->tok_chunk, cs, L->total_tokens, L->n_kv_heads,
                       L->head_dim, L->rope_layout, rotate);
  A3_CHECK_LAUNCH("a3_rope_realign_q8");
  return A3_OK;
}

// Host blocks of one layer's 8-bit chunk caches (records of a3_q8_row_bytes each, chunk_len[c] of them) into
// their packed rows: one copy per chunk.  Same rules as a3_chunk_cache_load.
extern "C" a3_status a3_chunk_cache_load_q8(const a3_layout *L, const int *chunk_start_host, const int *chunk_len_host,
                                            int n_chunks, const void *const *host_q8, void *cache_q8, void *stream) {
  a3_status s = a3_check_layout(L, "a3_chunk_cache_load_q8", false);
  if (s != A3_OK) return s;
  A3_REQUIRE(n_chunks >= 0, A3_ERR_INVALID_ARG, "a3_chunk_cache_load_q8: n_chunks %d is negative", n_chunks);
  if (n_chunks == 0) return A3_OK;
  A3_REQUIRE(chunk_start_host && chunk_len_host && host_q8 && cache_q8, A3_ERR_INVALID_ARG,
             "a3_chunk_cache_load_q8: NULL argument");
  const size_t row = q8_row_bytes(L->n_kv_heads, L->head_dim);
  for (int c = 0; c < n_chunks; ++c) {
    const int start = chunk_start_host[c], len = chunk_len_host[c];
    A3_REQUIRE(len >= 0 && start >= 0 && (long long)start + len <= L->total_tokens, A3_ERR_INVALID_ARG,
               "a3_chunk_cache_load_q8: chunk %d covers rows [%d, %d) outside [0, %d)", c, start, start + len,
               L->total_tokens);
    A3_REQUIRE(len == 0 || host_q8[c], A3_ERR_INVALID_ARG, "a3_chunk_cache_load_q8: chunk %d has no host block", c);
  }
  hipStream_t st = (hipStream_t)stream;
  for (int c = 0; c < n_chunks; ++c) {
    const size_t len = (size_t)chunk_len_host[c], start = (size_t)chunk_start_host[c];
    if (len == 0) continue;
    hipError_t e = hipMemcpyAsync((char *)cache_q8 + start * row, host_q8[c], len * row, hipMemcpyHostToDevice, st);
    if (e != hipSuccess) return a3_fail(A3_ERR_HIP, "a3_chunk_cache_load_q8: chunk %d: %s", c, hipGetErrorString(e));
  }
  return A3_OK;
}
