// Bandwidth-bound steps of the A^3 fusion path: layout tables, position recovery (Eq. 2)
// and the cache update (Eq. 5, middle lines).  Plain coalesced 16-byte streaming; one
// vector per lane, several vectors in flight per lane.
#include "a3_internal.h"

namespace {

constexpr int kBlock = 256;

// ---------------------------------------------------------------------------------------
// layout tables
// ---------------------------------------------------------------------------------------

// largest i in [0, n) with a[i] <= x, or -1
__device__ __forceinline__ int upper_index(const int *__restrict__ a, int n, int x) {
  int lo = 0, hi = n;   // invariant: a[lo-1] <= x < a[hi]
  while (lo < hi) {
    int mid = (lo + hi) >> 1;
    if (a[mid] <= x) lo = mid + 1; else hi = mid;
  }
  return lo - 1;
}

__global__ void __launch_bounds__(kBlock)
prepare_tokens_kernel(const int *__restrict__ seg_start, int n_req, const int *__restrict__ chunk_start,
                      const int *__restrict__ chunk_len, int n_chunks, int T, int *__restrict__ tok_pos,
                      int *__restrict__ tok_req, int *__restrict__ tok_chunk, const int *__restrict__ q_len,
                      int *__restrict__ q_start) {
  int t = blockIdx.x * kBlock + threadIdx.x;
  if (t == 0) {                          // n_req is small: a serial prefix sum is enough
    int run = 0;
    for (int r = 0; r < n_req; ++r) { q_start[r] = run; run += q_len[r]; }
    q_start[n_req] = run;
  }
  if (t >= T) return;
  int r = upper_index(seg_start, n_req, t);
  if (r < 0) r = 0;
  tok_req[t] = r;
  tok_pos[t] = t - seg_start[r];
  int c = n_chunks > 0 ? upper_index(chunk_start, n_chunks, t) : -1;
  if (c >= 0 && t >= chunk_start[c] + chunk_len[c]) c = -1;
  tok_chunk[t] = c;
}

// (cos, sin) of m * theta_i with theta_i = base^(-2i/d); angle formed and evaluated in double.
__global__ void __launch_bounds__(kBlock)
prepare_rope_kernel(const int *__restrict__ chunk_delta, int n_chunks, int n_pos, int half, double base,
                    float2 *__restrict__ chunk_cs, float2 *__restrict__ pos_cs) {
  long long gid = (long long)blockIdx.x * kBlock + threadIdx.x;
  long long total = (long long)(n_chunks + n_pos) * half;
  if (gid >= total) return;
  int row = (int)(gid / half), i = (int)(gid % half);
  double m = row < n_chunks ? (double)chunk_delta[row] : (double)(row - n_chunks);
  double theta = pow(base, -(double)i / (double)half);      // -2i/d with d = 2*half
  double s, c;
  sincos(m * theta, &s, &c);
  float2 v = make_float2((float)c, (float)s);
  if (row < n_chunks) chunk_cs[(size_t)row * half + i] = v;
  else pos_cs[(size_t)(row - n_chunks) * half + i] = v;
}

// ---------------------------------------------------------------------------------------
// step 1: position recovery
// ---------------------------------------------------------------------------------------

template <typename T> struct vec16 { uint4 raw; };

template <typename T, int N>
__device__ __forceinline__ void unpack(const uint4 &raw, float (&f)[N]) {
  const T *p = reinterpret_cast<const T *>(&raw);
#pragma unroll
  for (int i = 0; i < N; ++i) f[i] = a3_elem<T>::load(p + i);
}
template <typename T, int N>
__device__ __forceinline__ uint4 pack(const float (&f)[N]) {
  uint4 raw;
  T *p = reinterpret_cast<T *>(&raw);
#pragma unroll
  for (int i = 0; i < N; ++i) a3_elem<T>::store(p + i, f[i]);
  return raw;
}

// One work item rotates VEC/2 pairs (interleaved: one 16-byte vector; half layout: one vector
// from each half of the head).  items_per_row = work items per token over all KV heads.
template <typename T, int LAYOUT, int UNROLL>
__global__ void __launch_bounds__(kBlock)
rope_realign_kernel(const T *k_cat, T *k_fused,   /* may alias: each item reads its own elements first */
                    const int *__restrict__ tok_chunk,
                    const float2 *__restrict__ chunk_cs, int T_rows, int head_dim, int row_elems,
                    int items_per_row, int items_shift /* log2(items_per_row) or -1 */) {
  constexpr int VEC = a3_elem<T>::kVec;
  const int half = head_dim >> 1;
  // 32-bit indexing (the host checks T_rows * items_per_row < 2^31): 64-bit division is emulated
  const unsigned total = (unsigned)T_rows * (unsigned)items_per_row;
  const unsigned base = (blockIdx.x * UNROLL) * kBlock + threadIdx.x;

  uint4 va[UNROLL], vb[UNROLL];
  int chunk[UNROLL];
  size_t offa[UNROLL], offb[UNROLL];
  int pair0[UNROLL];
#pragma unroll
  for (int u = 0; u < UNROLL; ++u) {
    const unsigned gid = base + u * kBlock;
    chunk[u] = -1;
    if (gid < total) {
      const int t = items_shift >= 0 ? (int)(gid >> items_shift) : (int)(gid / (unsigned)items_per_row);
      const int j = (int)(gid - (unsigned)t * (unsigned)items_per_row);
      chunk[u] = tok_chunk[t];
      if (LAYOUT == A3_ROPE_INTERLEAVED) {
        int e = j * VEC;                       // element inside the row
        offa[u] = (size_t)t * row_elems + e;
        pair0[u] = (e % head_dim) >> 1;
        if (chunk[u] >= 0) va[u] = a3_nt_load(k_cat + offa[u]);
      } else {
        int per_head = half / VEC;             // work items per head
        int h = j / per_head, e = (j % per_head) * VEC;
        offa[u] = (size_t)t * row_elems + (size_t)h * head_dim + e;
        offb[u] = offa[u] + half;
        pair0[u] = e;
        if (chunk[u] >= 0) {
          va[u] = a3_nt_load(k_cat + offa[u]);
          vb[u] = a3_nt_load(k_cat + offb[u]);
        }
      }
    }
  }
#pragma unroll
  for (int u = 0; u < UNROLL; ++u) {
    if (chunk[u] < 0) continue;
    const float2 *cs = chunk_cs + (size_t)chunk[u] * half + pair0[u];
    if (LAYOUT == A3_ROPE_INTERLEAVED) {
      float x[VEC], y[VEC];
      unpack<T, VEC>(va[u], x);
#pragma unroll
      for (int p = 0; p < VEC / 2; ++p) {
        a3_rotate_pair(x[2 * p], x[2 * p + 1], cs[p], y[2 * p], y[2 * p + 1]);
      }
      a3_nt_store(k_fused + offa[u], pack<T, VEC>(y));
    } else {
      float xa[VEC], xb[VEC], ya[VEC], yb[VEC];
      unpack<T, VEC>(va[u], xa);
      unpack<T, VEC>(vb[u], xb);
#pragma unroll
      for (int p = 0; p < VEC; ++p) {
        a3_rotate_pair(xa[p], xb[p], cs[p], ya[p], yb[p]);
      }
      a3_nt_store(k_fused + offa[u], pack<T, VEC>(ya));
      a3_nt_store(k_fused + offb[u], pack<T, VEC>(yb));
    }
  }
}

// ---------------------------------------------------------------------------------------
// step 5: cache update
// ---------------------------------------------------------------------------------------

template <int UNROLL>
__global__ void __launch_bounds__(kBlock)
kv_scatter_kernel(const uint4 *__restrict__ k_new, const uint4 *__restrict__ v_new, const int *__restrict__ row_idx,
                  int n_rows, int vec_per_row, int vec_shift /* log2(vec_per_row) or -1 */,
                  uint4 *__restrict__ k_fused, uint4 *__restrict__ v_fused) {
  const uint4 *src = blockIdx.y == 0 ? k_new : v_new;
  uint4 *dst = blockIdx.y == 0 ? k_fused : v_fused;
  const unsigned total = (unsigned)n_rows * (unsigned)vec_per_row;     // < 2^31, checked on the host
  const unsigned base = (blockIdx.x * UNROLL) * kBlock + threadIdx.x;
  uint4 v[UNROLL];
  long long dsto[UNROLL];
#pragma unroll
  for (int u = 0; u < UNROLL; ++u) {
    const unsigned gid = base + u * kBlock;
    dsto[u] = -1;
    if (gid < total) {
      const int i = vec_shift >= 0 ? (int)(gid >> vec_shift) : (int)(gid / (unsigned)vec_per_row);
      const int j = (int)(gid - (unsigned)i * (unsigned)vec_per_row);
      v[u] = src[gid];
      dsto[u] = (long long)row_idx[i] * vec_per_row + j;
    }
  }
#pragma unroll
  for (int u = 0; u < UNROLL; ++u)
    if (dsto[u] >= 0) dst[dsto[u]] = v[u];
}

// ---------------------------------------------------------------------------------------
// active rows = selected rows then question rows, per request
// ---------------------------------------------------------------------------------------
__global__ void __launch_bounds__(kBlock)
active_rows_kernel(const int *__restrict__ sel_idx, const int *__restrict__ sel_start,
                   const int *__restrict__ q_start, const int *__restrict__ seg_start,
                   const int *__restrict__ ctx_len, int n_req, int n_act, int *__restrict__ act_idx) {
  int i = blockIdx.x * kBlock + threadIdx.x;
  if (i >= n_act) return;
  // largest r with sel_start[r] + q_start[r] <= i
  int lo = 0, hi = n_req;
  while (lo < hi) {
    int mid = (lo + hi) >> 1;
    if (sel_start[mid] + q_start[mid] <= i) lo = mid + 1; else hi = mid;
  }
  int r = lo - 1;
  if (r < 0) r = 0;
  int j = i - (sel_start[r] + q_start[r]);
  int k = sel_start[r + 1] - sel_start[r];
  act_idx[i] = j < k ? sel_idx[sel_start[r] + j] : seg_start[r] + ctx_len[r] + (j - k);
}

// ---------------------------------------------------------------------------------------
// alternative producers of the recompute list
// ---------------------------------------------------------------------------------------
// scores[t] = |v_true[t] - v_cat[t]|^2 over all KV heads for context rows, -inf for question rows.
// One wave per row, 16 bytes per lane and step, lanes added in a fixed tree.
template <typename T>
__global__ void __launch_bounds__(kBlock)
value_deviation_kernel(const T *__restrict__ a, const T *__restrict__ b, const int *__restrict__ tok_chunk,
                       float *__restrict__ scores, int n_rows, int row_elems) {
  constexpr int V = a3_elem<T>::kVec;
  typedef T vec_t __attribute__((ext_vector_type(V)));
  const int lane = threadIdx.x & 63, t = blockIdx.x * (kBlock / 64) + (threadIdx.x >> 6);
  if (t >= n_rows) return;
  if (tok_chunk[t] < 0) {
    if (lane == 0) scores[t] = -INFINITY;
    return;
  }
  const T *pa = a + (size_t)t * row_elems, *pb = b + (size_t)t * row_elems;
  float acc = 0.f;
  for (int v = lane; v < row_elems / V; v += 64) {
    const vec_t x = *reinterpret_cast<const vec_t *>(pa + v * V), y = *reinterpret_cast<const vec_t *>(pb + v * V);
#pragma unroll
    for (int e = 0; e < V; ++e) { const float d = (float)x[e] - (float)y[e]; acc = fmaf(d, d, acc); }
  }
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) acc += __shfl_xor(acc, o);
  if (lane == 0) scores[t] = acc;
}

// The first n_head and the last n_tail rows of every chunk (a chunk no longer than n_head + n_tail: all of
// its rows once), per request in ascending order.  One thread per chunk; its output offset is the request's
// start plus the counts of the request's earlier chunks.
__global__ void __launch_bounds__(kBlock)
chunk_edges_kernel(const int *__restrict__ chunk_start, const int *__restrict__ chunk_len,
                   const int *__restrict__ tok_req, const int *__restrict__ sel_start, int n_chunks, int n_head,
                   int n_tail, int total_k, int *__restrict__ sel_idx) {
  const int c = blockIdx.x * kBlock + threadIdx.x;
  if (c >= n_chunks) return;
  const int len = chunk_len[c];
  if (len <= 0) return;
  const int s = chunk_start[c], r = tok_req[s];
  int off = sel_start[r];
  for (int p = c - 1; p >= 0; --p) {
    const int pl = chunk_len[p];
    if (pl <= 0) continue;
    if (tok_req[chunk_start[p]] != r) break;
    off += min(pl, n_head + n_tail);
  }
  // (a sel_start that does not match the rule must not send a store outside the list)
  if (len <= n_head + n_tail) {
    for (int i = 0; i < len; ++i)
      if (off + i >= 0 && off + i < total_k) sel_idx[off + i] = s + i;
  } else {
    for (int i = 0; i < n_head; ++i)
      if (off + i >= 0 && off + i < total_k) sel_idx[off + i] = s + i;
    for (int i = 0; i < n_tail; ++i)
      if (off + n_head + i >= 0 && off + n_head + i < total_k) sel_idx[off + n_head + i] = s + len - n_tail + i;
  }
}

template <typename T>
a3_status launch_realign(const a3_layout *L, const void *k_cat, void *k_fused, hipStream_t st) {
  constexpr int VEC = a3_elem<T>::kVec;
  constexpr int UNROLL = 4;
  const int row_elems = L->n_kv_heads * L->head_dim;
  const bool inter = L->rope_layout == A3_ROPE_INTERLEAVED;
  const int items_per_row = inter ? row_elems / VEC : row_elems / (2 * VEC);
  const long long total = (long long)L->total_tokens * items_per_row;
  A3_REQUIRE(total < (1LL << 31), A3_ERR_UNSUPPORTED, "a3_rope_realign: cache too large for 32-bit indexing");
  const unsigned grid = (unsigned)((total + (long long)kBlock * UNROLL - 1) / ((long long)kBlock * UNROLL));
  const int items_shift = (items_per_row & (items_per_row - 1)) == 0 ? __builtin_ctz(items_per_row) : -1;
  auto fn = inter ? rope_realign_kernel<T, A3_ROPE_INTERLEAVED, UNROLL> : rope_realign_kernel<T, A3_ROPE_HALF, UNROLL>;
  hipLaunchKernelGGL(fn, dim3(grid), dim3(kBlock), 0, st, (const T *)k_cat, (T *)k_fused, L->tok_chunk,
                     (const float2 *)L->rope_chunk_cs, L->total_tokens, L->head_dim, row_elems, items_per_row, items_shift);
  A3_CHECK_LAUNCH("a3_rope_realign");
  return A3_OK;
}

}  // namespace

extern "C" a3_status a3_layout_prepare(const a3_layout *L, void *stream) {
  a3_status s = a3_check_layout(L, "a3_layout_prepare", true);
  if (s != A3_OK) return s;
  hipStream_t st = (hipStream_t)stream;
  const int T = L->total_tokens;
  hipLaunchKernelGGL(prepare_tokens_kernel, dim3((T + kBlock - 1) / kBlock), dim3(kBlock), 0, st, L->seg_start,
                     L->n_req, L->chunk_start, L->chunk_len, L->n_chunks, T, L->tok_pos, L->tok_req, L->tok_chunk,
                     L->q_len, L->q_start);
  A3_CHECK_LAUNCH("a3_layout_prepare(tokens)");
  const int half = L->head_dim / 2;
  const int n_pos = L->max_ctx_len + L->max_q_len;
  const long long total = (long long)(L->n_chunks + n_pos) * half;
  hipLaunchKernelGGL(prepare_rope_kernel, dim3((unsigned)((total + kBlock - 1) / kBlock)), dim3(kBlock), 0, st,
                     L->chunk_delta, L->n_chunks, n_pos, half, L->rope_base, (float2 *)L->rope_chunk_cs,
                     (float2 *)L->rope_pos_cs);
  A3_CHECK_LAUNCH("a3_layout_prepare(rope)");
  return A3_OK;
}

extern "C" a3_status a3_rope_realign(const a3_layout *L, const void *k_cat, void *k_fused, void *stream) {
  a3_status s = a3_check_layout(L, "a3_rope_realign", true);
  if (s != A3_OK) return s;
  A3_REQUIRE(k_cat && k_fused, A3_ERR_INVALID_ARG, "a3_rope_realign: k_cat/k_fused is NULL");
  A3_REQUIRE(a3_aligned16(k_cat) && a3_aligned16(k_fused), A3_ERR_INVALID_ARG,
             "a3_rope_realign: tensors must be 16-byte aligned");
  if (L->n_chunks == 0) return A3_OK;
  hipStream_t st = (hipStream_t)stream;
  return L->dtype == A3_BF16 ? launch_realign<bf16_t>(L, k_cat, k_fused, st) : launch_realign<float>(L, k_cat, k_fused, st);
}

extern "C" a3_status a3_kv_scatter(const a3_layout *L, const void *k_new, const void *v_new, const int *row_idx,
                                   int n_rows, void *k_fused, void *v_fused, void *stream) {
  a3_status s = a3_check_layout(L, "a3_kv_scatter", false);
  if (s != A3_OK) return s;
  A3_REQUIRE(n_rows >= 0 && n_rows <= L->total_tokens, A3_ERR_INVALID_ARG,
             "a3_kv_scatter: n_rows %d outside [0, %d]", n_rows, L->total_tokens);
  if (n_rows == 0) return A3_OK;
  A3_REQUIRE(k_new && v_new && row_idx && k_fused && v_fused, A3_ERR_INVALID_ARG, "a3_kv_scatter: NULL argument");
  A3_REQUIRE(a3_aligned16(k_new) && a3_aligned16(v_new) && a3_aligned16(k_fused) && a3_aligned16(v_fused),
             A3_ERR_INVALID_ARG, "a3_kv_scatter: tensors must be 16-byte aligned");
  constexpr int UNROLL = 4;
  const int esz = L->dtype == A3_BF16 ? 2 : 4;
  const int vec_per_row = L->n_kv_heads * L->head_dim * esz / 16;
  const long long total = (long long)n_rows * vec_per_row;
  A3_REQUIRE(total < (1LL << 31), A3_ERR_UNSUPPORTED, "a3_kv_scatter: too many rows for 32-bit indexing");
  const unsigned grid = (unsigned)((total + (long long)kBlock * UNROLL - 1) / ((long long)kBlock * UNROLL));
  const int vec_shift = (vec_per_row & (vec_per_row - 1)) == 0 ? __builtin_ctz(vec_per_row) : -1;
  hipLaunchKernelGGL(kv_scatter_kernel<UNROLL>, dim3(grid, 2), dim3(kBlock), 0, (hipStream_t)stream,
                     (const uint4 *)k_new, (const uint4 *)v_new, row_idx, n_rows, vec_per_row, vec_shift,
                     (uint4 *)k_fused, (uint4 *)v_fused);
  A3_CHECK_LAUNCH("a3_kv_scatter");
  return A3_OK;
}

extern "C" a3_status a3_active_rows(const a3_layout *L, const int *sel_idx, const int *sel_start, int n_act,
                                    int *act_idx, void *stream) {
  a3_status s = a3_check_layout(L, "a3_active_rows", true);
  if (s != A3_OK) return s;
  A3_REQUIRE(n_act >= 0 && n_act <= L->total_tokens, A3_ERR_INVALID_ARG, "a3_active_rows: n_act %d outside [0, %d]",
             n_act, L->total_tokens);
  if (n_act == 0) return A3_OK;
  A3_REQUIRE(sel_start && act_idx, A3_ERR_INVALID_ARG, "a3_active_rows: NULL argument");
  hipLaunchKernelGGL(active_rows_kernel, dim3((n_act + kBlock - 1) / kBlock), dim3(kBlock), 0, (hipStream_t)stream,
                     sel_idx, sel_start, L->q_start, L->seg_start, L->ctx_len, L->n_req, n_act, act_idx);
  A3_CHECK_LAUNCH("a3_active_rows");
  return A3_OK;
}

extern "C" a3_status a3_value_deviation_scores(const a3_layout *L, const void *v_true, const void *v_cat,
                                               float *scores, void *stream) {
  a3_status s = a3_check_layout(L, "a3_value_deviation_scores", true);
  if (s != A3_OK) return s;
  if (L->total_tokens == 0) return A3_OK;
  A3_REQUIRE(v_true && v_cat && scores, A3_ERR_INVALID_ARG, "a3_value_deviation_scores: NULL tensor");
  A3_REQUIRE(a3_aligned16(v_true) && a3_aligned16(v_cat), A3_ERR_INVALID_ARG,
             "a3_value_deviation_scores: tensors must be 16-byte aligned");
  const int row_elems = L->n_kv_heads * L->head_dim;
  const dim3 grid((L->total_tokens + kBlock / 64 - 1) / (kBlock / 64));
  if (L->dtype == A3_BF16) {
    A3_REQUIRE(row_elems % 8 == 0, A3_ERR_UNSUPPORTED, "a3_value_deviation_scores: row of %d elements", row_elems);
    hipLaunchKernelGGL(value_deviation_kernel<bf16_t>, grid, dim3(kBlock), 0, (hipStream_t)stream, (const bf16_t *)v_true,
                       (const bf16_t *)v_cat, L->tok_chunk, scores, L->total_tokens, row_elems);
  } else {
    A3_REQUIRE(row_elems % 4 == 0, A3_ERR_UNSUPPORTED, "a3_value_deviation_scores: row of %d elements", row_elems);
    hipLaunchKernelGGL(value_deviation_kernel<float>, grid, dim3(kBlock), 0, (hipStream_t)stream, (const float *)v_true,
                       (const float *)v_cat, L->tok_chunk, scores, L->total_tokens, row_elems);
  }
  A3_CHECK_LAUNCH("a3_value_deviation_scores");
  return A3_OK;
}

extern "C" a3_status a3_select_chunk_edges(const a3_layout *L, int n_head, int n_tail, const int *sel_start,
                                           int total_k, int *sel_idx, void *stream) {
  a3_status s = a3_check_layout(L, "a3_select_chunk_edges", true);
  if (s != A3_OK) return s;
  A3_REQUIRE(n_head >= 0 && n_tail >= 0, A3_ERR_INVALID_ARG, "a3_select_chunk_edges: n_head %d, n_tail %d", n_head, n_tail);
  A3_REQUIRE(total_k >= 0 && total_k <= L->total_tokens, A3_ERR_INVALID_ARG,
             "a3_select_chunk_edges: total_k %d outside [0, %d]", total_k, L->total_tokens);
  if (total_k == 0 || L->n_chunks == 0) return A3_OK;
  A3_REQUIRE(sel_start && sel_idx, A3_ERR_INVALID_ARG, "a3_select_chunk_edges: NULL argument");
  hipLaunchKernelGGL(chunk_edges_kernel, dim3((L->n_chunks + kBlock - 1) / kBlock), dim3(kBlock), 0, (hipStream_t)stream,
                     L->chunk_start, L->chunk_len, L->tok_req, sel_start, L->n_chunks, n_head, n_tail, total_k, sel_idx);
  A3_CHECK_LAUNCH("a3_select_chunk_edges");
  return A3_OK;
}
