// Step 3 of the A^3 fusion path: Re = top_p(s) (Eq. 3, second line).
//
// One workgroup of 16 wavefronts per request.  The k-th largest score is found exactly by a radix
// select on an order-preserving integer image of the float (8 bits per pass; the passes start at
// the highest bit in which the request's smallest and largest key differ), then the rows are
// compacted in index order with one workgroup-wide prefix sum.  Compacting in index order
// gives both rules of the selection for free: among equal scores the lowest rows are taken,
// and the output is ascending.  Integer work only: the result is unique and bit-exact.
// Requests of up to 36 K rows keep every key in a register of the lane that owns it (a contiguous
// run of rows per lane); longer ones re-read the scores from global memory in every pass.
#include "a3_internal.h"

namespace {

constexpr int kBlock = 1024;
constexpr int kWaves = kBlock / 64;

// Monotone map float -> uint32 (larger float <=> larger key); -0 is folded onto +0.
__device__ __forceinline__ uint32_t score_key(float s) {
  uint32_t b = __float_as_uint(s);
  if (b == 0x80000000u) b = 0u;
  return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}

// Exclusive prefix sum of one int per thread over the workgroup (threads in tid order).
__device__ __forceinline__ int block_exclusive_scan(int v, int *wave_tot /* [kWaves] LDS */) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  int inc = v;
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    int x = __shfl_up(inc, off, 64);
    if (lane >= off) inc += x;
  }
  __syncthreads();                       // wave_tot may still be read by a previous scan
  if (lane == 63) wave_tot[wave] = inc;
  __syncthreads();
  int before = 0;
  for (int w = 0; w < wave; ++w) before += wave_tot[w];
  return before + inc - v;
}

// Adds one to hist[bin] for every active lane.  Lanes of a wave that hit the same bin are merged
// into a single LDS atomic (the top byte of the scores takes only a handful of values, and
// thousands of same-address atomics would serialise).
__device__ __forceinline__ void hist_add_merged(uint32_t *hist, uint32_t bin, bool active) {
  unsigned long long todo = __ballot(active);
  const int lane = threadIdx.x & 63;
  while (todo) {
    const int leader = __ffsll(todo) - 1;
    const uint32_t lbin = __shfl(bin, leader, 64);
    const unsigned long long same = __ballot(active && bin == lbin);
    if (lane == leader) atomicAdd(&hist[lbin], (uint32_t)__popcll(same));
    todo &= ~same;
  }
}

// Suffix sums over the 256 bins, from the highest bin downwards, by the first wave: finds the bin
// that holds the need-th largest candidate and how many candidates of that bin are still needed.
__device__ __forceinline__ void find_bin(const uint32_t *hist, uint32_t need, uint32_t *sh_bin, uint32_t *sh_need) {
  const int tid = threadIdx.x;
  if (tid < 64) {
    uint32_t c[4], t = 0;                // lane owns bins 4*lane .. 4*lane+3
#pragma unroll
    for (int j = 0; j < 4; ++j) { c[j] = hist[4 * tid + j]; t += c[j]; }
    uint32_t suf = t;                    // sum over lanes >= this one
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
      uint32_t x = __shfl_down(suf, off, 64);
      if (tid + off < 64) suf += x;
    }
    uint32_t above = suf - t;            // candidates in bins of higher lanes
#pragma unroll
    for (int j = 3; j >= 0; --j) {
      if (above < need && above + c[j] >= need) { *sh_bin = 4 * tid + j; *sh_need = need - above; }
      above += c[j];
    }
  }
}

// Requests longer than the register kernel holds: 4 x 8-bit passes from the top byte, every pass
// re-reads the scores from global memory.
__global__ void __launch_bounds__(kBlock)
topk_select_kernel(const float *__restrict__ scores, const int *__restrict__ seg_start,
                   const int *__restrict__ ctx_len, const int *__restrict__ sel_start, int *__restrict__ sel_idx) {
  __shared__ uint32_t hist[256];
  __shared__ int wave_tot[kWaves];
  __shared__ uint32_t sh_bin, sh_need;

  const int r = blockIdx.x, tid = threadIdx.x;
  const int s = seg_start[r];
  const int N = ctx_len[r];
  int k = sel_start[r + 1] - sel_start[r];
  if (k > N) k = N;
  if (k <= 0) return;                    // uniform over the workgroup
  int *__restrict__ out = sel_idx + sel_start[r];
  const float *__restrict__ sc = scores + s;
  auto key_at = [&](int i) -> uint32_t { return score_key(sc[i]); };

  // ---- radix select: key of the k-th largest score -------------------------------------
  uint32_t prefix = 0, mask = 0, need = (uint32_t)k;
  for (int shift = 24; shift >= 0; shift -= 8) {
    if (tid < 256) hist[tid] = 0;
    __syncthreads();
    const int n_round = (N + kBlock - 1) / kBlock * kBlock;  // whole waves take part in the merged add
    for (int i = tid; i < n_round; i += kBlock) {
      const uint32_t u = i < N ? key_at(i) : 0u;
      const bool active = i < N && (u & mask) == prefix;
      const uint32_t bin = (u >> shift) & 255u;
      if (shift == 24) hist_add_merged(hist, bin, active);
      else if (active) atomicAdd(&hist[bin], 1u);
    }
    __syncthreads();
    find_bin(hist, need, &sh_bin, &sh_need);
    __syncthreads();
    prefix |= sh_bin << shift;
    mask |= 255u << shift;
    need = sh_need;
    __syncthreads();
  }
  const uint32_t tau = prefix;           // key of the k-th largest; `need` rows equal to it are taken

  // ---- ordered compaction: thread tid owns rows [lo, hi) ----------------------------------
  const int per = (N + kBlock - 1) / kBlock;
  const int lo = min(N, tid * per), hi = min(N, lo + per);
  int cnt_gt = 0, cnt_eq = 0;
  for (int i = lo; i < hi; ++i) {
    uint32_t u = key_at(i);
    cnt_gt += u > tau;
    cnt_eq += u == tau;
  }
  const int eq_before = block_exclusive_scan(cnt_eq, wave_tot);
  int take_eq = (int)need - eq_before;
  take_eq = take_eq < 0 ? 0 : (take_eq > cnt_eq ? cnt_eq : take_eq);
  int pos = block_exclusive_scan(cnt_gt + take_eq, wave_tot);
  for (int i = lo; i < hi; ++i) {
    uint32_t u = key_at(i);
    if (u > tau) out[pos++] = s + i;
    else if (u == tau && take_eq > 0) { out[pos++] = s + i; --take_eq; }
  }
}

// KPT = keys per lane (compile-time bound; the request's rows are split into runs of
// ceil(N / 1024) <= KPT consecutive rows).  The scores are read once, coalesced, into LDS and
// from there into the registers of their owners; every later step works on registers.
template <int KPT>
__global__ void __launch_bounds__(kBlock)
topk_select_reg_kernel(const float *__restrict__ scores, const int *__restrict__ seg_start,
                       const int *__restrict__ ctx_len, const int *__restrict__ sel_start, int *__restrict__ sel_idx) {
  extern __shared__ uint32_t keys[];                         // [N + N/32]
  __shared__ uint32_t hist[256];
  __shared__ uint32_t wave_min[kWaves], wave_max[kWaves];
  __shared__ int wave_gt[kWaves], wave_eq[kWaves];
  __shared__ uint32_t sh_bin, sh_need;

  const int r = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int s = seg_start[r];
  const int N = ctx_len[r];
  int k = sel_start[r + 1] - sel_start[r];
  if (k > N) k = N;
  if (k <= 0) return;                    // uniform over the workgroup
  int *__restrict__ out = sel_idx + sel_start[r];
  const float *__restrict__ sc = scores + s;

  const int per = (N + kBlock - 1) / kBlock;                 // <= KPT (checked by the host)
  const int first = min(N, tid * per), nv = min(N, first + per) - first;
  uint32_t key[KPT];
  uint32_t mn = 0xffffffffu, mx = 0u;
  if (per % 4 == 0 && (reinterpret_cast<uintptr_t>(sc) & 15) == 0) {
    // a lane's run starts on a 16-byte boundary: four scores per load, straight into the registers
#pragma unroll
    for (int q = 0; q < KPT / 4; ++q) {
      float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
      if (4 * q < nv) {
        if (4 * q + 4 <= nv) v = *reinterpret_cast<const float4 *>(sc + first + 4 * q);
        else {                                               // last lane with scores: the run ends inside this vector
          v.x = sc[first + 4 * q];
          if (4 * q + 1 < nv) v.y = sc[first + 4 * q + 1];
          if (4 * q + 2 < nv) v.z = sc[first + 4 * q + 2];
        }
      }
      key[4 * q] = score_key(v.x); key[4 * q + 1] = score_key(v.y);
      key[4 * q + 2] = score_key(v.z); key[4 * q + 3] = score_key(v.w);
    }
  } else {
    // coalesced through LDS.  One pad word per 32 keys: a lane reads a contiguous run, and without the pad
    // the runs of all lanes would start in the same few LDS banks
    for (int i = tid; i < N; i += kBlock) keys[i + (i >> 5)] = score_key(sc[i]);
    __syncthreads();
#pragma unroll
    for (int j = 0; j < KPT; ++j) {
      const int i = first + min(j, max(nv - 1, 0));
      key[j] = nv > 0 ? keys[i + (i >> 5)] : 0u;
    }
  }
#pragma unroll
  for (int j = 0; j < KPT; ++j)
    if (j < nv) { mn = min(mn, key[j]); mx = max(mx, key[j]); }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) {
    mn = min(mn, (uint32_t)__shfl_xor((int)mn, off, 64));
    mx = max(mx, (uint32_t)__shfl_xor((int)mx, off, 64));
  }
  if (lane == 0) { wave_min[wave] = mn; wave_max[wave] = mx; }
  __syncthreads();
#pragma unroll
  for (int w = 0; w < kWaves; ++w) { mn = min(mn, wave_min[w]); mx = max(mx, wave_max[w]); }

  // ---- radix select inside [lo, hi]: the key of the k-th largest score ------------------
  // Invariant: the wanted key lies in [lo, hi] and is the need-th largest of the keys in there.
  uint32_t lo = mn, hi = mx, need = (uint32_t)k;
  for (;;) {
    const uint32_t width = hi - lo;
    if (width == 0) break;                                   // every candidate is the same key
    const int shift = max(0, 24 - __clz((int)width));        // (width >> shift) < 256
    if (tid < 256) hist[tid] = 0;
    __syncthreads();
#pragma unroll
    for (int j = 0; j < KPT; ++j) {
      const uint32_t rel = key[j] - lo;
      if (j < nv && rel <= width) atomicAdd(&hist[rel >> shift], 1u);
    }
    __syncthreads();
    find_bin(hist, need, &sh_bin, &sh_need);
    __syncthreads();
    lo += sh_bin << shift;
    hi = min(hi, lo + ((1u << shift) - 1u));
    need = sh_need;
    __syncthreads();
    if (shift == 0) break;                                   // the bin was a single key
  }
  const uint32_t tau = lo;               // key of the k-th largest; `need` rows equal to it are taken

  // ---- ordered compaction: one scan over (rows above tau, rows equal to tau) per lane -------
  int cnt_gt = 0, cnt_eq = 0;
#pragma unroll
  for (int j = 0; j < KPT; ++j) {
    if (j < nv) { cnt_gt += key[j] > tau; cnt_eq += key[j] == tau; }
  }
  int inc_gt = cnt_gt, inc_eq = cnt_eq;
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const int xg = __shfl_up(inc_gt, off, 64), xe = __shfl_up(inc_eq, off, 64);
    if (lane >= off) { inc_gt += xg; inc_eq += xe; }
  }
  if (lane == 63) { wave_gt[wave] = inc_gt; wave_eq[wave] = inc_eq; }
  __syncthreads();
  int gt_before = inc_gt - cnt_gt, eq_before = inc_eq - cnt_eq;
  for (int w = 0; w < wave; ++w) { gt_before += wave_gt[w]; eq_before += wave_eq[w]; }
  // rows equal to tau are taken in index order until `need` of them are: min(eq_before, need) of
  // the earlier ones were taken
  int pos = gt_before + min(eq_before, (int)need);
  int take_eq = (int)need - eq_before;
  take_eq = take_eq < 0 ? 0 : (take_eq > cnt_eq ? cnt_eq : take_eq);
#pragma unroll
  for (int j = 0; j < KPT; ++j) {
    if (j < nv) {
      if (key[j] > tau) out[pos++] = s + first + j;
      else if (key[j] == tau && take_eq > 0) { out[pos++] = s + first + j; --take_eq; }
    }
  }
}

constexpr int kMaxLdsKeys = 36 * 1024;   // 148.5 KB of padded keys next to the small static arrays

}  // namespace

extern "C" a3_status a3_topk_select(const a3_layout *L, const float *scores, const int *sel_start, int total_k,
                                    int *sel_idx, void *ws, size_t ws_bytes, void *stream) {
  (void)ws; (void)ws_bytes;              // the select keeps everything in LDS
  a3_status s = a3_check_layout(L, "a3_topk_select", false);
  if (s != A3_OK) return s;
  A3_REQUIRE(total_k >= 0, A3_ERR_INVALID_ARG, "a3_topk_select: total_k %d is negative", total_k);
  A3_REQUIRE((long long)total_k <= (long long)L->max_ctx_len * L->n_req, A3_ERR_INVALID_ARG,
             "a3_topk_select: total_k %d exceeds the number of context rows", total_k);
  A3_REQUIRE(scores && sel_start, A3_ERR_INVALID_ARG, "a3_topk_select: scores/sel_start is NULL");
  if (total_k == 0) return A3_OK;
  A3_REQUIRE(sel_idx, A3_ERR_INVALID_ARG, "a3_topk_select: sel_idx is NULL");
  if (L->max_ctx_len <= kMaxLdsKeys) {
    const size_t lds = ((size_t)L->max_ctx_len + L->max_ctx_len / 32 + 1) * sizeof(uint32_t);
    static bool attr_done = false;
    if (!attr_done) {
      const int cap = (int)((kMaxLdsKeys + kMaxLdsKeys / 32 + 1) * sizeof(uint32_t));
      hipError_t e1 = hipFuncSetAttribute((const void *)topk_select_reg_kernel<4>, hipFuncAttributeMaxDynamicSharedMemorySize, cap);
      hipError_t e2 = hipFuncSetAttribute((const void *)topk_select_reg_kernel<16>, hipFuncAttributeMaxDynamicSharedMemorySize, cap);
      hipError_t e3 = hipFuncSetAttribute((const void *)topk_select_reg_kernel<36>, hipFuncAttributeMaxDynamicSharedMemorySize, cap);
      if (e1 != hipSuccess || e2 != hipSuccess || e3 != hipSuccess)
        return a3_fail(A3_ERR_HIP, "a3_topk_select: cannot raise the dynamic LDS limit");
      attr_done = true;
    }
    const int per = (L->max_ctx_len + kBlock - 1) / kBlock;  // keys per lane of the longest request
    if (per <= 4)
      hipLaunchKernelGGL(topk_select_reg_kernel<4>, dim3(L->n_req), dim3(kBlock), lds, (hipStream_t)stream, scores,
                         L->seg_start, L->ctx_len, sel_start, sel_idx);
    else if (per <= 16)
      hipLaunchKernelGGL(topk_select_reg_kernel<16>, dim3(L->n_req), dim3(kBlock), lds, (hipStream_t)stream, scores,
                         L->seg_start, L->ctx_len, sel_start, sel_idx);
    else
      hipLaunchKernelGGL(topk_select_reg_kernel<36>, dim3(L->n_req), dim3(kBlock), lds, (hipStream_t)stream, scores,
                         L->seg_start, L->ctx_len, sel_start, sel_idx);
  } else {
    hipLaunchKernelGGL(topk_select_kernel, dim3(L->n_req), dim3(kBlock), 0, (hipStream_t)stream, scores,
                       L->seg_start, L->ctx_len, sel_start, sel_idx);
  }
  A3_CHECK_LAUNCH("a3_topk_select");
  return A3_OK;
}
