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
#include "a3_attn_plan.h"

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

// What one workgroup ranks.  Selection of Eq. 3: the context rows of request blockIdx.x, k from sel_start.
// Eviction extension (skip != nullptr): blockIdx.y is a KV head with its own score row and output row; the
// first skip[r] context rows (system prompt) and the question rows are retained anyway and written by
// another kernel, so the candidates start behind the system prompt, the count leaves them out, and the
// output starts behind the system prompt's slots.
struct topk_problem {
  const int *seg_start, *ctx_len, *sel_start;
  const int *skip, *q_len;
  long score_stride, out_stride;
  // a batch of one request whose lengths the host knows (the layout's maxima add up to its rows): its context
  // length and count, so that the kernel starts without a chain of loads; otherwise -1
  int one_N = -1, one_k = -1;
};

struct topk_range { int s, N, k; const float *sc; int *out; };

__device__ __forceinline__ topk_range topk_range_of(const topk_problem &p, const float *scores, int *sel_idx) {
  topk_range t;
  if (p.one_N >= 0) {
    t.s = 0; t.N = p.one_N; t.k = min(p.one_k, p.one_N);
    t.sc = scores; t.out = sel_idx;
    return t;
  }
  const int r = blockIdx.x;
  const int sk = p.skip ? p.skip[r] : 0;
  t.s = p.seg_start[r] + sk;
  t.N = max(p.ctx_len[r] - sk, 0);
  t.k = p.sel_start[r + 1] - p.sel_start[r] - (p.skip ? sk + p.q_len[r] : 0);
  if (t.k > t.N) t.k = t.N;
  t.sc = scores + (size_t)blockIdx.y * p.score_stride + t.s;
  t.out = sel_idx + (size_t)blockIdx.y * p.out_stride + p.sel_start[r] + sk;
  return t;
}

// Requests longer than the register kernel holds: 4 x 8-bit passes from the top byte, every pass
// re-reads the scores from global memory.
__global__ void __launch_bounds__(kBlock)
topk_select_kernel(const float *__restrict__ scores, topk_problem prob, int *__restrict__ sel_idx) {
  __shared__ uint32_t hist[256];
  __shared__ int wave_tot[kWaves];
  __shared__ uint32_t sh_bin, sh_need;

  const int tid = threadIdx.x;
  const topk_range rg = topk_range_of(prob, scores, sel_idx);
  const int s = rg.s, N = rg.N, k = rg.k;
  if (k <= 0) return;                    // uniform over the workgroup
  int *__restrict__ out = rg.out;
  const float *__restrict__ sc = rg.sc;
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
__device__ __forceinline__ void topk_select_reg_body(const float *__restrict__ scores, const topk_problem &prob,
                                                     int *__restrict__ sel_idx, uint32_t *keys /* LDS [N + N/32] */) {
  __shared__ uint32_t hist[256];
  __shared__ uint32_t wave_min[kWaves], wave_max[kWaves];
  __shared__ int wave_gt[kWaves], wave_eq[kWaves];
  __shared__ uint32_t sh_bin, sh_need;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const topk_range rg = topk_range_of(prob, scores, sel_idx);
  const int s = rg.s, N = rg.N, k = rg.k;
  if (k <= 0) return;                    // uniform over the workgroup
  int *__restrict__ out = rg.out;
  const float *__restrict__ sc = rg.sc;

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
    const uint32_t in_bin = hist[sh_bin];                    // candidates left, need of them wanted
    __syncthreads();
    if (shift == 0) break;                                   // the bin was a single key
    if (in_bin <= 64) {
      // Few candidates left (the usual case after two rounds): they are gathered (in any order: what follows
      // does not depend on it) and one wave ranks them instead of two more rounds over all lanes.  The key v
      // with fewer than `need` candidates above it and at least `need` at or above it is the wanted one.
      uint32_t *cand = hist;                                 // free since the barrier above
      if (tid == 0) sh_bin = 0;
      __syncthreads();
#pragma unroll
      for (int j = 0; j < KPT; ++j)
        if (j < nv && key[j] - lo <= hi - lo) cand[atomicAdd(&sh_bin, 1u)] = key[j];
      __syncthreads();
      if (tid < 64) {
        const uint32_t mine = tid < (int)in_bin ? cand[tid] : 0u;
        uint32_t gt = 0, ge = 0;
        for (uint32_t i = 0; i < in_bin; ++i) { const uint32_t c = cand[i]; gt += c > mine; ge += c >= mine; }
        // (several lanes hold the wanted key when it occurs more than once: they store the same two numbers)
        if (tid < (int)in_bin && gt < need && need <= ge) { wave_min[0] = mine; sh_need = need - gt; }
      }
      __syncthreads();
      lo = hi = wave_min[0];
      need = sh_need;
      break;
    }
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

template <int KPT>
__global__ void __launch_bounds__(kBlock)
topk_select_reg_kernel(const float *__restrict__ scores, topk_problem prob, int *__restrict__ sel_idx) {
  extern __shared__ uint32_t keys[];
  topk_select_reg_body<KPT>(scores, prob, sel_idx, keys);
}

// Step 3, the active rows [Re, Q] and the layout of the attention's work in one launch, for a batch of one
// request (one workgroup ranks it anyway): the selection goes to sel_idx and to the head of act_idx, the question
// rows behind it, and the same workgroup then lays out the attention (a3_attn_plan.h) from the list it just wrote.
template <int KPT>
__global__ void __launch_bounds__(kBlock)
topk_select_plan_kernel(const float *__restrict__ scores, topk_problem prob, int *__restrict__ sel_idx,
                        int *act_idx, int n_act, attn_plan plan, int G, int wgs_per_head, int item_cost,
                        int lds_ints /* ints of dynamic LDS */) {
  extern __shared__ uint32_t keys[];
  __shared__ int wave_tot[kPlanThreads / 64];
  static_assert(kPlanThreads == kBlock, "one workgroup shape for both parts");
  topk_select_reg_body<KPT>(scores, prob, sel_idx, keys);
  __syncthreads();                                           // the selection is written (and has left this CU's L1 path)
  const int k = prob.one_N >= 0 ? prob.one_k : prob.sel_start[1] - prob.sel_start[0];
  const int s = prob.one_N >= 0 ? 0 : prob.seg_start[0], N = prob.one_N >= 0 ? prob.one_N : prob.ctx_len[0];
  if (sel_idx != act_idx)
    for (int i = threadIdx.x; i < k; i += kBlock) act_idx[i] = sel_idx[i];
  for (int i = threadIdx.x; k + i < n_act; i += kBlock) act_idx[k + i] = s + N + i;   // the question rows
  __threadfence_block();
  __syncthreads();
  // (the keys' LDS is free now: it serves as the plan's scratch)
  attn_plan_body(plan, act_idx, n_act, prob.seg_start, 1, G, wgs_per_head, item_cost, wave_tot,
                 reinterpret_cast<int *>(keys), lds_ints);
}

constexpr int kMaxLdsKeys = 36 * 1024;   // 148.5 KB of padded keys next to the small static arrays

// One launch of the ranking kernels over grid (requests, heads).
a3_status topk_launch(const a3_layout *L, const float *scores, const topk_problem &prob, int n_heads, int *sel_idx,
                      hipStream_t st, const char *who) {
  const dim3 grid(L->n_req, n_heads);
  if (L->max_ctx_len <= kMaxLdsKeys) {
    const size_t lds = ((size_t)L->max_ctx_len + L->max_ctx_len / 32 + 1) * sizeof(uint32_t);
    static a3_once_per_device lds_once;
    const hipError_t once_err = a3_once(lds_once, []() {
      const int cap = (int)((kMaxLdsKeys + kMaxLdsKeys / 32 + 1) * sizeof(uint32_t));
      hipError_t e1 = hipFuncSetAttribute((const void *)topk_select_reg_kernel<4>, hipFuncAttributeMaxDynamicSharedMemorySize, cap);
      hipError_t e2 = hipFuncSetAttribute((const void *)topk_select_reg_kernel<16>, hipFuncAttributeMaxDynamicSharedMemorySize, cap);
      hipError_t e3 = hipFuncSetAttribute((const void *)topk_select_reg_kernel<36>, hipFuncAttributeMaxDynamicSharedMemorySize, cap);
      return e1 != hipSuccess ? e1 : (e2 != hipSuccess ? e2 : e3);
    });
    if (once_err != hipSuccess) return a3_fail(A3_ERR_HIP, "%s: cannot raise the dynamic LDS limit", who);
    const int per = (L->max_ctx_len + kBlock - 1) / kBlock;  // keys per lane of the longest request
    if (per <= 4) hipLaunchKernelGGL(topk_select_reg_kernel<4>, grid, dim3(kBlock), lds, st, scores, prob, sel_idx);
    else if (per <= 16) hipLaunchKernelGGL(topk_select_reg_kernel<16>, grid, dim3(kBlock), lds, st, scores, prob, sel_idx);
    else hipLaunchKernelGGL(topk_select_reg_kernel<36>, grid, dim3(kBlock), lds, st, scores, prob, sel_idx);
  } else {
    hipLaunchKernelGGL(topk_select_kernel, grid, dim3(kBlock), 0, st, scores, prob, sel_idx);
  }
  A3_CHECK_LAUNCH(who);
  return A3_OK;
}

// ---------------------------------------------------------------------------------------
// eviction extension: pooling of the votes, the rows that are always retained, compaction
// ---------------------------------------------------------------------------------------
// 1-D pooling of stride 1 along the context rows of a request, per head.  mode 0: maximum over the rows
// inside the request's context; mode 1: sum / width (rows outside count as zero).  Other rows are copied.
__global__ void __launch_bounds__(256)
pool_votes_kernel(const float *__restrict__ in, float *__restrict__ out, const int *__restrict__ tok_req,
                  const int *__restrict__ tok_chunk, const int *__restrict__ seg_start,
                  const int *__restrict__ ctx_len, int T, int width, int mode) {
  const int t = blockIdx.x * 256 + threadIdx.x;
  if (t >= T) return;
  const float *row = in + (size_t)blockIdx.y * T;
  float v = row[t];
  if (tok_chunk[t] >= 0) {
    const int r = tok_req[t];
    const int s = seg_start[r], e = s + ctx_len[r];
    const int lo = max(s, t - width / 2), hi = min(e, t + width / 2 + 1);
    if (mode == 0) {
      for (int u = lo; u < hi; ++u) v = fmaxf(v, row[u]);
    } else {
      float sum = 0.f;
      for (int u = lo; u < hi; ++u) sum += row[u];           // ascending row order
      v = sum / (float)width;
    }
  }
  out[(size_t)blockIdx.y * T + t] = v;
}

// keep_idx[g][keep_start[r] + i] for the system-prompt rows (i < skip[r]) and the question rows (the last
// q_len[r] slots of the request)
__global__ void __launch_bounds__(256)
evict_fixed_rows_kernel(topk_problem p, int total_keep, int *__restrict__ keep_idx) {
  const int r = blockIdx.x;
  int *out = keep_idx + (size_t)blockIdx.y * p.out_stride;
  const int s = p.seg_start[r], N = p.ctx_len[r], nq = p.q_len[r], sk = p.skip[r];
  const int o0 = p.sel_start[r], o1 = p.sel_start[r + 1];
  // (a keep_start that does not match the rule must not send a store outside the list)
  for (int i = threadIdx.x; i < sk; i += 256)
    if (o0 + i >= 0 && o0 + i < total_keep) out[o0 + i] = s + i;
  for (int j = threadIdx.x; j < nq; j += 256)
    if (o1 - nq + j >= 0 && o1 - nq + j < total_keep) out[o1 - nq + j] = s + N + j;
}

// out[slot, g, :] = in[keep_idx[g][slot], g, :] for K and V; 16 bytes per lane
__global__ void __launch_bounds__(256)
evict_compact_kernel(const uint4 *__restrict__ k, const uint4 *__restrict__ v, const int *__restrict__ keep_idx,
                     int total_keep, int Hkv, int vec_per_head, uint4 *__restrict__ k_out, uint4 *__restrict__ v_out) {
  const long i = (long)blockIdx.x * 256 + threadIdx.x;
  const long per_slot = (long)Hkv * vec_per_head;
  if (i >= (long)total_keep * per_slot) return;
  const int slot = (int)(i / per_slot), rem = (int)(i % per_slot);
  const int g = rem / vec_per_head;
  const long src = (long)keep_idx[(size_t)g * total_keep + slot] * per_slot + rem;
  k_out[i] = k[src];
  v_out[i] = v[src];
}

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
  const topk_problem prob{L->seg_start, L->ctx_len, sel_start, nullptr, nullptr, 0, 0};
  return topk_launch(L, scores, prob, 1, sel_idx, (hipStream_t)stream, "a3_topk_select");
}

extern "C" size_t a3_evict_ws_bytes(const a3_layout *L) {
  if (L == nullptr || L->n_kv_heads <= 0 || L->total_tokens < 0) return 0;
  return a3_align_up((size_t)L->n_kv_heads * L->total_tokens * sizeof(float), 256) + 256;
}

extern "C" a3_status a3_evict_select(const a3_layout *L, const float *votes, const int *sys_len, const int *keep_start,
                                     int total_keep, int pool_width, int pool_mode, int *keep_idx, void *ws,
                                     size_t ws_bytes, void *stream) {
  a3_status s = a3_check_layout(L, "a3_evict_select", true);
  if (s != A3_OK) return s;
  A3_REQUIRE(total_keep >= 0 && total_keep <= L->total_tokens, A3_ERR_INVALID_ARG,
             "a3_evict_select: total_keep %d outside [0, %d]", total_keep, L->total_tokens);
  A3_REQUIRE(votes && sys_len && keep_start, A3_ERR_INVALID_ARG, "a3_evict_select: votes/sys_len/keep_start is NULL");
  A3_REQUIRE(pool_width >= 1 && pool_width % 2 == 1 && pool_width <= 63, A3_ERR_INVALID_ARG,
             "a3_evict_select: pool_width %d is not an odd number in [1, 63]", pool_width);
  A3_REQUIRE(pool_mode == A3_POOL_MAX || pool_mode == A3_POOL_AVG, A3_ERR_INVALID_ARG,
             "a3_evict_select: pool_mode %d", pool_mode);
  if (total_keep == 0 || L->n_req == 0) return A3_OK;
  A3_REQUIRE(keep_idx, A3_ERR_INVALID_ARG, "a3_evict_select: keep_idx is NULL");
  hipStream_t st = (hipStream_t)stream;
  const float *ranked = votes;
  if (pool_width > 1) {
    A3_REQUIRE(ws != nullptr && ws_bytes >= a3_evict_ws_bytes(L), A3_ERR_WORKSPACE,
               "a3_evict_select: workspace %zu bytes, need %zu", ws_bytes, a3_evict_ws_bytes(L));
    float *pooled = (float *)ws;
    hipLaunchKernelGGL(pool_votes_kernel, dim3((L->total_tokens + 255) / 256, L->n_kv_heads), dim3(256), 0, st, votes,
                       pooled, L->tok_req, L->tok_chunk, L->seg_start, L->ctx_len, L->total_tokens, pool_width,
                       pool_mode);
    ranked = pooled;
  }
  const topk_problem prob{L->seg_start, L->ctx_len, keep_start, sys_len, L->q_len, (long)L->total_tokens,
                          (long)total_keep};
  hipLaunchKernelGGL(evict_fixed_rows_kernel, dim3(L->n_req, L->n_kv_heads), dim3(256), 0, st, prob, total_keep, keep_idx);
  return topk_launch(L, ranked, prob, L->n_kv_heads, keep_idx, st, "a3_evict_select");
}

extern "C" a3_status a3_evict_compact(const a3_layout *L, const void *k_fused, const void *v_fused, const int *keep_idx,
                                      int total_keep, void *k_out, void *v_out, void *stream) {
  a3_status s = a3_check_layout(L, "a3_evict_compact", false);
  if (s != A3_OK) return s;
  A3_REQUIRE(total_keep >= 0 && total_keep <= L->total_tokens, A3_ERR_INVALID_ARG,
             "a3_evict_compact: total_keep %d outside [0, %d]", total_keep, L->total_tokens);
  if (total_keep == 0) return A3_OK;
  A3_REQUIRE(k_fused && v_fused && keep_idx && k_out && v_out, A3_ERR_INVALID_ARG, "a3_evict_compact: NULL tensor");
  A3_REQUIRE(a3_aligned16(k_fused) && a3_aligned16(v_fused) && a3_aligned16(k_out) && a3_aligned16(v_out),
             A3_ERR_INVALID_ARG, "a3_evict_compact: tensors must be 16-byte aligned");
  const int head_bytes = L->head_dim * (L->dtype == A3_BF16 ? 2 : 4);
  A3_REQUIRE(head_bytes % 16 == 0, A3_ERR_UNSUPPORTED, "a3_evict_compact: a head row of %d bytes", head_bytes);
  const long n = (long)total_keep * L->n_kv_heads * (head_bytes / 16);
  hipLaunchKernelGGL(evict_compact_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, (hipStream_t)stream,
                     (const uint4 *)k_fused, (const uint4 *)v_fused, keep_idx, total_keep, L->n_kv_heads, head_bytes / 16,
                     (uint4 *)k_out, (uint4 *)v_out);
  A3_CHECK_LAUNCH("a3_evict_compact");
  return A3_OK;
}

// Step 3 -> the rows [Re, Q] -> the layout of the attention's work, as one call: what a3_topk_select,
// a3_active_rows and a3_attention_plan do one after the other.  A batch of one request takes a single launch
// (the workgroup that ranks the request goes on to write the row list and the plan); larger batches run the
// three kernels.
extern "C" a3_status a3_topk_select_plan(const a3_layout *L, const float *scores, const int *sel_start, int total_k,
                                         int *sel_idx, int n_act, int *act_idx, void *ws, size_t ws_bytes,
                                         void *stream) {
  a3_status s = a3_check_layout(L, "a3_topk_select_plan", true);
  if (s != A3_OK) return s;
  A3_REQUIRE(total_k >= 0 && n_act >= total_k && n_act <= L->total_tokens, A3_ERR_INVALID_ARG,
             "a3_topk_select_plan: total_k %d, n_act %d (of %d rows)", total_k, n_act, L->total_tokens);
  A3_REQUIRE(scores && sel_start && act_idx && (sel_idx || total_k == 0), A3_ERR_INVALID_ARG,
             "a3_topk_select_plan: NULL argument");
  const bool one = L->n_req == 1 && L->dtype == A3_BF16 && L->max_ctx_len <= kMaxLdsKeys && total_k > 0 && n_act > 0;
  if (!one) {
    A3_REQUIRE(sel_idx != act_idx || L->n_req == 1, A3_ERR_INVALID_ARG,
               "a3_topk_select_plan: sel_idx may only be act_idx itself in a batch of one request");
    s = a3_topk_select(L, scores, sel_start, total_k, sel_idx, nullptr, 0, stream);
    if (s != A3_OK) return s;
    if (sel_idx == act_idx) {
      // one request, selection already at the head of act_idx: only the question rows are missing
      int *tmp = act_idx;   // a3_active_rows reads sel_idx[j] and writes act_idx[j] for the same j: in place is fine
      s = a3_active_rows(L, tmp, sel_start, n_act, act_idx, stream);
    } else {
      s = a3_active_rows(L, sel_idx, sel_start, n_act, act_idx, stream);
    }
    if (s != A3_OK) return s;
    return a3_attention_plan(L, act_idx, n_act, ws, ws_bytes, stream);
  }
  A3_REQUIRE((long long)total_k <= (long long)L->max_ctx_len, A3_ERR_INVALID_ARG,
             "a3_topk_select_plan: total_k %d exceeds the number of context rows", total_k);
  A3_REQUIRE(ws != nullptr && ws_bytes >= a3_attn_ws_bytes(L, n_act), A3_ERR_WORKSPACE,
             "a3_topk_select_plan: workspace %zu bytes, need %zu", ws_bytes, a3_attn_ws_bytes(L, n_act));
  attn_plan plan;
  attn_plan_carve(L, n_act, ws, ws_bytes, &plan);
  topk_problem prob{L->seg_start, L->ctx_len, sel_start, nullptr, nullptr, 0, 0};
  if (L->max_ctx_len + L->max_q_len == L->total_tokens) {   // the one request's lengths are the layout's maxima
    prob.one_N = L->max_ctx_len;
    prob.one_k = total_k;
  }
  const size_t lds = ((size_t)L->max_ctx_len + L->max_ctx_len / 32 + 1) * sizeof(uint32_t);
  static a3_once_per_device lds_once;
  const hipError_t once_err = a3_once(lds_once, []() {
    const int cap = (int)((kMaxLdsKeys + kMaxLdsKeys / 32 + 1) * sizeof(uint32_t));
    hipError_t e1 = hipFuncSetAttribute((const void *)topk_select_plan_kernel<4>, hipFuncAttributeMaxDynamicSharedMemorySize, cap);
    hipError_t e2 = hipFuncSetAttribute((const void *)topk_select_plan_kernel<16>, hipFuncAttributeMaxDynamicSharedMemorySize, cap);
    hipError_t e3 = hipFuncSetAttribute((const void *)topk_select_plan_kernel<36>, hipFuncAttributeMaxDynamicSharedMemorySize, cap);
    return e1 != hipSuccess ? e1 : (e2 != hipSuccess ? e2 : e3);
  });
  if (once_err != hipSuccess) return a3_fail(A3_ERR_HIP, "a3_topk_select_plan: cannot raise the dynamic LDS limit");
  hipStream_t st = (hipStream_t)stream;
  const int G = L->n_q_heads / L->n_kv_heads, wgs = plan.max_wgs, cost = attn_item_cost();
  const int per = (L->max_ctx_len + kBlock - 1) / kBlock;
  if (per <= 4)
    hipLaunchKernelGGL(topk_select_plan_kernel<4>, dim3(1), dim3(kBlock), lds, st, scores, prob, sel_idx, act_idx, n_act, plan, G, wgs, cost, (int)(lds / sizeof(int)));
  else if (per <= 16)
    hipLaunchKernelGGL(topk_select_plan_kernel<16>, dim3(1), dim3(kBlock), lds, st, scores, prob, sel_idx, act_idx, n_act, plan, G, wgs, cost, (int)(lds / sizeof(int)));
  else
    hipLaunchKernelGGL(topk_select_plan_kernel<36>, dim3(1), dim3(kBlock), lds, st, scores, prob, sel_idx, act_idx, n_act, plan, G, wgs, cost, (int)(lds / sizeof(int)));
  A3_CHECK_LAUNCH("a3_topk_select_plan");
  return A3_OK;
}
