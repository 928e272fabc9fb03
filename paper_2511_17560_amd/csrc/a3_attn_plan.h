// The layout of the attention's work (Eq. 4 / Eq. 5, last line): which workgroup attends which part of which tile
// of active rows.  It depends only on the list of active rows, so it is made right behind the selection (one
// workgroup) - by a kernel of its own, or at the tail of the kernel that selects (a3_topk.hip).  Shared by
// a3_attn.hip and a3_topk.hip; device code is inlined into both (no relocatable device code).
#pragma once

#include "a3_internal.h"

namespace {

constexpr int kTM = 256;            // packed (row, head) pairs per work item: 32 per wave of the attention kernel
constexpr int kTK = 64;             // keys per tile
constexpr int kPlanThreads = 1024;
constexpr int kPlanLdsInts = 4096;  // LDS the plan kernel sets aside for the plan's small arrays (16 KB)

// Work decomposition written by the plan kernel.
//   tile  = 256 consecutive packed (row, head) pairs of one request and one KV head group; it needs
//           ceil(visible keys of its last row / 64) key steps
//   The key steps of all tiles, laid end to end, are cut into P equal shares, one per workgroup of a
//   KV head (P = workgroups per head, at most one share per 8 steps): every workgroup gets the same
//   amount of work whatever the mix of short and long tiles.
//   item  = the part of one share that lies in one tile: (tile, k_begin, k_end).  A tile that lies inside
//           one share is finished by that workgroup; the others are cut into 2 or more items whose
//           unnormalised partial results are merged afterwards, in key order.
struct attn_plan {
  int *a_lo;         // [n_req+1] first active row of each request
  int *tile_start;   // [n_req+1] first tile of each request
  int4 *tile_a;      // [max_tiles] (request, first m, visible keys of the last row, rows*G of the request)
  int2 *tile_b;      // [max_tiles] (first item, number of items)
  int *tile_pre;     // [max_tiles+1] key steps of all earlier tiles
  int4 *items;       // [max_items] (tile, k_begin, k_end, 0), in work order
  int *wg_start;     // [max_wgs+1] first item of each workgroup of a head
  int *counters;     // n_tiles, n_items, P, max_wgs the plan was made with (first in the workspace: its place
                     // does not depend on the sizes of the other arrays)
  float *part_o;     // [Hkv * max_items][256][128] unnormalised partial O of cut tiles
  float2 *part_ml;   // [Hkv * max_items][256]      (exponent reference in the exp2 domain, sum)
  int max_tiles, max_items, max_wgs;
};

__device__ __forceinline__ int lower_bound_i32(const int *__restrict__ a, int n, int x) {
  int lo = 0, hi = n;            // first index with a[i] >= x
  while (lo < hi) {
    int mid = (lo + hi) >> 1;
    if (a[mid] < x) lo = mid + 1; else hi = mid;
  }
  return lo;
}
__device__ __forceinline__ int upper_bound_i32(const int *a, int n, int x) {
  int lo = 0, hi = n;            // first index with a[i] > x
  while (lo < hi) {
    int mid = (lo + hi) >> 1;
    if (a[mid] <= x) lo = mid + 1; else hi = mid;
  }
  return lo;
}

// exclusive prefix sum over the workgroup (threads in tid order); *total receives the sum
__device__ __forceinline__ int plan_scan(int v, int *wave_tot, int *total) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  int inc = v;
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    int x = __shfl_up(inc, off, 64);
    if (lane >= off) inc += x;
  }
  __syncthreads();               // wave_tot may still be read by a previous scan
  if (lane == 63) wave_tot[wave] = inc;
  __syncthreads();
  int before = 0, all = 0;
  for (int w2 = 0; w2 < kPlanThreads / 64; ++w2) { if (w2 < wave) before += wave_tot[w2]; all += wave_tot[w2]; }
  *total = all;
  return before + inc - v;
}

// The whole plan, by one workgroup of kPlanThreads threads.  wave_tot: [kPlanThreads / 64] ints of LDS.
// lds: lds_ints ints of LDS.  The searches below each are a chain of dependent reads; when the small arrays they
// run over (row range and first tile of each request, running cost and key count of each tile) fit there, they
// are kept in LDS beside their copies in the workspace (which the attention kernels read) and the chains run
// at LDS latency instead of a round trip to the L2 per step.
__device__ __forceinline__ void attn_plan_body(const attn_plan &p, const int *act_idx, int n_act,
                                               const int *__restrict__ seg_start, int n_req, int G, int wgs_per_head,
                                               int item_cost, int *wave_tot, int *lds, int lds_ints) {
  const int tid = threadIdx.x;
  const bool in_lds = 2 * (n_req + 1) + 2 * p.max_tiles + 1 <= lds_ints;
  int *a_lo = in_lds ? lds : p.a_lo;
  int *tile_start = in_lds ? lds + (n_req + 1) : p.tile_start;
  int *tile_pre = in_lds ? lds + 2 * (n_req + 1) : p.tile_pre;
  int *tile_kv = in_lds ? lds + 2 * (n_req + 1) + p.max_tiles + 1 : nullptr;
  // active rows are ascending, so the rows of request r are a contiguous range found by bisection (a batch of one
  // request: all of them)
  for (int r = tid; r <= n_req; r += kPlanThreads) {
    const int v = r == n_req ? n_act : (r == 0 && n_req == 1 ? 0 : lower_bound_i32(act_idx, n_act, seg_start[r]));
    a_lo[r] = v;
    if (in_lds) p.a_lo[r] = v;
  }
  __syncthreads();
  if (tid == 0) {
    int t = 0;
    for (int r = 0; r < n_req; ++r) {
      tile_start[r] = t;
      if (in_lds) p.tile_start[r] = t;
      t += ((a_lo[r + 1] - a_lo[r]) * G + kTM - 1) / kTM;
    }
    tile_start[n_req] = t;
    if (in_lds) p.tile_start[n_req] = t;
  }
  __syncthreads();
  const int n_tiles = min(tile_start[n_req], p.max_tiles);

  // ---- tiles and their running cost -------------------------------------------------------
  // A tile is laid out as `item_cost` units of start-up (fetching its queries and first keys, storing its
  // result: measured at six to seven key steps) followed by one unit per key step.
  int carry = 0;
  for (int base = 0; base < n_tiles; base += kPlanThreads) {
    const int t = base + tid;
    int steps = 0;
    if (t < n_tiles) {
      const int r = upper_bound_i32(tile_start, n_req, t) - 1;       // last r with tile_start[r] <= t
      const int j = t - tile_start[r];
      const int nr = a_lo[r + 1] - a_lo[r];
      int last = ((j + 1) * kTM - 1) / G;
      if (last > nr - 1) last = nr - 1;
      const int kv = act_idx[a_lo[r] + last] - seg_start[r] + 1;
      steps = (kv + kTK - 1) / kTK;
      p.tile_a[t] = make_int4(r, j * kTM, kv, nr * G);
      if (in_lds) tile_kv[t] = kv;
    }
    int total;
    const int before = plan_scan(t < n_tiles ? steps + item_cost : 0, wave_tot, &total);
    if (t < n_tiles) {
      tile_pre[t] = carry + before;
      if (in_lds) p.tile_pre[t] = carry + before;
    }
    carry += total;
  }
  const int W = carry;                                       // cost of one head, >= n_tiles
  if (tid == 0) {
    tile_pre[n_tiles] = W;
    if (in_lds) p.tile_pre[n_tiles] = W;
  }
  __syncthreads();

  // ---- equal shares ------------------------------------------------------------------------
  int P = (W - n_tiles * item_cost + 7) / 8;                  // at least 8 key steps per share
  if (P > wgs_per_head) P = wgs_per_head;
  if (P > p.max_wgs) P = p.max_wgs;
  if (P < 1) P = 1;
  int t0 = 0, cnt = 0;
  long long s_beg = 0, s_end = 0;
  if (tid < P && W > 0) {
    s_beg = (long long)tid * W / P;
    s_end = (long long)(tid + 1) * W / P;
    if (s_end > s_beg) {
      t0 = upper_bound_i32(tile_pre, n_tiles + 1, (int)s_beg) - 1;      // tile that holds position s_beg
      const int t1 = lower_bound_i32(tile_pre, n_tiles + 1, (int)s_end) - 1;     // ... and position s_end - 1
      // the last tile only counts if the share reaches past its start-up units
      cnt = t1 - t0 + 1 - (s_end <= (long long)tile_pre[t1] + item_cost ? 1 : 0);
    }
  }
  int n_items;
  const int first = plan_scan(cnt, wave_tot, &n_items);
  if (tid < P) p.wg_start[tid] = min(first, p.max_items);
  if (tid == 0) p.wg_start[P] = min(n_items, p.max_items);
  for (int i = 0; i < cnt; ++i) {
    const int t = t0 + i, idx = first + i;
    if (idx >= p.max_items) break;
    const int pre = tile_pre[t] + item_cost, nxt = tile_pre[t + 1];      // key step s of the tile sits at pre + s
    const int it_b = (int)(s_beg > pre ? s_beg - pre : 0), it_e = (int)((s_end < nxt ? s_end : nxt) - pre);
    const int kv = in_lds ? tile_kv[t] : p.tile_a[t].z;
    p.items[idx] = make_int4(t, it_b * kTK, min(kv, it_e * kTK), 0);
    if (it_b == 0) p.tile_b[t].x = idx;
  }
  // items of a tile = share boundaries strictly inside it + 1; boundary q lies at floor(q W / P)
  for (int t = tid; t < n_tiles; t += kPlanThreads) {
    const long long x = (long long)tile_pre[t] + item_cost, y = tile_pre[t + 1];
    const long long ub = ((x + 1) * P + W - 1) / W;          // first q with floor(q W / P) > x
    const long long lb = (y * P + W - 1) / W;                // first q with floor(q W / P) >= y
    p.tile_b[t].y = (int)(lb > ub ? lb - ub : 0) + 1;
  }
  if (tid == 0) {
    p.counters[0] = n_tiles;
    p.counters[1] = min(n_items, p.max_items);
    p.counters[2] = P;
    p.counters[3] = p.max_wgs;
  }
}


int attn_max_tiles(const a3_layout *L, int n_act) {
  const int G = L->n_q_heads / L->n_kv_heads;
  return (int)(((long long)n_act * G + kTM - 1) / kTM) + L->n_req;
}

// Workgroups per KV head: one per CU over all heads (256 CUs), or the tuning value "attn_wgs".
int attn_wgs_per_head(const a3_layout *L) {
  int w = (256 + L->n_kv_heads - 1) / L->n_kv_heads;
  const int v = a3_knob(A3_KNOB_ATTN_WGS);
  if (v >= 1 && v <= kPlanThreads) w = v;
  return w;
}

// Start-up cost of an item in key steps (what the share boundaries are balanced with), or the tuning
// value "attn_item_cost".
int attn_item_cost() {
  const int v = a3_knob(A3_KNOB_ATTN_ITEM_COST);
  return v >= 0 && v <= 64 ? v : 7;
}

// every tile starts an item, every share boundary inside a tile starts another
int attn_max_items(const a3_layout *L, int n_act) { return attn_max_tiles(L, n_act) + attn_wgs_per_head(L); }


// carves the plan's arrays out of the workspace (the same way in every call that shares a plan)
inline void attn_plan_carve(const a3_layout *L, int n_act, void *ws, size_t ws_bytes, attn_plan *p) {
  const int max_tiles = attn_max_tiles(L, n_act), max_items = attn_max_items(L, n_act);
  const int wgs_per_head = attn_wgs_per_head(L);
  const int Hkv = L->n_kv_heads;
  a3_ws_cursor cur(ws, ws_bytes);
  p->counters = (int *)cur.take(4 * sizeof(int));
  p->a_lo = (int *)cur.take((size_t)(L->n_req + 1) * sizeof(int));
  p->tile_start = (int *)cur.take((size_t)(L->n_req + 1) * sizeof(int));
  p->tile_a = (int4 *)cur.take((size_t)max_tiles * sizeof(int4));
  p->tile_b = (int2 *)cur.take((size_t)max_tiles * sizeof(int2));
  p->tile_pre = (int *)cur.take((size_t)(max_tiles + 1) * sizeof(int));
  p->items = (int4 *)cur.take((size_t)max_items * sizeof(int4));
  p->wg_start = (int *)cur.take((size_t)(wgs_per_head + 1) * sizeof(int));
  p->part_o = (float *)cur.take((size_t)max_items * Hkv * kTM * 128 * sizeof(float));
  p->part_ml = (float2 *)cur.take((size_t)max_items * Hkv * kTM * sizeof(float2));
  p->max_tiles = max_tiles; p->max_items = max_items; p->max_wgs = wgs_per_head;
}

}  // namespace
