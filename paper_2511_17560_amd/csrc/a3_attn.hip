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
#include <stdlib.h>
#include <string.h>

#include "a3_internal.h"
#include "a3_attn_plan.h"

namespace {

constexpr float kLog2e = 1.4426950408889634f;
constexpr int kD = 128;
constexpr int kAttnWaves = kTM / 32;   // waves per workgroup: 0-3 also stage the next K/V tile
constexpr int kAttnThreads = 64 * kAttnWaves;
constexpr int kKRowBytes = kD * 2;   // K tile  [key][d]   256-byte rows, unpadded; 16-byte pieces XOR-swizzled by key % 16
constexpr int kVStride = kTK + 8;   // V^T tile [d][key]  row stride in elements (144 B)
constexpr int kKTile = kTK * kD;     // elements
constexpr int kVTile = kD * kVStride;
constexpr size_t kAttnLds = (size_t)2 * (kKTile + kVTile) * sizeof(bf16_t);   // double buffered: 69632 B

__global__ void __launch_bounds__(kPlanThreads)
attn_plan_kernel(attn_plan p, const int *__restrict__ act_idx, int n_act, const int *__restrict__ seg_start,
                 int n_req, int G, int wgs_per_head, int item_cost) {
  __shared__ int wave_tot[kPlanThreads / 64];
  __shared__ int small[kPlanLdsInts];
  attn_plan_body(p, act_idx, n_act, seg_start, n_req, G, wgs_per_head, item_cost, wave_tot, small, kPlanLdsInts);
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

// v_exp_f32: 2^x, about 1 ulp, -inf -> 0, results below the normal range flush to 0
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
// Combine a value across the two 32-lane halves of the wave with v_permlane32_swap (no LDS round
// trip): after the swap one result holds the low-half values in every lane and the other the
// high-half values, so max / sum of the two results is the combined value in all 64 lanes.
__device__ __forceinline__ float halves_max(float x) {
  const uint32_t u = __float_as_uint(x);
  auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float halves_sum(float x) {
  const uint32_t u = __float_as_uint(x);
  auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}
__device__ __forceinline__ uint32_t pack_lo(uint32_t a, uint32_t b) { return (a & 0xffffu) | (b << 16); }
__device__ __forceinline__ uint32_t pack_hi(uint32_t a, uint32_t b) { return (a >> 16) | (b & 0xffff0000u); }

// One workgroup per share of a KV head's work: it runs the items of its share in order.
__global__ void __launch_bounds__(kAttnThreads, 1)
attn_bf16_kernel(attn_args a) {
  extern __shared__ __align__(16) unsigned char lds_raw[];
  bf16_t *Ks = reinterpret_cast<bf16_t *>(lds_raw);          // [2][64][128], swizzled
  bf16_t *Vt = Ks + 2 * kKTile;                              // [2][128][kVStride]

  const int g = blockIdx.x % a.Hkv, wg = blockIdx.x / a.Hkv;
  // a plan made with another number of workgroups per head lies elsewhere in the workspace: touch nothing
  if (a.plan.counters[3] != a.plan.max_wgs || wg >= a.plan.counters[2]) return;
  const int item_begin = a.plan.wg_start[wg], item_end = a.plan.wg_start[wg + 1];
  const int G = a.Hq / a.Hkv;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, lhi = lane >> 5;
  const bf16_t *__restrict__ Q = (const bf16_t *)a.q;
  const bf16_t *__restrict__ K = (const bf16_t *)a.k;
  const bf16_t *__restrict__ V = (const bf16_t *)a.v;
  const float c2 = a.scale2;

  // K tile: global memory -> LDS directly (global_load_lds, 16 bytes per lane, lane i lands at base + 16 i).
  // One wave instruction brings 4 keys x 256 B; instruction j of wave w < 4 covers keys 4 (4 j + w) .. +3.
  // The lane fetches piece (slot ^ key % 16) of its key, so LDS slot s of key r holds piece s ^ (r % 16)
  // and the 16 keys a quarter wave reads at one piece index touch all 64 banks once.
  const int dwave = wave & 3;                                // K loads are issued by waves 0..3
  const int drow = 4 * dwave + (lane >> 4);                  // key of the lane in instruction 0
  const int dpiece = (lane & 15) ^ (drow & 15);              // (4 (4 j + w) + lane/16) % 16 does not depend on j
  const uint32_t lds_k = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char *)lds_raw;
  // fragment read: key b*32 + l32, piece 2 ks + lhi -> slot (2 ks + lhi) ^ (l32 % 16)
  const int kfrag = l32 * kKRowBytes, kswz = (lhi ^ (l32 & 15)) * 16;
  // V tile: lane = (4 keys, 8 dims), transposed in registers on its way into LDS.
  // 16 consecutive lanes take 16 different key groups: their 8-byte transposed stores land in 128
  // contiguous bytes of one V^T row (all 32 LDS banks) instead of 16 rows at a bank-aligned stride
  // Both tiles are staged by waves 0..3: the SIMD serves the older of its two waves first, so these
  // waves run ahead of waves 4..7 and would otherwise idle at the barrier of every tile
  const int vkg = tid & 15, vc = (tid & 255) >> 4;
  const int vpos = ((4 * vkg) & ~12) | (((4 * vkg) & 4) << 1) | (((4 * vkg) & 8) >> 1);   // swap key bits 2 and 3

  for (int item = item_begin; item < item_end; ++item) {
    __syncthreads();                                       // the LDS tiles of the previous item are free
    const int4 it = a.plan.items[item];
    const int4 ta = a.plan.tile_a[it.x];
    const int nseg = a.plan.tile_b[it.x].y;
    const int r = ta.x, m0 = ta.y, kv_len = ta.z, m_end = ta.w;
    const int k_begin = it.y, k_end = it.z;
    const int a0 = a.plan.a_lo[r];
    const int base = a.seg_start[r];

    // this lane's query row
    const int m = m0 + wave * 32 + l32;
    const bool valid = m < m_end;
    const int mc = valid ? m : m_end - 1;
    const int arow = a0 + mc / G, hq = g * G + mc % G;
    const int limit = a.act_idx[arow] - base;              // last visible key (request-relative)
    int wave_min_limit = limit, wave_max_limit = limit;
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
      wave_min_limit = min(wave_min_limit, __shfl_xor(wave_min_limit, off, 64));
      wave_max_limit = max(wave_max_limit, __shfl_xor(wave_max_limit, off, 64));
    }

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
    float row_ref = -INFINITY, row_sum = 0.f;               // exponent reference in raw logit units

    // Next tile staged in registers while the current one is being consumed.  Loads are branch
    // free (rows past the last visible key are clamped onto it and masked later) so that nothing
    // forces the loaded registers to be touched before the LDS store at the end of the iteration.
    uint4 vr_0, vr_1, vr_2, vr_3;
    const uint32_t pitch_b = (uint32_t)a.Hkv * kD * sizeof(bf16_t);
    const char *kb = reinterpret_cast<const char *>(K + ((size_t)base * a.Hkv + g) * kD);
    const char *vb = reinterpret_cast<const char *>(V + ((size_t)base * a.Hkv + g) * kD);
    const uint32_t k_last = (uint32_t)(kv_len - 1) * pitch_b + dpiece * 16, v_last = (uint32_t)(kv_len - 1) * pitch_b + vc * 16;
    const uint32_t ko_0 = (uint32_t)drow * pitch_b + dpiece * 16;
    const uint32_t vo_0 = (uint32_t)(4 * vkg) * pitch_b + vc * 16, vo_1 = vo_0 + pitch_b, vo_2 = vo_0 + 2 * pitch_b,
                   vo_3 = vo_0 + 3 * pitch_b;
    // Inline assembly on purpose: the compiler then neither treats these as LDS writes (it would wait
    // for all of them before every LDS read) nor moves memory accesses across them.  They are issued
    // right after the V loads of the same tile: the hardware counter the compiler waits on before
    // using the V registers counts them too, so that wait (which ends at zero, just before the
    // barrier that publishes the tile) covers them; issued before the V loads they would instead
    // be waited for at the top of the loop, where the compiler guards the reuse of the V registers.
#define A3_KDMA(BUF, K0)                                                                                     \
    _Pragma("unroll") for (int j = 0; j < 4; ++j) {                                                          \
      const char *gp_ = kb + min(ko_0 + ((uint32_t)(K0) + 16u * j) * pitch_b, k_last);                       \
      asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off"                                     \
                   :: "s"(__builtin_amdgcn_readfirstlane(lds_k + (BUF) * (kKTile * 2) + 4 * (4 * j + dwave) * kKRowBytes)), \
                      "v"(gp_) : "memory");                                                                  \
    }
#define A3_GLOAD(K0)                                                                       \
    {                                                                                      \
      const uint32_t t_off = (uint32_t)(K0) * pitch_b;                                     \
      vr_0 = *reinterpret_cast<const uint4 *>(vb + min(vo_0 + t_off, v_last));             \
      vr_1 = *reinterpret_cast<const uint4 *>(vb + min(vo_1 + t_off, v_last));             \
      vr_2 = *reinterpret_cast<const uint4 *>(vb + min(vo_2 + t_off, v_last));             \
      vr_3 = *reinterpret_cast<const uint4 *>(vb + min(vo_3 + t_off, v_last));             \
    }
#define A3_V_TRANSPOSE_STORE(VD, W, C)                                                                       \
    {                                                                                                        \
      uint2 even = make_uint2(pack_lo(vr_0.C, vr_1.C), pack_lo(vr_2.C, vr_3.C)); /* dim 8vc+2W,   4 keys */  \
      uint2 odd = make_uint2(pack_hi(vr_0.C, vr_1.C), pack_hi(vr_2.C, vr_3.C));  /* dim 8vc+2W+1, 4 keys */  \
      *reinterpret_cast<uint2 *>((VD) + (8 * vc + 2 * W) * kVStride + vpos) = even;                          \
      *reinterpret_cast<uint2 *>((VD) + (8 * vc + 2 * W + 1) * kVStride + vpos) = odd;                       \
    }
#define A3_LSTORE(BUF)                                                                                       \
    {                                                                                                        \
      bf16_t *vd = Vt + (BUF) * kVTile;                                                                      \
      A3_V_TRANSPOSE_STORE(vd, 0, x)                                                                         \
      A3_V_TRANSPOSE_STORE(vd, 1, y)                                                                         \
      A3_V_TRANSPOSE_STORE(vd, 2, z)                                                                         \
      A3_V_TRANSPOSE_STORE(vd, 3, w)                                                                         \
    }

    if (k_begin < k_end) {
      if (wave < 4) {
        A3_GLOAD(k_begin)
        A3_KDMA(0, k_begin)
        A3_LSTORE(0)
      }
    }
    // Everything loaded so far (Q fragments, first tile) has arrived: inside the loop the compiler's
    // waits then only concern the V registers of the loop itself.  (Its counter arithmetic does not
    // know about the direct-to-LDS loads; a pending Q load would make it wait for fresh V loads
    // in the middle of the MFMAs.)
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();
    int buf = 0;
    for (int k0 = k_begin; k0 < k_end; k0 += kTK, buf ^= 1) {
      const bool more = k0 + kTK < k_end;
      if (wave < 4) {
        A3_GLOAD(k0 + kTK)                                   // next tile: in flight during everything below
        if (more) { A3_KDMA(buf ^ 1, k0 + kTK) }
      }
      // The tile's keys run up to the last row of the workgroup's 256; a wave whose own rows all end before
      // the tile has nothing in it (every P would be 0) and only takes part in the staging and the barrier.
      if (k0 <= wave_max_limit) {
      const unsigned char *kt = reinterpret_cast<const unsigned char *>(Ks) + buf * (kKTile * 2) + kfrag;
      const bf16_t *vt = Vt + buf * kVTile + l32 * kVStride + lhi * 8;

      // ---- S^T = K Q^T : two 32-key blocks, K fragments read one step ahead -----------------
      f32x16 st[2];
#pragma unroll
      for (int b = 0; b < 2; ++b)
#pragma unroll
        for (int x = 0; x < 16; ++x) st[b][x] = 0.f;
      // The scheduling barriers pin the order "reads of step ks + 1, then MFMAs of step ks": left alone
      // the compiler sinks every read to just before its use and the LDS latency is exposed
      bf16x8 kf[2][2];
#pragma unroll
      for (int b = 0; b < 2; ++b)
        kf[0][b] = *reinterpret_cast<const bf16x8 *>(kt + b * 32 * kKRowBytes + (0 ^ kswz));
#pragma unroll
      for (int ks = 0; ks < kD / 16; ++ks) {
        if (ks + 1 < kD / 16) {
#pragma unroll
          for (int b = 0; b < 2; ++b)
            kf[(ks + 1) & 1][b] = *reinterpret_cast<const bf16x8 *>(kt + b * 32 * kKRowBytes + ((32 * (ks + 1)) ^ kswz));
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int b = 0; b < 2; ++b)
          st[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[ks & 1][b], qf[ks], st[b], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
      }

      // first V^T fragments: their LDS latency hides behind the softmax arithmetic
      bf16x8 vf[2][4];
#pragma unroll
      for (int db = 0; db < 4; ++db)
        vf[0][db] = *reinterpret_cast<const bf16x8 *>(vt + db * 32 * kVStride);

      // ---- online softmax for this lane's row (accumulator x of block b: key k0 + 32b + 8(x/4) + 4 lhi + x%4)
      if (k0 + kTK - 1 > wave_min_limit) {                  // tile touches the causal boundary of some row
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
          for (int x = 0; x < 16; ++x) {
            int key = k0 + 32 * b + 8 * (x >> 2) + 4 * lhi + (x & 3);
            if (key > limit) st[b][x] = -INFINITY;
          }
      }
      float mx = st[0][0];
#pragma unroll
      for (int b = 0; b < 2; ++b)
#pragma unroll
        for (int x = 0; x < 16; ++x) mx = fmaxf(mx, st[b][x]);
      mx = halves_max(mx);
      // Lazy rescaling: the exponent reference `row_ref` only has to stay within 2^8 of the running
      // maximum, not equal to it, so the accumulators are rescaled a handful of times per row
      // instead of whenever the maximum moves (64 multiplies each time).  P then ranges up to 256.
      if (__any((mx - row_ref) * c2 > 8.0f)) {              // also true for the first visible key (-inf reference)
        const float new_ref = fmaxf(row_ref, mx);
        const float alpha = new_ref == -INFINITY ? 1.0f : fast_exp2((row_ref - new_ref) * c2);
        row_ref = new_ref;
        row_sum *= alpha;
#pragma unroll
        for (int b = 0; b < 4; ++b)
#pragma unroll
          for (int x = 0; x < 16; ++x) o[b][x] *= alpha;
      }
      const float nref = row_ref == -INFINITY ? 0.f : -row_ref * c2;   // no visible key yet: every P is 0
      float psum = 0.f;
#pragma unroll
      for (int b = 0; b < 2; ++b)
#pragma unroll
        for (int x = 0; x < 16; ++x) {
          float pv = fast_exp2(fmaf(st[b][x], c2, nref));
          st[b][x] = pv;
          psum += pv;
        }
      row_sum += psum;                                      // per lane half; halves are added at the end

      // ---- O^T += V^T P^T, V^T fragments read one step ahead ------------------------------------
#pragma unroll
      for (int step = 0; step < 4; ++step) {                // step = 2 b + s2: keys 32 b + 16 s2 ..
        if (step + 1 < 4) {
#pragma unroll
          for (int db = 0; db < 4; ++db)
            vf[(step + 1) & 1][db] = *reinterpret_cast<const bf16x8 *>(vt + db * 32 * kVStride + (step + 1) * 16);
        }
        bf16x8 pf;
#pragma unroll
        for (int e = 0; e < 8; ++e) pf[e] = a3_f2bf(st[step >> 1][8 * (step & 1) + e]);
#pragma unroll
        for (int db = 0; db < 4; ++db)
          o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[step & 1][db], pf, o[db], 0, 0, 0);
      }
      }
      if (more) {
        if (wave < 4) {
          A3_LSTORE(buf ^ 1)
          __builtin_amdgcn_s_waitcnt(0x0f70);               // vmcnt(0): this wave's K loads have landed
        }
      }
      __syncthreads();
    }
#undef A3_KDMA
#undef A3_GLOAD
#undef A3_LSTORE
#undef A3_V_TRANSPOSE_STORE

    row_sum = halves_sum(row_sum);
    if (nseg == 1) {
      if (valid) {
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
    } else {
      const size_t pidx = (size_t)g * a.plan.max_items + item;
      const int ml = wave * 32 + l32;
      float *po = a.plan.part_o + (pidx * kTM + ml) * kD;
#pragma unroll
      for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
          f32x4 v;
#pragma unroll
          for (int e = 0; e < 4; ++e) v[e] = o[db][4 * q4 + e];
          *reinterpret_cast<f32x4 *>(po + 32 * db + 8 * q4 + 4 * lhi) = v;
        }
      if (lhi == 0) a.plan.part_ml[pidx * kTM + ml] = make_float2(row_ref * c2, row_sum);
    }
  }
}

// Merges the partial results of tiles that were cut into key segments, in segment order.
// One workgroup per (tile, KV head, quarter of the tile's rows); 8 lanes share a row, 16 dims each.
__global__ void __launch_bounds__(256)
attn_combine_kernel(attn_args a) {
  const int t = blockIdx.x, g = blockIdx.y;
  if (a.plan.counters[3] != a.plan.max_wgs || t >= a.plan.counters[0]) return;
  const int2 tb = a.plan.tile_b[t];
  const int nseg = tb.y;
  if (nseg <= 1) return;
  const int4 ta = a.plan.tile_a[t];
  const int G = a.Hq / a.Hkv;
  const int ml = blockIdx.z * 32 + (threadIdx.x >> 3), d0 = (threadIdx.x & 7) * 16;
  const int m = ta.y + ml;
  if (m >= ta.w) return;
  const int arow = a.plan.a_lo[ta.x] + m / G, hq = g * G + m % G;
  const size_t p0 = (size_t)g * a.plan.max_items + tb.x;
  float M = -INFINITY;
  for (int s = 0; s < nseg; ++s) M = fmaxf(M, a.plan.part_ml[(p0 + s) * kTM + ml].x);
  float acc[16];
#pragma unroll
  for (int i = 0; i < 16; ++i) acc[i] = 0.f;
  float L = 0.f;
  for (int s = 0; s < nseg; ++s) {
    const float2 st = a.plan.part_ml[(p0 + s) * kTM + ml];
    const float wgt = exp2f(st.x - M);                      // 0 for a segment this row sees nothing of
    L += st.y * wgt;
    const f32x4 *po = reinterpret_cast<const f32x4 *>(a.plan.part_o + ((p0 + s) * kTM + ml) * kD + d0);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      f32x4 v = po[i];
#pragma unroll
      for (int e = 0; e < 4; ++e) acc[4 * i + e] = fmaf(v[e], wgt, acc[4 * i + e]);
    }
  }
  const float inv = 1.0f / L;
  bf16_t *orow = (bf16_t *)a.out + ((size_t)arow * a.Hq + hq) * kD + d0;
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    bf16x8 v;
#pragma unroll
    for (int e = 0; e < 8; ++e) v[e] = a3_f2bf(acc[8 * i + e] * inv);
    *reinterpret_cast<bf16x8 *>(orow + 8 * i) = v;
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

}  // namespace

size_t a3_attn_ws_bytes(const a3_layout *L, int max_active_rows) {
  if (L->dtype != A3_BF16) return 256;
  const size_t per_req = a3_align_up((size_t)(L->n_req + 1) * sizeof(int), 256);
  const size_t tiles = attn_max_tiles(L, max_active_rows), items = attn_max_items(L, max_active_rows);
  return 2 * per_req + a3_align_up(tiles * sizeof(int4), 256) + a3_align_up(tiles * sizeof(int2), 256) +
         a3_align_up((tiles + 1) * sizeof(int), 256) + a3_align_up(items * sizeof(int4), 256) +
         a3_align_up((size_t)(attn_wgs_per_head(L) + 1) * sizeof(int), 256) + 256 +
         a3_align_up(items * L->n_kv_heads * kTM * kD * sizeof(float), 256) +
         a3_align_up(items * L->n_kv_heads * kTM * sizeof(float2), 256) + 2048;
}

// parts & 1: lay out the work (plan kernel); parts & 2: attend and merge.  The plan only depends on the list of
// active rows, so a caller may have it made beside whatever else precedes the attention.
static a3_status attn_launch(const a3_layout *L, const void *q_act, const int *act_idx, int n_act,
                             const void *k_fused, const void *v_fused, void *out, void *ws, size_t ws_bytes,
                             void *stream, int parts, hipEvent_t ev_begin = nullptr, hipEvent_t ev_end = nullptr) {
  a3_status s = a3_check_layout(L, "a3_fused_attention", true);
  if (s != A3_OK) return s;
  A3_REQUIRE(n_act >= 0 && n_act <= L->total_tokens, A3_ERR_INVALID_ARG,
             "a3_fused_attention: n_act %d outside [0, %d]", n_act, L->total_tokens);
  if (n_act == 0) return A3_OK;
  A3_REQUIRE(act_idx != nullptr, A3_ERR_INVALID_ARG, "a3_fused_attention: act_idx is NULL");
  if (parts & 2) {
    A3_REQUIRE(q_act && k_fused && v_fused && out, A3_ERR_INVALID_ARG, "a3_fused_attention: NULL argument");
    A3_REQUIRE(a3_aligned16(q_act) && a3_aligned16(k_fused) && a3_aligned16(v_fused) && a3_aligned16(out),
               A3_ERR_INVALID_ARG, "a3_fused_attention: tensors must be 16-byte aligned");
  }
  hipStream_t st = (hipStream_t)stream;
  attn_args a;
  a.q = q_act; a.k = k_fused; a.v = v_fused; a.out = out;
  a.act_idx = act_idx; a.seg_start = L->seg_start; a.tok_req = L->tok_req;
  a.n_act = n_act; a.Hq = L->n_q_heads; a.Hkv = L->n_kv_heads; a.d = L->head_dim;
  a.scale2 = a3_scale_of(L) * kLog2e;
  memset(&a.plan, 0, sizeof(a.plan));
  if (L->dtype == A3_BF16) {
    // the kernel addresses a request's K/V rows with 32-bit byte offsets
    A3_REQUIRE(((long long)L->max_ctx_len + L->max_q_len + 128) * L->n_kv_heads * kD * 2 < (1LL << 32), A3_ERR_UNSUPPORTED,
               "a3_fused_attention: a request of %d rows is too long for 32-bit cache offsets",
               L->max_ctx_len + L->max_q_len);
    A3_REQUIRE(ws != nullptr, A3_ERR_WORKSPACE, "a3_fused_attention: workspace is NULL");
    A3_REQUIRE(ws_bytes >= a3_attn_ws_bytes(L, n_act), A3_ERR_WORKSPACE,
               "a3_fused_attention: workspace %zu bytes, need %zu", ws_bytes, a3_attn_ws_bytes(L, n_act));
    static a3_once_per_device lds_once;
    const hipError_t e = a3_once(lds_once, []() {
      return hipFuncSetAttribute((const void *)attn_bf16_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)kAttnLds);
    });
    if (e != hipSuccess) return a3_fail(A3_ERR_HIP, "a3_fused_attention: %s", hipGetErrorString(e));
    attn_plan_carve(L, n_act, ws, ws_bytes, &a.plan);
    const int wgs_per_head = a.plan.max_wgs, max_tiles = a.plan.max_tiles, Hkv = L->n_kv_heads;
    if (parts & 1)
      hipLaunchKernelGGL(attn_plan_kernel, dim3(1), dim3(kPlanThreads), 0, st, a.plan, act_idx, n_act, L->seg_start,
                         L->n_req, L->n_q_heads / L->n_kv_heads, wgs_per_head, attn_item_cost());
    if (parts & 2) {
      // blockIdx % Hkv = KV head, so with 8 KV heads each XCD's L2 serves the K/V of one head
      if (ev_begin) (void)hipEventRecord(ev_begin, st);
      hipLaunchKernelGGL(attn_bf16_kernel, dim3((unsigned)wgs_per_head * Hkv), dim3(kAttnThreads), kAttnLds, st, a);
      if (ev_end) (void)hipEventRecord(ev_end, st);
      hipLaunchKernelGGL(attn_combine_kernel, dim3((unsigned)max_tiles, Hkv, kTM / 32), dim3(256), 0, st, a);
    }
  } else if (parts & 2) {
    hipLaunchKernelGGL(attn_f32_kernel, dim3(n_act, L->n_q_heads), dim3(256), 0, st, a);
  }
  A3_CHECK_LAUNCH("a3_fused_attention");
  return A3_OK;
}

extern "C" a3_status a3_fused_attention(const a3_layout *L, const void *q_act, const int *act_idx, int n_act,
                                        const void *k_fused, const void *v_fused, void *out, void *ws,
                                        size_t ws_bytes, void *stream) {
  return attn_launch(L, q_act, act_idx, n_act, k_fused, v_fused, out, ws, ws_bytes, stream, 3);
}

extern "C" a3_status a3_attention_plan(const a3_layout *L, const int *act_idx, int n_act, void *ws, size_t ws_bytes,
                                       void *stream) {
  return attn_launch(L, nullptr, act_idx, n_act, nullptr, nullptr, nullptr, ws, ws_bytes, stream, 1);
}

extern "C" a3_status a3_fused_attention_planned(const a3_layout *L, const void *q_act, const int *act_idx, int n_act,
                                                const void *k_fused, const void *v_fused, void *out, void *ws,
                                                size_t ws_bytes, void *stream) {
  return attn_launch(L, q_act, act_idx, n_act, k_fused, v_fused, out, ws, ws_bytes, stream, 2);
}

// a3_fused_attention_planned with two HIP events recorded on the stream right before and right after the main
// kernel (the merge of the partial results follows the second one): for measurements of that kernel alone.
extern "C" a3_status a3_fused_attention_planned_events(const a3_layout *L, const void *q_act, const int *act_idx,
                                                       int n_act, const void *k_fused, const void *v_fused, void *out,
                                                       void *ws, size_t ws_bytes, void *stream, void *ev_main_begin,
                                                       void *ev_main_end) {
  return attn_launch(L, q_act, act_idx, n_act, k_fused, v_fused, out, ws, ws_bytes, stream, 2, (hipEvent_t)ev_main_begin,
                     (hipEvent_t)ev_main_end);
}
