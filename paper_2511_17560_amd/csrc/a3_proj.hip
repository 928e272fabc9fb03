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
#include <stdlib.h>

#include "a3_internal.h"
#include "a3_gemm_tile.h"

namespace {

// ---------------------------------------------------------------------------------------
// bf16 MFMA kernel
// ---------------------------------------------------------------------------------------
// The 128 B/clk LDS feeds at most one 16-byte fragment read per 32x32x16 MFMA issued on the CU,
// so a wave has to reuse every fragment several times.  A wave therefore owns one head
// (128 features = 4 blocks) x 32*TB listed rows (TB = 2, 3 or 4 blocks): (4 + TB) fragment reads
// per 4*TB MFMAs, accumulators in up to 256 registers, one wave per SIMD.  The workgroup is
// 2 (heads) x 2 (row halves) waves: 256 features x 64*TB rows, both operands staged through LDS
// with full 128-byte row segments per 8 lanes.  TB is chosen per launch: larger tiles need less
// LDS and L2 traffic per flop, smaller ones fill the 256 CUs better.
// Loads go from global memory straight into LDS (global_load_lds, 16 bytes per lane, no staging
// registers), three 32-wide k-slabs ahead of the MFMAs in a ring of four LDS stages; rows are
// unpadded and the 16-byte pieces of a row are XOR-swizzled against bank conflicts.
constexpr int kHeadDim = 128;
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
  int n_pairs, n_tok_tiles;
  int scatter_kv;        // K and V go to row row_idx[i] of their output (the caches) instead of row i
};

struct head_sel { int which, head, heads_out; };

__device__ __forceinline__ head_sel select_head(int h, int Hq, int Hkv) {
  head_sel r;
  if (h < Hq) { r.which = 0; r.head = h; r.heads_out = Hq; }
  else if (h < Hq + Hkv) { r.which = 1; r.head = h - Hq; r.heads_out = Hkv; }
  else { r.which = 2; r.head = h - Hq - Hkv; r.heads_out = Hkv; }
  return r;
}

template <int TB, bool K64>
__global__ void __launch_bounds__(256, TB == 2 ? 2 : 1)
proj_bf16_kernel(proj_args a) {
  constexpr int kTokTile = 64 * TB;
  extern __shared__ __align__(16) unsigned char lds[];

  // workgroup -> (head pair, row tile).  Consecutive workgroup ids go to different XCDs; all row
  // tiles of one head pair are kept on one XCD so its L2 holds that pair's weights.
  const int xcd = blockIdx.x & 7, q = blockIdx.x >> 3;
  const int hp = xcd + 8 * (q / a.n_tok_tiles), tt = q % a.n_tok_tiles;
  if (hp >= a.n_pairs) return;
  const int n_heads = a.Hq + 2 * a.Hkv;
  {
    // a pair whose two heads both have no output (Q-only or K/V-only calls) has nothing to do
    const head_sel h0 = select_head(min(2 * hp, n_heads - 1), a.Hq, a.Hkv);
    const head_sel h1 = select_head(min(2 * hp + 1, n_heads - 1), a.Hq, a.Hkv);
    if (a.out[h0.which] == nullptr && (2 * hp + 1 >= n_heads || a.out[h1.which] == nullptr)) return;
  }
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, lhi = lane >> 5;
  const int fh = wave & 1, th = wave >> 1;

  // ---- this wave's head and rows ---------------------------------------------------------------------
  const int my_head = 2 * hp + fh;
  const head_sel hs = select_head(min(my_head, n_heads - 1), a.Hq, a.Hkv);
  bf16_t *__restrict__ out = my_head < n_heads ? a.out[hs.which] : nullptr;
  const bool compute = out != nullptr;
  const int tok0 = tt * kTokTile + th * 32 * TB;

  // ---- the product: weight-tile row r is row r % 128 of head 2 hp + r / 128, activation-tile row r the
  // hidden row of listed row tt * kTokTile + r
  f32x16 acc[4][TB];
  gemm_tile_mainloop<TB, K64>(
      acc, lds, a.K,
      [&](int row) -> const bf16_t * {
        const head_sel hsl = select_head(min(2 * hp + (row >> 7), n_heads - 1), a.Hq, a.Hkv);
        const bf16_t *wb = a.w[hsl.which];
        int hh = hsl.head;
        if (wb == nullptr) { wb = a.w[0] ? a.w[0] : (a.w[1] ? a.w[1] : a.w[2]); hh = 0; }   // unused head: any valid tile
        return wb + ((size_t)hh * kHeadDim + (row & 127)) * a.K;
      },
      [&](int row) -> const bf16_t * {
        const int m = min(tt * kTokTile + row, a.n_rows - 1);    // clamp: computed but never stored
        return a.hidden + (size_t)(a.row_idx ? a.row_idx[m] : m) * a.K;
      });
  // (a wave whose head has no output multiplies all the same: its partner in the pair sets the pace, and
  // a guard around the MFMAs turns into execution-mask juggling and branches between them)
  // ---- epilogue: bias, RoPE, one rounding, store -------------------------------------------------------
  // In the accumulators a lane holds one row and, per register quad, 4 consecutive features: stored
  // from there, every instruction would touch 64 different cache lines, and the (cos, sin) reads
  // likewise.  Each wave therefore turns its tile through its own piece of the (now free) LDS, one
  // 32-row block at a time: fp32 [32 rows][128 features], row stride padded to 528 bytes.  Read back,
  // a lane holds features 4c..4c+3 and 64+4c..64+4c+3 of one row (both RoPE pairings stay inside the
  // lane), 16 lanes cover a row, and every global access of the wave is made of whole 128-byte runs.
  __syncthreads();                                           // every wave's tail loads have landed
  if (!compute) return;
  constexpr int kEpiStride = 528;                            // bytes per LDS row: 512 + 16 (bank spread)
  unsigned char *epi = lds + wave * (32 * kEpiStride);
  const int which = hs.which, head = hs.head, heads_out = hs.heads_out;
  const bf16_t *bias = a.bias[which];
  const int ec = lane & 15, er = lane >> 4;                  // read-back role: chunk of 4 features, row er + 4 j
  const bool inter = a.rope_layout == A3_ROPE_INTERLEAVED;
  // rows of this lane in the read-back role and their (cos, sin) table rows, for all blocks at once: the
  // two dependent index loads of every row are in flight together
  int src_row[TB][8];
  const float2 *csrow[TB][8];
#pragma unroll
  for (int tb = 0; tb < TB; ++tb)
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const int tok = min(tok0 + tb * 32 + er + 4 * j, a.n_rows - 1);
      src_row[tb][j] = a.row_idx ? a.row_idx[tok] : tok;
    }
#pragma unroll
  for (int tb = 0; tb < TB; ++tb)
#pragma unroll
    for (int j = 0; j < 8; ++j) csrow[tb][j] = a.pos_cs + (size_t)a.tok_pos[src_row[tb][j]] * (kHeadDim / 2);
  float bl[4], bh[4];
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    bl[e] = bias ? a3_bf2f(bias[head * kHeadDim + 4 * ec + e]) : 0.f;
    bh[e] = bias ? a3_bf2f(bias[head * kHeadDim + 64 + 4 * ec + e]) : 0.f;
  }
#pragma unroll
  for (int tb = 0; tb < TB; ++tb) {
    // accumulator block (fb, tb), register r of this lane: feature 32 fb + 8 (r/4) + 4 lhi + r%4, row l32
#pragma unroll
    for (int fb = 0; fb < 4; ++fb)
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        f32x4 v;
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] = acc[fb][tb][4 * q4 + e];
        *reinterpret_cast<f32x4 *>(epi + l32 * kEpiStride + (32 * fb + 8 * q4 + 4 * lhi) * 4) = v;
      }
    // (same wave writes and reads: the compiler's wait for the LDS writes is all the ordering needed)
    // all (cos, sin) reads of the block first, then the arithmetic and the stores
    float4 t0[8], t1[8];
    if (which != 2) {
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        // interleaved: pairs 2 ec, 2 ec + 1 and 32 + 2 ec, ..; half: pairs 4 ec .. 4 ec + 3
        t0[j] = *reinterpret_cast<const float4 *>(csrow[tb][j] + (inter ? 2 * ec : 4 * ec));
        t1[j] = *reinterpret_cast<const float4 *>(csrow[tb][j] + (inter ? 32 + 2 * ec : 4 * ec + 2));
      }
    }
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const int row = er + 4 * j;
      const int tok = tok0 + tb * 32 + row;
      f32x4 lo = *reinterpret_cast<const f32x4 *>(epi + row * kEpiStride + ec * 16);          // features 4 ec ..
      f32x4 hi = *reinterpret_cast<const f32x4 *>(epi + row * kEpiStride + 256 + ec * 16);    // features 64 + 4 ec ..
#pragma unroll
      for (int e = 0; e < 4; ++e) { lo[e] += bl[e]; hi[e] += bh[e]; }
      if (which != 2) {
        const float4 c0 = t0[j], c1 = t1[j];
        if (inter) {
          f32x4 x = lo;
          lo[0] = x[0] * c0.x - x[1] * c0.y; lo[1] = x[0] * c0.y + x[1] * c0.x;
          lo[2] = x[2] * c0.z - x[3] * c0.w; lo[3] = x[2] * c0.w + x[3] * c0.z;
          x = hi;
          hi[0] = x[0] * c1.x - x[1] * c1.y; hi[1] = x[0] * c1.y + x[1] * c1.x;
          hi[2] = x[2] * c1.z - x[3] * c1.w; hi[3] = x[2] * c1.w + x[3] * c1.z;
        } else {
          const f32x4 xl = lo, xh = hi;
          lo[0] = xl[0] * c0.x - xh[0] * c0.y; hi[0] = xl[0] * c0.y + xh[0] * c0.x;
          lo[1] = xl[1] * c0.z - xh[1] * c0.w; hi[1] = xl[1] * c0.w + xh[1] * c0.z;
          lo[2] = xl[2] * c1.x - xh[2] * c1.y; hi[2] = xl[2] * c1.y + xh[2] * c1.x;
          lo[3] = xl[3] * c1.z - xh[3] * c1.w; hi[3] = xl[3] * c1.w + xh[3] * c1.z;
        }
      }
      if (tok < a.n_rows) {
        const int out_row = (a.scatter_kv && which != 0) ? src_row[tb][j] : tok;
        bf16_t *orow = out + ((size_t)out_row * heads_out + head) * kHeadDim;
        bf16x4 vlo, vhi;
#pragma unroll
        for (int e = 0; e < 4; ++e) { vlo[e] = a3_f2bf(lo[e]); vhi[e] = a3_f2bf(hi[e]); }
        *reinterpret_cast<bf16x4 *>(orow + 4 * ec) = vlo;
        *reinterpret_cast<bf16x4 *>(orow + 64 + 4 * ec) = vhi;
      }
    }
  }
}

// ---------------------------------------------------------------------------------------
// bf16 kernels for few rows (the question tokens): weight-streaming bound
// ---------------------------------------------------------------------------------------
// Last step of both few-row kernels for one lane = one listed row: adds the NW partial tiles in wave
// order (partial w of accumulator register r is part[w * wave_stride + r * 64]), then bias, RoPE
// and the single rounding.  A workgroup holds 32 features of one head: 16 sb + (0..15) and the same
// + 64, so both RoPE pairings are inside it; accumulator register r is MFMA row
// i = 8 (r/4) + 4 lhi + r%4, and i < 16 is the first half of the head, i >= 16 the second.
template <int NW>
__device__ __forceinline__ void small_finish(const proj_args &a, const head_sel hs, int sb, int tok, int lhi,
                                             const float *part, int wave_stride) {
  if (tok >= a.n_rows) return;
  float v[16];
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    float t = 0.f;
#pragma unroll
    for (int w = 0; w < NW; ++w) t += part[w * wave_stride + r * 64];   // fixed order
    v[r] = t;
  }
  auto feat_of = [&](int r) {
    int i = 8 * (r >> 2) + 4 * lhi + (r & 3);
    return i < 16 ? 16 * sb + i : 64 + 16 * sb + (i - 16);
  };
  const bf16_t *bias = a.bias[hs.which];
  if (bias) {
#pragma unroll
    for (int r = 0; r < 16; ++r) v[r] += a3_bf2f(bias[hs.head * kHeadDim + feat_of(r)]);
  }
  const int src_row = a.row_idx ? a.row_idx[tok] : tok;
  if (hs.which != 2) {
    const float2 *cs = a.pos_cs + (size_t)a.tok_pos[src_row] * (kHeadDim / 2);
    if (a.rope_layout == A3_ROPE_INTERLEAVED) {
#pragma unroll
      for (int r = 0; r < 16; r += 2) {
        const float2 t = cs[feat_of(r) >> 1];
        float x0 = v[r], x1 = v[r + 1];
        v[r] = x0 * t.x - x1 * t.y;
        v[r + 1] = x0 * t.y + x1 * t.x;
      }
    } else {
#pragma unroll
      for (int r = 0; r < 8; ++r) {                            // register r + 8 holds feature + 64
        const float2 t = cs[feat_of(r)];
        float xlo = v[r], xhi = v[r + 8];
        v[r] = xlo * t.x - xhi * t.y;
        v[r + 8] = xlo * t.y + xhi * t.x;
      }
    }
  }
  const int out_row = (a.scatter_kv && hs.which != 0) ? src_row : tok;
  bf16_t *orow = a.out[hs.which] + ((size_t)out_row * hs.heads_out + hs.head) * kHeadDim;
#pragma unroll
  for (int q4 = 0; q4 < 4; ++q4) {
    bf16x4 o;
#pragma unroll
    for (int e = 0; e < 4; ++e) o[e] = a3_f2bf(v[4 * q4 + e]);
    *reinterpret_cast<bf16x4 *>(orow + feat_of(4 * q4)) = o;
  }
}

// Hidden size a multiple of 256.  With ~64 rows the GEMM is a stream over the 48 MB of weights.  To
// put every CU on that stream a workgroup takes only 32 features of one head x 64 rows, and its 4
// waves split the reduction dimension four ways.  Each wave runs its own pipeline with no workgroup
// barrier: stages of 64 reduction elements (32 weight rows + 64 hidden rows, 128 bytes each) go
// from global memory straight into the wave's private ring of three LDS stages with fully coalesced
// direct-to-LDS loads (8 lanes per 128-byte row), two stages ahead of the MFMAs.  (Fragments loaded
// straight into registers would touch 32 different cache lines per instruction, and the address
// path of the L1, not HBM, then sets the pace.)  LDS slot s of row r holds the 16-byte piece
// s ^ ((r/2) % 8) of the row's 128 bytes: the 16 consecutive rows a quarter wave reads at one piece
// index touch all 64 banks once.
// RB = row blocks of 32 per workgroup: 2 (64 rows), or 1 when that leaves more than half of the CUs without a
// workgroup (a call with few heads: Q of the question rows alone): twice the workgroups, each re-reading half as
// many hidden rows.
constexpr int kSmRing = 3;
constexpr int sm_stage_bytes(int rb) { return (32 + 32 * rb) * 128; }
constexpr size_t sm_lds_bytes(int rb) { return (size_t)4 * kSmRing * sm_stage_bytes(rb); }      // 144 KB / 96 KB

template <int RB>
__global__ void __launch_bounds__(256)
proj_small_dma_bf16_kernel(proj_args a) {
  constexpr int kSmStageBytes = sm_stage_bytes(RB);
  constexpr int kSmLoads = 4 + 4 * RB;                         // direct-to-LDS loads per stage
  extern __shared__ __align__(16) unsigned char lds[];

  const int head_all = blockIdx.x >> 2, sb = blockIdx.x & 3;
  const head_sel hs = select_head(head_all, a.Hq, a.Hkv);
  if (a.out[hs.which] == nullptr) return;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, lhi = lane >> 5;
  const int tok0 = blockIdx.y * 32 * RB;
  const int kq = a.K / 4;                                      // this wave's share: a multiple of 64

  // loading role: one instruction brings 8 rows x 128 B, lane -> (row lane/8, slot lane%8)
  const int drow = lane >> 3, dslot = lane & 7;
  const char *wsrc[4], *xsrc[4 * RB];
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int row = 8 * j + drow;                              // MFMA row of the weight block
    const int feat = row < 16 ? 16 * sb + row : 64 + 16 * sb + (row - 16);
    wsrc[j] = reinterpret_cast<const char *>(a.w[hs.which] + ((size_t)hs.head * kHeadDim + feat) * a.K + wave * kq) +
              16 * (dslot ^ ((row >> 1) & 7));
  }
#pragma unroll
  for (int j = 0; j < 4 * RB; ++j) {
    const int row = 8 * j + drow;
    const int m = min(tok0 + row, a.n_rows - 1);               // clamp: computed but never stored
    const int src_row = a.row_idx ? a.row_idx[m] : m;
    xsrc[j] = reinterpret_cast<const char *>(a.hidden + (size_t)src_row * a.K + wave * kq) +
              16 * (dslot ^ ((row >> 1) & 7));
  }
  unsigned char *ring = lds + wave * (kSmRing * kSmStageBytes);
  const uint32_t lds_ring = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char *)ring;
  // Inline assembly as in the large kernel: lane i's 16 bytes land at M0 + 16 i, the compiler does not
  // track these loads, and the waits for them are the explicit s_waitcnt below.
#define A3_SM_ISSUE(SLOT, K0)                                                                                  \
  {                                                                                                            \
    _Pragma("unroll") for (int j = 0; j < 4; ++j)                                                              \
      asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off"                                       \
                   :: "s"(__builtin_amdgcn_readfirstlane(lds_ring + (SLOT) * kSmStageBytes + 1024 * j)),       \
                      "v"(wsrc[j] + 2 * (K0)) : "memory");                                                     \
    _Pragma("unroll") for (int j = 0; j < 4 * RB; ++j)                                                         \
      asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off"                                       \
                   :: "s"(__builtin_amdgcn_readfirstlane(lds_ring + (SLOT) * kSmStageBytes + 4096 + 1024 * j)), \
                      "v"(xsrc[j] + 2 * (K0)) : "memory");                                                     \
  }
  f32x16 acc[RB];
#pragma unroll
  for (int tb = 0; tb < RB; ++tb)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[tb][r] = 0.f;
  // everything the compiler loaded itself (row indices) has arrived: from here on only the
  // direct-to-LDS loads are outstanding and the counts below are exact
  __builtin_amdgcn_s_waitcnt(0);
  const int n_st = kq / 64;
  A3_SM_ISSUE(0, 0)
  if (n_st > 1) A3_SM_ISSUE(1, 64)
  const int frag = l32 * 128, fswz = (l32 >> 1) & 7;           // rows 32 tb + l32 swizzle like row l32
  int slot = 0, slot2 = 2;
  for (int s = 0; s < n_st; ++s) {
    if (s + 2 < n_st) {
      A3_SM_ISSUE(slot2, 64 * (s + 2))
      __builtin_amdgcn_s_waitcnt(vmcnt_imm(2 * kSmLoads));     // stage s has landed: two younger ones may be on their way
    } else if (s + 1 < n_st) {
      __builtin_amdgcn_s_waitcnt(vmcnt_imm(kSmLoads));
    } else {
      __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
    }
    asm volatile("" ::: "memory");
    const unsigned char *st = ring + slot * kSmStageBytes + frag;
    bf16x8 wf[4], xa[4], xb[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int po = 16 * ((2 * u + lhi) ^ fswz);
      wf[u] = *reinterpret_cast<const bf16x8 *>(st + po);
      xa[u] = *reinterpret_cast<const bf16x8 *>(st + 4096 + po);
      if (RB == 2) xb[u] = *reinterpret_cast<const bf16x8 *>(st + 8192 + po);
    }
    __builtin_amdgcn_sched_barrier(0);                         // all twelve reads in flight before the first MFMA
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      acc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[u], xa[u], acc[0], 0, 0, 0);
      if (RB == 2) acc[RB - 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[u], xb[u], acc[RB - 1], 0, 0, 0);
    }
    // the fragments are in registers before the next trip overwrites the slot read two trips ago
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    slot = slot == kSmRing - 1 ? 0 : slot + 1;
    slot2 = slot2 == kSmRing - 1 ? 0 : slot2 + 1;
  }
#undef A3_SM_ISSUE
  // the wave's own ring is free now: it holds the wave's partial tile, [row block][register][lane]
  float *red = reinterpret_cast<float *>(ring);
#pragma unroll
  for (int tb = 0; tb < RB; ++tb)
#pragma unroll
    for (int r = 0; r < 16; ++r) red[(tb * 16 + r) * 64 + lane] = acc[tb][r];
  __syncthreads();
  if (wave >= RB) return;
  const int tb = wave;                                         // one wave per row block finishes it
  small_finish<4>(a, hs, sb, tok0 + tb * 32 + l32, lhi, reinterpret_cast<const float *>(lds) + tb * 16 * 64 + lane,
                  kSmRing * kSmStageBytes / 4);
}

// Any other hidden size that is a multiple of 64: fragments straight from global memory.
// A workgroup takes 32 features of one head (16 from each half of the head, so both RoPE
// pairings stay inside it) x 64 rows, and its NW waves (2 when the hidden size is a multiple of
// 128, else 1) split the reduction dimension NW ways in shares of whole 64-wide stages; fragments
// are read straight from global memory and the partial tiles are added in LDS in wave order.
template <int NW>                                               // waves per workgroup = ways the reduction is split
__global__ void __launch_bounds__(64 * NW)
proj_small_bf16_kernel(proj_args a) {
  __shared__ float red[NW][2][16][64];                         // [wave][row block][register][lane]

  const int head_all = blockIdx.x >> 2, sb = blockIdx.x & 3;
  const head_sel hs = select_head(head_all, a.Hq, a.Hkv);
  bf16_t *__restrict__ out = a.out[hs.which];
  if (out == nullptr) return;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, lhi = lane >> 5;
  const int tok0 = blockIdx.y * 64;
  // MFMA row i of this workgroup's weight block <-> feature of the head
  const int feat = l32 < 16 ? 16 * sb + l32 : 64 + 16 * sb + (l32 - 16);
  const int kq = a.K / NW;                                     // this wave's share of the reduction
  const bf16_t *wp = a.w[hs.which] + ((size_t)hs.head * kHeadDim + feat) * a.K + wave * kq + lhi * 8;
  const bf16_t *xp0, *xp1;
  {
    int m = min(tok0 + l32, a.n_rows - 1);
    xp0 = a.hidden + (size_t)(a.row_idx ? a.row_idx[m] : m) * a.K + wave * kq + lhi * 8;
    m = min(tok0 + 32 + l32, a.n_rows - 1);
    xp1 = a.hidden + (size_t)(a.row_idx ? a.row_idx[m] : m) * a.K + wave * kq + lhi * 8;
  }
  f32x16 acc[2];
#pragma unroll
  for (int tb = 0; tb < 2; ++tb)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[tb][r] = 0.f;
  // Two register stages of four k-steps each: the loads of one stage are in flight while the other
  // is multiplied, so every wave always has weight bytes on their way from HBM.  The share kq is a
  // multiple of 64 (one stage).
  bf16x8 wf0[4], wf1[4], xa0[4], xa1[4], xb0[4], xb1[4];
#define A3_SMALL_LOAD(WF, XA, XB, K0)                                            \
  _Pragma("unroll") for (int u = 0; u < 4; ++u) {                                \
    WF[u] = *reinterpret_cast<const bf16x8 *>(wp + (K0) + 16 * u);               \
    XA[u] = *reinterpret_cast<const bf16x8 *>(xp0 + (K0) + 16 * u);              \
    XB[u] = *reinterpret_cast<const bf16x8 *>(xp1 + (K0) + 16 * u);              \
  }
#define A3_SMALL_MMA(WF, XA, XB)                                                 \
  _Pragma("unroll") for (int u = 0; u < 4; ++u) {                                \
    acc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(WF[u], XA[u], acc[0], 0, 0, 0); \
    acc[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(WF[u], XB[u], acc[1], 0, 0, 0); \
  }
  A3_SMALL_LOAD(wf0, xa0, xb0, 0)
  int k = 0;
  for (; k + 128 <= kq; k += 128) {
    A3_SMALL_LOAD(wf1, xa1, xb1, k + 64)
    A3_SMALL_MMA(wf0, xa0, xb0)
    const int kn = min(k + 128, kq - 64);                      // past the end: the last stage again, unused
    A3_SMALL_LOAD(wf0, xa0, xb0, kn)
    A3_SMALL_MMA(wf1, xa1, xb1)
  }
  if (k < kq) { A3_SMALL_MMA(wf0, xa0, xb0) }                  // odd number of stages
#undef A3_SMALL_LOAD
#undef A3_SMALL_MMA
#pragma unroll
  for (int tb = 0; tb < 2; ++tb)
#pragma unroll
    for (int r = 0; r < 16; ++r) red[wave][tb][r][lane] = acc[tb][r];
  __syncthreads();
  if (wave >= 2) return;
  for (int tb = wave; tb < 2; tb += (NW > 1 ? 2 : 1))          // waves 0 and 1 finish one row block each
    small_finish<NW>(a, hs, sb, tok0 + tb * 32 + l32, lhi, &red[0][tb][0][lane], 2 * 16 * 64);
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
  int scatter_kv;
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
    const int out_row = (a.scatter_kv && which != 0) ? (a.row_idx ? a.row_idx[m] : m) : m;
    float *orow = out + ((size_t)out_row * heads_out + head) * d;
    orow[ia] = ya;
    orow[ib] = yb;
  }
}

}  // namespace

static a3_status proj_launch(const a3_layout *L, const void *hidden, const int *row_idx, int n_rows, const void *wq,
                             const void *wk, const void *wv, const void *bq, const void *bk, const void *bv,
                             void *q_out, void *k_out, void *v_out, int scatter_kv, void *stream) {
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
    A3_REQUIRE(L->hidden % 64 == 0, A3_ERR_UNSUPPORTED, "a3_selected_qkv_proj: bf16 needs hidden %% 64 == 0, got %d",
               L->hidden);
    A3_REQUIRE((long long)L->total_tokens * L->hidden * 2 < (1LL << 32), A3_ERR_UNSUPPORTED,
               "a3_selected_qkv_proj: hidden tensor larger than 4 GiB");
    proj_args a;
    a.hidden = (const bf16_t *)hidden; a.row_idx = row_idx; a.n_rows = n_rows;
    a.w[0] = (const bf16_t *)wq; a.w[1] = (const bf16_t *)wk; a.w[2] = (const bf16_t *)wv;
    a.bias[0] = (const bf16_t *)bq; a.bias[1] = (const bf16_t *)bk; a.bias[2] = (const bf16_t *)bv;
    a.out[0] = (bf16_t *)q_out; a.out[1] = (bf16_t *)k_out; a.out[2] = (bf16_t *)v_out;
    a.tok_pos = L->tok_pos; a.pos_cs = (const float2 *)L->rope_pos_cs;
    a.K = L->hidden; a.Hq = L->n_q_heads; a.Hkv = L->n_kv_heads; a.rope_layout = L->rope_layout;
    a.n_pairs = (n_heads_total + 1) / 2;
    a.n_tok_tiles = 0;
    a.scatter_kv = scatter_kv;
    const int ntw_knob = a3_knob(A3_KNOB_PROJ_NTW);            // tuning value "proj_ntw": the GEMM kernel in this width
    if (n_rows <= 192 && L->hidden % 64 == 0 && ntw_knob < 0) {
      // few rows: stream the weights with 4 x n_heads x ceil(rows/64) small workgroups
      const dim3 grid(4 * n_heads_total, (n_rows + 63) / 64);
      if (L->hidden % 256 == 0) {
        static a3_once_per_device small_once;
        const hipError_t once_err = a3_once(small_once, []() {
          hipError_t e = hipFuncSetAttribute((const void *)proj_small_dma_bf16_kernel<2>,
                                             hipFuncAttributeMaxDynamicSharedMemorySize, (int)sm_lds_bytes(2));
          hipError_t e1 = hipFuncSetAttribute((const void *)proj_small_dma_bf16_kernel<1>,
                                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)sm_lds_bytes(1));
          return e != hipSuccess ? e : e1;
        });
        if (once_err != hipSuccess) return a3_fail(A3_ERR_HIP, "a3_selected_qkv_proj: cannot raise the dynamic LDS limit");
        // workgroups that have an output: 4 per head of the tensors asked for, per 64 rows
        const int heads_out = (q_out ? L->n_q_heads : 0) + (k_out ? L->n_kv_heads : 0) + (v_out ? L->n_kv_heads : 0);
        if (4 * heads_out * (int)grid.y <= 128 && n_rows > 32)
          hipLaunchKernelGGL(proj_small_dma_bf16_kernel<1>, dim3(grid.x, (n_rows + 31) / 32), dim3(256), sm_lds_bytes(1), st, a);
        else
          hipLaunchKernelGGL(proj_small_dma_bf16_kernel<2>, grid, dim3(256), sm_lds_bytes(2), st, a);
      } else if (L->hidden % 128 == 0) {
        hipLaunchKernelGGL(proj_small_bf16_kernel<2>, grid, dim3(128), 0, st, a);
      } else {
        hipLaunchKernelGGL(proj_small_bf16_kernel<1>, grid, dim3(64), 0, st, a);
      }
      A3_CHECK_LAUNCH("a3_selected_qkv_proj");
      return A3_OK;
    }
    // rows per workgroup: 128, 192 or 256.  Estimate each choice by (useful rows / padded rows) x (how
    // evenly the workgroups fill 256 CUs) x a bonus for the lower L2 traffic of larger tiles.
    int ntw = 2;
    if (ntw_knob >= 0) ntw = ntw_knob;
    else {
      double best = -1.0;
      for (int c = 2; c <= 4; ++c) {
        const int tiles = (n_rows + 64 * c - 1) / (64 * c);
        const long wgs = (long)tiles * a.n_pairs;
        const int per_cu = c == 2 ? 2 : 1;                    // co-resident workgroups
        const long rounds = (wgs + 256L * per_cu - 1) / (256L * per_cu);
        const double fill = (double)wgs / (double)(rounds * 256L * per_cu);
        const double pad = (double)n_rows / (double)(tiles * 64 * c);
        const double traffic = 256.0 * 64 * c / (256.0 + 64 * c) / 128.0;   // flop per L2 byte, relative to 256x256
        const double score = pad * fill * (0.5 + 0.5 * traffic);
        if (score > best) { best = score; ntw = c; }
      }
    }
    if (ntw < 2 || ntw > 4) ntw = 2;
    a.n_tok_tiles = (n_rows + 64 * ntw - 1) / (64 * ntw);
    const unsigned grid = 8u * (unsigned)((a.n_pairs + 7) / 8) * (unsigned)a.n_tok_tiles;
    // 128-byte row pieces for the 192- and 256-row tiles when the hidden size allows (tuning value "proj_k64" = 0:
    // the 64-byte loop)
    bool k64 = ntw >= 3 && L->hidden % 64 == 0;
    if (a3_knob(A3_KNOB_PROJ_K64) == 0) k64 = false;
    static a3_once_per_device lds_once;
    const hipError_t once_err = a3_once(lds_once, []() {
      hipError_t e1 = hipFuncSetAttribute((const void *)proj_bf16_kernel<2, false>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)gemm_tile_lds_bytes(2));
      hipError_t e2 = hipFuncSetAttribute((const void *)proj_bf16_kernel<3, false>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)gemm_tile_lds_bytes(3));
      hipError_t e3 = hipFuncSetAttribute((const void *)proj_bf16_kernel<4, false>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)gemm_tile_lds_bytes(4));
      hipError_t e4 = hipFuncSetAttribute((const void *)proj_bf16_kernel<3, true>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)gemm_tile_lds_bytes_k64(3));
      hipError_t e5 = hipFuncSetAttribute((const void *)proj_bf16_kernel<4, true>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)gemm_tile_lds_bytes_k64(4));
      for (hipError_t e : {e1, e2, e3, e4, e5}) if (e != hipSuccess) return e;
      return hipSuccess;
    });
    if (once_err != hipSuccess) return a3_fail(A3_ERR_HIP, "a3_selected_qkv_proj: cannot raise the dynamic LDS limit");
    if (ntw == 2) hipLaunchKernelGGL((proj_bf16_kernel<2, false>), dim3(grid), dim3(256), gemm_tile_lds_bytes(2), st, a);
    else if (ntw == 3 && k64) hipLaunchKernelGGL((proj_bf16_kernel<3, true>), dim3(grid), dim3(256), gemm_tile_lds_bytes_k64(3), st, a);
    else if (ntw == 3) hipLaunchKernelGGL((proj_bf16_kernel<3, false>), dim3(grid), dim3(256), gemm_tile_lds_bytes(3), st, a);
    else if (k64) hipLaunchKernelGGL((proj_bf16_kernel<4, true>), dim3(grid), dim3(256), gemm_tile_lds_bytes_k64(4), st, a);
    else hipLaunchKernelGGL((proj_bf16_kernel<4, false>), dim3(grid), dim3(256), gemm_tile_lds_bytes(4), st, a);
  } else {
    proj_args_f32 a;
    a.hidden = (const float *)hidden; a.row_idx = row_idx; a.n_rows = n_rows;
    a.w[0] = (const float *)wq; a.w[1] = (const float *)wk; a.w[2] = (const float *)wv;
    a.bias[0] = (const float *)bq; a.bias[1] = (const float *)bk; a.bias[2] = (const float *)bv;
    a.out[0] = (float *)q_out; a.out[1] = (float *)k_out; a.out[2] = (float *)v_out;
    a.tok_pos = L->tok_pos; a.pos_cs = (const float2 *)L->rope_pos_cs;
    a.K = L->hidden; a.Hq = L->n_q_heads; a.Hkv = L->n_kv_heads; a.d = L->head_dim; a.rope_layout = L->rope_layout;
    a.scatter_kv = scatter_kv;
    dim3 grid(n_heads_total, (n_rows + kF32Rows - 1) / kF32Rows);
    hipLaunchKernelGGL(proj_f32_kernel, grid, dim3(256), 0, st, a);
  }
  A3_CHECK_LAUNCH("a3_selected_qkv_proj");
  return A3_OK;
}

extern "C" a3_status a3_selected_qkv_proj(const a3_layout *L, const void *hidden, const int *row_idx, int n_rows,
                                          const void *wq, const void *wk, const void *wv, const void *bq,
                                          const void *bk, const void *bv, void *q_out, void *k_out, void *v_out,
                                          void *stream) {
  return proj_launch(L, hidden, row_idx, n_rows, wq, wk, wv, bq, bk, bv, q_out, k_out, v_out, 0, stream);
}

extern "C" a3_status a3_selected_qkv_proj_scatter(const a3_layout *L, const void *hidden, const int *row_idx,
                                                  int n_rows, const void *wq, const void *wk, const void *wv,
                                                  const void *bq, const void *bk, const void *bv, void *q_out,
                                                  void *k_fused, void *v_fused, void *stream) {
  return proj_launch(L, hidden, row_idx, n_rows, wq, wk, wv, bq, bk, bv, q_out, k_fused, v_fused, 1, stream);
}
