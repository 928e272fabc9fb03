// The main loop of the row-tiled bf16 MFMA GEMM that the Q/K/V projection (Eq. 5, first lines; a3_proj.hip)
// and the three GEMMs of H(.) (a3_block.hip) share.  One workgroup of four waves forms
//     acc[256 weight rows][64 TB activation rows] = W_tile X_tile^T      over the whole reduction dimension,
// wave (fh, th) = (wave & 1, wave >> 1) owning weight rows 128 fh .. + 127 (4 blocks of 32) and activation rows
// 32 TB th .. (TB blocks of 32): 4 + TB fragment reads per 4 TB MFMAs, one wave per SIMD.  Both operands are
// reduction-contiguous in memory and go from global memory straight into LDS (global_load_lds, 16 bytes per
// lane, no staging registers); LDS rows are unpadded and their 16-byte pieces XOR-swizzled against bank
// conflicts.  Which memory row an LDS row is - a head's weight row, a gate or an up row, a gathered hidden row -
// is the caller's business: it passes two functions from the tile's row number to the start of that row.
// Device code, inlined into both translation units (no relocatable device code).
#pragma once

#include "a3_internal.h"

namespace {

constexpr int kGemmBK = 32;                      // reduction slab per barrier of the 64-byte-piece loop
constexpr int kGemmRowBytes = kGemmBK * 2;       // there an LDS row is one 64-byte k-slab of a weight or activation row
// LDS stages of the 64-byte-piece loop: loads run stages-1 slabs ahead of the MFMAs.  The 128-row tile keeps 3
// stages (72 KB) so that two workgroups share a CU and cover each other's barriers; the larger tiles run alone with 4.
constexpr int gemm_tile_stages(int tb) { return tb == 2 ? 3 : 4; }
constexpr size_t gemm_tile_lds_bytes(int tb) { return (size_t)gemm_tile_stages(tb) * (256 + 64 * tb) * kGemmRowBytes; }
// the loop with 128-byte row pieces: 3 weight stages and 2 stages of activation rows
constexpr size_t gemm_tile_lds_bytes_k64(int tb) { return (size_t)3 * 256 * 128 + (size_t)2 * 64 * tb * 128; }

// s_waitcnt immediate that waits until at most n vector-memory operations are outstanding and
// nothing else (gfx9 encoding: vmcnt in bits 3:0 and 15:14, expcnt 6:4, lgkmcnt 11:8)
constexpr int vmcnt_imm(int n) { return (n & 15) | ((n >> 4) << 14) | (7 << 4) | (15 << 8); }

// w_row(r): start of the memory row behind weight-tile row r (0..255); x_row(r): the same for activation-tile row
// r (0..64 TB - 1; rows past the end of the list are clamped by the caller: computed, never stored).  K is a
// multiple of 64.  On return every load has landed (the caller still needs a barrier before it reuses LDS).
template <int TB, bool K64, class WRow, class XRow>
__device__ __forceinline__ void gemm_tile_mainloop(f32x16 (&acc)[4][TB], unsigned char *lds, int K, WRow w_row, XRow x_row) {
  constexpr int kTokTile = 64 * TB;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, lhi = lane >> 5;
  const int fh = wave & 1, th = wave >> 1;
#pragma unroll
  for (int fb = 0; fb < 4; ++fb)
#pragma unroll
    for (int tb = 0; tb < TB; ++tb)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[fb][tb][r] = 0.f;

  // global_load_lds: lane i's 16 bytes land at (M0 = wave-uniform LDS byte address) + 16 i.  Issued as
  // inline assembly on purpose: the compiler then neither tracks these as LDS writes (it would put
  // a full vmcnt(0) in front of every LDS read and undo the lookahead) nor reorders memory accesses
  // across them; the waits for them are the explicit s_waitcnt below.  M0 is not used by anything
  // else in these kernels (LDS instructions need no M0 on gfx9 and later).  The s_nop is the wait state this
  // chip wants between a scalar write of M0 and a direct-to-LDS load that reads it (the compiler puts the same
  // one behind its own M0 writes; it does not look into an asm statement).
  const uint32_t lds_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char *)lds;
#define A3_DMA(GPTR, LDS_OFF)                                                                                 \
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off"                                \
               :: "s"(__builtin_amdgcn_readfirstlane(lds_base + (uint32_t)(LDS_OFF))), "v"(GPTR) : "memory")
  // A wave that issues an LDS read or a vector-memory instruction is held until the unit takes it, and
  // with one wave per SIMD nothing else fills that time: a batch of seven reads in front of twelve
  // MFMAs costs about a sixth of their run time (measured on a register-only copy of this loop).  So
  // every read and every load is issued on its own, right after an MFMA, whose 32 cycles in the matrix
  // pipe cover it.  A3_FENCE keeps the compiler from regrouping them.
#define A3_FENCE __builtin_amdgcn_sched_barrier(0);
  if constexpr (!K64) {
    // ---- 64-byte row pieces: 32-wide k-slabs, loads run stages-1 slabs ahead ----------------------------------
    // One wave instruction brings 16 rows x 64 B: lane -> (row lane/4, slot lane%4), and the lane fetches the
    // 16-byte piece (slot ^ swz(row)) of its row, so that LDS slot s of row r holds piece s ^ swz(r),
    // swz(r) = (r/4) % 4: the 16 consecutive rows that one quarter of a wave reads at one piece index then
    // touch all 64 LDS banks (256 bytes) exactly once.  Wave w issues weight rows 16 (4 j + w) .. +15
    // (j = 0..3) and activation rows 16 (4 j + w) .. +15 (j = 0..TB-1).
    constexpr int kStages = gemm_tile_stages(TB);
    constexpr int kWBytes = 256 * kGemmRowBytes;               // weight part of a stage
    constexpr int kStageBytes = kWBytes + kTokTile * kGemmRowBytes;
    constexpr int kLoads = 4 + TB;                             // direct-to-LDS loads per wave per slab
    const int lrow = lane >> 2, slot = lane & 3;
    const int piece = slot ^ ((lrow >> 2) & 3);
    const char *wsrc[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) wsrc[j] = reinterpret_cast<const char *>(w_row(16 * (4 * j + wave) + lrow) + piece * 8);
    const char *xsrc[TB];
#pragma unroll
    for (int j = 0; j < TB; ++j) xsrc[j] = reinterpret_cast<const char *>(x_row(16 * (4 * j + wave) + lrow) + piece * 8);
#define A3_ISSUE(STAGE, K0)                                                                                   \
    {                                                                                                         \
      const uint32_t st_ = (STAGE) * kStageBytes;                                                             \
      const size_t kb_ = (size_t)(K0) * sizeof(bf16_t);                                                       \
      _Pragma("unroll") for (int j = 0; j < 4; ++j) A3_DMA(wsrc[j] + kb_, st_ + 16 * (4 * j + wave) * kGemmRowBytes); \
      _Pragma("unroll") for (int j = 0; j < TB; ++j)                                                          \
        A3_DMA(xsrc[j] + kb_, st_ + kWBytes + 16 * (4 * j + wave) * kGemmRowBytes);                           \
    }
    // fragment addresses: row base + swizzled slot of piece 2 ks + lhi
    const int swz = (l32 >> 2) & 3;
    const int frag_w = (fh * 128 + l32) * kGemmRowBytes, frag_x = kWBytes + (th * 32 * TB + l32) * kGemmRowBytes;
    const int slot_k0 = ((lhi) ^ swz) * 16, slot_k1 = ((2 + lhi) ^ swz) * 16;
    // the I-th fragment read of a k-step: activation rows first, then the weights
#define A3_FRAG1(I, WF, XF, ST, SLOT)                                                                          \
    if ((I) < TB) XF[(I) < TB ? (I) : 0] = *reinterpret_cast<const bf16x8 *>((ST) + frag_x + ((I) < TB ? (I) : 0) * 32 * kGemmRowBytes + (SLOT)); \
    else if ((I) < TB + 4) WF[(I) - TB < 4 && (I) >= TB ? (I) - TB : 0] = *reinterpret_cast<const bf16x8 *>((ST) + frag_w + ((I) - TB < 4 && (I) >= TB ? (I) - TB : 0) * 32 * kGemmRowBytes + (SLOT));
    // One wave per SIMD, so LDS latency has to be hidden inside the wave: the fragments of the second
    // k-step of a slab are read while the MFMAs of the first run, and the fragments of the next slab's
    // first k-step are read (right after its barrier) while the MFMAs of this slab's second k-step run.
    const int n_slabs = K / kGemmBK;
    const int k_last = K - kGemmBK;
#pragma unroll
    for (int s0 = 0; s0 < kStages - 1; ++s0) A3_ISSUE(s0, min(s0 * kGemmBK, k_last))
    bf16x8 wf0[4], xf0[TB], wf1[4], xf1[TB];
    __builtin_amdgcn_s_waitcnt(vmcnt_imm((kStages - 2) * kLoads));   // this wave's loads of slab 0 have landed
    __builtin_amdgcn_s_barrier();                                     // ... and everybody's
    A3_ISSUE(kStages - 1, min((kStages - 1) * kGemmBK, k_last))
#pragma unroll
    for (int i = 0; i < TB + 4; ++i) { A3_FRAG1(i, wf0, xf0, lds, slot_k0) }
    for (int sl = 0; sl < n_slabs; ++sl) {
      const unsigned char *st = lds + (sl % kStages) * kStageBytes;
      // first k-step of the slab; the fragments of its second k-step are read underneath
      A3_FENCE
#pragma unroll
      for (int i = 0; i < 4 * TB; ++i) {
        const int fb = i / TB, tb = i % TB;
        acc[fb][tb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf0[fb], xf0[tb], acc[fb][tb], 0, 0, 0);
        A3_FENCE
        A3_FRAG1(i, wf1, xf1, st, slot_k1)
        A3_FENCE
      }
      // Slab sl+1: this wave's loads have landed once only the 2 younger slabs are outstanding, and
      // after the barrier everybody's have.  The barrier also says that every wave has fetched its last
      // fragments of slab sl (lgkmcnt(0) first), whose stage the loads issued next will overwrite.
      // (Bare barrier: a fence here would wait for the loads in flight.)
      __builtin_amdgcn_s_waitcnt(vmcnt_imm((kStages - 2) * kLoads) & ~(15 << 8));
      __builtin_amdgcn_s_barrier();
      const unsigned char *sn = lds + ((sl + 1) % kStages) * kStageBytes;
      // second k-step; underneath, the fragments of the next slab's first k-step (past the last slab: a
      // stale stage, unused) and the loads of slab sl + kStages
      {
        const uint32_t st_ = ((sl + kStages) % kStages) * kStageBytes;
        const size_t kb_ = (size_t)min((sl + kStages) * kGemmBK, k_last) * sizeof(bf16_t);
        A3_FENCE
#pragma unroll
        for (int i = 0; i < 4 * TB; ++i) {
          const int fb = i / TB, tb = i % TB;
          acc[fb][tb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf1[fb], xf1[tb], acc[fb][tb], 0, 0, 0);
          A3_FENCE
          A3_FRAG1(i, wf0, xf0, sn, slot_k0)
          if (i < 4) A3_DMA(wsrc[i] + kb_, st_ + 16 * (4 * i + wave) * kGemmRowBytes);
          else if (i < kLoads) A3_DMA(xsrc[i - 4] + kb_, st_ + kWBytes + 16 * (4 * (i - 4) + wave) * kGemmRowBytes);
          A3_FENCE
        }
      }
    }
#undef A3_FRAG1
#undef A3_ISSUE
  } else {
    // ---- 128-byte row pieces: a slab is 64 elements of the reduction dimension ------------------------------
    // The L1 path moves a wave instruction of 8 rows x 128 B (whole cache lines) a third faster than one of
    // 16 rows x 64 B (half lines), and at these tile sizes that path, not the matrix pipe, sets the pace of
    // the loop.  LDS: a ring of 3 weight stages [256 rows][128 B] and a ring of 2 stages of activation rows
    // [64 TB rows][128 B]; the weights, which come from HBM the first time an XCD asks for them, are
    // requested two slabs ahead, the activation rows (shared by all weight tiles, L2 hits) one slab ahead.
    // LDS slot s of row r holds piece s ^ ((r >> 1) & 7): the 16 consecutive rows a quarter wave reads at one
    // piece index then touch all 64 banks once.
    constexpr int kRowB = 128, kWStage = 256 * kRowB, kXStage = kTokTile * kRowB, kXBase = 3 * kWStage;
    constexpr int kLW = 8, kLX = 2 * TB;                       // direct-to-LDS loads per wave and slab
    const int row8 = lane >> 3, slot8 = lane & 7;
    const int piece8 = slot8 ^ ((4 * (wave & 1) + (row8 >> 1)) & 7);   // rows 8 (4 j + wave) + row8: (row >> 1) & 7
    const char *wsrc[kLW];
#pragma unroll
    for (int j = 0; j < kLW; ++j) wsrc[j] = reinterpret_cast<const char *>(w_row(8 * (4 * j + wave) + row8) + piece8 * 8);
    const char *xsrc[kLX];
#pragma unroll
    for (int j = 0; j < kLX; ++j) xsrc[j] = reinterpret_cast<const char *>(x_row(8 * (4 * j + wave) + row8) + piece8 * 8);
    const int n_slabs = K / 64;
#define A3_KB(SLAB) ((size_t)min((SLAB), n_slabs - 1) * 128)     /* byte offset of a slab in a row; past the end: the last one, unused */
#define A3_W_LOAD(J, WOFF, SLAB) A3_DMA(wsrc[J] + A3_KB(SLAB), (WOFF) + (4 * (J) + wave) * 1024);
#define A3_X_LOAD(J, XOFF, SLAB) A3_DMA(xsrc[J] + A3_KB(SLAB), (XOFF) + (4 * (J) + wave) * 1024);
    // fragment addresses: row base + swizzled slot of piece 2 ks + lhi
    const int swz8 = (l32 >> 1) & 7;
    const int frag_w = (fh * 128 + l32) * kRowB, frag_x = (th * 32 * TB + l32) * kRowB;
    int slot[4];
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) slot[ks] = ((2 * ks + lhi) ^ swz8) * 16;
    // the I-th fragment read of a k-step: activation rows first, then the weights
#define A3_FRAG8(I, WF, XF, WOFF, XOFF, SLOT)                                                                   \
    if ((I) < TB) XF[(I) < TB ? (I) : 0] = *reinterpret_cast<const bf16x8 *>(lds + (XOFF) + frag_x + ((I) < TB ? (I) : 0) * 32 * kRowB + (SLOT)); \
    else if ((I) < TB + 4) WF[(I) >= TB && (I) - TB < 4 ? (I) - TB : 0] = *reinterpret_cast<const bf16x8 *>(lds + (WOFF) + frag_w + ((I) >= TB && (I) - TB < 4 ? (I) - TB : 0) * 32 * kRowB + (SLOT));
    // one k-step: its MFMAs, and behind each of them at most one fragment read and one load
#define A3_KSTEP(WA, XA, WB, XB, WOFF, XOFF, SLOT, LOADS)                                                       \
    A3_FENCE                                                                                                    \
    _Pragma("unroll") for (int i = 0; i < 4 * TB; ++i) {                                                        \
      const int fb = i / TB, tb = i % TB;                                                                       \
      acc[fb][tb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(WA[fb], XA[tb], acc[fb][tb], 0, 0, 0);              \
      A3_FENCE                                                                                                  \
      A3_FRAG8(i, WB, XB, WOFF, XOFF, SLOT)                                                                     \
      LOADS                                                                                                     \
      A3_FENCE                                                                                                  \
    }
    // request order: W(0) X(0) W(1) X(1), then per slab sl: W(sl+2) under its first k-step and X(sl+2) under
    // its last one, so that at the barrier of slab sl only the 8 loads of W(sl+2) may still be on their way
    int w_cur = 0, w_nxt = kWStage, w_nn = 2 * kWStage;        // weight stages of slabs sl, sl + 1, sl + 2
    int x_cur = kXBase, x_nxt = kXBase + kXStage;
#pragma unroll
    for (int j = 0; j < kLW; ++j) A3_W_LOAD(j, w_cur, 0)
#pragma unroll
    for (int j = 0; j < kLX; ++j) A3_X_LOAD(j, x_cur, 0)
#pragma unroll
    for (int j = 0; j < kLW; ++j) A3_W_LOAD(j, w_nxt, 1)
#pragma unroll
    for (int j = 0; j < kLX; ++j) A3_X_LOAD(j, x_nxt, 1)
    bf16x8 wf0[4], xf0[TB], wf1[4], xf1[TB];
    __builtin_amdgcn_s_waitcnt(vmcnt_imm(kLW + kLX));          // this wave's loads of slab 0 have landed
    __builtin_amdgcn_s_barrier();                              // ... and everybody's
#pragma unroll
    for (int i = 0; i < TB + 4; ++i) { A3_FRAG8(i, wf0, xf0, w_cur, x_cur, slot[0]) }
    for (int sl = 0; sl < n_slabs; ++sl) {
      A3_KSTEP(wf0, xf0, wf1, xf1, w_cur, x_cur, slot[1], if (i < kLW) A3_W_LOAD(i, w_nn, sl + 2))
      A3_KSTEP(wf1, xf1, wf0, xf0, w_cur, x_cur, slot[2], )
      A3_KSTEP(wf0, xf0, wf1, xf1, w_cur, x_cur, slot[3], )
      // Slab sl + 1 is complete once only the 8 youngest loads (W(sl+2)) are outstanding; the barrier also says
      // that every wave has fetched its last fragments of slab sl (LDS counter at zero first), whose stage of
      // activation rows the loads issued next overwrite (and whose weight stage W(sl+3) will).
      __builtin_amdgcn_s_waitcnt(vmcnt_imm(kLW) & ~(15 << 8));
      __builtin_amdgcn_s_barrier();
      A3_KSTEP(wf1, xf1, wf0, xf0, w_nxt, x_nxt, slot[0], if (i < kLX) A3_X_LOAD(i, x_cur, sl + 2))
      { const int t = w_cur; w_cur = w_nxt; w_nxt = w_nn; w_nn = t; }
      { const int t = x_cur; x_cur = x_nxt; x_nxt = t; }
    }
#undef A3_KSTEP
#undef A3_FRAG8
#undef A3_W_LOAD
#undef A3_X_LOAD
#undef A3_KB
  }
#undef A3_FENCE
#undef A3_DMA
  __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));                    // drain the tail loads before LDS is released
}

}  // namespace
