// Internal helpers shared by the HIP translation units of liba3 (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "a3.h"

#define A3_VERSION 100

// ---- error reporting -------------------------------------------------------------------
a3_status a3_fail(a3_status code, const char *fmt, ...);
a3_status a3_check_layout(const a3_layout *L, const char *who, bool need_tables);

#define A3_REQUIRE(cond, code, ...)                 \
  do {                                              \
    if (!(cond)) return a3_fail(code, __VA_ARGS__); \
  } while (0)

#define A3_CHECK_LAUNCH(who)                                                              \
  do {                                                                                    \
    hipError_t e_ = hipGetLastError();                                                    \
    if (e_ != hipSuccess) return a3_fail(A3_ERR_HIP, "%s: %s", who, hipGetErrorString(e_)); \
  } while (0)

static inline bool a3_aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
static inline float a3_scale_of(const a3_layout *L) {
  return L->sm_scale != 0.f ? L->sm_scale : 1.0f / sqrtf((float)L->head_dim);
}
static inline size_t a3_align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// ---- set-up that has to happen once per device (kernel attributes): thread-safe, per device ----------
#include <mutex>
constexpr int kA3MaxDevices = 64;
struct a3_once_per_device {
  std::once_flag flag[kA3MaxDevices];
  hipError_t err[kA3MaxDevices];
};
// runs fn() (returning a hipError_t) the first time it is called with the current device; returns what fn returned
template <typename F>
static inline hipError_t a3_once(a3_once_per_device &o, F fn) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kA3MaxDevices) return hipErrorInvalidDevice;
  std::call_once(o.flag[dev], [&]() { o.err[dev] = fn(); });
  return o.err[dev];
}

// ---- tuning values (a3_set_tuning): process-wide, -1 = the library's own choice ------------------------
enum a3_knob {
  A3_KNOB_ATTN_WGS = 0,        // workgroups (shares) per KV head in the attention plan
  A3_KNOB_ATTN_ITEM_COST,      // start-up cost of a tile in the plan, in key steps
  A3_KNOB_PROJ_NTW,            // row-tile width (2, 3, 4 x 64 rows) of the projection GEMM; also sends few rows there
  A3_KNOB_PROJ_K64,            // 0: the projection's main loop on 64-byte row pieces
  A3_KNOB_GEMM_TB,             // row-tile width of the GEMMs of H(.)
  A3_KNOB_GEMM_K64,            // 0: their main loop on 64-byte row pieces
  A3_KNOB_COUNT
};
int a3_knob(int which);

// ---- device-side numeric helpers ----------------------------------------------------------
typedef __bf16 bf16_t;
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

__device__ __forceinline__ float a3_bf2f(bf16_t x) { return (float)x; }
__device__ __forceinline__ bf16_t a3_f2bf(float x) { return (bf16_t)x; }   // round-to-nearest-even

// (x0, x1) turned by the angle whose (cos, sin) is cs.  One definition, with the contraction written out,
// for every kernel that realigns cached keys (Eq. 2): they then round alike, bit for bit.
__device__ __forceinline__ void a3_rotate_pair(float x0, float x1, float2 cs, float &y0, float &y1) {
  y0 = __fmaf_rn(x0, cs.x, -__fmul_rn(x1, cs.y));
  y1 = __fmaf_rn(x0, cs.y, __fmul_rn(x1, cs.x));
}

template <typename T> struct a3_elem;
template <> struct a3_elem<float> {
  static constexpr int kVec = 4;   // elements per 16-byte vector
  __device__ static __forceinline__ float load(const float *p) { return *p; }
  __device__ static __forceinline__ void store(float *p, float v) { *p = v; }
};
template <> struct a3_elem<bf16_t> {
  static constexpr int kVec = 8;
  __device__ static __forceinline__ float load(const bf16_t *p) { return (float)*p; }
  __device__ static __forceinline__ void store(bf16_t *p, float v) { *p = (bf16_t)v; }
};

// ---- workspace carving (host) ---------------------------------------------------------------
struct a3_ws_cursor {
  char *base;
  size_t off, cap;
  a3_ws_cursor(void *p, size_t n) : base((char *)p), off(0), cap(n) {}
  void *take(size_t bytes) {
    off = a3_align_up(off, 256);
    void *r = base ? base + off : nullptr;
    off += bytes;
    return r;
  }
  bool fits() const { return off <= cap; }
};

// ---- streaming accesses: for tensors every byte of which is touched once per kernel (a cache copied, expanded,
// realigned), nontemporal loads and stores keep them from displacing what the caches should hold and run measurably
// faster on this chip (position recovery of 32 MiB: 14.9 -> 13.3 us) -------------------------------------------
typedef unsigned int a3_u32x4 __attribute__((ext_vector_type(4)));
template <typename P> __device__ __forceinline__ void a3_nt_store(P *p, uint4 v) {
  a3_u32x4 w = {v.x, v.y, v.z, v.w};
  __builtin_nontemporal_store(w, reinterpret_cast<a3_u32x4 *>(p));
}
template <typename P> __device__ __forceinline__ uint4 a3_nt_load(const P *p) {
  const a3_u32x4 w = __builtin_nontemporal_load(reinterpret_cast<const a3_u32x4 *>(p));
  return make_uint4(w.x, w.y, w.z, w.w);
}

// ---- per-step launchers (one per translation unit) ---------------------------------------------
size_t a3_scores_ws_bytes(const a3_layout *L);
size_t a3_attn_ws_bytes(const a3_layout *L, int max_active_rows);
