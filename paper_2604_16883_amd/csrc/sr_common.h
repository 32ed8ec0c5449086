// SinkRouter decode attention for MI355X: constants, bf16 helpers and cache addressing shared by the kernels.
#ifndef SR_COMMON_H
#define SR_COMMON_H

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "sr_config.h"

#ifndef SR_P_SPLIT
#define SR_P_SPLIT 1      // softmax weights enter the P.V MFMA as bf16 hi + bf16 lo (1) or bf16 only (0)
#endif

namespace {

constexpr int kOStride = kD + 4;     // LDS row stride (floats) of the per-wave output tile

// Timeline build: thread 0 of the workgroup stores the chip-wide wall clock into slot i of its row.
#if SR_TIMELINE
#define SR_STAMP(buf, per_group, i) do { if ((buf) && threadIdx.x == 0) (buf)[(size_t)blockIdx.x * (per_group) + (i)] = wall_clock64(); } while (0)
#else
#define SR_STAMP(buf, per_group, i) do { } while (0)
#endif

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

// 128-bit streaming load: V rows are read exactly once per step, so they are fetched with the
// non-temporal hint and do not displace the queries and partial records from the caches.
__device__ __forceinline__ uint4 load_stream(const uint4* p) {
  const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));
  return make_uint4(v.x, v.y, v.z, v.w);
}

__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

__device__ __forceinline__ uint32_t f32_to_bf16_rne(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return 0x7fc0u;
  u += 0x7fffu + ((u >> 16) & 1u);
  return u >> 16;
}

// K_0 of (sequence, KV group) bg: row bg of the separately cached anchors [B,H_kv,D] when the caller
// keeps them (Section 4.3 layout), else token 0 of the group's key cache.
__device__ __forceinline__ const uint4* anchor_row(const void* k_cache, const void* k0, int bg, int Lmax, int Hkv,
                                                   const PageMap& pm) {
  if (k0) return static_cast<const uint4*>(k0) + (size_t)bg * (kD / 8);
  if (pm.table) {
    const int b = bg / Hkv, g = bg - b * Hkv;
    return static_cast<const uint4*>(k_cache) + paged_offset(pm, page_of(pm, b, 0), Hkv, g, 0);
  }
  return static_cast<const uint4*>(k_cache) + (size_t)bg * Lmax * (kD / 8);
}

}  // namespace

#endif
