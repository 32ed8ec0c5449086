// SinkRouter decode attention for MI355X: the routing signal (Section 4.2), the standalone probe kernel
// and the prefill-side anchor kernel.
#ifndef SR_ROUTE_H
#define SR_ROUTE_H

#include "sr_common.h"

namespace {

// ------------------------------------------------------------------------------------------
// Routing signal (Section 4.2).  Four adjacent lanes share one query head: lane4 owns the 16-byte
// chunks lane4, lane4+4, lane4+8, lane4+12 of the 256-byte row.  The standalone probe kernel and
// the probe fused into the balanced partial kernel run exactly this arithmetic, in this order, so
// their decisions are identical.
// ------------------------------------------------------------------------------------------
// x + x of the lane whose index differs in bit 0 (kXor1) or bit 1 of the quad: one DPP move each.
template <int kCtrl>
__device__ __forceinline__ float quad_swap_add(float x) {
  const int y = __builtin_amdgcn_update_dpp(0, __float_as_int(x), kCtrl, 0xF, 0xF, false);
  return x + __int_as_float(y);
}

// a.lo * b.lo + a.hi * b.hi + acc on one 32-bit word of two bf16 (v_dot2c_f32_bf16: the products of bf16
// values are exact in fp32), a fifth of the instructions that unpacking to fp32 and three FMAs take.
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ float dot2_bf16(uint32_t a, uint32_t b, float acc) {
  return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, a), __builtin_bit_cast(bf16x2, b), acc, false);
}

// Square root for the norms of Eq. 7 and Eq. 11: the hardware instruction (1 ulp), not the correctly rounded
// library sequence; the probe sits in front of every workgroup's first K/V load, so its instruction count matters.
// The probe, the fused probe and the anchor kernel all take their norms from here, so they agree bit for bit.
__device__ __forceinline__ float norm_of(float sumsq) { return __builtin_amdgcn_sqrtf(sumsq); }

// Sum of squares of one 256-byte row held by a quad (4 chunks per lane): ||K_0||^2 of Eq. 7.
__device__ __forceinline__ float quad_sumsq(const uint4 (&kw)[4]) {
  float kk = 0.f;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const uint32_t ks[4] = {kw[j].x, kw[j].y, kw[j].z, kw[j].w};
#pragma unroll
    for (int e = 0; e < 4; ++e) kk = dot2_bf16(ks[e], ks[e], kk);
  }
  kk = quad_swap_add<0xB1>(kk);
  return quad_swap_add<0x4E>(kk);
}

// Eq. 11 for one head; qw / kw are this lane's four chunks of the query and of K_0.
// anchor_norm < 0 means "recompute ||K_0||".  All 4 lanes of the head must be active.
__device__ __forceinline__ float head_cosine(const uint4 (&qw)[4], const uint4 (&kw)[4], float anchor_norm) {
  float dot = 0.f, qq = 0.f;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const uint32_t qs[4] = {qw[j].x, qw[j].y, qw[j].z, qw[j].w}, ks[4] = {kw[j].x, kw[j].y, kw[j].z, kw[j].w};
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      dot = dot2_bf16(qs[e], ks[e], dot);
      qq = dot2_bf16(qs[e], qs[e], qq);
    }
  }
  dot = quad_swap_add<0xB1>(dot); qq = quad_swap_add<0xB1>(qq);   // quad_perm [1,0,3,2]
  dot = quad_swap_add<0x4E>(dot); qq = quad_swap_add<0x4E>(qq);   // quad_perm [2,3,0,1]
  const float nk = anchor_norm >= 0.f ? anchor_norm : norm_of(quad_sumsq(kw));
  const float den = norm_of(qq) * nk;
  return (den > 0.f) ? dot * __builtin_amdgcn_rcpf(den) : 0.f;
}

// Eq. 12-13 and the cubic threshold of Appendix A.  cosines: the G values of the group, in head order.
__device__ __forceinline__ bool route_decide(const float* cosines, int G, int L, const RouteRule& r, float* S_out) {
  float S = 0.f;
  for (int j = 0; j < G; ++j) S += cosines[j];
  S *= __builtin_amdgcn_rcpf((float)G);        // hardware reciprocal (1 ulp; exact for the usual power-of-two G)
  const float x = r.len_norm > 0.f ? (float)L * __builtin_amdgcn_rcpf(r.len_norm) : 0.f;
  const float tau = ((r.tau[0] * x + r.tau[1]) * x + r.tau[2]) * x + r.tau[3];
  *S_out = S;
  return r.routing && L > 0 && S > tau;       // strict; NaN compares false, so the group stays active
}

// Standalone probe.  grid = B*H_kv, block = 64: 4 lanes per head, up to 16 heads.
struct ProbeArgs {
  const uint4* q;
  const void* k;
  const void* k0;          // optional separate anchors
  const int32_t* seq_lens;
  const float* k0_norm;    // optional
  float* group_score;      // optional
  uint8_t* mask;
  int Hq, Hkv, G, Lmax;
  RouteRule rule;
  PageMap pm;
};

__global__ __launch_bounds__(64) void sr_probe_kernel(ProbeArgs a) {
  __shared__ float cosv[kMaxGroup];
  const int bg = blockIdx.x;
  const int b = bg / a.Hkv, g = bg - b * a.Hkv;
  const int lane4 = threadIdx.x & 3, i = threadIdx.x >> 2;
  const int hd = i < a.G ? i : 0;
  const uint4* krow = anchor_row(a.k, a.k0, bg, a.Lmax, a.Hkv, a.pm);
  const uint4* qrow = a.q + ((size_t)b * a.Hq + (size_t)g * a.G + hd) * (kD / 8);
  uint4 qw[4], kw[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) { qw[j] = qrow[lane4 + 4 * j]; kw[j] = krow[lane4 + 4 * j]; }
  const float c = head_cosine(qw, kw, a.k0_norm ? a.k0_norm[bg] : -1.f);
  if (lane4 == 0 && i < a.G) cosv[i] = c;
  __syncthreads();
  if (threadIdx.x == 0) {
    float S;
    const bool skip = route_decide(cosv, a.G, clamp_len(a.seq_lens[b], a.Lmax), a.rule, &S);
    if (a.group_score) a.group_score[bg] = S;
    a.mask[bg] = skip ? 1 : 0;
  }
}

// Prefill-side anchor caching (Section 4.1): copies row 0 of every group's key cache to
// k0_out [B,H_kv,D] and its norm to k0_norm_out [B,H_kv].  One quad per group; the norm is computed
// exactly as the probe recomputes it, so decisions do not depend on which of the two is used.
__global__ __launch_bounds__(64) void sr_anchor_kernel(const void* k_cache, uint4* k0_out, float* k0_norm_out, int NG, int Lmax,
                                                       int Hkv, PageMap pm) {
  const int lane4 = threadIdx.x & 3;
  int bg = blockIdx.x * 16 + (threadIdx.x >> 2);
  const bool ok = bg < NG;
  bg = ok ? bg : NG - 1;
  const uint4* krow = anchor_row(k_cache, nullptr, bg, Lmax, Hkv, pm);
  uint4 kw[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) kw[j] = krow[lane4 + 4 * j];
  const float kk = quad_sumsq(kw);
  if (ok) {
    if (k0_out) {
#pragma unroll
      for (int j = 0; j < 4; ++j) k0_out[(size_t)bg * (kD / 8) + lane4 + 4 * j] = kw[j];
    }
    if (k0_norm_out && lane4 == 0) k0_norm_out[bg] = norm_of(kk);
  }
}

}  // namespace

#endif
