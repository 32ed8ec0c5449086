// SinkRouter decode attention for MI355X (gfx950, CDNA4): kernels and the C ABI.
//
// Kernels of one decode step, all on the caller's stream:
//   sr_probe_kernel    routing signal of Section 4.2 (Eq. 11-13): one wavefront per
//                      (sequence, KV group), four lanes per query head; reads the group's query
//                      heads and token 0 of K only.  Normally fused into the balanced partial
//                      kernel (every workgroup evaluates the rule for all groups itself); launched
//                      on its own for large batches, fixed chunks and sinkrouter_probe.
//   sr_partial_*       Split-K partial attention of Section 4.3 for Active Groups only.
//                      Each wavefront streams 64-token K/V blocks straight from HBM into
//                      registers with 128-bit loads and feeds them to the matrix cores: all
//                      query heads of the group form the N dimension of the MFMA tile, so one
//                      K/V fetch serves every head of the group without expansion (the
//                      paper's group-centric layout) and without an LDS round trip.  Online
//                      softmax per block.  The 4 wavefronts of a workgroup interleave blocks
//                      and merge their results through LDS into one partial (m, l, o) per
//                      (head, workgroup).  Two schedules:
//        balanced  (default) one workgroup per compute unit; every workgroup first obtains the
//                  skip decisions of all groups (fused probe, or the mask of sr_probe_kernel), so
//                  the 64-token blocks of the Active Groups only are dealt out in equal contiguous
//                  shares.  Sink Groups cost nothing and the chip stays
//                  full whatever the skip pattern is.
//        fixed     the paper's literal Split-K: [0, L) cut into num_splits chunks, one
//                  workgroup per (chunk, sequence, KV group); workgroups of Sink Groups
//                  leave at once.
//   sr_combine_kernel  log-sum-exp merge of the partials, bf16 output; zeros for Sink Groups
//                      (Eq. 14).
//
// Register layout of the MFMA shape used for both products (lane = 0..63, r16 = lane % 16, kg = lane / 16):
//   v_mfma_f32_16x16x32_bf16  A: row r16, 8 consecutive k of k-group kg; B: column r16, same k;
//                             D: column r16, rows 4*kg + {0,1,2,3} in the 4 result registers.
// Only "A row = lane%16, B column = lane%16, both operands use the same k slot" is relied on,
// so any consistent assignment of head-dimension elements to k slots gives the right dot product.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "sinkrouter.h"

#ifndef SR_P_SPLIT
#define SR_P_SPLIT 1      // softmax weights enter the P.V MFMA as bf16 hi + bf16 lo (1) or bf16 only (0)
#endif

namespace {

constexpr int kD = 128;              // head dimension
constexpr int kBlock = 64;           // tokens per online-softmax block (B_K)
#ifndef SR_WAVES
#define SR_WAVES 4
#endif
constexpr int kWaves = SR_WAVES;     // wavefronts per partial workgroup
constexpr int kThreads = 64 * kWaves;
constexpr int kMaxGroup = 16;        // query heads per KV group that fit the MFMA tile
constexpr int kChunkUnit = kBlock * kWaves;
constexpr int kOStride = kD + 4;     // LDS row stride (floats) of the per-wave output tile
constexpr int kCombineThreads = 1024;
#ifndef SR_GRID
#define SR_GRID 256
#endif
constexpr int kBalancedGrid = SR_GRID;   // one workgroup per compute unit: measured best (512 and 1024 are 3-6% slower)
constexpr int kMaxSchedGroups = 2048;  // (sequence, KV group) pairs the balanced schedule scans in LDS
constexpr int kMaxFusedHeads = 512;    // query heads (all sequences) the balanced kernel probes itself

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

__device__ __forceinline__ int clamp_len(int L, int Lmax) { return L < 0 ? 0 : (L > Lmax ? Lmax : L); }

// Paged KV cache: pages of 2^page_shift tokens laid out [n_pages, H_kv, page_tokens, D]; logical
// page j of sequence b is physical page table[b * pages_per_seq + j] (clamped to the pool, so a
// bad entry reads a wrong page but never leaves the allocation).  table == NULL: contiguous cache.
struct PageMap {
  const int32_t* table;
  int page_shift, pages_per_seq, n_pages;
};

__device__ __forceinline__ int page_of(const PageMap& pm, int b, int tok) {
  int pg = pm.table[(size_t)b * pm.pages_per_seq + (tok >> pm.page_shift)];
  pg = pg < 0 ? 0 : pg;
  return pg < pm.n_pages ? pg : pm.n_pages - 1;
}

// Offset (in 16-byte units) of token `tok` of group g in a page pool, given its physical page.
__device__ __forceinline__ size_t paged_offset(const PageMap& pm, int page, int Hkv, int g, int tok) {
  return ((((size_t)page * Hkv + g) << pm.page_shift) + (tok & ((1 << pm.page_shift) - 1))) * (kD / 8);
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

// ------------------------------------------------------------------------------------------
// Routing signal (Section 4.2).  Four adjacent lanes share one query head: lane4 owns the 16-byte
// chunks lane4, lane4+4, lane4+8, lane4+12 of the 256-byte row.  The standalone probe kernel and
// the probe fused into the balanced partial kernel run exactly this arithmetic, in this order, so
// their decisions are identical.
// ------------------------------------------------------------------------------------------
struct RouteRule {
  float tau[4], len_norm;
  int routing;
};

// x + x of the lane whose index differs in bit 0 (kXor1) or bit 1 of the quad: one DPP move each.
template <int kCtrl>
__device__ __forceinline__ float quad_swap_add(float x) {
  const int y = __builtin_amdgcn_update_dpp(0, __float_as_int(x), kCtrl, 0xF, 0xF, false);
  return x + __int_as_float(y);
}

// Sum of squares of one 256-byte row held by a quad (4 chunks per lane): ||K_0||^2 of Eq. 7.
__device__ __forceinline__ float quad_sumsq(const uint4 (&kw)[4]) {
  float kk = 0.f;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const uint32_t ks[4] = {kw[j].x, kw[j].y, kw[j].z, kw[j].w};
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const float k0 = bf16_lo(ks[e]), k1 = bf16_hi(ks[e]);
      kk = fmaf(k0, k0, kk);
      kk = fmaf(k1, k1, kk);
    }
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
      const float q0 = bf16_lo(qs[e]), q1 = bf16_hi(qs[e]), k0 = bf16_lo(ks[e]), k1 = bf16_hi(ks[e]);
      dot = fmaf(q0, k0, dot); dot = fmaf(q1, k1, dot);
      qq = fmaf(q0, q0, qq);   qq = fmaf(q1, q1, qq);
    }
  }
  dot = quad_swap_add<0xB1>(dot); qq = quad_swap_add<0xB1>(qq);   // quad_perm [1,0,3,2]
  dot = quad_swap_add<0x4E>(dot); qq = quad_swap_add<0x4E>(qq);   // quad_perm [2,3,0,1]
  const float nk = anchor_norm >= 0.f ? anchor_norm : sqrtf(quad_sumsq(kw));
  const float den = sqrtf(qq) * nk;
  return (den > 0.f) ? dot / den : 0.f;
}

// Eq. 12-13 and the cubic threshold of Appendix A.  cosines: the G values of the group, in head order.
__device__ __forceinline__ bool route_decide(const float* cosines, int G, int L, const RouteRule& r, float* S_out) {
  float S = 0.f;
  for (int j = 0; j < G; ++j) S += cosines[j];
  S /= (float)G;
  const float x = r.len_norm > 0.f ? (float)L / r.len_norm : 0.f;
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
    if (k0_norm_out && lane4 == 0) k0_norm_out[bg] = sqrtf(kk);
  }
}

// ------------------------------------------------------------------------------------------
// Split-K partial attention.
// ------------------------------------------------------------------------------------------
struct PartialArgs {
  const uint16_t* q;
  const uint16_t* k;
  const uint16_t* v;
  const int32_t* seq_lens;
  uint8_t* mask;    // [B*Hkv] read (written first when the probe is fused)
  const void* k0;         // fused probe: optional separate anchors [B,H_kv,D]
  const float* k0_norm;   // fused probe: optional cached ||K_0||
  float* group_score;     // fused probe: S_g out
  RouteRule rule;         // fused probe
  float* part_o;    // [B*Hq, slots, D]  sum_t 2^(z_t - m) v_t
  float* part_ml;   // [B*Hq, slots, 2]  m (log2 domain), l
  int32_t* sched;   // balanced schedule only: U, c, start[0..NG]
  int Hq, Hkv, G, Lmax, NG;
  int chunk;        // fixed schedule: tokens per chunk
  int slots;        // partial records per head
  float scale_log2; // softmax scale * log2(e)
  PageMap pm;
};

// Loads of one 64-token block whose first row is row0 of the slab at Kbase / Vbase (a contiguous
// (sequence, group) cache, or one group's part of a page: a block never straddles a page).
// row_last is the slab row of the last valid token of the sequence: rows are clamped to it, so a
// ragged tail never reads beyond seq_len.
//
// K tile T, step j: lane (r16, kg) holds row row0+16T+r16, elements (4j+kg)*8 .. +8.
// A row reaches the wavefront as 64-byte pieces, two loads per 128-byte line, so these stay
// ordinary cached loads (the second piece of a line hits); a non-temporal hint here costs bandwidth.
__device__ __forceinline__ void load_k_tile(uint4 (&kr)[4], const uint4* __restrict__ Kbase, int row0, int T,
                                            int r16, int kg, int row_last) {
  int row = row0 + 16 * T + r16;
  row = row < row_last ? row : row_last;
  const uint4* p = Kbase + (size_t)row * 16 + kg;
#pragma unroll
  for (int j = 0; j < 4; ++j) kr[j] = p[4 * j];
}

// V tile T, row r: lane (r16, kg) holds row row0+16T+4kg+r, elements 8*r16 .. +8: each load
// instruction covers four whole 256-byte rows.
__device__ __forceinline__ void load_v_tile(uint4 (&vr)[4], const uint4* __restrict__ Vbase, int row0, int T,
                                            int r16, int kg, int row_last) {
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    int row = row0 + 16 * T + 4 * kg + r;
    row = row < row_last ? row : row_last;
    vr[r] = load_stream(Vbase + (size_t)row * 16 + r16);
  }
}

struct WaveState {
  float m_run;     // running max of head r16 (log2 domain), same in the 4 lane groups
  float l_run;     // this lane's share of the running sum
  f32x4 acc[8];    // acc[e][vv] = O[head r16][32*kg + 8*vv + e]
};

// One 64-token block: scores, online softmax, P.V.  With kPrefetch the loads of the block at
// `next` are issued tile by tile, each as soon as the registers it overwrites have been consumed,
// so the loop body has no conditional loads and the wait counts the compiler inserts stay exact.
// The scheduling barriers keep the compiler from hoisting a prefetch above the MFMAs that still
// read its registers (it would need a second register set) or sinking it to the end of the block.
template <bool kPrefetch>
__device__ __forceinline__ void block_step(WaveState& w, uint4 (&kr)[4][4], uint4 (&vr)[4][4], const bf16x8 (&qb)[4],
                                           const uint4* __restrict__ Kn, const uint4* __restrict__ Vn, int row0_n, int row_last_n,
                                           int tok0, int t_end, int r16, int kg, float scale_log2) {
  // ---- scores: sc[T][r] = q_{r16} . k_{tok0+16T+4kg+r}
  f32x4 sc[4];
#pragma unroll
  for (int T = 0; T < 4; ++T) {
    sc[T] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int j = 0; j < 4; ++j)
      sc[T] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, kr[T][j]), qb[j], sc[T], 0, 0, 0);
    __builtin_amdgcn_sched_barrier(0);
    if (kPrefetch) load_k_tile(kr[T], Kn, row0_n, T, r16, kg, row_last_n);
    __builtin_amdgcn_sched_barrier(0);
  }
  // ---- online softmax over the block
  float bm = -INFINITY;
#pragma unroll
  for (int T = 0; T < 4; ++T)
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int tok = tok0 + 16 * T + 4 * kg + r;
      float z = sc[T][r] * scale_log2;
      z = tok < t_end ? z : -INFINITY;
      sc[T][r] = z;
      bm = fmaxf(bm, z);
    }
  bm = fmaxf(bm, __shfl_xor(bm, 16, 64));
  bm = fmaxf(bm, __shfl_xor(bm, 32, 64));
  const float m_new = fmaxf(w.m_run, bm);
  const float alpha = __builtin_amdgcn_exp2f(w.m_run - m_new);
  float ps = 0.f;
#pragma unroll
  for (int T = 0; T < 4; ++T)
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const float p = __builtin_amdgcn_exp2f(sc[T][r] - m_new);
      sc[T][r] = p;
      ps += p;
    }
  w.l_run = w.l_run * alpha + ps;
  w.m_run = m_new;
#pragma unroll
  for (int e = 0; e < 8; ++e) w.acc[e] *= alpha;
  // ---- O^T += V^T P^T on the bf16 matrix cores, two 16-token tiles per MFMA (k = 32).
  // A = V^T: row = this lane's 16-byte column chunk r16, and the lane's k slots are the 8 tokens it
  // loaded for tiles T and T+1 (4kg + r each): for one element e of the chunk, v_perm gathers its
  // 8 token values out of the 8 loaded rows, so V needs no transpose through LDS.
  // B = P^T: column = head r16, same 8 tokens - the lane's own probabilities.  P enters as bf16
  // hi + bf16 lo (two MFMAs), which keeps ~16 mantissa bits; products accumulate in fp32.
#pragma unroll
  for (int T = 0; T < 4; T += 2) {
    bf16x8 bhi, blo;
    {
      float pv[8] = {sc[T][0], sc[T][1], sc[T][2], sc[T][3], sc[T + 1][0], sc[T + 1][1], sc[T + 1][2], sc[T + 1][3]};
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const __bf16 hv = (__bf16)pv[i];
        bhi[i] = hv;
#if SR_P_SPLIT
        blo[i] = (__bf16)(pv[i] - (float)hv);
#endif
      }
    }
    const uint32_t wa[4][4] = {{vr[T][0].x, vr[T][0].y, vr[T][0].z, vr[T][0].w}, {vr[T][1].x, vr[T][1].y, vr[T][1].z, vr[T][1].w},
                               {vr[T][2].x, vr[T][2].y, vr[T][2].z, vr[T][2].w}, {vr[T][3].x, vr[T][3].y, vr[T][3].z, vr[T][3].w}};
    const uint32_t wb[4][4] = {{vr[T + 1][0].x, vr[T + 1][0].y, vr[T + 1][0].z, vr[T + 1][0].w}, {vr[T + 1][1].x, vr[T + 1][1].y, vr[T + 1][1].z, vr[T + 1][1].w},
                               {vr[T + 1][2].x, vr[T + 1][2].y, vr[T + 1][2].z, vr[T + 1][2].w}, {vr[T + 1][3].x, vr[T + 1][3].y, vr[T + 1][3].z, vr[T + 1][3].w}};
#pragma unroll
    for (int m = 0; m < 4; ++m) {                 // 32-bit word m of the chunk = elements 2m, 2m+1
#pragma unroll
      for (int half = 0; half < 2; ++half) {
        const uint32_t sel = half ? 0x07060302u : 0x05040100u;   // high / low bf16 of both words
        uint4 av;
        av.x = __builtin_amdgcn_perm(wa[1][m], wa[0][m], sel);
        av.y = __builtin_amdgcn_perm(wa[3][m], wa[2][m], sel);
        av.z = __builtin_amdgcn_perm(wb[1][m], wb[0][m], sel);
        av.w = __builtin_amdgcn_perm(wb[3][m], wb[2][m], sel);
        const bf16x8 am = __builtin_bit_cast(bf16x8, av);
        const int e = 2 * m + half;
        w.acc[e] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(am, bhi, w.acc[e], 0, 0, 0);
#if SR_P_SPLIT
        w.acc[e] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(am, blo, w.acc[e], 0, 0, 0);
#endif
      }
    }
    __builtin_amdgcn_sched_barrier(0);
    if (kPrefetch) { load_v_tile(vr[T], Vn, row0_n, T, r16, kg, row_last_n); load_v_tile(vr[T + 1], Vn, row0_n, T + 1, r16, kg, row_last_n); }
    __builtin_amdgcn_sched_barrier(0);
  }
}

// Attention of the G heads of group (b, g) over tokens [t_begin, t_end) (t_begin a multiple of 64,
// t_begin < t_end <= L), by the whole workgroup; writes partial record `slot` of each head.
// Every thread of the workgroup must call it (it synchronises).
template <bool kPaged>
__device__ __forceinline__ void attend_range(const PartialArgs& a, int b, int g, int L, int t_begin, int t_end, int slot) {
  __shared__ float lds_o[kWaves][kMaxGroup][kOStride];
  __shared__ float lds_m[kWaves][kMaxGroup];
  __shared__ float lds_l[kWaves][kMaxGroup];
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int r16 = lane & 15, kg = lane >> 4;
  const int G = a.G;
  const int bg = b * a.Hkv + g;
  const int last = L - 1;

  // B operand of Q.K^T: column r16 = query head (zero beyond the group), same k slots as K.
  bf16x8 qb[4];
  {
    const bool ok = r16 < G;
    const uint4* qrow = reinterpret_cast<const uint4*>(a.q + ((size_t)b * a.Hq + (size_t)g * G + (ok ? r16 : 0)) * kD);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      uint4 x = qrow[4 * j + kg];
      if (!ok) x = make_uint4(0, 0, 0, 0);
      qb[j] = __builtin_bit_cast(bf16x8, x);
    }
  }
  // Slab = the rows that share one base pointer: the whole (sequence, group) cache, or the group's
  // part of one page.  slab_base(page) is its offset in 16-byte units, slab_row(tok) the row of a token.
  const uint4* K4 = reinterpret_cast<const uint4*>(a.k);
  const uint4* V4 = reinterpret_cast<const uint4*>(a.v);
  const int page_mask = kPaged ? (1 << a.pm.page_shift) - 1 : 0;
  auto slab_base = [&](int page) -> size_t {
    return kPaged ? (((size_t)page * a.Hkv + g) << a.pm.page_shift) * (kD / 8) : (size_t)bg * a.Lmax * (kD / 8);
  };
  auto slab_row = [&](int tok) -> int { return kPaged ? (tok & page_mask) : tok; };

  WaveState w;
  w.m_run = -INFINITY;
  w.l_run = 0.f;
#pragma unroll
  for (int e = 0; e < 8; ++e) w.acc[e] = f32x4{0.f, 0.f, 0.f, 0.f};

  constexpr int kStep = kWaves * kBlock;   // the wavefronts of the workgroup interleave 64-token blocks
  int tok0 = t_begin + wave * kBlock;
  if (tok0 < t_end) {
    uint4 kr[4][4], vr[4][4];
    {
      const size_t base = slab_base(kPaged ? page_of(a.pm, b, tok0) : 0);
      const int row0 = slab_row(tok0), row_last = row0 + (last - tok0);
#pragma unroll
      for (int T = 0; T < 4; ++T) load_k_tile(kr[T], K4 + base, row0, T, r16, kg, row_last);
#pragma unroll
      for (int T = 0; T < 4; ++T) load_v_tile(vr[T], V4 + base, row0, T, r16, kg, row_last);
    }
    int next = tok0 + kStep;
    // paged: the page of a block is looked up one iteration before the block is prefetched
    int page_n = (kPaged && next < t_end) ? page_of(a.pm, b, next) : 0;
    while (next < t_end) {
      const size_t base = slab_base(page_n);
      const int row0 = slab_row(next), row_last = row0 + (last - next);
      if (kPaged) page_n = page_of(a.pm, b, min(next + kStep, last));
      block_step<true>(w, kr, vr, qb, K4 + base, V4 + base, row0, row_last, tok0, t_end, r16, kg, a.scale_log2);
      tok0 = next;
      next += kStep;
    }
    block_step<false>(w, kr, vr, qb, K4, V4, 0, 0, tok0, t_end, r16, kg, a.scale_log2);
  }

  // ---- merge the 4 wavefronts through LDS, write one partial per head
  float l_run = w.l_run;
  l_run += __shfl_xor(l_run, 16, 64);
  l_run += __shfl_xor(l_run, 32, 64);
  if (r16 < G) {
    float* row = &lds_o[wave][r16][32 * kg];
#pragma unroll
    for (int vv = 0; vv < 4; ++vv) {
      *reinterpret_cast<float4*>(row + 8 * vv) = make_float4(w.acc[0][vv], w.acc[1][vv], w.acc[2][vv], w.acc[3][vv]);
      *reinterpret_cast<float4*>(row + 8 * vv + 4) = make_float4(w.acc[4][vv], w.acc[5][vv], w.acc[6][vv], w.acc[7][vv]);
    }
    if (kg == 0) { lds_m[wave][r16] = w.m_run; lds_l[wave][r16] = l_run; }
  }
  __syncthreads();
  const int c4 = threadIdx.x & 31;            // float4 column
  for (int h = threadIdx.x >> 5; h < G; h += kThreads / 32) {
    float M = lds_m[0][h];
#pragma unroll
    for (int u = 1; u < kWaves; ++u) M = fmaxf(M, lds_m[u][h]);
    float4 o = make_float4(0.f, 0.f, 0.f, 0.f);
    float l = 0.f;
#pragma unroll
    for (int u = 0; u < kWaves; ++u) {
      const float wt = __builtin_amdgcn_exp2f(lds_m[u][h] - M);   // wave 0 always holds a block, so M is finite
      const float4 x = *reinterpret_cast<const float4*>(&lds_o[u][h][4 * c4]);
      o.x += wt * x.x; o.y += wt * x.y; o.z += wt * x.z; o.w += wt * x.w;
      l += wt * lds_l[u][h];
    }
    const size_t rec = ((size_t)b * a.Hq + (size_t)g * G + h) * a.slots + slot;
    *reinterpret_cast<float4*>(a.part_o + rec * kD + 4 * c4) = o;
    if (c4 == 0) *reinterpret_cast<float2*>(a.part_ml + rec * 2) = make_float2(M, l);
  }
}

// Fixed schedule.  grid = (num_splits, B*H_kv), block = 256.
template <bool kPaged>
__global__ __launch_bounds__(kThreads, 2) void sr_partial_fixed_kernel(PartialArgs a) {
  const int s = blockIdx.x;
  const int bg = blockIdx.y;
  if (a.mask[bg]) return;                       // Sink Group: no K/V row is touched
  const int b = bg / a.Hkv, g = bg - b * a.Hkv;
  const int L = clamp_len(a.seq_lens[b], a.Lmax);
  const int t_begin = s * a.chunk;
  if (t_begin >= L) return;                     // chunk lies beyond this sequence
  attend_range<kPaged>(a, b, g, L, t_begin, min(t_begin + a.chunk, L), s);
}

// Balanced schedule.  grid = kBalancedGrid, block = 256.  Unit = one 64-token block of an Active
// Group; units are numbered group after group; workgroup p owns units [p*c, (p+1)*c), c = ceil(U/P).
// Partial record j of a group belongs to workgroup (start/c + j).  Workgroup 0 leaves the schedule
// (U, c, start[]) in `sched` for the merge kernel.
// With kFused every workgroup first evaluates the routing rule for all groups itself (the queries
// and anchor rows are a few tens of KB, served by L2), as the paper's kernel does inline, so no
// separate probe launch precedes it; workgroup 0 writes skip mask and group scores.  Otherwise
// the mask written by sr_probe_kernel is read.
template <bool kFused, bool kPaged>
__global__ __launch_bounds__(kThreads, 2) void sr_partial_balanced_kernel(PartialArgs a) {
  __shared__ int start[kMaxSchedGroups + 1];
  __shared__ int lens[kMaxSchedGroups];
  __shared__ float cosv[kFused ? kMaxFusedHeads : 1];
  __shared__ int wsum[kWaves];
  __shared__ int first_group;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int NG = a.NG, G = a.G;
  // share index = workgroup index: the stream has no reuse, so which XCD works on which share is
  // immaterial (giving each XCD one contiguous eighth of the blocks measured the same)
  const int p = blockIdx.x, P = gridDim.x;
  // the first length load is issued here and parked in a register, so that it and the probe's query /
  // anchor loads are in flight together (one memory round trip at kernel start instead of two)
  int len_first = 0;
  if (tid < NG) len_first = a.seq_lens[tid / a.Hkv];
  if (kFused && a.rule.routing) {
    const int NH = NG * G, lane4 = tid & 3;
    const uint4* q4 = reinterpret_cast<const uint4*>(a.q);
    for (int h0 = 0; h0 < NH; h0 += kThreads / 2) {      // kThreads/4 heads per sweep, two sweeps in flight
      uint4 qw[2][4], kw[2][4];
      float kn[2];
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        int hd = h0 + (kThreads / 4) * u + (tid >> 2);
        hd = hd < NH ? hd : NH - 1;
        const int i = hd / G;
        const uint4* qrow = q4 + (size_t)hd * (kD / 8);
        const uint4* krow = anchor_row(a.k, a.k0, i, a.Lmax, a.Hkv, a.pm);
#pragma unroll
        for (int j = 0; j < 4; ++j) { qw[u][j] = qrow[lane4 + 4 * j]; kw[u][j] = krow[lane4 + 4 * j]; }
        kn[u] = a.k0_norm ? a.k0_norm[i] : -1.f;
      }
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        const int hd = h0 + (kThreads / 4) * u + (tid >> 2);
        const float cs = head_cosine(qw[u], kw[u], kn[u]);
        if (lane4 == 0 && hd < NH) cosv[hd] = cs;
      }
    }
  }
  if (tid < NG) lens[tid] = clamp_len(len_first, a.Lmax);
  for (int i = tid + kThreads; i < NG; i += kThreads) lens[i] = clamp_len(a.seq_lens[i / a.Hkv], a.Lmax);
  __syncthreads();
  int carry = 0;
  for (int base = 0; base < NG; base += kThreads) {
    const int i = base + tid;
    int u = 0;
    if (i < NG) {
      bool skip;
      if (kFused) {
        float S = 0.f;
        skip = a.rule.routing ? route_decide(cosv + i * G, G, lens[i], a.rule, &S) : false;
        if (p == 0) { a.mask[i] = skip ? 1 : 0; if (a.group_score) a.group_score[i] = S; }
      } else {
        skip = a.mask[i] != 0;
      }
      if (!skip) u = (lens[i] + kBlock - 1) / kBlock;
    }
    int x = u;                                   // inclusive scan inside the wavefront
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
      const int y = __shfl_up(x, o, 64);
      if (lane >= o) x += y;
    }
    if (lane == 63) wsum[wave] = x;
    __syncthreads();
    int woff = 0;
#pragma unroll
    for (int u2 = 0; u2 < kWaves; ++u2) if (u2 < wave) woff += wsum[u2];
    int tot = 0;
#pragma unroll
    for (int u2 = 0; u2 < kWaves; ++u2) tot += wsum[u2];
    if (i < NG) start[i] = carry + woff + x - u;
    carry += tot;
    __syncthreads();
  }
  const int U = carry;
  if (tid == 0) start[NG] = U;
  const int c = (U + P - 1) / P;
  __syncthreads();
  if (p == 0) {
    if (tid == 0) { a.sched[0] = U; a.sched[1] = c; }
    for (int i = tid; i <= NG; i += kThreads) a.sched[2 + i] = start[i];
  }
  const int u_lo = p * c, u_hi = min(u_lo + c, U);
  if (u_lo >= u_hi) return;
  for (int i = tid; i < NG; i += kThreads)
    if (start[i] <= u_lo && u_lo < start[i + 1]) first_group = i;   // exactly one group holds u_lo
  __syncthreads();
  for (int i = first_group; i < NG && start[i] < u_hi; ++i) {
    const int s0 = start[i], s1 = start[i + 1];
    if (s1 == s0) continue;                     // Sink Group or empty sequence
    const int b = i / a.Hkv, g = i - b * a.Hkv;
    const int L = lens[i];
    const int blk_lo = max(u_lo, s0) - s0, blk_hi = min(u_hi, s1) - s0;
    attend_range<kPaged>(a, b, g, L, blk_lo * kBlock, min(blk_hi * kBlock, L), p - s0 / c);
    __syncthreads();                            // LDS of attend_range is reused by the next segment
  }
}

// ------------------------------------------------------------------------------------------
// Merge of the partials.  grid = B*H_q, block = 1024 (16 wavefronts; lane owns 2 columns).
// ------------------------------------------------------------------------------------------
struct CombineArgs {
  const float* part_o;
  const float* part_ml;
  const int32_t* seq_lens;
  const uint8_t* mask;
  const int32_t* sched;   // balanced schedule, else NULL
  uint32_t* out;          // bf16 pairs
  int Hq, Hkv, G, Lmax, chunk, slots;
  // diagnostics (optional): log-sum-exp of the scaled scores and softmax mass on token 0 per head
  const uint32_t* q;      // bf16 pairs
  const void* k;          // contiguous key cache (diagnostics are not offered for paged caches)
  float* lse_out;
  float* alpha0_out;
  float scale_log2;
  // concentration mode (max_rest_out set): the partials cover tokens 1..L-1 of the cache whose row 0
  // is at k; token 0 is folded in here.  lens_full holds the unshifted lengths.
  const int32_t* lens_full;
  float* max_rest_out;
  float* mean_rest_out;
};

__global__ __launch_bounds__(kCombineThreads) void sr_combine_kernel(CombineArgs a) {
  constexpr int NW = kCombineThreads / 64;
  constexpr int UN = 8;
  const int bh = blockIdx.x;
  const int b = bh / a.Hq, h = bh - b * a.Hq, g = h / a.G;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int L = clamp_len(a.seq_lens[b], a.Lmax);
  const int bg = b * a.Hkv + g;
  uint32_t* orow = a.out + (size_t)bh * (kD / 2);
  int n = 0;                                     // partial records of this head
  if (!a.mask[bg] && L > 0) {
    if (a.sched) {
      const int c = a.sched[1], s0 = a.sched[2 + bg], s1 = a.sched[3 + bg];
      if (s1 > s0) n = (s1 - 1) / c - s0 / c + 1;
    } else {
      n = (L + a.chunk - 1) / a.chunk;
    }
  }
  if (n == 0) {                                  // zero surrogate (Eq. 14) / empty sequence
    if (wave == 0) orow[lane] = 0u;
    if (threadIdx.x == 0) {                      // not computed for Sink Groups; an empty row has lse = -inf
      const float nan = __int_as_float(0x7fc00000);
      if (a.max_rest_out) {                      // a one-token cache has all its weight on token 0
        const bool one = clamp_len(a.lens_full[b], a.Lmax) == 1;
        a.alpha0_out[bh] = one ? 1.f : nan;
        a.max_rest_out[bh] = one ? 0.f : nan;
        a.mean_rest_out[bh] = one ? 0.f : nan;
      } else {
        if (a.lse_out) a.lse_out[bh] = (L == 0) ? -INFINITY : nan;
        if (a.alpha0_out) a.alpha0_out[bh] = nan;
      }
    }
    return;
  }
  const float2* ml = reinterpret_cast<const float2*>(a.part_ml) + (size_t)bh * a.slots;
  const float2* po = reinterpret_cast<const float2*>(a.part_o) + (size_t)bh * a.slots * (kD / 2);

  __shared__ float red_m[NW];
  __shared__ float red_l[NW];
  __shared__ float2 red_o[NW][64];
  float mx = -INFINITY;
  for (int s = threadIdx.x; s < n; s += kCombineThreads) mx = fmaxf(mx, ml[s].x);
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o, 64));
  if (lane == 0) red_m[wave] = mx;
  __syncthreads();
  float M = red_m[0];
#pragma unroll
  for (int u = 1; u < NW; ++u) M = fmaxf(M, red_m[u]);

  float2 acc = make_float2(0.f, 0.f);
  float lsum = 0.f;
  for (int s0 = wave; s0 < n; s0 += NW * UN) {   // UN rows in flight per wavefront
    float2 st[UN], o[UN];
#pragma unroll
    for (int u = 0; u < UN; ++u) {
      const int s = s0 + u * NW;
      const bool ok = s < n;
      st[u] = ok ? ml[s] : make_float2(-INFINITY, 0.f);
      o[u] = ok ? po[(size_t)s * (kD / 2) + lane] : make_float2(0.f, 0.f);
    }
#pragma unroll
    for (int u = 0; u < UN; ++u) {
      const float wt = __builtin_amdgcn_exp2f(st[u].x - M);
      acc.x += wt * o[u].x;
      acc.y += wt * o[u].y;
      lsum += wt * st[u].y;
    }
  }
  red_o[wave][lane] = acc;
  if (lane == 0) red_l[wave] = lsum;
  __syncthreads();
  if (wave == 0) {
    float2 t = red_o[0][lane];
    float l = red_l[0];
#pragma unroll
    for (int u = 1; u < NW; ++u) { t.x += red_o[u][lane].x; t.y += red_o[u][lane].y; l += red_l[u]; }
    const float inv = 1.0f / l;
    orow[lane] = f32_to_bf16_rne(t.x * inv) | (f32_to_bf16_rne(t.y * inv) << 16);
    if (a.lse_out || a.alpha0_out) {
      const float lse2 = M + __builtin_amdgcn_logf(l);                  // log2 domain (v_log_f32 is log2)
      if (a.alpha0_out) {                                               // alpha_0 = exp(z_0 - lse), Section 4.2
        const uint32_t qw = a.q[(size_t)bh * (kD / 2) + lane];
        const uint32_t kw = reinterpret_cast<const uint32_t*>(a.k)[(size_t)bg * a.Lmax * (kD / 2) + lane];   // token 0 of the cache itself
        float d = bf16_lo(qw) * bf16_lo(kw) + bf16_hi(qw) * bf16_hi(kw);
#pragma unroll
        for (int o = 32; o >= 1; o >>= 1) d += __shfl_xor(d, o, 64);
        if (a.max_rest_out) {                                           // Table 1 (Section 3): lse2 and M are those of tokens >= 1
          const float z0 = d * a.scale_log2;
          const float hi = fmaxf(z0, lse2);
          const float full = hi + __builtin_amdgcn_logf(__builtin_amdgcn_exp2f(z0 - hi) + __builtin_amdgcn_exp2f(lse2 - hi));
          if (lane == 0) {
            a.alpha0_out[bh] = __builtin_amdgcn_exp2f(z0 - full);
            a.max_rest_out[bh] = __builtin_amdgcn_exp2f(M - full);
            a.mean_rest_out[bh] = __builtin_amdgcn_exp2f(lse2 - full) / (float)L;
          }
        } else if (lane == 0) {
          a.alpha0_out[bh] = __builtin_amdgcn_exp2f(d * a.scale_log2 - lse2);
        }
      }
      if (a.lse_out && lane == 0) a.lse_out[bh] = lse2 * 0.6931471805599453f;
    }
  }
}

// Lengths of the caches with token 0 taken off, for the concentration statistics.
__global__ __launch_bounds__(256) void sr_rest_lens_kernel(const int32_t* seq_lens, int32_t* rest, int B, int Lmax) {
  const int b = blockIdx.x * 256 + threadIdx.x;
  if (b < B) rest[b] = max(clamp_len(seq_lens[b], Lmax) - 1, 0);
}

// ------------------------------------------------------------------------------------------
// Measurement helpers.
// ------------------------------------------------------------------------------------------
constexpr int kProbeGrid = 1024;

// Streaming read at the pattern that measured fastest on MI355X: every wavefront reads whole 16 KB
// pieces (16 non-temporal 128-bit loads per lane in flight), pieces dealt round-robin to the wavefronts.
__global__ __launch_bounds__(256) void sr_read_probe_kernel(const uint4* __restrict__ p, size_t n16, uint32_t* sink) {
  constexpr int U = 16;
  const int lane = threadIdx.x & 63;
  const size_t wave = (size_t)blockIdx.x * 4 + (threadIdx.x >> 6), nw = (size_t)gridDim.x * 4;
  const size_t piece = (size_t)U * 64;                     // 128-bit words per piece
  uint32_t x = 0;
  size_t c = wave * piece;
  for (; c + piece <= n16; c += nw * piece) {
    uint4 a[U];
#pragma unroll
    for (int u = 0; u < U; ++u) a[u] = load_stream(p + c + (size_t)u * 64 + lane);
#pragma unroll
    for (int u = 0; u < U; ++u) x ^= a[u].x ^ a[u].y ^ a[u].z ^ a[u].w;
  }
  // the tail that does not fill a whole round of pieces
  const size_t done = n16 / piece * piece;
  for (size_t i = done + (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += (size_t)gridDim.x * 256) {
    const uint4 a = p[i];
    x ^= a.x ^ a.y ^ a.z ^ a.w;
  }
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) x ^= __shfl_xor(x, o, 64);
  __shared__ uint32_t red[4];
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = x;
  __syncthreads();
  if (threadIdx.x == 0) sink[blockIdx.x] = red[0] ^ red[1] ^ red[2] ^ red[3];
}

__global__ __launch_bounds__(256) void sr_copy_probe_kernel(uint4* __restrict__ dst, const uint4* __restrict__ src, size_t n16) {
  const size_t stride = (size_t)gridDim.x * 256;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += stride) dst[i] = src[i];
}

// ------------------------------------------------------------------------------------------
// Host side.
// ------------------------------------------------------------------------------------------
inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

struct Layout {
  sr_plan plan;
  size_t off_o, off_ml, off_score, off_sched, off_lens;
};

int make_layout(const sr_route_params* p, Layout* lay) {
  if (!p) return SR_ERR_NULL;
  if (p->struct_size != sizeof(sr_route_params)) return SR_ERR_UNSUPPORTED;
  if (p->batch < 1 || p->n_q_heads < 1 || p->n_kv_heads < 1 || p->max_seq_len < 1 || p->num_splits < 0)
    return SR_ERR_SHAPE;
  if (p->n_q_heads % p->n_kv_heads != 0) return SR_ERR_SHAPE;
  if ((int64_t)p->batch * p->n_kv_heads > 65535) return SR_ERR_SHAPE;
  if ((int64_t)p->batch * p->n_q_heads > (int64_t)1 << 24) return SR_ERR_SHAPE;
  if (p->max_seq_len > (1 << 24)) return SR_ERR_SHAPE;          // 32-bit token arithmetic stays exact
  if (p->head_dim != kD || p->kv_block != kBlock) return SR_ERR_UNSUPPORTED;
  const int G = p->n_q_heads / p->n_kv_heads;
  if (G > kMaxGroup) return SR_ERR_UNSUPPORTED;
  if (!(p->sm_scale >= 0.f) || p->sm_scale > 1e30f) return SR_ERR_SHAPE;

  const int NG = p->batch * p->n_kv_heads;
  const int blocks = (p->max_seq_len + kBlock - 1) / kBlock;
  sr_plan& pl = lay->plan;
  pl.group_size = G;
  if (p->num_splits == 0 && NG <= kMaxSchedGroups && (int64_t)NG * blocks < ((int64_t)1 << 30)) {
    pl.schedule = 1;
    pl.chunk_tokens = 0;
    pl.num_splits = 0;
    pl.partial_grid = kBalancedGrid;
    pl.slots_per_head = blocks < kBalancedGrid + 1 ? blocks : kBalancedGrid + 1;
  } else {
    int chunk;
    if (p->num_splits > 0) {
      const int per = (p->max_seq_len + p->num_splits - 1) / p->num_splits;
      chunk = (int)align_up((size_t)per, kChunkUnit);
    } else {
      // too many groups to schedule in LDS: plain chunks sized so that, with about 40% of the
      // groups active (the paper's retained budget, Section 5.1), some 2048 workgroups have work
      const double active_tokens = 0.4 * (double)NG * p->max_seq_len;
      int units = (int)(active_tokens / (2048.0 * kChunkUnit));
      units = units < 1 ? 1 : (units > 8 ? 8 : units);
      chunk = units * kChunkUnit;
    }
    pl.schedule = 0;
    pl.chunk_tokens = chunk;
    pl.num_splits = (p->max_seq_len + chunk - 1) / chunk;
    pl.partial_grid = pl.num_splits * NG;
    pl.slots_per_head = pl.num_splits;
  }
  const size_t heads = (size_t)p->batch * p->n_q_heads;
  const size_t S = (size_t)pl.slots_per_head;
  lay->off_o = 0;
  lay->off_ml = align_up(heads * S * kD * sizeof(float), 256);
  lay->off_score = lay->off_ml + align_up(heads * S * 2 * sizeof(float), 256);
  lay->off_sched = lay->off_score + align_up((size_t)NG * sizeof(float), 256);
  lay->off_lens = lay->off_sched + align_up((size_t)(NG + 3) * sizeof(int32_t), 256);
  pl.workspace_bytes = lay->off_lens + align_up((size_t)p->batch * sizeof(int32_t), 256);
  return SR_OK;
}

inline bool misaligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) != 0; }

RouteRule make_rule(const sr_route_params* p) {
  RouteRule r;
  for (int i = 0; i < 4; ++i) r.tau[i] = p->tau_coef[i];
  r.len_norm = p->len_norm;
  r.routing = p->routing_enabled != 0;
  return r;
}

int launch_probe(const void* q, const void* k, const int32_t* seq_lens, const sr_route_params* p,
                 const Layout& lay, float* score, uint8_t* mask, hipStream_t st, const PageMap& pm) {
  ProbeArgs a;
  a.pm = pm;
  a.q = static_cast<const uint4*>(q);
  a.k = k;
  a.k0 = p->k0;
  a.seq_lens = seq_lens;
  a.k0_norm = p->k0_norm;
  a.group_score = score;
  a.mask = mask;
  a.Hq = p->n_q_heads; a.Hkv = p->n_kv_heads; a.G = lay.plan.group_size; a.Lmax = p->max_seq_len;
  a.rule = make_rule(p);
  hipLaunchKernelGGL(sr_probe_kernel, dim3(p->batch * p->n_kv_heads), dim3(64), 0, st, a);
  return hipGetLastError() == hipSuccess ? SR_OK : SR_ERR_HIP;
}

// Outputs of the concentration statistics; decode_impl then attends over tokens 1..L-1 only.
struct RestStats {
  float* max_rest;
  float* mean_rest;
};

int decode_impl(const void* q, const void* k, const void* v, const int32_t* seq_lens,
                const sr_route_params* p, void* out, uint8_t* mask, float* stage_us,
                float* lse_out = nullptr, float* alpha0_out = nullptr, const PageMap* pages = nullptr,
                const RestStats* rest = nullptr) {
  if (!q || !k || !v || !seq_lens || !p || !out || !mask) return SR_ERR_NULL;
  Layout lay;
  int rc = make_layout(p, &lay);
  if (rc != SR_OK) return rc;
  if (misaligned(q, 16) || misaligned(k, 16) || misaligned(v, 16) || misaligned(out, 16) || misaligned(seq_lens, 4) ||
      misaligned(p->k0, 16) || misaligned(p->k0_norm, 4) || misaligned(lse_out, 4) || misaligned(alpha0_out, 4) ||
      (rest && (misaligned(rest->max_rest, 4) || misaligned(rest->mean_rest, 4))))
    return SR_ERR_ALIGN;
  if (!p->workspace || misaligned(p->workspace, 256) || p->workspace_bytes < lay.plan.workspace_bytes)
    return SR_ERR_WORKSPACE;
  hipStream_t st = static_cast<hipStream_t>(p->stream);
  char* ws = static_cast<char*>(p->workspace);
  float* part_o = reinterpret_cast<float*>(ws + lay.off_o);
  float* part_ml = reinterpret_cast<float*>(ws + lay.off_ml);
  float* score = reinterpret_cast<float*>(ws + lay.off_score);
  int32_t* sched = reinterpret_cast<int32_t*>(ws + lay.off_sched);
  const bool balanced = lay.plan.schedule == 1;
  PageMap pm = {nullptr, 0, 0, 0};
  if (pages) pm = *pages;
  const bool paged = pm.table != nullptr;
  const bool fused = balanced && (int64_t)p->batch * p->n_q_heads <= kMaxFusedHeads;
  // Concentration statistics: the caches are entered one row later with lengths one shorter, so the
  // partial kernels see tokens 1..L-1 (row L-1 is the last one read, as in a plain call).
  const void* k_anchor = k;
  const int32_t* lens_full = seq_lens;
  if (rest) {
    int32_t* lens_rest = reinterpret_cast<int32_t*>(ws + lay.off_lens);
    hipLaunchKernelGGL(sr_rest_lens_kernel, dim3((p->batch + 255) / 256), dim3(256), 0, st, seq_lens, lens_rest,
                       p->batch, p->max_seq_len);
    if (hipGetLastError() != hipSuccess) return SR_ERR_HIP;
    seq_lens = lens_rest;
    k = static_cast<const uint16_t*>(k) + kD;
    v = static_cast<const uint16_t*>(v) + kD;
  }

  hipEvent_t ev[4] = {nullptr, nullptr, nullptr, nullptr};
  if (stage_us) {
    for (int i = 0; i < 4; ++i)
      if (hipEventCreate(&ev[i]) != hipSuccess) {
        for (int j = 0; j < i; ++j) (void)hipEventDestroy(ev[j]);
        return SR_ERR_HIP;
      }
  }
  auto mark = [&](int i) { return !stage_us || hipEventRecord(ev[i], st) == hipSuccess; };
  bool ok = mark(0);
  if (ok && !fused) ok = launch_probe(q, k_anchor, seq_lens, p, lay, score, mask, st, pm) == SR_OK;
  if (ok) ok = mark(1);
  if (ok) {
    PartialArgs a;
    a.q = static_cast<const uint16_t*>(q);
    a.k = static_cast<const uint16_t*>(k);
    a.v = static_cast<const uint16_t*>(v);
    a.seq_lens = seq_lens; a.mask = mask; a.part_o = part_o; a.part_ml = part_ml; a.sched = sched;
    a.k0 = p->k0; a.k0_norm = p->k0_norm; a.group_score = score; a.rule = make_rule(p);
    a.Hq = p->n_q_heads; a.Hkv = p->n_kv_heads; a.G = lay.plan.group_size; a.Lmax = p->max_seq_len;
    a.NG = p->batch * p->n_kv_heads;
    a.chunk = lay.plan.chunk_tokens; a.slots = lay.plan.slots_per_head;
    const float scale = p->sm_scale > 0.f ? p->sm_scale : 0.08838834764831845f;   // 1/sqrt(128)
    a.scale_log2 = scale * 1.4426950408889634f;
    a.pm = pm;
    const dim3 blk(kThreads), fixed_grid(lay.plan.num_splits, a.NG);
    if (fused && paged)       hipLaunchKernelGGL((sr_partial_balanced_kernel<true, true>), dim3(kBalancedGrid), blk, 0, st, a);
    else if (fused)           hipLaunchKernelGGL((sr_partial_balanced_kernel<true, false>), dim3(kBalancedGrid), blk, 0, st, a);
    else if (balanced && paged) hipLaunchKernelGGL((sr_partial_balanced_kernel<false, true>), dim3(kBalancedGrid), blk, 0, st, a);
    else if (balanced)        hipLaunchKernelGGL((sr_partial_balanced_kernel<false, false>), dim3(kBalancedGrid), blk, 0, st, a);
    else if (paged)           hipLaunchKernelGGL(sr_partial_fixed_kernel<true>, fixed_grid, blk, 0, st, a);
    else                      hipLaunchKernelGGL(sr_partial_fixed_kernel<false>, fixed_grid, blk, 0, st, a);
    ok = hipGetLastError() == hipSuccess;
  }
  const float scale_log2 = (p->sm_scale > 0.f ? p->sm_scale : 0.08838834764831845f) * 1.4426950408889634f;
  if (ok) ok = mark(2);
  if (ok) {
    CombineArgs c;
    c.q = static_cast<const uint32_t*>(q); c.k = k_anchor;
    c.lse_out = lse_out; c.alpha0_out = alpha0_out; c.scale_log2 = scale_log2;
    c.lens_full = lens_full;
    c.max_rest_out = rest ? rest->max_rest : nullptr;
    c.mean_rest_out = rest ? rest->mean_rest : nullptr;
    c.part_o = part_o; c.part_ml = part_ml; c.seq_lens = seq_lens; c.mask = mask;
    c.sched = balanced ? sched : nullptr;
    c.out = static_cast<uint32_t*>(out);
    c.Hq = p->n_q_heads; c.Hkv = p->n_kv_heads; c.G = lay.plan.group_size; c.Lmax = p->max_seq_len;
    c.chunk = lay.plan.chunk_tokens; c.slots = lay.plan.slots_per_head;
    hipLaunchKernelGGL(sr_combine_kernel, dim3(p->batch * p->n_q_heads), dim3(kCombineThreads), 0, st, c);
    ok = hipGetLastError() == hipSuccess;
  }
  if (ok) ok = mark(3);
  if (stage_us) {
    if (ok) ok = hipEventSynchronize(ev[3]) == hipSuccess;
    if (ok) {
      for (int i = 0; i < 3 && ok; ++i) {
        float ms = 0.f;
        ok = hipEventElapsedTime(&ms, ev[i], ev[i + 1]) == hipSuccess;
        stage_us[i] = ms * 1000.f;
      }
      float ms = 0.f;
      if (ok) ok = hipEventElapsedTime(&ms, ev[0], ev[3]) == hipSuccess;
      stage_us[3] = ms * 1000.f;
    }
    for (int i = 0; i < 4; ++i) (void)hipEventDestroy(ev[i]);
  }
  return ok ? SR_OK : SR_ERR_HIP;
}

}  // namespace

extern "C" {

int sinkrouter_plan(const sr_route_params* params, sr_plan* plan) {
  if (!params || !plan) return SR_ERR_NULL;
  Layout lay;
  const int rc = make_layout(params, &lay);
  if (rc != SR_OK) return rc;
  *plan = lay.plan;
  return SR_OK;
}

size_t sinkrouter_workspace_bytes(const sr_route_params* params) {
  Layout lay;
  if (make_layout(params, &lay) != SR_OK) return 0;
  return lay.plan.workspace_bytes;
}

int sinkrouter_decode(const void* q, const void* k_cache, const void* v_cache, const int32_t* seq_lens,
                      const sr_route_params* params, void* out, uint8_t* skip_mask_out) {
  return decode_impl(q, k_cache, v_cache, seq_lens, params, out, skip_mask_out, nullptr);
}

int sinkrouter_decode_profiled(const void* q, const void* k_cache, const void* v_cache, const int32_t* seq_lens,
                               const sr_route_params* params, void* out, uint8_t* skip_mask_out,
                               float* stage_us) {
  if (!stage_us) return SR_ERR_NULL;
  return decode_impl(q, k_cache, v_cache, seq_lens, params, out, skip_mask_out, stage_us);
}

int sinkrouter_probe(const void* q, const void* k_cache, const int32_t* seq_lens,
                     const sr_route_params* params, float* group_score_out, uint8_t* skip_mask_out) {
  if (!q || !k_cache || !seq_lens || !params || !skip_mask_out) return SR_ERR_NULL;
  Layout lay;
  const int rc = make_layout(params, &lay);
  if (rc != SR_OK) return rc;
  if (misaligned(q, 16) || misaligned(k_cache, 16) || misaligned(seq_lens, 4) || misaligned(group_score_out, 4) ||
      misaligned(params->k0, 16) || misaligned(params->k0_norm, 4))
    return SR_ERR_ALIGN;
  const PageMap none = {nullptr, 0, 0, 0};
  return launch_probe(q, k_cache, seq_lens, params, lay, group_score_out, skip_mask_out,
                      static_cast<hipStream_t>(params->stream), none);
}

int sinkrouter_decode_diag(const void* q, const void* k_cache, const void* v_cache, const int32_t* seq_lens,
                           const sr_route_params* params, void* out, uint8_t* skip_mask_out,
                           float* lse_out, float* alpha0_out) {
  if (!lse_out && !alpha0_out) return SR_ERR_NULL;
  return decode_impl(q, k_cache, v_cache, seq_lens, params, out, skip_mask_out, nullptr, lse_out, alpha0_out);
}

int sinkrouter_concentration(const void* q, const void* k_cache, const void* v_cache, const int32_t* seq_lens,
                             const sr_route_params* params, void* out_rest, uint8_t* skip_mask_out,
                             float* alpha0_out, float* max_rest_out, float* mean_rest_out) {
  if (!params || !alpha0_out || !max_rest_out || !mean_rest_out) return SR_ERR_NULL;
  if (params->struct_size != sizeof(sr_route_params)) return SR_ERR_UNSUPPORTED;
  sr_route_params dense = *params;              // every head is measured: no routing, no cached anchors
  dense.routing_enabled = 0;
  dense.k0 = nullptr;
  dense.k0_norm = nullptr;
  const RestStats rest = {max_rest_out, mean_rest_out};
  return decode_impl(q, k_cache, v_cache, seq_lens, &dense, out_rest, skip_mask_out, nullptr, nullptr, alpha0_out,
                     nullptr, &rest);
}

int sinkrouter_decode_paged(const void* q, const void* k_pages, const void* v_pages, const int32_t* block_table,
                            const int32_t* seq_lens, const sr_route_params* params, const sr_paged_layout* layout,
                            void* out, uint8_t* skip_mask_out) {
  if (!block_table || !layout || !params) return SR_ERR_NULL;
  if (layout->struct_size != sizeof(sr_paged_layout)) return SR_ERR_UNSUPPORTED;
  const int pt = layout->page_tokens;
  if (pt < kBlock || (pt & (pt - 1)) != 0) return SR_ERR_UNSUPPORTED;       // power of two, >= one block
  if (layout->n_pages < 1 || layout->pages_per_seq < 1) return SR_ERR_SHAPE;
  if (params->max_seq_len < 1 || (int64_t)layout->pages_per_seq * pt < params->max_seq_len) return SR_ERR_SHAPE;
  if (misaligned(block_table, 4)) return SR_ERR_ALIGN;
  PageMap pm;
  pm.table = block_table;
  pm.page_shift = __builtin_ctz((unsigned)pt);
  pm.pages_per_seq = layout->pages_per_seq;
  pm.n_pages = layout->n_pages;
  return decode_impl(q, k_pages, v_pages, seq_lens, params, out, skip_mask_out, nullptr, nullptr, nullptr, &pm);
}

int sinkrouter_extract_anchor(const void* k_cache, const sr_route_params* params, void* k0_out, float* k0_norm_out) {
  if (!k_cache || !params || (!k0_out && !k0_norm_out)) return SR_ERR_NULL;
  Layout lay;
  const int rc = make_layout(params, &lay);
  if (rc != SR_OK) return rc;
  if (misaligned(k_cache, 16) || misaligned(k0_out, 16) || misaligned(k0_norm_out, 4)) return SR_ERR_ALIGN;
  const int NG = params->batch * params->n_kv_heads;
  const PageMap none = {nullptr, 0, 0, 0};
  hipLaunchKernelGGL(sr_anchor_kernel, dim3((NG + 15) / 16), dim3(64), 0, static_cast<hipStream_t>(params->stream),
                     k_cache, static_cast<uint4*>(k0_out), k0_norm_out, NG, params->max_seq_len, params->n_kv_heads, none);
  return hipGetLastError() == hipSuccess ? SR_OK : SR_ERR_HIP;
}

int sinkrouter_hbm_read_probe(const void* buf, size_t bytes, void* sink, void* stream) {
  if (!buf || !sink) return SR_ERR_NULL;
  if (bytes == 0 || bytes % 16 != 0) return SR_ERR_SHAPE;
  if (misaligned(buf, 16) || misaligned(sink, 4)) return SR_ERR_ALIGN;
  hipLaunchKernelGGL(sr_read_probe_kernel, dim3(kProbeGrid), dim3(256), 0, static_cast<hipStream_t>(stream),
                     static_cast<const uint4*>(buf), bytes / 16, static_cast<uint32_t*>(sink));
  return hipGetLastError() == hipSuccess ? SR_OK : SR_ERR_HIP;
}

int sinkrouter_hbm_copy_probe(void* dst, const void* src, size_t bytes, void* stream) {
  if (!dst || !src) return SR_ERR_NULL;
  if (bytes == 0 || bytes % 16 != 0) return SR_ERR_SHAPE;
  if (misaligned(dst, 16) || misaligned(src, 16)) return SR_ERR_ALIGN;
  hipLaunchKernelGGL(sr_copy_probe_kernel, dim3(kProbeGrid * 2), dim3(256), 0, static_cast<hipStream_t>(stream),
                     static_cast<uint4*>(dst), static_cast<const uint4*>(src), bytes / 16);
  return hipGetLastError() == hipSuccess ? SR_OK : SR_ERR_HIP;
}

const char* sinkrouter_status_string(int status) {
  switch (status) {
    case SR_OK: return "ok";
    case SR_ERR_NULL: return "a required pointer is NULL";
    case SR_ERR_SHAPE: return "invalid or inconsistent sizes";
    case SR_ERR_UNSUPPORTED: return "unsupported configuration (head_dim must be 128, kv_block 64, group size <= 16, struct_size must match)";
    case SR_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case SR_ERR_ALIGN: return "tensor pointer not 16-byte aligned";
    case SR_ERR_HIP: return "HIP runtime error";
    default: return "unknown status";
  }
}

int sinkrouter_abi_version(void) { return SINKROUTER_ABI_VERSION; }

}  // extern "C"
