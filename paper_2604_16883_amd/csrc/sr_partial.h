// SinkRouter decode attention for MI355X: Split-K partial attention (Section 4.3) on the bf16 matrix cores,
// fixed and balanced schedules.
//
// Register layout of the MFMA shape used for both products (lane = 0..63, r16 = lane % 16, kg = lane / 16):
//   v_mfma_f32_16x16x32_bf16  A: row r16, 8 consecutive k of k-group kg; B: column r16, same k;
//                             D: column r16, rows 4*kg + {0,1,2,3} in the 4 result registers.
// Only "A row = lane%16, B column = lane%16, both operands use the same k slot" is relied on,
// so any consistent assignment of head-dimension elements to k slots gives the right dot product.
#ifndef SR_PARTIAL_H
#define SR_PARTIAL_H

#include "sr_common.h"
#include "sr_route.h"

namespace {

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
  uint32_t g_magic, hkv_magic;   // div_magic(G), div_magic(Hkv)
  int chunk;        // fixed schedule: tokens per chunk
  int slots;        // partial records per head
  float scale_log2; // softmax scale * log2(e)
  PageMap pm;
  long long* timeline;   // timeline build: [grid, 8] stamps; NULL otherwise
};

// Loads of one 64-token block whose first row is row0 of the slab at Kbase / Vbase (a contiguous
// (sequence, group) cache, or one group's part of a page: a block never straddles a page).
// row_last is the slab row of the last valid token of the sequence: rows are clamped to it, so a
// ragged tail never reads beyond seq_len.
//
// K tile T, step j: lane (r16, kg) holds row row0+16T+r16, elements (4j+kg)*8 .. +8.
// A row reaches the wavefront as 64-byte pieces, two loads per 128-byte line, so these stay
// ordinary cached loads (the second piece of a line hits); a non-temporal hint here costs bandwidth.
// kExact: the whole block lies inside the sequence, so no row is clamped; the address is then a wavefront-uniform
// base plus a lane offset that never changes (lane_k / lane_v below), which needs no vector address arithmetic.
template <bool kExact>
__device__ __forceinline__ void load_k_tile(uint4 (&kr)[4], const uint4* __restrict__ Kbase, int row0, int T,
                                            int r16, int kg, int row_last) {
  if (kExact) {
    const uint4* p = Kbase + (size_t)(row0 + 16 * T) * 16;          // uniform
    const unsigned lane_k = (unsigned)(r16 * 16 + kg);
#pragma unroll
    for (int j = 0; j < 4; ++j) kr[j] = p[lane_k + 4u * j];
    return;
  }
  int row = row0 + 16 * T + r16;
  row = row < row_last ? row : row_last;
  const uint4* p = Kbase + (size_t)row * 16 + kg;
#pragma unroll
  for (int j = 0; j < 4; ++j) kr[j] = p[4 * j];
}

// V tile T, row r: lane (r16, kg) holds row row0+16T+4kg+r, elements 8*r16 .. +8: each load
// instruction covers four whole 256-byte rows.
template <bool kExact>
__device__ __forceinline__ void load_v_tile(uint4 (&vr)[4], const uint4* __restrict__ Vbase, int row0, int T,
                                            int r16, int kg, int row_last) {
  if (kExact) {
    const uint4* p = Vbase + (size_t)(row0 + 16 * T) * 16;          // uniform
    const unsigned lane_v = (unsigned)(kg * 64 + r16);
#pragma unroll
    for (int r = 0; r < 4; ++r) vr[r] = load_stream(p + (lane_v + 16u * r));
    return;
  }
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
// kExact: the current block lies inside [0, t_end) (no score is masked) and the prefetched one inside the sequence (no row
// is clamped): every block but the last one or two of a range.
template <bool kPrefetch, bool kExact>
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
    if (kPrefetch) load_k_tile<kExact>(kr[T], Kn, row0_n, T, r16, kg, row_last_n);
    __builtin_amdgcn_sched_barrier(0);
  }
  // ---- online softmax over the block
  float bm = -INFINITY;
#pragma unroll
  for (int T = 0; T < 4; ++T)
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      float z = sc[T][r] * scale_log2;
      if (!kExact) {
        const int tok = tok0 + 16 * T + 4 * kg + r;
        z = tok < t_end ? z : -INFINITY;
      }
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
    if (kPrefetch) { load_v_tile<kExact>(vr[T], Vn, row0_n, T, r16, kg, row_last_n); load_v_tile<kExact>(vr[T + 1], Vn, row0_n, T + 1, r16, kg, row_last_n); }
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
      for (int T = 0; T < 4; ++T) load_k_tile<false>(kr[T], K4 + base, row0, T, r16, kg, row_last);
#pragma unroll
      for (int T = 0; T < 4; ++T) load_v_tile<false>(vr[T], V4 + base, row0, T, r16, kg, row_last);
    }
    int next = tok0 + kStep;
    // paged: the page of a block is looked up one iteration before the block is prefetched
    int page_n = (kPaged && next < t_end) ? page_of(a.pm, b, next) : 0;
#if SR_TIMELINE
    bool first_step = a.timeline && a.timeline[(size_t)blockIdx.x * kTimelinePartialStamps + 4] == 0;
#endif
    // every block but the last of a range lies inside [0, t_end), and the prefetched one inside the sequence unless it is
    // the sequence's ragged last block: those steps mask no score and clamp no row
    while (next + kBlock <= t_end) {
      const size_t base = slab_base(page_n);
      const int row0 = slab_row(next);
      if (kPaged) page_n = page_of(a.pm, b, min(next + kStep, last));
      block_step<true, true>(w, kr, vr, qb, K4 + base, V4 + base, row0, 0, tok0, t_end, r16, kg, a.scale_log2);
#if SR_TIMELINE
      if (first_step) { SR_STAMP(a.timeline, kTimelinePartialStamps, 4); first_step = false; }
#endif
      tok0 = next;
      next += kStep;
    }
    if (next < t_end) {                     // the range ends with a ragged block, and it is this wavefront's
      const size_t base = slab_base(page_n);
      const int row0 = slab_row(next), row_last = row0 + (last - next);
      block_step<true, false>(w, kr, vr, qb, K4 + base, V4 + base, row0, row_last, tok0, t_end, r16, kg, a.scale_log2);
#if SR_TIMELINE
      if (first_step) { SR_STAMP(a.timeline, kTimelinePartialStamps, 4); first_step = false; }
#endif
      tok0 = next;
    }
    block_step<false, false>(w, kr, vr, qb, K4, V4, 0, 0, tok0, t_end, r16, kg, a.scale_log2);
#if SR_TIMELINE
    if (first_step) SR_STAMP(a.timeline, kTimelinePartialStamps, 4);
#endif
  }
  SR_STAMP(a.timeline, kTimelinePartialStamps, 5);

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
  SR_STAMP(a.timeline, kTimelinePartialStamps, 6);
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

// Balanced schedule.  grid = kBalancedGrid (P), block = 256.  Unit = one 64-token block of an Active Group.
//   per-group shares (at most P/2 Active Groups): group i gets n_i workgroups in proportion to its blocks
//     (share_count), each a run of share_blocks consecutive blocks: every workgroup streams one group only.  A
//     workgroup that changes groups drains and refills its load pipeline while the rest of the chip keeps the
//     memory queues full, which costs it 3-4 us: with contiguous shares those workgroups ended the kernel.
//   contiguous shares (more Active Groups than that, or per-group shares that would occupy less than three quarters of
//     the workgroups: per_group_fills): units are numbered group after group and workgroup p
//     owns units [p*c, (p+1)*c), c = ceil(U/P); partial record j of a group belongs to workgroup (start/c + j).
// Workgroup 0 leaves the schedule in `sched` for the merge kernel: mode (1 = per-group), c, then per group
// (blocks, workgroups) or (first unit, end unit).
// With kFused every workgroup first evaluates the routing rule for all groups itself (the queries
// and anchor rows are a few tens of KB, served by L2), as the paper's kernel does inline, so no
// separate probe launch precedes it; workgroup 0 writes skip mask and group scores.  Otherwise
// the mask written by sr_probe_kernel is read.
// Inclusive prefix sum over the 64 lanes without LDS traffic: shifts inside each row of 16 lanes, then the
// totals of the rows are carried over with the two row-broadcast moves (lane 15 -> next row, lane 31 ->
// upper half).  Lanes without a source add 0.
__device__ __forceinline__ int wave_inclusive_scan(int x) {
  x += __builtin_amdgcn_update_dpp(0, x, 0x111, 0xF, 0xF, false);   // row_shr:1
  x += __builtin_amdgcn_update_dpp(0, x, 0x112, 0xF, 0xF, false);   // row_shr:2
  x += __builtin_amdgcn_update_dpp(0, x, 0x114, 0xF, 0xF, false);   // row_shr:4
  x += __builtin_amdgcn_update_dpp(0, x, 0x118, 0xF, 0xF, false);   // row_shr:8
  x += __builtin_amdgcn_update_dpp(0, x, 0x142, 0xA, 0xF, false);   // row_bcast:15 into rows 1 and 3
  x += __builtin_amdgcn_update_dpp(0, x, 0x143, 0xC, 0xF, false);   // row_bcast:31 into rows 2 and 3
  return x;
}

template <bool kFused, bool kPaged>
// (The measurement build's stamps take a few registers more than two workgroups per compute unit leave: it is built for one,
// which is what the persistent grid runs anyway.)
__global__ __launch_bounds__(kThreads, SR_TIMELINE ? 1 : 2) void sr_partial_balanced_kernel(PartialArgs a) {
  __shared__ int start[kMaxSchedGroups + 1];
  __shared__ int lens[kMaxSchedGroups];
  __shared__ float cosv[kFused ? kMaxFusedHeads : 1];
  __shared__ int wsum[2 * kWaves];
  __shared__ int first_group;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int NG = a.NG, G = a.G;
  // share index = workgroup index: the stream has no reuse, so which XCD works on which share is
  // immaterial (giving each XCD one contiguous eighth of the blocks measured the same)
  const int p = blockIdx.x;
  constexpr int P = kBalancedGrid;               // the host launches exactly this grid
  // the first length load is issued here and parked in a register, so that it and the probe's query /
  // anchor loads are in flight together (one memory round trip at kernel start instead of two)
  SR_STAMP(a.timeline, kTimelinePartialStamps, 0);
  int len_first = 0;
  if (tid < NG) len_first = a.seq_lens[div_by(tid, a.hkv_magic)];
  if (kFused && a.rule.routing) {
    const int NH = NG * G, lane4 = tid & 3;
    const uint4* q4 = reinterpret_cast<const uint4*>(a.q);
    // anchor of (sequence, group) i: row i of the separate K_0 tensor, else token 0 of its cache (contiguous caches:
    // a fixed stride; paged ones go through the block table)
    const uint4* kbase = static_cast<const uint4*>(a.k0 ? a.k0 : static_cast<const void*>(a.k));
    const size_t kstride = a.k0 ? (size_t)(kD / 8) : (size_t)a.Lmax * (kD / 8);
    for (int h0 = 0; h0 < NH; h0 += kThreads / 2) {      // kThreads/4 heads per sweep, two sweeps in flight
      uint4 qw[2][4], kw[2][4];
      float kn[2];
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        int hd = h0 + (kThreads / 4) * u + (tid >> 2);
        hd = hd < NH ? hd : NH - 1;
        const int i = div_by(hd, a.g_magic);
        const uint4* qrow = q4 + (size_t)hd * (kD / 8);
        const uint4* krow = (kPaged && !a.k0) ? anchor_row(a.k, a.k0, i, a.Lmax, a.Hkv, a.pm) : kbase + (size_t)i * kstride;
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
  SR_STAMP(a.timeline, kTimelinePartialStamps, 1);
  __syncthreads();
  SR_STAMP(a.timeline, kTimelinePartialStamps, 2);
  if (NG <= 64) {
    // Up to 64 groups: every wavefront builds the whole schedule in registers (lane = group), so no
    // further barrier or LDS round trip stands between the routing decision and the first K/V load.
    const bool live = lane < NG;
    const int len_i = live ? lens[lane] : 0;
    bool skip = false;
    float S = 0.f;
    if (live) {
      if (kFused) skip = a.rule.routing ? route_decide(cosv + lane * G, G, len_i, a.rule, &S) : false;
      else skip = a.mask[lane] != 0;
    }
    if (kFused && p == 0 && wave == 0 && live) { a.mask[lane] = skip ? 1 : 0; if (a.group_score) a.group_score[lane] = S; }
    const int u = (live && !skip) ? (len_i + kBlock - 1) / kBlock : 0;
    const int x = wave_inclusive_scan(u);        // over the groups
    const int U = __builtin_amdgcn_readlane(x, 63);
    const int A = __popcll(__ballot(u > 0));
    // at most 64 Active Groups, fewer than half the workgroups: always per-group shares
    static_assert(2 * 64 <= kBalancedGrid, "the register-built schedule relies on per-group shares");
    const int n = share_count(u, U, P, A);
    const int ns = wave_inclusive_scan(n) - n;    // first workgroup of the group
    if (p == 0 && wave == 0) {
      if (lane == 0) { a.sched[0] = 1; a.sched[1] = 0; }
      if (live) { a.sched[2 + 2 * lane] = u; a.sched[3 + 2 * lane] = n; }
    }
    SR_STAMP(a.timeline, kTimelinePartialStamps, 3);
    const unsigned long long holds = __ballot(n > 0 && ns <= p && p < ns + n);   // at most one group
    if (!holds) return;                           // fewer shares than workgroups, or nothing active
    const int i = __ffsll(holds) - 1;
    const int ui = __builtin_amdgcn_readlane(u, i), j = p - __builtin_amdgcn_readlane(ns, i);
    const int cb = share_blocks(ui, __builtin_amdgcn_readlane(n, i));
    const int blk_lo = j * cb, blk_hi = min(blk_lo + cb, ui);
    if (blk_lo >= blk_hi) return;                 // more workgroups than the group has blocks
    const int L = __builtin_amdgcn_readlane(len_i, i);
    const int b = div_by(i, a.hkv_magic), g = i - b * a.Hkv;
    attend_range<kPaged>(a, b, g, L, blk_lo * kBlock, min(blk_hi * kBlock, L), j);
    SR_STAMP(a.timeline, kTimelinePartialStamps, 7);
    return;
  }
  // More than 64 groups: the schedule is built in LDS.  Pass 1: decisions, blocks per group (a Sink Group's length
  // is kept as -1 - L so that it counts no blocks), their total and the number of Active Groups.
  int my_U = 0, my_A = 0;
  for (int i = tid; i < NG; i += kThreads) {
    bool skip;
    if (kFused) {
      float S = 0.f;
      skip = a.rule.routing ? route_decide(cosv + i * G, G, lens[i], a.rule, &S) : false;
      if (p == 0) { a.mask[i] = skip ? 1 : 0; if (a.group_score) a.group_score[i] = S; }
    } else {
      skip = a.mask[i] != 0;
    }
    if (skip) lens[i] = -1 - lens[i];
    const int u = skip ? 0 : (lens[i] + kBlock - 1) / kBlock;
    my_U += u;
    my_A += u > 0;
  }
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) { my_U += __shfl_xor(my_U, o, 64); my_A += __shfl_xor(my_A, o, 64); }
  if (lane == 0) { wsum[wave] = my_U; wsum[kWaves + wave] = my_A; }
  __syncthreads();
  int U = 0, A = 0;
#pragma unroll
  for (int u2 = 0; u2 < kWaves; ++u2) { U += wsum[u2]; A += wsum[kWaves + u2]; }
  bool per_group = per_group_shares(A, P);
  __syncthreads();                                // wsum is reused by the scan
  // Pass 2: prefix sums of the workgroups per group (per-group shares) or of the blocks per group (contiguous).  Per-group
  // shares that would leave more than a quarter of the workgroups idle are dropped for contiguous ones: one more scan.
  int carry = 0;
  for (int attempt = 0; attempt < 2; ++attempt) {
    carry = 0;
    for (int base = 0; base < NG; base += kThreads) {
      const int i = base + tid;
      int v = 0;
      if (i < NG) {
        const int u = lens[i] > 0 ? (lens[i] + kBlock - 1) / kBlock : 0;
        v = per_group ? share_count(u, U, P, A) : u;
      }
      int x = v;                                   // inclusive scan inside the wavefront
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
      if (i < NG) start[i] = carry + woff + x - v;
      carry += tot;
      __syncthreads();
    }
    if (!per_group || per_group_fills(carry, P)) break;      // carry is the same in every thread
    per_group = false;
  }
  if (tid == 0) { start[NG] = carry; first_group = -1; }
  const int c = per_group ? 0 : (U + P - 1) / P;
  __syncthreads();
  if (p == 0) {
    if (tid == 0) { a.sched[0] = per_group ? 1 : 0; a.sched[1] = c; }
    for (int i = tid; i < NG; i += kThreads) {
      const int u = lens[i] > 0 ? (lens[i] + kBlock - 1) / kBlock : 0;
      a.sched[2 + 2 * i] = per_group ? u : start[i];
      a.sched[3 + 2 * i] = per_group ? start[i + 1] - start[i] : start[i + 1];
    }
  }
  SR_STAMP(a.timeline, kTimelinePartialStamps, 3);
  if (per_group) {
    for (int i = tid; i < NG; i += kThreads)
      if (start[i] <= p && p < start[i + 1]) first_group = i;        // at most one group
    __syncthreads();
    const int i = first_group;
    if (i < 0) return;                            // fewer shares than workgroups
    const int L = lens[i], ui = (L + kBlock - 1) / kBlock, j = p - start[i];
    const int cb = share_blocks(ui, start[i + 1] - start[i]);
    const int blk_lo = j * cb, blk_hi = min(blk_lo + cb, ui);
    if (blk_lo >= blk_hi) return;                 // more workgroups than the group has blocks
    const int b = i / a.Hkv, g = i - b * a.Hkv;
    attend_range<kPaged>(a, b, g, L, blk_lo * kBlock, min(blk_hi * kBlock, L), j);
    SR_STAMP(a.timeline, kTimelinePartialStamps, 7);
    return;
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
  SR_STAMP(a.timeline, kTimelinePartialStamps, 7);
}

}  // namespace

#endif
