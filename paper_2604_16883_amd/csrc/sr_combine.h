// SinkRouter decode attention for MI355X: log-sum-exp merge of the partials, diagnostics, zero surrogate.
#ifndef SR_COMBINE_H
#define SR_COMBINE_H

#include "sr_common.h"

namespace {

// ------------------------------------------------------------------------------------------
// Merge of the partials.  grid = B*H_q*CP, block = NW wavefronts (8 on whole rows where heads have few records, 4 on
// an eighth of a head's columns where they have many: the launch of a workgroup's wavefronts is part of the step's
// latency, and so is the time one compute unit takes to pull a head's records).
// ------------------------------------------------------------------------------------------
struct CombineArgs {
  const float* part_o;
  const float* part_ml;
  const int32_t* seq_lens;
  const uint8_t* mask;
  const int32_t* sched;   // balanced schedule (mode, c, one pair per group), else NULL
  uint32_t* out;          // bf16 pairs
  int Hq, Hkv, G, Lmax, chunk, slots;
  int spec;               // records of a head requested before their number is known (1..slots)
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
  long long* timeline;    // timeline build: [heads, 4] stamps (entry, records loaded, merged, exit); NULL otherwise
};

// One pass: every wavefront keeps a running (max, sum, weighted rows) over the records it owns and the NW
// wavefronts are merged through LDS.  A workgroup merges one head's columns [cp 128/CP, (cp+1) 128/CP): CP = 1
// where heads have few records, CP = 8 where a few Active Groups hold all 256 shares (hundreds of records per
// head, and as few as 8 busy heads: one compute unit per head then takes longer to pull a head's 130 KB of
// records than the memory round trip itself).  A record's slice is read by LPR = 32/CP lanes x 16 bytes, so one
// load instruction of a wavefront covers RPL = 64/LPR records: record s belongs to wavefront s % NW, lane group
// (s / NW) % RPL, row s / (NW RPL); UN rows are in flight, one sweep takes NW RPL UN records (64 / 256 for
// the two instantiations: the balanced schedule never makes more than 256 records per head).
// The first `spec` records are requested at kernel entry, before the number of records is known (it takes a load
// of the mask and of the schedule to know it); when spec covers the head's records the merge costs one memory
// round trip.  What was fetched beyond the last record is discarded.  The host sets spec (combine_spec_records).
template <int NW, int CP, int UN>
__global__ __launch_bounds__(NW * 64) void sr_combine_kernel(CombineArgs a) {
  constexpr int LPR = 32 / CP, RPL = 64 / LPR;
  const int bh = blockIdx.x / CP, cp = blockIdx.x % CP;
#if SR_TIMELINE
  long long* tl = (a.timeline && blockIdx.x < kTimelineMergeGroups) ? a.timeline : nullptr;
#endif
  SR_STAMP(tl, kTimelineMergeStamps, 0);
  const int b = bh / a.Hq, h = bh - b * a.Hq, g = h / a.G;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const float2* ml = reinterpret_cast<const float2*>(a.part_ml) + (size_t)bh * a.slots;
  const int sub = lane / LPR, ll = lane % LPR;
  const float4* po = reinterpret_cast<const float4*>(a.part_o) + (size_t)bh * a.slots * (kD / 4) + cp * LPR + ll;
  float2 st[UN];
  float4 o[UN];
#pragma unroll
  for (int u = 0; u < UN; ++u) {
    const int s = wave + NW * (RPL * u + sub);
    if (s < a.spec) {                            // spec <= slots
      st[u] = ml[s];
      o[u] = po[(size_t)s * (kD / 4)];
    }
  }
  // Everything the head's record count depends on is requested here, unconditionally and together with the
  // speculative rows, as vector loads: the sequence length and the four schedule entries by lanes 0..4 of
  // one load instruction (broadcast afterwards), the mask byte by another.  One memory round trip covers
  // them all; a mask test in front of the schedule loads, or scalar loads (which have to be waited for
  // one batch at a time), made it three dependent ones.
  const int bg = b * a.Hkv + g;
  const int32_t* src = a.seq_lens + b;                                       // lane 0 (and the idle lanes)
  if (a.sched && lane >= 1 && lane <= 4) src = a.sched + (lane <= 2 ? lane - 1 : 2 * bg + lane - 1);   // mode, c, the group's pair
  const int word = *src;
  const int sink = a.mask[bg];
  const int len_raw = __builtin_amdgcn_readlane(word, 0);
  const int mode = __builtin_amdgcn_readlane(word, 1), c = __builtin_amdgcn_readlane(word, 2);
  const int e0 = __builtin_amdgcn_readlane(word, 3), e1 = __builtin_amdgcn_readlane(word, 4);
  const int L = clamp_len(len_raw, a.Lmax);
  uint32_t* orow = a.out + (size_t)bh * (kD / 2) + cp * (64 / CP);
  int n = 0;                                     // partial records of this head
  if (!sink && L > 0) {
    if (!a.sched) n = (L + a.chunk - 1) / a.chunk;                          // fixed chunks
    else if (mode) n = share_records(e0, e1);                               // per-group shares: (blocks, workgroups)
    else if (e1 > e0) n = (e1 - 1) / c - e0 / c + 1;                        // contiguous shares: units [e0, e1)
  }
  if (n == 0) {                                  // zero surrogate (Eq. 14) / empty sequence
    if (wave == 0 && lane < 64 / CP) orow[lane] = 0u;
    if (threadIdx.x == 0 && cp == 0) {           // not computed for Sink Groups; an empty row has lse = -inf
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
    SR_STAMP(tl, kTimelineMergeStamps, 3);
    return;
  }
  __shared__ float red_m[NW];
  __shared__ float red_l[NW];
  __shared__ float4 red_o[NW][LPR];
  float m_run = -INFINITY, lsum = 0.f;
  float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
  for (int s0 = wave; s0 < n; s0 += NW * RPL * UN) {   // UN rows in flight per lane group
    const int have = s0 == wave ? a.spec : 0;    // records of this sweep that are already here
#pragma unroll
    for (int u = 0; u < UN; ++u) {
      const int s = s0 + NW * (RPL * u + sub);
      if (s >= have && s < n) {
        st[u] = ml[s];
        o[u] = po[(size_t)s * (kD / 4)];
      }
    }
    float bm = m_run;
#pragma unroll
    for (int u = 0; u < UN; ++u) {
      if (s0 + NW * (RPL * u + sub) >= n) st[u] = make_float2(-INFINITY, 0.f);
      bm = fmaxf(bm, st[u].x);
    }
    // a lane group may own no record at all: everything of it is then weighted 0
    const float keep = m_run > -INFINITY ? __builtin_amdgcn_exp2f(m_run - bm) : 0.f;
    acc.x *= keep; acc.y *= keep; acc.z *= keep; acc.w *= keep; lsum *= keep;
#pragma unroll
    for (int u = 0; u < UN; ++u) {
      const bool ok = s0 + NW * (RPL * u + sub) < n;
      const float wt = ok ? __builtin_amdgcn_exp2f(st[u].x - bm) : 0.f;
      acc.x += ok ? wt * o[u].x : 0.f;
      acc.y += ok ? wt * o[u].y : 0.f;
      acc.z += ok ? wt * o[u].z : 0.f;
      acc.w += ok ? wt * o[u].w : 0.f;
      lsum += ok ? wt * st[u].y : 0.f;
    }
    m_run = bm;
  }
  // fold the lane groups into the first one (lanes ll, ll + LPR, ... hold the same 4 columns)
#pragma unroll
  for (int off = LPR; off < 64; off <<= 1) {
    const float m_o = __shfl_xor(m_run, off, 64), l_o = __shfl_xor(lsum, off, 64);
    const float ax = __shfl_xor(acc.x, off, 64), ay = __shfl_xor(acc.y, off, 64), az = __shfl_xor(acc.z, off, 64), aw = __shfl_xor(acc.w, off, 64);
    const float mm = fmaxf(m_run, m_o);
    const float w_s = m_run > -INFINITY ? __builtin_amdgcn_exp2f(m_run - mm) : 0.f;
    const float w_o = m_o > -INFINITY ? __builtin_amdgcn_exp2f(m_o - mm) : 0.f;
    acc.x = w_s * acc.x + w_o * ax; acc.y = w_s * acc.y + w_o * ay; acc.z = w_s * acc.z + w_o * az; acc.w = w_s * acc.w + w_o * aw;
    lsum = w_s * lsum + w_o * l_o;
    m_run = mm;
  }
  SR_STAMP(tl, kTimelineMergeStamps, 1);
  if (sub == 0) red_o[wave][ll] = acc;           // columns 4 ll .. 4 ll + 3 of the slice
  if (lane == 0) { red_m[wave] = m_run; red_l[wave] = lsum; }
  __syncthreads();
  SR_STAMP(tl, kTimelineMergeStamps, 2);
  float M = red_m[0];                            // wavefront 0 owns record 0, so M is finite
#pragma unroll
  for (int u = 1; u < NW; ++u) M = fmaxf(M, red_m[u]);
  if (wave == 0) {
    float2 t = make_float2(0.f, 0.f);
    float l = 0.f;
    const int pair = lane < 64 / CP ? lane : 0;  // lane -> columns 2 lane, 2 lane + 1 of the slice
#pragma unroll
    for (int u = 0; u < NW; ++u) {
      const float wt = __builtin_amdgcn_exp2f(red_m[u] - M);   // 0 for a wavefront without records
      const float2 r = reinterpret_cast<const float2*>(red_o[u])[pair];
      t.x += wt * r.x; t.y += wt * r.y; l += wt * red_l[u];
    }
    const float inv = 1.0f / l;
    if (lane < 64 / CP) orow[lane] = f32_to_bf16_rne(t.x * inv) | (f32_to_bf16_rne(t.y * inv) << 16);
    if (cp == 0 && (a.lse_out || a.alpha0_out)) {
      const float lse2 = M + __builtin_amdgcn_logf(l);                  // log2 domain (v_log_f32 is log2)
      if (a.alpha0_out) {                                               // alpha_0 = exp(z_0 - lse), Section 4.2
        const uint32_t qw = a.q[(size_t)bh * (kD / 2) + lane];
        const uint32_t kw = reinterpret_cast<const uint32_t*>(a.k)[(size_t)bg * a.Lmax * (kD / 2) + lane];   // token 0 of the cache itself
        float d = bf16_lo(qw) * bf16_lo(kw) + bf16_hi(qw) * bf16_hi(kw);
#pragma unroll
        for (int o2 = 32; o2 >= 1; o2 >>= 1) d += __shfl_xor(d, o2, 64);
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
  SR_STAMP(tl, kTimelineMergeStamps, 3);
}

// Lengths of the caches with token 0 taken off, for the concentration statistics.
__global__ __launch_bounds__(256) void sr_rest_lens_kernel(const int32_t* seq_lens, int32_t* rest, int B, int Lmax) {
  const int b = blockIdx.x * 256 + threadIdx.x;
  if (b < B) rest[b] = max(clamp_len(seq_lens[b], Lmax) - 1, 0);
}

}  // namespace

#endif
