// SinkRouter decode attention for MI355X (gfx950, CDNA4): the C ABI over the kernels in this directory.
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
//                  the 64-token blocks of the Active Groups only are dealt out: workgroups per
//                  group in proportion to its blocks, one group per workgroup (or equal runs of
//                  the blocks laid end to end when more than half as many groups are active as
//                  there are workgroups, or when shares per group would leave a quarter of the
//                  workgroups idle).  Sink Groups cost nothing and the chip stays full
//                  whatever the skip pattern is.
//        fixed     the paper's literal Split-K: [0, L) cut into num_splits chunks, one
//                  workgroup per (chunk, sequence, KV group); workgroups of Sink Groups
//                  leave at once.
//   sr_combine_kernel  log-sum-exp merge of the partials, bf16 output; zeros for Sink Groups
//                      (Eq. 14).
//
// sr_common.h, sr_route.h, sr_partial.h, sr_combine.h and sr_measure.h hold the kernels, sr_config.h the
// constants and index arithmetic host and device share, sr_host.h the argument checks, launch plan and
// workspace layout (plain C++, no GPU needed); this file launches.
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>

#include <mutex>

#include "sinkrouter.h"

#include "sr_host.h"
#include "sr_common.h"
#include "sr_route.h"
#include "sr_partial.h"
#include "sr_combine.h"
#include "sr_measure.h"

static_assert(kStaticScratchBytes == SINKROUTER_STATIC_SCRATCH_BYTES, "header and kernels disagree on the static scratch size");

// Scratch of the allocation-free entry point (sinkrouter_decode_static): the workspace of one decode call,
// held by every GPU the library runs on until the process ends.  In host code this name is only a handle
// for hipGetSymbolAddress; kernels receive the device address looked up once per device.
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {

// ------------------------------------------------------------------------------------------
// Host side: launches.  Argument checks, plan and workspace layout are in sr_host.h.
// ------------------------------------------------------------------------------------------
// Plain launch, or (benchmarks) a launch whose own begin and end times are left in two events.
template <typename Kernel, typename Args>
bool launch(Kernel kernel, dim3 grid, dim3 block, hipStream_t st, const Args& args, hipEvent_t begin, hipEvent_t end) {
  if (begin) hipExtLaunchKernelGGL(kernel, grid, block, 0, st, begin, end, 0, args);
  else hipLaunchKernelGGL(kernel, grid, block, 0, st, args);
  return hipGetLastError() == hipSuccess;
}

int launch_probe(const void* q, const void* k, const int32_t* seq_lens, const sr_route_params* p,
                 const Layout& lay, float* score, uint8_t* mask, hipStream_t st, const PageMap& pm,
                 hipEvent_t begin = nullptr, hipEvent_t end = nullptr) {
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
  return launch(sr_probe_kernel, dim3(p->batch * p->n_kv_heads), dim3(64), st, a, begin, end) ? SR_OK : SR_ERR_HIP;
}

// Device address of `scratch` on the current device, looked up on the first call per device (each GPU
// holds its own copy of the array at its own address).  No allocation: the array is part of the
// library's code object.
bool static_scratch(void** ptr) {
  constexpr int kMaxDevices = 64;
  static void* addr[kMaxDevices] = {};
  static std::mutex guard;
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return false;
  std::lock_guard<std::mutex> lock(guard);
  if (!addr[dev]) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return false;
    addr[dev] = p;
  }
  *ptr = addr[dev];
  return true;
}

// Outputs of the concentration statistics; decode_impl then attends over tokens 1..L-1 only.
struct RestStats {
  float* max_rest;
  float* mean_rest;
};

int decode_impl(const void* q, const void* k, const void* v, const int32_t* seq_lens,
                const sr_route_params* p, void* out, uint8_t* mask, float* stage_us,
                float* lse_out = nullptr, float* alpha0_out = nullptr, const PageMap* pages = nullptr,
                const RestStats* rest = nullptr, void* own_workspace = nullptr) {
  Layout lay;
  const DecodeExtras extras = {lse_out, alpha0_out, rest ? rest->max_rest : nullptr, rest ? rest->mean_rest : nullptr};
  const int rc = check_decode_args(q, k, v, seq_lens, p, out, mask, extras, own_workspace == nullptr, &lay);
  if (rc != SR_OK) return rc;
  hipStream_t st = static_cast<hipStream_t>(p->stream);
  char* ws = static_cast<char*>(own_workspace ? own_workspace : p->workspace);
  float* part_o = reinterpret_cast<float*>(ws + lay.off_o);
  float* part_ml = reinterpret_cast<float*>(ws + lay.off_ml);
  float* score = reinterpret_cast<float*>(ws + lay.off_score);
  int32_t* sched = reinterpret_cast<int32_t*>(ws + lay.off_sched);
  const bool balanced = lay.plan.schedule == 1;
  PageMap pm = {nullptr, 0, 0, 0};
  if (pages) pm = *pages;
  const bool paged = pm.table != nullptr;
  // the balanced kernel evaluates the routing rule itself for batches of up to kMaxFusedHeads query heads; with routing off
  // there is nothing to evaluate (it writes a mask of zeros), so no probe launch precedes it either
  const bool fused = balanced && ((int64_t)p->batch * p->n_q_heads <= kMaxFusedHeads || !p->routing_enabled);
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

  // timing: ev[0] / ev[7] are recorded on the stream around the whole call; ev[1..2], ev[3..4], ev[5..6]
  // receive the begin and end times of the probe, partial and merge kernels themselves
  constexpr int kEvents = 8;
  hipEvent_t ev[kEvents] = {nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr};
  if (stage_us) {
    for (int i = 0; i < kEvents; ++i)
      if (hipEventCreate(&ev[i]) != hipSuccess) {
        for (int j = 0; j < i; ++j) (void)hipEventDestroy(ev[j]);
        return SR_ERR_HIP;
      }
  }
  bool ok = !stage_us || hipEventRecord(ev[0], st) == hipSuccess;
  if (ok && !fused) ok = launch_probe(q, k_anchor, seq_lens, p, lay, score, mask, st, pm, ev[1], ev[2]) == SR_OK;
  if (ok) {
    PartialArgs a;
    a.q = static_cast<const uint16_t*>(q);
    a.k = static_cast<const uint16_t*>(k);
    a.v = static_cast<const uint16_t*>(v);
    a.seq_lens = seq_lens; a.mask = mask; a.part_o = part_o; a.part_ml = part_ml; a.sched = sched;
    a.k0 = p->k0; a.k0_norm = p->k0_norm; a.group_score = score; a.rule = make_rule(p);
    a.Hq = p->n_q_heads; a.Hkv = p->n_kv_heads; a.G = lay.plan.group_size; a.Lmax = p->max_seq_len;
    a.NG = p->batch * p->n_kv_heads;
    a.g_magic = div_magic((uint32_t)a.G); a.hkv_magic = div_magic((uint32_t)a.Hkv);
    a.chunk = lay.plan.chunk_tokens; a.slots = lay.plan.slots_per_head;
    a.scale_log2 = scale_log2_of(p);
    a.pm = pm;
    a.timeline = (SR_TIMELINE && balanced) ? reinterpret_cast<long long*>(ws + lay.off_timeline) : nullptr;
    const dim3 blk(kThreads), fixed_grid(lay.plan.num_splits, a.NG);
    const dim3 grid = balanced ? dim3(kBalancedGrid) : fixed_grid;
    if (fused && paged)       ok = launch(sr_partial_balanced_kernel<true, true>, grid, blk, st, a, ev[3], ev[4]);
    else if (fused)           ok = launch(sr_partial_balanced_kernel<true, false>, grid, blk, st, a, ev[3], ev[4]);
    else if (balanced && paged) ok = launch(sr_partial_balanced_kernel<false, true>, grid, blk, st, a, ev[3], ev[4]);
    else if (balanced)        ok = launch(sr_partial_balanced_kernel<false, false>, grid, blk, st, a, ev[3], ev[4]);
    else if (paged)           ok = launch(sr_partial_fixed_kernel<true>, grid, blk, st, a, ev[3], ev[4]);
    else                      ok = launch(sr_partial_fixed_kernel<false>, grid, blk, st, a, ev[3], ev[4]);
  }
  if (ok) {
    CombineArgs c;
    c.q = static_cast<const uint32_t*>(q); c.k = k_anchor;
    c.lse_out = lse_out; c.alpha0_out = alpha0_out; c.scale_log2 = scale_log2_of(p);
    c.lens_full = lens_full;
    c.max_rest_out = rest ? rest->max_rest : nullptr;
    c.mean_rest_out = rest ? rest->mean_rest : nullptr;
    c.part_o = part_o; c.part_ml = part_ml; c.seq_lens = seq_lens; c.mask = mask;
    c.sched = balanced ? sched : nullptr;
    c.out = static_cast<uint32_t*>(out);
    c.Hq = p->n_q_heads; c.Hkv = p->n_kv_heads; c.G = lay.plan.group_size; c.Lmax = p->max_seq_len;
    c.chunk = lay.plan.chunk_tokens; c.slots = lay.plan.slots_per_head;
    c.timeline = SR_TIMELINE ? reinterpret_cast<long long*>(ws + lay.off_timeline) + (size_t)kBalancedGrid * kTimelinePartialStamps : nullptr;
    const int NG = p->batch * p->n_kv_heads;
    c.spec = combine_spec_records(lay, NG);
    const dim3 groups((unsigned)(p->batch * p->n_q_heads * combine_parts(lay, NG)));
    if (combine_narrow(lay, NG))
      ok = launch(sr_combine_kernel<kCombineWavesNarrow, kCombinePartsNarrow, kCombineRowsNarrow>, groups, dim3(64 * kCombineWavesNarrow), st, c, ev[5], ev[6]);
    else
      ok = launch(sr_combine_kernel<kCombineWavesWide, kCombinePartsWide, kCombineRowsWide>, groups, dim3(64 * kCombineWavesWide), st, c, ev[5], ev[6]);
  }
  if (stage_us) {
    if (ok) ok = hipEventRecord(ev[7], st) == hipSuccess;
    if (ok) ok = hipEventSynchronize(ev[7]) == hipSuccess;
    auto span_us = [&](int i, int j, float* us) {
      float ms = 0.f;
      if (hipEventElapsedTime(&ms, ev[i], ev[j]) != hipSuccess) return false;
      *us = ms * 1000.f;
      return true;
    };
    stage_us[0] = 0.f;
    if (ok && !fused) ok = span_us(1, 2, &stage_us[0]);
    if (ok) ok = span_us(3, 4, &stage_us[1]);
    if (ok) ok = span_us(5, 6, &stage_us[2]);
    if (ok) ok = span_us(0, 7, &stage_us[3]);
    for (int i = 0; i < kEvents; ++i) (void)hipEventDestroy(ev[i]);
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
  PageMap pm;
  const int rc = check_paged_args(block_table, layout, params, &pm);
  if (rc != SR_OK) return rc;
  return decode_impl(q, k_pages, v_pages, seq_lens, params, out, skip_mask_out, nullptr, nullptr, nullptr, &pm);
}

int sinkrouter_decode_static(const void* q, const void* k_cache, const void* v_cache, const int32_t* seq_lens,
                             const sr_route_params* params, void* out, uint8_t* skip_mask_out) {
  // every host-side check first, the size limit included, so that error paths touch no GPU
  Layout lay;
  const DecodeExtras none = {nullptr, nullptr, nullptr, nullptr};
  const int rc = check_decode_args(q, k_cache, v_cache, seq_lens, params, out, skip_mask_out, none, false, &lay);
  if (rc != SR_OK) return rc;
  if (lay.plan.workspace_bytes > kStaticScratchBytes) return SR_ERR_STATIC_LIMIT;
  void* ws = nullptr;
  if (!static_scratch(&ws)) return SR_ERR_HIP;
  return decode_impl(q, k_cache, v_cache, seq_lens, params, out, skip_mask_out, nullptr, nullptr, nullptr, nullptr,
                     nullptr, ws);
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
    case SR_ERR_STATIC_LIMIT: return "shape needs more workspace than the library's static scratch holds (SINKROUTER_STATIC_SCRATCH_BYTES): use sinkrouter_decode with a caller workspace";
    default: return "unknown status";
  }
}

int sinkrouter_abi_version(void) { return SINKROUTER_ABI_VERSION; }

// Timeline (measurement) build only: bytes of wall-clock stamps at the end of the workspace, 0 in the product build.
size_t sinkrouter_timeline_bytes(void) { return kTimelineBytes; }

}  // extern "C"