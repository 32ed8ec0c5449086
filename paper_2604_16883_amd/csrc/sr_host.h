// SinkRouter decode attention for MI355X: the host side of the C ABI that needs no GPU - argument checks,
// launch plan and workspace layout.  Plain C++ (no HIP types), so a CPU build with sanitizers can sweep it.
#ifndef SR_HOST_H
#define SR_HOST_H

#include "sinkrouter.h"
#include "sr_config.h"

namespace {

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

inline bool misaligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) != 0; }

// Byte offsets of the pieces of the workspace, in this order: partial outputs [heads, slots, D] fp32,
// partial (m, l) [heads, slots, 2] fp32, group scores [NG] fp32, schedule table (mode, c, one pair per group) int32,
// shifted lengths [B] int32 (concentration statistics only), wall-clock stamps (timeline build only).  Every piece starts on a 256-byte boundary.
struct Layout {
  sr_plan plan;
  size_t off_o, off_ml, off_score, off_sched, off_lens, off_timeline;
};

// Shape checks, launch plan and workspace layout for params.  All size products are formed in 64 bits.
inline int make_layout(const sr_route_params* p, Layout* lay) {
  if (!p) return SR_ERR_NULL;
  if (p->struct_size != sizeof(sr_route_params)) return SR_ERR_UNSUPPORTED;
  if (p->batch < 1 || p->n_q_heads < 1 || p->n_kv_heads < 1 || p->max_seq_len < 1 || p->num_splits < 0)
    return SR_ERR_SHAPE;
  if (p->n_q_heads % p->n_kv_heads != 0) return SR_ERR_SHAPE;
  if ((int64_t)p->batch * p->n_kv_heads > kMaxGroupsTotal) return SR_ERR_SHAPE;
  if ((int64_t)p->batch * p->n_q_heads > kMaxHeadsTotal) return SR_ERR_SHAPE;
  if (p->max_seq_len > kMaxSeqLen) return SR_ERR_SHAPE;
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
      const int64_t per = ((int64_t)p->max_seq_len + p->num_splits - 1) / p->num_splits;   // <= max_seq_len
      chunk = (int)align_up((size_t)per, kChunkUnit);
    } else {
      // too many groups to schedule in LDS: plain chunks sized so that, with about 40% of the
      // groups active (the paper's retained budget, Section 5.1), some 2048 workgroups have work
      const double active_tokens = 0.4 * (double)NG * p->max_seq_len;
      int units = (int)(active_tokens / (2048.0 * kChunkUnit));
      units = units < 1 ? 1 : (units > 8 ? 8 : units);
      chunk = units * kChunkUnit;
    }
    const int splits = (p->max_seq_len + chunk - 1) / chunk;
    if ((int64_t)splits * NG > INT32_MAX) return SR_ERR_SHAPE;   // more workgroups than a launch can name
    pl.schedule = 0;
    pl.chunk_tokens = chunk;
    pl.num_splits = splits;
    pl.partial_grid = splits * NG;
    pl.slots_per_head = splits;
  }
  const size_t heads = (size_t)p->batch * p->n_q_heads;
  const size_t S = (size_t)pl.slots_per_head;
  lay->off_o = 0;
  lay->off_ml = align_up(heads * S * kD * sizeof(float), 256);
  lay->off_score = lay->off_ml + align_up(heads * S * 2 * sizeof(float), 256);
  lay->off_sched = lay->off_score + align_up((size_t)NG * sizeof(float), 256);
  lay->off_lens = lay->off_sched + align_up((size_t)(2 * NG + 2) * sizeof(int32_t), 256);
  lay->off_timeline = lay->off_lens + align_up((size_t)p->batch * sizeof(int32_t), 256);
  pl.workspace_bytes = lay->off_timeline + kTimelineBytes;      // no stamps in the product build
  return SR_OK;
}

inline RouteRule make_rule(const sr_route_params* p) {
  RouteRule r;
  for (int i = 0; i < 4; ++i) r.tau[i] = p->tau_coef[i];
  r.len_norm = p->len_norm;
  r.routing = p->routing_enabled != 0;
  return r;
}

// Softmax scale in the log2 domain, as the kernels use it.
inline float scale_log2_of(const sr_route_params* p) {
  const float scale = p->sm_scale > 0.f ? p->sm_scale : 0.08838834764831845f;   // 1/sqrt(128)
  return scale * 1.4426950408889634f;
}

// Optional per-head outputs of the diagnostic entry points; all may be NULL.
struct DecodeExtras {
  const float* lse_out;
  const float* alpha0_out;
  const float* max_rest_out;
  const float* mean_rest_out;
};

// Every check of a decode call that precedes the first HIP call: pointers, shape (make_layout),
// alignment, workspace.  with_workspace = false skips the workspace test (the allocation-free entry
// point brings its own).
inline int check_decode_args(const void* q, const void* k, const void* v, const int32_t* seq_lens,
                             const sr_route_params* p, const void* out, const uint8_t* mask,
                             const DecodeExtras& x, bool with_workspace, Layout* lay) {
  if (!q || !k || !v || !seq_lens || !p || !out || !mask) return SR_ERR_NULL;
  const int rc = make_layout(p, lay);
  if (rc != SR_OK) return rc;
  if (misaligned(q, 16) || misaligned(k, 16) || misaligned(v, 16) || misaligned(out, 16) || misaligned(seq_lens, 4) ||
      misaligned(p->k0, 16) || misaligned(p->k0_norm, 4) || misaligned(x.lse_out, 4) || misaligned(x.alpha0_out, 4) ||
      misaligned(x.max_rest_out, 4) || misaligned(x.mean_rest_out, 4))
    return SR_ERR_ALIGN;
  if (with_workspace &&
      (!p->workspace || misaligned(p->workspace, 256) || p->workspace_bytes < lay->plan.workspace_bytes))
    return SR_ERR_WORKSPACE;
  return SR_OK;
}

// Checks of the paged layout; fills *pm (table pointer included) when they pass.
inline int check_paged_args(const int32_t* block_table, const sr_paged_layout* layout, const sr_route_params* p,
                            PageMap* pm) {
  if (!block_table || !layout || !p) return SR_ERR_NULL;
  if (layout->struct_size != sizeof(sr_paged_layout)) return SR_ERR_UNSUPPORTED;
  const int pt = layout->page_tokens;
  if (pt < kBlock || (pt & (pt - 1)) != 0) return SR_ERR_UNSUPPORTED;       // power of two, >= one block
  if (layout->n_pages < 1 || layout->pages_per_seq < 1) return SR_ERR_SHAPE;
  if (p->max_seq_len < 1 || (int64_t)layout->pages_per_seq * pt < p->max_seq_len) return SR_ERR_SHAPE;
  if (misaligned(block_table, 4)) return SR_ERR_ALIGN;
  pm->table = block_table;
  pm->page_shift = __builtin_ctz((unsigned)pt);
  pm->pages_per_seq = layout->pages_per_seq;
  pm->n_pages = layout->n_pages;
  return SR_OK;
}

// Records a head has when every group is active: shares / groups + 1 in the balanced schedule, else the chunks.
inline int expected_records(const Layout& lay, int NG) {
  return lay.plan.schedule == 1 ? kBalancedGrid / NG + 1 : lay.plan.num_splits;
}

// Shape of the merge workgroups.  Narrow (8 wavefronts on a head's whole row) where heads are expected to have at
// most 16 records (more than 16 groups share the 256 workgroups); else a head is split into column parts of 4
// wavefronts each: with few Active Groups a head has hundreds of records and only a few heads have any, and one
// compute unit per head takes longer to pull a head's 130 KB of records than a memory round trip (200K-token
// workload: 8 busy heads, -1.1 us per step with the split).  The narrow shape on the 128K-token batch: 4 wavefronts
// x 2 or 4 parts +0.1-0.2 us, 2 wavefronts x 4 or 8 parts +0.3-0.4 us.
inline bool combine_narrow(const Layout& lay, int NG) { return expected_records(lay, NG) <= 16; }
inline int combine_waves(const Layout& lay, int NG) { return combine_narrow(lay, NG) ? kCombineWavesNarrow : kCombineWavesWide; }

// Column parts a head's merge is split into (workgroups per head): 1 for the narrow shape, kCombinePartsWide else.
inline int combine_parts(const Layout& lay, int NG) {
  return combine_narrow(lay, NG) ? kCombinePartsNarrow : kCombinePartsWide;
}

// Records of a head the merge kernel requests before it knows how many the head has: enough for a head when every
// group is active (narrow shape: rounded up to what one load instruction of the workgroup covers), at most one
// sweep and never more than the slots a head has.  Every head requests them, Sink Groups' heads included; what is
// not a record is dropped.  Four times as many (a head covered down to a quarter of the groups being active) measured
// the same on the 200K- and 512K-token workloads: the second request follows the first by much less than a cold
// round trip.
inline int combine_spec_records(const Layout& lay, int NG) {
  const int e = expected_records(lay, NG);
  int spec;
  if (combine_narrow(lay, NG)) {
    const int per_row = 2 * kCombinePartsNarrow * kCombineWavesNarrow;
    spec = (e + per_row - 1) / per_row * per_row;
    if (spec > per_row * kCombineRowsNarrow) spec = per_row * kCombineRowsNarrow;
  } else {
    const int sweep = kCombineWavesWide * 2 * kCombinePartsWide * kCombineRowsWide;   // 64 / (32 / parts) records per load
    spec = e > sweep ? sweep : e;
  }
  if (spec > lay.plan.slots_per_head) spec = lay.plan.slots_per_head;
  return spec < 1 ? 1 : spec;
}

}  // namespace

#endif
