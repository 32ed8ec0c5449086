// SinkRouter decode attention for MI355X: compile-time constants and the pure index arithmetic that host and
// device share (length clamp, page addressing, the routing rule's parameters).  Nothing here needs the HIP
// runtime, so the host side of the library (sr_host.h) and its CPU tests build with a plain C++ compiler.
#ifndef SR_CONFIG_H
#define SR_CONFIG_H

#include <stddef.h>
#include <stdint.h>

#if defined(__HIPCC__)
#define SR_HD __host__ __device__ __forceinline__
#else
#define SR_HD inline
#endif

#ifndef SR_WAVES
#define SR_WAVES 4
#endif
#ifndef SR_GRID
#define SR_GRID 256
#endif

// SR_TIMELINE=1 builds the measurement variant of the library: every workgroup of the balanced partial
// kernel and of the merge kernel leaves wall-clock stamps (100 MHz counter) behind the workspace, which
// grows by kTimelineBytes.  The product build (0) contains none of it.
#ifndef SR_TIMELINE
#define SR_TIMELINE 0
#endif

namespace {

constexpr int kD = 128;              // head dimension
constexpr int kBlock = 64;           // tokens per online-softmax block (B_K)
constexpr int kWaves = SR_WAVES;     // wavefronts per partial workgroup
constexpr int kThreads = 64 * kWaves;
constexpr int kMaxGroup = 16;        // query heads per KV group that fit the MFMA tile
constexpr int kChunkUnit = kBlock * kWaves;
// Merge workgroups come in two shapes (see combine_narrow).  Few records per head: 8 wavefronts on a head's whole
// row, 4 record rows in flight (64 records per sweep).  Many records per head: a head is split into 8 column parts,
// one workgroup of 4 wavefronts each, 4 rows in flight (256 records per sweep, all a head can have in the balanced
// schedule).  Measured on the 200K- and 512K-token workloads: 16 wavefronts x 4 parts x 2 rows +0.2 / +0.4 us per step,
// 8 x 4 x 4 and 8 x 8 x 2 within 0.1 us, 16 x 8 x 1 +0.3 / +1.2 us, 16 wavefronts on whole rows (8 rows in flight) +1.3 / +1.0 us.
constexpr int kCombineWavesWide = 4, kCombineWavesNarrow = 8;
constexpr int kCombinePartsWide = 8, kCombinePartsNarrow = 1;
constexpr int kCombineRowsWide = 4, kCombineRowsNarrow = 4;
constexpr int kBalancedGrid = SR_GRID;   // persistent workgroups of the balanced schedule: one per compute unit
constexpr int kMaxSchedGroups = 2048;  // (sequence, KV group) pairs the balanced schedule scans in LDS
// Query heads (all sequences) up to which the balanced kernel probes itself.  Every workgroup evaluates all heads, 128 per
// sweep, so the cost grows with the batch while a separate probe launch costs a fixed ~4.7 us.  Measured on an 8B-shaped
// layer (step with the fused / the separate probe): 160 heads 46.9 / 47.6 us, 192: 30.3 / 31.1, 256: 21.9 / 22.6,
// 320: 42.7 / 42.2, 384: 32.3 / 31.7, 512: 37.4 / 35.9, 640: 44.1 / 41.7, 1024: 69.1 / 64.2.
constexpr int kMaxFusedHeads = 256;
constexpr int kMaxGroupsTotal = 65535; // (sequence, KV group) pairs per call: the y extent of the fixed grid
constexpr int kMaxSeqLen = 1 << 24;    // 32-bit token arithmetic stays exact up to here
constexpr int64_t kMaxHeadsTotal = (int64_t)1 << 24;
// The allocation-free entry point keeps its partial records in a device array of this size.
constexpr size_t kStaticScratchBytes = (size_t)32 << 20;

// Timeline build: 8 stamps per partial workgroup, then 4 per merge workgroup (the first kTimelineMergeGroups).
constexpr int kTimelinePartialStamps = 8, kTimelineMergeStamps = 4, kTimelineMergeGroups = 1024;
constexpr size_t kTimelineBytes =
    SR_TIMELINE ? ((size_t)kBalancedGrid * kTimelinePartialStamps + (size_t)kTimelineMergeGroups * kTimelineMergeStamps) * 8 : 0;

// Division by a run-time constant as one multiply: magic = ceil(2^32 / d) made on the host, x / d == umulhi(x, magic)
// for every x with x * d < 2^32 (d == 1 is marked by magic 0).  The kernels use it where a workgroup's first loads wait
// for a quotient (head -> group, group -> sequence).
inline uint32_t div_magic(uint32_t d) { return d <= 1 ? 0u : (uint32_t)((((uint64_t)1) << 32) / d + 1); }
SR_HD uint32_t div_by(uint32_t x, uint32_t magic) {
#if defined(__HIP_DEVICE_COMPILE__)
  return magic ? __umulhi(x, magic) : x;
#else
  return magic ? (uint32_t)(((uint64_t)x * magic) >> 32) : x;
#endif
}

// Balanced schedule, "per-group shares" (used when at most half as many groups are active as there are workgroups):
// with U blocks in A Active Groups and P workgroups, group i with u_i blocks gets n_i = ceil(u_i (P - A) / U) >= 1
// workgroups (their sum is at most P), each taking ceil(u_i / n_i) consecutive blocks, so no workgroup works on two
// groups.  share_records is the number of workgroups of a group that get any block: its partial records.
SR_HD bool per_group_shares(int A, int P) { return A > 0 && 2 * A <= P; }
// ... and only if the shares then occupy at least three quarters of the workgroups.  share_count leaves up to A of
// them idle: 128 equally long Active Groups would get one workgroup each and half the chip would stand still, where
// contiguous shares give every group two.  (Up to 64 Active Groups always pass: their shares occupy P - A >= 192.)
SR_HD bool per_group_fills(int shares, int P) { return 4 * shares >= 3 * P; }
SR_HD int share_count(int u, int U, int P, int A) {        // u (P - A) < 2^18 * 2^8: 32-bit arithmetic is exact
  return u > 0 ? (int)(((uint32_t)u * (uint32_t)(P - A) + (uint32_t)U - 1u) / (uint32_t)U) : 0;
}
SR_HD int share_blocks(int u, int n) { return (u + n - 1) / n; }
SR_HD int share_records(int u, int n) { return u > 0 ? (u + share_blocks(u, n) - 1) / share_blocks(u, n) : 0; }

// seq_lens[b] as the kernels use it: values outside [0, L_max] are clamped.
SR_HD int clamp_len(int L, int Lmax) { return L < 0 ? 0 : (L > Lmax ? Lmax : L); }

// Paged KV cache: pages of 2^page_shift tokens laid out [n_pages, H_kv, page_tokens, D]; logical
// page j of sequence b is physical page table[b * pages_per_seq + j] (clamped to the pool, so a
// bad entry reads a wrong page but never leaves the allocation).  table == NULL: contiguous cache.
struct PageMap {
  const int32_t* table;
  int page_shift, pages_per_seq, n_pages;
};

SR_HD int page_of(const PageMap& pm, int b, int tok) {
  int pg = pm.table[(size_t)b * pm.pages_per_seq + (tok >> pm.page_shift)];
  pg = pg < 0 ? 0 : pg;
  return pg < pm.n_pages ? pg : pm.n_pages - 1;
}

// Offset (in 16-byte units) of token `tok` of group g in a page pool, given its physical page.
SR_HD size_t paged_offset(const PageMap& pm, int page, int Hkv, int g, int tok) {
  return ((((size_t)page * Hkv + g) << pm.page_shift) + (tok & ((1 << pm.page_shift) - 1))) * (kD / 8);
}

// Parameters of the routing rule (Section 4.2, Appendix A) as the kernels receive them.
struct RouteRule {
  float tau[4], len_norm;
  int routing;
};

}  // namespace

#endif
