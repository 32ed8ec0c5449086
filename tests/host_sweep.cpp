// CPU sweep of the library's host-side arithmetic (argument checks, launch plan, workspace layout) and of
// the index arithmetic host and device share (length clamp, page addressing), meant to be built with
// -fsanitize=address,undefined: any signed overflow, bad shift or out-of-bounds access aborts the run.
// Prints "ok <n>" with the number of shapes checked; exits non-zero on the first violated invariant.
#include <limits.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <vector>

#include "sr_host.h"

#define CHECK(cond)                                                                                 \
  do {                                                                                              \
    if (!(cond)) {                                                                                  \
      fprintf(stderr, "%s:%d: check failed: %s  (B %d Hq %d Hkv %d L %d splits %d)\n", __FILE__, __LINE__, #cond, cur.batch, \
              cur.n_q_heads, cur.n_kv_heads, cur.max_seq_len, cur.num_splits);                       \
      exit(1);                                                                                      \
    }                                                                                               \
  } while (0)

static sr_route_params cur;

static sr_route_params shape(int B, int Hq, int Hkv, int L, int splits) {
  sr_route_params p;
  memset(&p, 0, sizeof p);
  p.struct_size = sizeof p;
  p.batch = B; p.n_q_heads = Hq; p.n_kv_heads = Hkv; p.head_dim = 128; p.max_seq_len = L; p.kv_block = 64;
  p.num_splits = splits; p.routing_enabled = 1;
  p.tau_coef[3] = 0.55f;
  return p;
}

typedef unsigned __int128 u128;
static u128 up256(u128 x) { return (x + 255) / 256 * 256; }

// One valid shape: the plan and the layout against an independent 128-bit evaluation.
static void check_valid(const sr_route_params& p) {
  cur = p;
  Layout lay;
  CHECK(make_layout(&p, &lay) == SR_OK);
  const sr_plan& pl = lay.plan;
  const long long NG = (long long)p.batch * p.n_kv_heads, heads = (long long)p.batch * p.n_q_heads;
  const long long blocks = ((long long)p.max_seq_len + 63) / 64;
  CHECK(pl.group_size == p.n_q_heads / p.n_kv_heads);
  if (pl.schedule == 1) {
    CHECK(p.num_splits == 0 && NG <= 2048 && NG * blocks < (1LL << 30));
    CHECK(pl.partial_grid == 256 && pl.num_splits == 0 && pl.chunk_tokens == 0);
    CHECK(pl.slots_per_head == (blocks < 257 ? blocks : 257));
  } else {
    CHECK(pl.schedule == 0 && pl.chunk_tokens > 0 && pl.chunk_tokens % 256 == 0);
    CHECK((long long)pl.num_splits * pl.chunk_tokens >= p.max_seq_len);
    CHECK((long long)(pl.num_splits - 1) * pl.chunk_tokens < p.max_seq_len);
    CHECK((long long)pl.partial_grid == (long long)pl.num_splits * NG);
    CHECK(pl.slots_per_head == pl.num_splits);
    if (p.num_splits > 0) CHECK(pl.num_splits <= p.num_splits);
  }
  CHECK(pl.slots_per_head >= 1 && pl.partial_grid >= 1);
  const u128 S = (u128)pl.slots_per_head;
  const u128 off_ml = up256((u128)heads * S * 128 * 4);
  const u128 off_score = off_ml + up256((u128)heads * S * 2 * 4);
  const u128 off_sched = off_score + up256((u128)NG * 4);
  const u128 off_lens = off_sched + up256((u128)(2 * NG + 2) * 4);
  const u128 total = off_lens + up256((u128)p.batch * 4);
  CHECK(total <= (u128)SIZE_MAX);
  CHECK(lay.off_o == 0 && (u128)lay.off_ml == off_ml && (u128)lay.off_score == off_score);
  CHECK((u128)lay.off_sched == off_sched && (u128)lay.off_lens == off_lens && (u128)pl.workspace_bytes == total);
  CHECK(lay.off_o < lay.off_ml && lay.off_ml < lay.off_score && lay.off_score < lay.off_sched);
  CHECK(lay.off_sched < lay.off_lens && lay.off_lens < pl.workspace_bytes);
  CHECK(lay.off_ml % 256 == 0 && lay.off_score % 256 == 0 && lay.off_sched % 256 == 0 && lay.off_lens % 256 == 0);
  const int spec = combine_spec_records(lay, (int)NG), cw = combine_waves(lay, (int)NG), parts = combine_parts(lay, (int)NG);
  CHECK(spec >= 1 && spec <= pl.slots_per_head && (cw == kCombineWavesNarrow || cw == kCombineWavesWide) &&
        parts == (combine_narrow(lay, (int)NG) ? kCombinePartsNarrow : kCombinePartsWide));
  CHECK(spec <= 2 * cw * parts * (combine_narrow(lay, (int)NG) ? kCombineRowsNarrow : kCombineRowsWide));   // one sweep at most
  CHECK((int64_t)p.batch * p.n_q_heads * parts <= INT32_MAX);                                       // the merge grid
  CHECK(!combine_narrow(lay, (int)NG) || expected_records(lay, (int)NG) <= 16);
  // the whole argument check on fake, suitably aligned addresses
  sr_route_params q = p;
  q.workspace = (void*)0x7000000;
  q.workspace_bytes = pl.workspace_bytes;
  const DecodeExtras none = {nullptr, nullptr, nullptr, nullptr};
  Layout l2;
  CHECK(check_decode_args((void*)0x10000, (void*)0x20000, (void*)0x30000, (const int32_t*)0x40000, &q, (void*)0x50000,
                          (const uint8_t*)0x60000, none, true, &l2) == SR_OK);
  q.workspace_bytes -= 1;
  CHECK(check_decode_args((void*)0x10000, (void*)0x20000, (void*)0x30000, (const int32_t*)0x40000, &q, (void*)0x50000,
                          (const uint8_t*)0x60000, none, true, &l2) == SR_ERR_WORKSPACE);
  CHECK(check_decode_args((void*)0x10000, (void*)0x20000, (void*)0x30000, (const int32_t*)0x40000, &q, (void*)0x50000,
                          (const uint8_t*)0x60000, none, false, &l2) == SR_OK);
}

static void check_rejected(const sr_route_params& p, int want) {
  cur = p;
  Layout lay;
  CHECK(make_layout(&p, &lay) == want);
}

// Page addressing on a host-side pool: every table entry, good or bad, lands inside the pool.
static void check_pages() {
  cur = shape(0, 0, 0, 0, 0);
  const int bad[] = {-1, INT_MIN, INT_MAX, 0, 1};
  for (int shift = 6; shift <= 12; shift += 3) {
    for (int n_pages : {1, 2, 7}) {
      const int B = 3, Hkv = 5, pps = 9, pt = 1 << shift;
      std::vector<int32_t> table((size_t)B * pps);
      for (size_t i = 0; i < table.size(); ++i) table[i] = (i % 4 == 3) ? bad[(i / 4) % 5] : (int32_t)(i % n_pages);
      table[0] = n_pages;          // one past the pool
      const PageMap pm = {table.data(), shift, pps, n_pages};
      const size_t pool16 = (size_t)n_pages * Hkv * pt * (kD / 8);      // pool size in 16-byte units
      for (int b = 0; b < B; ++b)
        for (int tok = 0; tok < pps * pt; tok += (tok % 64 == 63 ? 1 : 21)) {
          const int pg = page_of(pm, b, tok);
          CHECK(pg >= 0 && pg < n_pages);
          const int32_t raw = table[(size_t)b * pps + tok / pt];
          if (raw >= 0 && raw < n_pages) CHECK(pg == raw);
          for (int g = 0; g < Hkv; ++g) {
            const size_t off = paged_offset(pm, pg, Hkv, g, tok);
            CHECK(off + kD / 8 <= pool16);
            CHECK(off == (((size_t)pg * Hkv + g) * pt + (size_t)(tok % pt)) * (kD / 8));
          }
        }
    }
  }
  // the largest pool the interface can name: offsets are formed in 64 bits
  const int32_t one = INT_MAX;
  const PageMap pm = {&one, 12, 1, INT_MAX};
  CHECK(page_of(pm, 0, 4095) == INT_MAX - 1);
  CHECK(paged_offset(pm, INT_MAX - 1, 65535, 65534, 4095) ==
        ((((size_t)(INT_MAX - 1) * 65535 + 65534) << 12) + 4095) * 16);
  CHECK(clamp_len(INT_MIN, 5) == 0 && clamp_len(-1, 5) == 0 && clamp_len(0, 5) == 0 && clamp_len(5, 5) == 5);
  CHECK(clamp_len(6, 5) == 5 && clamp_len(INT_MAX, 1 << 24) == (1 << 24));
  // division by multiplication, on the domains the kernels use (x * d < 2^32)
  for (uint32_t d : {1u, 2u, 3u, 4u, 5u, 7u, 8u, 12u, 16u, 40u, 255u, 256u, 257u, 2047u, 2048u, 40000u, 65535u}) {
    const uint32_t m = div_magic(d);
    const uint32_t top = (uint32_t)(((uint64_t)1 << 32) / d);
    for (uint32_t x = 0; x < 70000u && x < top; ++x) CHECK(div_by(x, m) == x / d);
    for (uint32_t x = top > 5000u ? top - 5000u : 0u; x < top; ++x) CHECK(div_by(x, m) == x / d);
  }
  // per-group shares: every group gets at least one workgroup, the workgroups suffice, the shares cover the blocks
  {
    const int P = kBalancedGrid;
    unsigned seed = 12345;
    for (int round = 0; round < 4000; ++round) {
      seed = seed * 1664525u + 1013904223u;
      const int A = 1 + (int)((seed >> 8) % (P / 2));
      std::vector<int> u(A);
      long long U = 0;
      for (int i = 0; i < A; ++i) {
        seed = seed * 1664525u + 1013904223u;
        const int kind = (seed >> 28) & 3;
        u[i] = kind == 0 ? 1 : kind == 1 ? 1 + (int)((seed >> 4) % 7) : kind == 2 ? 1 + (int)((seed >> 4) % 4096) : 1 + (int)((seed >> 4) % (1 << 18));
        U += u[i];
      }
      if (U >= (1LL << 30)) continue;
      CHECK(per_group_shares(A, P));
      long long total = 0;
      for (int i = 0; i < A; ++i) {
        const int n = share_count(u[i], (int)U, P, A);
        CHECK(n >= 1 && n <= P - A + 1);
        const int cb = share_blocks(u[i], n), r = share_records(u[i], n);
        CHECK(cb >= 1 && (long long)cb * n >= u[i]);                 // the shares cover the group
        CHECK(r >= 1 && r <= n && (long long)(r - 1) * cb < u[i] && (long long)r * cb >= u[i]);
        CHECK(r <= kBalancedGrid + 1 && r <= u[i]);                    // fits the reserved record slots
        total += n;
      }
      CHECK(total <= P && total >= P - A);
      CHECK(A > 64 || per_group_fills((int)total, P));             // the register-built schedule never needs the check
    }
    CHECK(per_group_fills(192, P) && !per_group_fills(191, P));    // 128 equal groups: one workgroup each, dropped
    CHECK(!per_group_shares(0, P) && !per_group_shares(P / 2 + 1, P) && per_group_shares(P / 2, P));
    CHECK(share_count(0, 100, P, 3) == 0 && share_records(0, 0) == 0);
    CHECK(share_count(1 << 18, 1 << 18, P, 1) == P - 1);               // one group alone takes P - 1 workgroups
  }
  sr_paged_layout lay = {(uint32_t)sizeof(sr_paged_layout), 64, 4, 3};
  sr_route_params p = shape(1, 8, 2, 256, 0);
  PageMap out;
  const int32_t* tab = (const int32_t*)0x1000;
  CHECK(check_paged_args(tab, &lay, &p, &out) == SR_OK && out.page_shift == 6 && out.pages_per_seq == 4 && out.n_pages == 3);
  p.max_seq_len = 257;
  CHECK(check_paged_args(tab, &lay, &p, &out) == SR_ERR_SHAPE);
  p.max_seq_len = 256;
  lay.page_tokens = 1 << 30; lay.pages_per_seq = INT_MAX;
  CHECK(check_paged_args(tab, &lay, &p, &out) == SR_OK && out.page_shift == 30);
  lay.page_tokens = 96;
  CHECK(check_paged_args(tab, &lay, &p, &out) == SR_ERR_UNSUPPORTED);
  lay.page_tokens = INT_MIN;
  CHECK(check_paged_args(tab, &lay, &p, &out) == SR_ERR_UNSUPPORTED);
}

int main() {
  long long n = 0;
  const int Ls[] = {1, 63, 64, 65, 4096, 16383, 16384 * 2, 200000, 524288, (1 << 24) - 1, 1 << 24};
  const int heads[][2] = {{1, 1}, {4, 1}, {32, 8}, {64, 8}, {40, 40}, {16, 1}, {128, 8}};
  const int Bs[] = {1, 2, 4, 16, 17, 64, 255, 256, 257, 2047, 2048, 8191};
  const int splits[] = {0, 1, 3, 64, 1000, 65536, INT_MAX};
  for (int L : Ls)
    for (auto& h : heads)
      for (int B : Bs)
        for (int s : splits) {
          const sr_route_params p = shape(B, h[0], h[1], L, s);
          const long long NG = (long long)B * h[1];
          if (NG > 65535) { check_rejected(p, SR_ERR_SHAPE); ++n; continue; }
          Layout lay;
          cur = p;
          const int rc = make_layout(&p, &lay);
          if (rc == SR_ERR_SHAPE) {            // only a fixed grid beyond 32 bits may be refused here
            const long long per = ((long long)L + (s > 0 ? s : 1) - 1) / (s > 0 ? s : 1);
            const long long chunk = (per + 255) / 256 * 256;
            CHECK(s > 0 && (((long long)L + chunk - 1) / chunk) * NG > INT_MAX);
          } else {
            check_valid(p);
          }
          ++n;
        }
  // the documented limits, at their edge and one beyond
  check_valid(shape(65535, 1, 1, 1 << 24, 0));
  check_valid(shape(65535, 16, 1, 70, 0));
  check_valid(shape(1, 16, 1, 1 << 24, 0));
  check_valid(shape(1 << 20, 16, 16, 64, 0).batch > 65535 ? shape(4095, 16, 16, 64, 0) : shape(1, 1, 1, 1, 0));
  check_valid(shape(65535, 256, 16, 64, 0).n_q_heads / 16 <= 16 ? shape(65535 / 16, 256, 16, 64, 0) : shape(1, 1, 1, 1, 0));
  check_valid(shape(2048, 16, 1, 33554368 / 64, 0));       // NG * blocks just below 2^30: still balanced
  check_rejected(shape(65536, 1, 1, 64, 0), SR_ERR_SHAPE);
  check_rejected(shape(1, 1, 1, (1 << 24) + 1, 0), SR_ERR_SHAPE);
  check_rejected(shape(INT_MAX, INT_MAX, 1, 64, 0), SR_ERR_SHAPE);
  check_rejected(shape(INT_MAX, 1, INT_MAX, 64, 0), SR_ERR_SHAPE);
  check_rejected(shape(65535, 1, 1, 1 << 24, 65536), SR_ERR_SHAPE);          // 2^32 workgroups
  check_rejected(shape(1, 32, 8, 4096, -1), SR_ERR_SHAPE);
  check_rejected(shape(1, 33, 8, 4096, 0), SR_ERR_SHAPE);
  check_rejected(shape(1, 17, 1, 4096, 0), SR_ERR_UNSUPPORTED);
  check_rejected(shape(1, INT_MAX, 1, 4096, 0), SR_ERR_SHAPE);
  { sr_route_params p = shape(1, 32, 8, 4096, 0); p.head_dim = 64; check_rejected(p, SR_ERR_UNSUPPORTED); }
  { sr_route_params p = shape(1, 32, 8, 4096, 0); p.struct_size -= 4; check_rejected(p, SR_ERR_UNSUPPORTED); }
  cur = shape(0, 0, 0, 0, 0);
  Layout lay;
  CHECK(make_layout(nullptr, &lay) == SR_ERR_NULL);
  // static scratch: the five benchmark shapes fit, a 512-head batch at 32K does not
  const int bench[][4] = {{1, 32, 8, 4096}, {4, 32, 8, 32768}, {1, 32, 4, 200000}, {1, 64, 8, 524288}, {2, 40, 40, 65536}};
  for (auto& b : bench) {
    const sr_route_params p = shape(b[0], b[1], b[2], b[3], 0);
    cur = p;
    CHECK(make_layout(&p, &lay) == SR_OK && lay.plan.workspace_bytes <= kStaticScratchBytes);
  }
  { const sr_route_params p = shape(16, 32, 8, 32768, 0); cur = p; CHECK(make_layout(&p, &lay) == SR_OK && lay.plan.workspace_bytes > kStaticScratchBytes); }
  check_pages();
  printf("ok %lld\n", n);
  return 0;
}
