// Host planner: Alg. 1 prefill loop (stable partition of chunks by bitwidth),
// block layout of the packed cache, and the static split of the decode work.
#include <hip/hip_runtime.h>

#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <algorithm>
#include <cstring>
#include <vector>

#include "../../include/cocktail.h"
#include "common.h"
#include "plan.h"

namespace cocktail {

static thread_local char g_err[512] = "";

int fail(int code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return code;
}

int check_shape(const cocktail_shape* s) {
  if (!s) return fail(COCKTAIL_EINVAL, "shape is NULL");
  if (s->batch < 1 || s->num_q_heads < 1 || s->num_kv_heads < 1 || s->chunk_size < 1)
    return fail(COCKTAIL_EINVAL, "batch, head counts and chunk_size must be >= 1");
  if (s->num_q_heads % s->num_kv_heads != 0)
    return fail(COCKTAIL_EINVAL, "num_q_heads %d is not a multiple of num_kv_heads %d", s->num_q_heads,
                s->num_kv_heads);
  if (s->head_dim < 64 || s->head_dim % 64 != 0 || s->head_dim > 512)
    return fail(COCKTAIL_EINVAL, "head_dim %d must be a multiple of 64 in [64, 512]", s->head_dim);
  if (s->group_size != 32 && s->group_size != 64 && s->group_size != 128)
    return fail(COCKTAIL_EINVAL, "group_size %d must be 32, 64 or 128", s->group_size);
  if (s->head_dim % s->group_size != 0)
    return fail(COCKTAIL_EINVAL, "group_size %d does not divide head_dim %d", s->group_size, s->head_dim);
  return COCKTAIL_OK;
}

constexpr int64_t kCostWeightInt2 = 115, kCostWeightInt4 = 120, kCostWeightFp16 = 64;
// Share of every class that is cut into small late-dispatched items, and the size of one item (K+V bytes).
// Measured on MI355X: such items do not pay (their start-up latency costs more than the balance gains),
// so the share is zero; the planner and the kernel still support them.
constexpr int kDynamicPercent = 0;
constexpr int64_t kDynamicItemBytes = 40 * 1024;

static inline int32_t align16(int64_t x) { return static_cast<int32_t>((x + 15) & ~int64_t(15)); }

}  // namespace cocktail

using namespace cocktail;

extern "C" const char* cocktail_last_error(void) { return g_err; }
extern "C" int cocktail_version(void) { return (0 << 16) | 4; }

extern "C" int cocktail_plan(const cocktail_shape* shape, const int32_t* seq_lens, const uint8_t* chunk_bits,
                             int32_t num_workers, cocktail_sizes* sizes, void* plan_host, size_t plan_capacity,
                             int32_t* class_tokens, int32_t* perm) {
  if (int rc = check_shape(shape)) return rc;
  if (!seq_lens || !sizes) return fail(COCKTAIL_EINVAL, "seq_lens and sizes must not be NULL");
  if (num_workers < 1 || num_workers > (1 << 20))
    return fail(COCKTAIL_EINVAL, "num_workers %d out of range [1, 2^20]", num_workers);
  const int B = shape->batch, Hkv = shape->num_kv_heads, D = shape->head_dim, C = shape->chunk_size,
            G = shape->group_size;
  const int P = num_workers;

  int64_t total_chunks = 0, total_tokens = 0;
  for (int b = 0; b < B; ++b) {
    if (seq_lens[b] < 0) return fail(COCKTAIL_EINVAL, "seq_lens[%d] = %d is negative", b, seq_lens[b]);
    total_chunks += seq_lens[b] / C;
    total_tokens += seq_lens[b];
  }
  if (total_chunks > 0 && !chunk_bits) return fail(COCKTAIL_EINVAL, "chunk_bits is NULL");
  if (total_tokens >= (int64_t(1) << 31)) return fail(COCKTAIL_EINVAL, "more than 2^31 tokens in one call");
  for (int64_t i = 0; i < total_chunks; ++i) {
    const uint8_t v = chunk_bits[i];
    if (v != 2 && v != 4 && v != 16)
      return fail(COCKTAIL_EINVAL, "chunk_bits[%lld] = %d is not one of 2, 4, 16", (long long)i, int(v));
  }

  const int bits_of[3] = {2, 4, 16};
  int32_t row_bytes[3], block_bytes[3], algo_row[3];
  for (int c = 0; c < 3; ++c) {
    const int meta = (c == 2) ? 0 : 4 * (D / G);
    row_bytes[c] = D * bits_of[c] / 8;
    block_bytes[c] = kTB * (row_bytes[c] + meta);
    algo_row[c] = row_bytes[c] + meta;
  }

  // ---- Alg. 1 prefill loop: class lists in loop order, concatenated INT2 | INT4 | FP16 ----
  std::vector<int32_t> v_perm(total_chunks), v_chunk_off(B + 1, 0), v_ct(3 * B), v_cc0(3 * B), v_nblk(3 * B),
      v_blk_base(3 * (B + 1), 0);
  std::vector<int64_t> v_cum(B + 1, 0);
  int64_t class_tokens_tot[3] = {0, 0, 0};
  int64_t packed = 0;
  for (int b = 0; b < B; ++b) {
    const int n = seq_lens[b] / C;
    const uint8_t* bits = chunk_bits ? chunk_bits + v_chunk_off[b] : nullptr;
    int32_t* pb = v_perm.data() + v_chunk_off[b];
    int pos = 0;
    for (int c = 0; c < 3; ++c) {
      v_cc0[3 * b + c] = pos;
      for (int i = 0; i < n; ++i)
        if (bits[i] == bits_of[c]) pb[pos++] = i;
      int64_t ntok = int64_t(pos - v_cc0[3 * b + c]) * C;
      if (c == 2) ntok += seq_lens[b] - n * C;  // Sec. III-A: the remainder stays FP16
      v_ct[3 * b + c] = static_cast<int32_t>(ntok);
      v_nblk[3 * b + c] = static_cast<int32_t>((ntok + kTB - 1) / kTB);
      class_tokens_tot[c] += ntok;
      packed += 2 * int64_t(Hkv) * ntok * algo_row[c];
      const int64_t nb = int64_t(v_blk_base[3 * b + c]) + int64_t(Hkv) * v_nblk[3 * b + c];
      if (nb >= (int64_t(1) << 31)) return fail(COCKTAIL_EINVAL, "class %d needs more than 2^31 blocks", c);
      v_blk_base[3 * (b + 1) + c] = static_cast<int32_t>(nb);
    }
    v_chunk_off[b + 1] = v_chunk_off[b] + n;
    v_cum[b + 1] = v_cum[b] + seq_lens[b];
  }

  // Relative time per byte of the three classes in the decode kernel (1/64 units).  The FP16 class is
  // a pure stream; the quantised classes also keep the vector ALU busy, so a byte of them takes longer.
  // Measured on MI355X with all three classes running side by side.
  int64_t weight[3] = {kCostWeightInt2, kCostWeightInt4, kCostWeightFp16};
  if (const char* e = std::getenv("COCKTAIL_COST_WEIGHTS")) {   // tuning aid: "w2,w4,w16"
    long a = 0, b2 = 0, c2 = 0;
    if (std::sscanf(e, "%ld,%ld,%ld", &a, &b2, &c2) == 3 && a > 0 && b2 > 0 && c2 > 0) weight[0] = a, weight[1] = b2, weight[2] = c2;
  }

  int dyn_percent = kDynamicPercent;
  if (const char* e = std::getenv("COCKTAIL_DYNAMIC_PERCENT")) {   // tuning aid
    const int v = std::atoi(e);
    if (v >= 0 && v <= 90) dyn_percent = v;
  }

  // ---- physical runs of the class buffers: (class, b, h) order, each a contiguous run of blocks ----
  struct Run {
    int b, h, cls, nb, ntok, blk0;
  };
  std::vector<Run> runs;
  int64_t class_nblk[3] = {0, 0, 0};
  for (int c = 0; c < 3; ++c)
    for (int b = 0; b < B; ++b)
      for (int h = 0; h < Hkv; ++h) {
        const int nb = v_nblk[3 * b + c];
        if (nb == 0) continue;
        runs.push_back({b, h, c, nb, v_ct[3 * b + c], v_blk_base[3 * b + c] + h * nb});
        class_nblk[c] += nb;
      }
  int64_t tot_blocks = class_nblk[0] + class_nblk[1] + class_nblk[2];
  if (tot_blocks >= (int64_t(1) << 31)) return fail(COCKTAIL_EINVAL, "more than 2^31 blocks in one call");

  // ---- segments: the leading (100 - dyn)% of every class is split statically over the P workgroups,
  //      the trailing part is cut into small items that are dispatched as wave slots become free ----
  int64_t class_static[3];
  for (int c = 0; c < 3; ++c) class_static[c] = class_nblk[c] - class_nblk[c] * dyn_percent / 100;
  std::vector<Segment> segs;
  std::vector<int64_t> seg_cost0;   // cumulative cost (weighted bytes of K+V) at the start of each static segment
  int64_t gblk = 0, cost = 0;
  int32_t first_dyn_seg[3] = {0, 0, 0}, dyn_g0[3] = {0, 0, 0}, dyn_g1[3] = {0, 0, 0};
  for (int part = 0; part < 2; ++part) {
    if (part == 1) seg_cost0.push_back(cost);
    for (int c = 0; c < 3; ++c) {
      if (part == 1) first_dyn_seg[c] = static_cast<int32_t>(segs.size()), dyn_g0[c] = static_cast<int32_t>(gblk);
      int64_t seen = 0;   // blocks of class c passed so far
      for (const Run& r : runs) {
        if (r.cls != c) continue;
        // blocks [lo, hi) of this run belong to the current part
        const int64_t cut = class_static[c] - seen;   // blocks of this run that are static
        const int lo = part == 0 ? 0 : static_cast<int>(cut < 0 ? 0 : (cut > r.nb ? r.nb : cut));
        const int hi = part == 0 ? static_cast<int>(cut < 0 ? 0 : (cut > r.nb ? r.nb : cut)) : r.nb;
        seen += r.nb;
        if (hi <= lo) continue;
        Segment sgm;
        sgm.b = r.b, sgm.h = r.h, sgm.cls = c, sgm.ntok = r.ntok - lo * kTB;
        sgm.blk0 = r.blk0 + lo, sgm.nblk = hi - lo;
        sgm.gblk0 = static_cast<int32_t>(gblk);
        sgm.bh = r.b * Hkv + r.h;
        segs.push_back(sgm);
        if (part == 0) seg_cost0.push_back(cost);
        gblk += sgm.nblk;
        cost += int64_t(sgm.nblk) * 2 * block_bytes[c] * weight[c];
      }
      if (part == 1) dyn_g1[c] = static_cast<int32_t>(gblk);
    }
  }
  const int S = static_cast<int>(segs.size());
  const int S_static = static_cast<int>(seg_cost0.size()) - 1;   // segments of the static part
  const int64_t W = seg_cost0[S_static];      // cost of the static part
  const int32_t g_static = S_static < S ? segs[S_static].gblk0 : static_cast<int32_t>(gblk);

  // ---- work items: P static ranges of equal cost, then the dynamic items ----
  struct Item {
    int32_t g0, g1, seg0, pid0;
    double key;
  };
  std::vector<Item> items(P);
  {
    std::vector<int32_t> bound(P + 1), bseg(P + 1);
    int s = 0;
    for (int w = 0; w <= P; ++w) {
      const int64_t target = static_cast<int64_t>((static_cast<__int128>(W) * w) / P);
      while (s < S_static && seg_cost0[s + 1] <= target) ++s;
      if (s >= S_static) {
        bound[w] = g_static, bseg[w] = S_static;
      } else {
        const int64_t per = 2 * int64_t(block_bytes[segs[s].cls]) * weight[segs[s].cls];
        int64_t j = (target - seg_cost0[s] + per / 2) / per;
        if (j > segs[s].nblk) j = segs[s].nblk;
        bound[w] = segs[s].gblk0 + static_cast<int32_t>(j);
        bseg[w] = (j == segs[s].nblk) ? s + 1 : s;
      }
    }
    bound[0] = 0, bseg[0] = 0, bound[P] = g_static, bseg[P] = S_static;
    for (int w = 0; w < P; ++w) items[w] = {bound[w], bound[w + 1], bseg[w], 0, 0.0};
  }
  {
    std::vector<Item> dyn;
    for (int c = 0; c < 3; ++c) {
      const int n = dyn_g1[c] - dyn_g0[c];
      if (n <= 0) continue;
      int per = static_cast<int>(kDynamicItemBytes / (2 * int64_t(block_bytes[c])));
      if (per < 1) per = 1;
      int sidx = first_dyn_seg[c];
      for (int g0 = dyn_g0[c]; g0 < dyn_g1[c]; g0 += per) {
        const int g1 = g0 + per < dyn_g1[c] ? g0 + per : dyn_g1[c];
        while (segs[sidx].gblk0 + segs[sidx].nblk <= g0) ++sidx;
        // interleave the classes in the queue by relative position inside their dynamic part
        dyn.push_back({g0, g1, sidx, 0, (double(g0 - dyn_g0[c]) + 0.5 * (g1 - g0)) / double(n)});
      }
    }
    std::stable_sort(dyn.begin(), dyn.end(), [](const Item& x, const Item& y) { return x.key < y.key; });
    items.insert(items.end(), dyn.begin(), dyn.end());
  }
  const int Q = static_cast<int>(items.size()) - P;

  // partial ids: one per (item, class, (b, kv head)) intersection, numbered in the global block order so
  // that the ids of one (b, kv head, class, part) are contiguous
  const int BH = B * Hkv;
  std::vector<int32_t> bh_pid(size_t(BH) * 12, 0);   // [bh][class][static|dynamic][begin, end)
  int32_t npart = 0;
  {
    std::vector<int> order(items.size());
    for (size_t i = 0; i < order.size(); ++i) order[i] = static_cast<int>(i);
    std::stable_sort(order.begin(), order.end(), [&](int x, int y) { return items[x].g0 < items[y].g0; });
    for (int idx : order) {
      Item& it = items[idx];
      it.pid0 = npart;
      const int part = idx < P ? 0 : 1;
      int s = it.seg0;
      int32_t g = it.g0;
      int cur = -1, cur_cls = -1;
      while (g < it.g1) {
        const Segment& sg = segs[s];
        if (sg.bh != cur || sg.cls != cur_cls) {
          cur = sg.bh, cur_cls = sg.cls;
          int32_t* range = &bh_pid[((size_t(cur) * 3 + cur_cls) * 2 + part) * 2];
          if (range[1] == range[0]) range[0] = npart;
          range[1] = npart + 1;
          ++npart;
        }
        const int32_t end = sg.gblk0 + sg.nblk;
        g = end < it.g1 ? end : it.g1;
        ++s;
      }
    }
  }

  // ---- sizes and blob layout ----
  PlanHeader hd;
  std::memset(&hd, 0, sizeof(hd));
  hd.magic = kPlanMagic, hd.version = kPlanVersion;
  hd.batch = B, hd.num_q_heads = shape->num_q_heads, hd.num_kv_heads = Hkv, hd.head_dim = D;
  hd.chunk_size = C, hd.group_size = G, hd.rep = shape->num_q_heads / Hkv;
  hd.num_workers = P, hd.num_segments = S, hd.num_partials = npart, hd.num_items = Q;
  hd.total_gblocks = static_cast<int32_t>(gblk);
  hd.total_chunks = total_chunks, hd.total_tokens = total_tokens, hd.packed_bytes = packed;
  for (int c = 0; c < 3; ++c) {
    hd.class_blocks[c] = v_blk_base[3 * B + c];
    hd.class_bytes[c] = hd.class_blocks[c] * block_bytes[c];
    hd.block_bytes[c] = block_bytes[c];
    hd.row_bytes[c] = row_bytes[c];
  }
  hd.workspace_bytes = int64_t(npart > 0 ? npart : 1) * hd.rep * (D + kPartialFloats) * int64_t(sizeof(float));
  int64_t off = align16(sizeof(PlanHeader));
  auto place = [&](int32_t& field, int64_t bytes) {
    field = static_cast<int32_t>(off);
    off = align16(off + bytes);
  };
  place(hd.off_seq_len, 4 * int64_t(B));
  place(hd.off_cum_tokens, 8 * int64_t(B + 1));
  place(hd.off_chunk_off, 4 * int64_t(B + 1));
  place(hd.off_perm, 4 * total_chunks);
  place(hd.off_class_tokens, 12 * int64_t(B));
  place(hd.off_class_chunk0, 12 * int64_t(B));
  place(hd.off_blk_base, 12 * int64_t(B + 1));
  place(hd.off_nblk, 12 * int64_t(B));
  place(hd.off_segments, int64_t(sizeof(Segment)) * S);
  place(hd.off_bh_pid, 48 * int64_t(BH));
  place(hd.off_worker_rec, int64_t(sizeof(WorkerRec)) * (P + Q));
  if (off >= (int64_t(1) << 31)) return fail(COCKTAIL_EINVAL, "plan larger than 2 GiB");
  hd.plan_bytes = off;

  std::memset(sizes, 0, sizeof(*sizes));
  sizes->total_chunks = total_chunks;
  for (int c = 0; c < 3; ++c) {
    sizes->class_tokens[c] = class_tokens_tot[c];
    sizes->class_blocks[c] = hd.class_blocks[c];
    sizes->class_bytes[c] = hd.class_bytes[c];
  }
  sizes->plan_bytes = hd.plan_bytes;
  sizes->workspace_bytes = hd.workspace_bytes;
  sizes->packed_bytes = packed;
  sizes->num_workers = P, sizes->num_partials = npart, sizes->num_segments = S;

  if (class_tokens) std::memcpy(class_tokens, v_ct.data(), sizeof(int32_t) * v_ct.size());
  if (perm && total_chunks) std::memcpy(perm, v_perm.data(), sizeof(int32_t) * v_perm.size());

  if (plan_host) {
    if (plan_capacity < static_cast<size_t>(hd.plan_bytes))
      return fail(COCKTAIL_ENOSPACE, "plan buffer holds %zu bytes, %lld needed", plan_capacity,
                  (long long)hd.plan_bytes);
    char* p = static_cast<char*>(plan_host);
    std::memset(p, 0, hd.plan_bytes);
    std::memcpy(p, &hd, sizeof(hd));
    auto put = [&](int32_t o, const void* src, size_t bytes) {
      if (bytes) std::memcpy(p + o, src, bytes);
    };
    put(hd.off_seq_len, seq_lens, 4 * size_t(B));
    put(hd.off_cum_tokens, v_cum.data(), 8 * size_t(B + 1));
    put(hd.off_chunk_off, v_chunk_off.data(), 4 * size_t(B + 1));
    put(hd.off_perm, v_perm.data(), 4 * size_t(total_chunks));
    put(hd.off_class_tokens, v_ct.data(), 12 * size_t(B));
    put(hd.off_class_chunk0, v_cc0.data(), 12 * size_t(B));
    put(hd.off_blk_base, v_blk_base.data(), 12 * size_t(B + 1));
    put(hd.off_nblk, v_nblk.data(), 12 * size_t(B));
    put(hd.off_segments, segs.data(), sizeof(Segment) * size_t(S));
    put(hd.off_bh_pid, bh_pid.data(), 48 * size_t(BH));
    std::vector<WorkerRec> recs(P + Q);
    std::memset(recs.data(), 0, sizeof(WorkerRec) * recs.size());
    for (int w = 0; w < P + Q; ++w) {
      recs[w].g0 = items[w].g0, recs[w].g1 = items[w].g1;
      recs[w].seg0 = items[w].seg0, recs[w].pid0 = items[w].pid0;
      if (items[w].g0 < items[w].g1) recs[w].first = segs[items[w].seg0];
    }
    put(hd.off_worker_rec, recs.data(), sizeof(WorkerRec) * recs.size());

  }
  g_err[0] = 0;
  return COCKTAIL_OK;
}
