// Host planner: Alg. 1 prefill loop (stable partition of chunks by bitwidth),
// block layout of the packed cache, and the static split of the decode work.
#include <hip/hip_runtime.h>

#include <cstdarg>
#include <cstdio>
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

static inline int32_t align16(int64_t x) { return static_cast<int32_t>((x + 15) & ~int64_t(15)); }

}  // namespace cocktail

using namespace cocktail;

extern "C" const char* cocktail_last_error(void) { return g_err; }
extern "C" int cocktail_version(void) { return (0 << 16) | 3; }

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

  // ---- segments in the global order (b, h, class, block) ----
  std::vector<Segment> segs;
  int64_t gblk = 0;
  std::vector<int64_t> seg_cost0;  // cumulative cost (bytes of K+V) at the start of each segment
  int64_t cost = 0;
  for (int b = 0; b < B; ++b)
    for (int h = 0; h < Hkv; ++h)
      for (int c = 0; c < 3; ++c) {
        const int nb = v_nblk[3 * b + c];
        if (nb == 0) continue;
        Segment s;
        s.b = b, s.h = h, s.cls = c, s.ntok = v_ct[3 * b + c];
        s.blk0 = v_blk_base[3 * b + c] + h * nb;
        s.nblk = nb;
        s.gblk0 = static_cast<int32_t>(gblk);
        s.bh = b * Hkv + h;
        segs.push_back(s);
        seg_cost0.push_back(cost);
        gblk += nb;
        cost += int64_t(nb) * 2 * block_bytes[c];
        if (gblk >= (int64_t(1) << 31)) return fail(COCKTAIL_EINVAL, "more than 2^31 blocks in one call");
      }
  const int S = static_cast<int>(segs.size());
  seg_cost0.push_back(cost);
  const int64_t W = cost;

  // ---- equal-byte split of the block stream over P workers ----
  std::vector<int32_t> w_gblk(P + 1), w_seg(P + 1), w_pid(P + 1);
  {
    int s = 0;
    for (int w = 0; w <= P; ++w) {
      // target = w * W / P without overflow (W < 2^62 / P is guaranteed by the 2^31 block limit for sane P)
      const int64_t target = static_cast<int64_t>((static_cast<__int128>(W) * w) / P);
      while (s < S && seg_cost0[s + 1] <= target) ++s;
      if (s >= S) {
        w_gblk[w] = static_cast<int32_t>(gblk);
        w_seg[w] = S;
      } else {
        const int64_t per = 2 * int64_t(block_bytes[segs[s].cls]);
        int64_t j = (target - seg_cost0[s] + per / 2) / per;
        if (j > segs[s].nblk) j = segs[s].nblk;
        w_gblk[w] = segs[s].gblk0 + static_cast<int32_t>(j);
        w_seg[w] = s;
        if (j == segs[s].nblk) w_seg[w] = s + 1;  // boundary falls on the segment end
      }
    }
    w_gblk[0] = 0, w_seg[0] = 0;
    w_gblk[P] = static_cast<int32_t>(gblk), w_seg[P] = S;
  }
  // partial ids: one per (worker, (b, kv head)) intersection, numbered in global order
  const int BH = B * Hkv;
  std::vector<int32_t> bh_pid(BH + 1, 0);
  std::vector<int32_t> bh_count(BH, 0);
  int32_t npart = 0;
  for (int w = 0; w < P; ++w) {
    w_pid[w] = npart;
    int s = w_seg[w];
    int32_t g = w_gblk[w];
    const int32_t g1 = w_gblk[w + 1];
    int cur = -1;
    while (g < g1) {
      const Segment& sg = segs[s];
      if (sg.bh != cur) {
        cur = sg.bh;
        ++npart;
        ++bh_count[cur];
      }
      const int32_t end = sg.gblk0 + sg.nblk;
      g = end < g1 ? end : g1;
      ++s;
    }
  }
  w_pid[P] = npart;
  for (int i = 0; i < BH; ++i) bh_pid[i + 1] = bh_pid[i] + bh_count[i];

  // ---- sizes and blob layout ----
  PlanHeader hd;
  std::memset(&hd, 0, sizeof(hd));
  hd.magic = kPlanMagic, hd.version = kPlanVersion;
  hd.batch = B, hd.num_q_heads = shape->num_q_heads, hd.num_kv_heads = Hkv, hd.head_dim = D;
  hd.chunk_size = C, hd.group_size = G, hd.rep = shape->num_q_heads / Hkv;
  hd.num_workers = P, hd.num_segments = S, hd.num_partials = npart;
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
  place(hd.off_worker_gblk, 4 * int64_t(P + 1));
  place(hd.off_worker_seg, 4 * int64_t(P + 1));
  place(hd.off_worker_pid, 4 * int64_t(P + 1));
  place(hd.off_bh_pid, 4 * int64_t(BH + 1));
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
    put(hd.off_worker_gblk, w_gblk.data(), 4 * size_t(P + 1));
    put(hd.off_worker_seg, w_seg.data(), 4 * size_t(P + 1));
    put(hd.off_worker_pid, w_pid.data(), 4 * size_t(P + 1));
    put(hd.off_bh_pid, bh_pid.data(), 4 * size_t(BH + 1));
  }
  g_err[0] = 0;
  return COCKTAIL_OK;
}
