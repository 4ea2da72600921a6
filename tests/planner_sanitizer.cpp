// Host-side fuzz of the planner, meant to be built with AddressSanitizer and UndefinedBehaviorSanitizer
// (tests/test_planner_sanitizers.py does that; no GPU is involved).  For thousands of random shapes it calls
// cocktail_plan_ex the way a caller does (size query, then the fill), then walks the plan blob the way the
// decode and reorder+quantize kernels do and checks that every index they would follow stays inside the
// blob and the buffers it describes: every 32-token unit is read exactly once, every partial id is written
// exactly once, every reorder+quantize record names rows that exist.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <random>
#include <vector>

#include "../include/cocktail.h"
#include "../paper_2503_23294_amd/csrc/plan.h"

using namespace cocktail;

#define REQUIRE(cond)                                                                     \
  do {                                                                                    \
    if (!(cond)) {                                                                        \
      std::fprintf(stderr, "case %d: %s:%d: requirement failed: %s\n", g_case, __FILE__, __LINE__, #cond); \
      std::exit(1);                                                                       \
    }                                                                                     \
  } while (0)

static int g_case = -1;

template <class T>
static const T* view(const std::vector<char>& blob, int64_t off, int64_t count) {
  REQUIRE(off >= 0 && off % 4 == 0 && off + int64_t(sizeof(T)) * count <= int64_t(blob.size()));
  return reinterpret_cast<const T*>(blob.data() + off);
}

static void check_plan(const cocktail_shape& sh, const std::vector<int32_t>& lens, const std::vector<uint8_t>& bits,
                       int workers, const cocktail_plan_options& opt, std::mt19937_64& rng) {
  cocktail_sizes sz;
  std::vector<int32_t> ct(kNumClasses * sh.batch), perm(bits.size() + 1);
  int rc = cocktail_plan_ex(&sh, lens.data(), bits.empty() ? nullptr : bits.data(), workers, &opt, &sz, nullptr, 0,
                            nullptr, nullptr);
  REQUIRE(rc == COCKTAIL_OK);
  std::vector<char> blob(sz.plan_bytes);
  // an undersized buffer must be refused without a write
  if (sz.plan_bytes > 16) {
    std::vector<char> small(sz.plan_bytes - 16);
    REQUIRE(cocktail_plan_ex(&sh, lens.data(), bits.empty() ? nullptr : bits.data(), workers, &opt, &sz, small.data(),
                             small.size(), nullptr, nullptr) == COCKTAIL_ENOSPACE);
  }
  rc = cocktail_plan_ex(&sh, lens.data(), bits.empty() ? nullptr : bits.data(), workers, &opt, &sz, blob.data(),
                        blob.size(), ct.data(), perm.data());
  REQUIRE(rc == COCKTAIL_OK);
  const PlanHeader& hd = *view<PlanHeader>(blob, 0, 1);
  REQUIRE(hd.magic == kPlanMagic && hd.plan_bytes == int64_t(blob.size()));
  const int B = sh.batch, Hkv = sh.num_kv_heads, C = sh.chunk_size, P = hd.num_workers;
  REQUIRE(P >= 1 && P <= workers && P == sz.num_workers && (P == workers || P % 64 == 0));   // the request is an upper bound
  const int UPB = sh.head_dim == 64 ? 1 : 2;   // units (what a wave handles at a time) per 64-token block
  const int Hw = hd.work_heads;   // heads of the decode work split: Hkv, or Hq with one wave per query head
  REQUIRE(hd.work_rep >= 1 && hd.work_rep <= 8 && Hw * hd.work_rep == sh.num_q_heads && Hw % Hkv == 0);
  const int share = Hw / Hkv;
  const int S = hd.num_segments, NG = hd.num_groups, NPS = hd.num_pool_segs, BH = B * Hw;
  const Segment* segs = view<Segment>(blob, hd.off_segments, S);
  const WorkerRec* recs = view<WorkerRec>(blob, hd.off_worker_rec, P);
  const GroupRec* groups = view<GroupRec>(blob, hd.off_group_rec, NG);
  const PoolSeg* psegs = view<PoolSeg>(blob, hd.off_pool_seg, NPS);
  const int32_t* bh_off = view<int32_t>(blob, hd.off_bh_off, BH + 1);
  const uint32_t* counters = view<uint32_t>(blob, hd.off_counters, int64_t(NG) * kCounterStride);
  const int32_t* chunk_off = view<int32_t>(blob, hd.off_chunk_off, B + 1);
  const int32_t* pperm = view<int32_t>(blob, hd.off_perm, hd.total_chunks);
  const int32_t* cc0 = view<int32_t>(blob, hd.off_class_chunk0, kNumClasses * B);
  const int32_t* ctok = view<int32_t>(blob, hd.off_class_tokens, kNumClasses * B);
  const int32_t* seq_len = view<int32_t>(blob, hd.off_seq_len, B);
  // layout: blocks per head that hold tokens, blocks per head the run is laid out with, first block per sequence
  const int32_t* used_blk = view<int32_t>(blob, hd.off_nblk, kNumClasses * B);
  const int32_t* run_blk = view<int32_t>(blob, hd.off_run_blocks, kNumClasses * B);
  const int32_t* base_blk = view<int32_t>(blob, hd.off_blk_base, kNumClasses * (B + 1));
  int64_t nblocks = 0, nrecords = 0;   // blocks with tokens (the decode work); blocks of the buffers (one record each)
  for (int c = 0; c < kNumClasses; ++c) {
    nrecords += hd.class_blocks[c];
    REQUIRE(base_blk[c] == 0 && base_blk[kNumClasses * B + c] == hd.class_blocks[c] && sz.class_blocks[c] == hd.class_blocks[c]);
    for (int b = 0; b < B; ++b) {
      const int64_t n = ctok[kNumClasses * b + c];
      const int64_t room = (c == kFp16Class && opt.max_seq_lens) ? opt.max_seq_lens[b] - lens[b] : 0;
      REQUIRE(used_blk[kNumClasses * b + c] == (n + kTB - 1) / kTB && run_blk[kNumClasses * b + c] == (n + room + kTB - 1) / kTB);
      REQUIRE(base_blk[kNumClasses * (b + 1) + c] - base_blk[kNumClasses * b + c] == int64_t(Hkv) * run_blk[kNumClasses * b + c]);
      nblocks += int64_t(Hkv) * used_blk[kNumClasses * b + c];
    }
  }
  const RQItem* items = view<RQItem>(blob, hd.off_rq_items, nrecords);
  for (int64_t i = 0; i < int64_t(NG) * kCounterStride; ++i) REQUIRE(counters[i] == 0);
  REQUIRE(hd.off_counters % 128 == 0);

  // Alg. 1's partition: perm is a permutation per sequence, classes ascending, stable
  for (int b = 0; b < B; ++b) {
    const int n = lens[b] / C;
    REQUIRE(chunk_off[b + 1] - chunk_off[b] == n && seq_len[b] == lens[b]);
    std::vector<int> seen(n, 0);
    int prev_cls = -1, prev_idx = -1;
    for (int j = 0; j < n; ++j) {
      const int i = pperm[chunk_off[b] + j];
      REQUIRE(i >= 0 && i < n && !seen[i]);
      seen[i] = 1;
      const int v = bits[chunk_off[b] + i], cls = v == 2 ? 0 : v == 4 ? 1 : v == 8 ? 2 : 3;
      REQUIRE(cls > prev_cls || (cls == prev_cls && i > prev_idx));
      prev_cls = cls, prev_idx = i;
      REQUIRE(perm[chunk_off[b] + j] == i);
    }
    int64_t tot = 0;
    for (int c = 0; c < kNumClasses; ++c) {
      tot += ctok[kNumClasses * b + c];
      REQUIRE(ct[kNumClasses * b + c] == ctok[kNumClasses * b + c]);
    }
    REQUIRE(tot == lens[b]);
  }

  // segments tile every class buffer exactly once and are listed in global order
  std::vector<std::vector<uint8_t>> phys(kNumClasses);
  for (int c = 0; c < kNumClasses; ++c) phys[c].assign(hd.class_blocks[c], 0);
  int64_t g = 0;
  for (int s = 0; s < S; ++s) {
    const Segment& sg = segs[s];
    REQUIRE(sg.cls >= 0 && sg.cls < kNumClasses && sg.b >= 0 && sg.b < B && sg.h >= 0 && sg.h < Hw);
    REQUIRE(sg.gblk0 == g && sg.nblk > 0 && int64_t(sg.nblk - 1) * kTB < sg.ntok);
    REQUIRE(sg.blk0 >= 0 && int64_t(sg.blk0) + sg.nblk <= hd.class_blocks[sg.cls]);
    for (int i = 0; i < sg.nblk; ++i) REQUIRE(phys[sg.cls][sg.blk0 + i]++ < share);
    g += sg.nblk;
  }
  REQUIRE(g == hd.total_gblocks && g == nblocks * share);
  // every block that holds tokens once per work head of its kv head; blocks that are only room to grow never
  for (int c = 0; c < kNumClasses; ++c) {
    std::vector<uint8_t> want(hd.class_blocks[c], 0);
    for (int b = 0; b < B; ++b)
      for (int h = 0; h < Hkv; ++h)
        for (int i = 0; i < used_blk[kNumClasses * b + c]; ++i)
          want[base_blk[kNumClasses * b + c] + int64_t(h) * run_blk[kNumClasses * b + c] + i] = uint8_t(share);
    REQUIRE(phys[c] == want);
  }

  // the walk of every worker: own range, then the pool tickets of its group (handed out at random)
  std::vector<uint8_t> unit_seen(UPB * g, 0);
  std::vector<uint8_t> pid_seen(hd.num_partials, 0);
  auto claim_pid = [&](int pid, const Segment& sg) {
    REQUIRE(pid >= 0 && pid < hd.num_partials && !pid_seen[pid]);
    pid_seen[pid] = 1;
    const int bh = sg.b * Hw + sg.h;
    REQUIRE(bh_off[bh] <= pid && pid < bh_off[bh + 1]);
  };
  std::vector<std::vector<int>> members(NG);
  for (int w = 0; w < P; ++w) {
    REQUIRE(recs[w].group >= 0 && recs[w].group < NG);
    members[recs[w].group].push_back(w);
  }
  for (int gi = 0; gi < NG; ++gi) {
    const GroupRec& gr = groups[gi];
    REQUIRE(int(members[gi].size()) == gr.nworkers && gr.nps >= 0 && gr.nps <= kMaxPoolSegments);
    REQUIRE(gr.pseg0 >= 0 && gr.pseg0 + gr.nps <= NPS && gr.ngran >= 0);
    std::vector<std::vector<int>> tickets(gr.nworkers);
    for (int t = 0; t < gr.ngran; ++t) tickets[rng() % gr.nworkers].push_back(t);
    for (int w : members[gi]) {
      const WorkerRec& rc_ = recs[w];
      const int rank = rc_.rank_nps & 0xffff;
      REQUIRE(rank < gr.nworkers && (rc_.rank_nps >> 16) == gr.nps && rc_.ngran == gr.ngran && rc_.pseg0 == gr.pseg0);
      int u = UPB * rc_.g0, u1 = UPB * rc_.g1, s = rc_.seg0, pid = rc_.pid0, last_seg = -1;
      REQUIRE(rc_.g0 <= rc_.g1 && rc_.g1 <= g);
      if (u < u1) {
        REQUIRE(s >= 0 && s < S && std::memcmp(&rc_.first, &segs[s], sizeof(Segment)) == 0);
      }
      while (u < u1) {
        REQUIRE(s < S);
        if (u >= UPB * (segs[s].gblk0 + segs[s].nblk)) {
          ++s;
          REQUIRE(s < S);
          pid = segs[s].pid0;
          continue;
        }
        REQUIRE(u >= UPB * segs[s].gblk0);
        if (s != last_seg) {
          claim_pid(pid, segs[s]);
          last_seg = s;
        }
        const int end = std::min(u1, UPB * (segs[s].gblk0 + segs[s].nblk));
        const int nu = std::min(kIterUnits[segs[s].cls], end - u);
        REQUIRE(nu > 0);
        for (int i = 0; i < nu; ++i) REQUIRE(unit_seen[u + i]++ == 0);
        u += nu;
      }
      uint32_t used = 0;
      for (int t : tickets[rank]) {
        int pi = -1;
        for (int i = 0; i < gr.nps; ++i)
          if (psegs[gr.pseg0 + i].gran0 <= t) pi = i;
        REQUIRE(pi >= 0);
        const PoolSeg& ps = psegs[gr.pseg0 + pi];
        REQUIRE(ps.seg >= 0 && ps.seg < S && ps.seg >= last_seg);
        const Segment& sg = segs[ps.seg];
        const int J = kIterUnits[sg.cls];
        const int us = ps.unit0 + (t - ps.gran0) * J, nu = std::min(J, ps.unit0 + ps.nunits - us);
        REQUIRE(nu > 0 && us >= 0 && us + nu <= UPB * sg.nblk);
        if (ps.seg != last_seg) {
          REQUIRE(rank < ps.nslots);
          claim_pid(ps.slot0 + rank, sg);
          used |= 1u << pi;
          last_seg = ps.seg;
        }
        for (int i = 0; i < nu; ++i) REQUIRE(unit_seen[UPB * sg.gblk0 + us + i]++ == 0);
      }
      for (int i = 0; i < gr.nps; ++i)   // slots the worker fills with the neutral state
        if (!((used >> i) & 1u) && rank < psegs[gr.pseg0 + i].nslots)
          claim_pid(psegs[gr.pseg0 + i].slot0 + rank, segs[psegs[gr.pseg0 + i].seg]);
    }
  }
  for (int64_t i = 0; i < UPB * g; ++i) REQUIRE(unit_seen[i] == 1);
  // the last partials of every (sequence, kv head) belong to the appended tokens, one per slice of the append buffer
  REQUIRE(hd.append_slices == (hd.append_blocks + kAppendSliceBlocks - 1) / kAppendSliceBlocks);
  for (int bh = 0; bh < BH; ++bh)
    for (int sl = 1; sl <= hd.append_slices; ++sl) {
      REQUIRE(bh_off[bh + 1] - sl >= bh_off[bh] && !pid_seen[bh_off[bh + 1] - sl]);
      pid_seen[bh_off[bh + 1] - sl] = 1;
    }
  for (int i = 0; i < hd.num_partials; ++i) REQUIRE(pid_seen[i] == 1);
  REQUIRE(bh_off[0] == 0 && bh_off[BH] == hd.num_partials);

  // reorder+quantize records: every block of every class buffer, its rows inside the source
  int64_t idx = 0;
  for (int c = 0; c < kNumClasses; ++c)
    for (int64_t i = 0; i < hd.class_blocks[c]; ++i, ++idx) {
      const RQItem& it = items[idx];
      const int cls = it.cls_nvalid & 0xff, nvalid = it.cls_nvalid >> 8;
      REQUIRE(cls == c && nvalid >= 0 && nvalid <= kTB && it.b >= 0 && it.b < B && it.h >= 0 && it.h < Hkv);
      const int T = lens[it.b], N = T / C;
      const int ntok = ctok[kNumClasses * it.b + c], chunk_tokens = c == kFp16Class ? ntok - (T - N * C) : ntok;
      // record i describes block i of the class buffer: block j of the run of (b, h)
      REQUIRE(i == base_blk[kNumClasses * it.b + c] + int64_t(it.h) * run_blk[kNumClasses * it.b + c] + it.j);
      REQUIRE(it.j >= 0 && it.j < run_blk[kNumClasses * it.b + c]);
      REQUIRE(nvalid == std::max<int64_t>(0, std::min<int64_t>(kTB, ntok - int64_t(it.j) * kTB)));
      if (nvalid == 0) {   // room to grow: written as zeros, nothing is read
        REQUIRE(c == kFp16Class && it.t0 == 0);
        continue;
      }
      if (it.t0 >= 0) {
        REQUIRE(it.t0 + nvalid <= T);
      } else {
        for (int r = it.j * kTB; r < it.j * kTB + nvalid; ++r) {
          int t;
          if (r < chunk_tokens) {
            const int slot = r / C;
            REQUIRE(cc0[kNumClasses * it.b + c] + slot < N);
            t = pperm[chunk_off[it.b] + cc0[kNumClasses * it.b + c] + slot] * C + (r - slot * C);
          } else {
            t = N * C + (r - chunk_tokens);
          }
          REQUIRE(t >= 0 && t < T);
        }
      }
    }
  REQUIRE(idx == nrecords);

  // the debugging accessor agrees with the header
  int64_t v = -1;
  REQUIRE(cocktail_plan_field(blob.data(), "num_partials", 0, &v) == COCKTAIL_OK && v == hd.num_partials);
  REQUIRE(cocktail_plan_field(blob.data(), "class_blocks", 2, &v) == COCKTAIL_OK && v == hd.class_blocks[2]);
  REQUIRE(cocktail_plan_field(blob.data(), "class_blocks", kNumClasses, &v) == COCKTAIL_EINVAL);
  REQUIRE(cocktail_plan_field(blob.data(), "no_such_field", 0, &v) == COCKTAIL_EINVAL);
}

int main(int argc, char** argv) {
  const int cases = argc > 1 ? std::atoi(argv[1]) : 2000;
  const uint64_t seed = argc > 2 ? std::strtoull(argv[2], nullptr, 10) : 1;
  std::mt19937_64 rng(seed);
  auto pick = [&](std::initializer_list<int> xs) { return *(xs.begin() + rng() % xs.size()); };
  for (g_case = 0; g_case < cases; ++g_case) {
    cocktail_shape sh;
    sh.batch = 1 + int(rng() % 6);
    sh.num_kv_heads = 1 + int(rng() % 4);
    sh.num_q_heads = sh.num_kv_heads * pick({1, 1, 2, 3, 4, 5, 8, 11, 12, 16});
    sh.head_dim = pick({64, 128, 128});
    sh.group_size = sh.head_dim == 64 ? pick({32, 64}) : pick({32, 64, 128});
    sh.chunk_size = pick({1, 8, 17, 32, 64, 100, 256, 1000});
    std::vector<int32_t> lens(sh.batch);
    std::vector<uint8_t> bits;
    const int scale = pick({70, 700, 7000, 40000});
    const int mix = int(rng() % 7);   // 0..3: a single class, 4..6: mixed
    for (int b = 0; b < sh.batch; ++b) {
      lens[b] = (rng() % 5 == 0) ? int(rng() % sh.chunk_size) : int(rng() % scale);
      for (int i = 0; i < lens[b] / sh.chunk_size; ++i) {
        const int c = mix < 4 ? mix : int(rng() % 4);
        bits.push_back(uint8_t(kClassBits[c]));
      }
    }
    const int workers = pick({1, 2, 3, 5, 8, 16, 33, 64, 200, 2048});
    cocktail_plan_options opt;
    std::memset(&opt, 0, sizeof(opt));
    opt.append_capacity = pick({0, 0, 1, 64, 130, 1500});
    opt.reproducible = int(rng() % 4 == 0);
    opt.vector_alu_only = int(rng() % 5 == 0);
    std::vector<int32_t> most(lens);
    if (rng() % 3 == 0) {   // FP16 runs with room to grow
      for (int b = 0; b < sh.batch; ++b) most[b] += pick({0, 1, 63, 64, 65, 1000});
      opt.max_seq_lens = most.data();
    }
    check_plan(sh, lens, bits, workers, opt, rng);
  }
  // extremes: the longest sequence the planner accepts, and one it has to refuse
  {
    g_case = -2;
    cocktail_shape sh{1, 1, 1, 128, 1 << 16, 32};
    const int32_t longest = (1 << 24) - 64;
    std::vector<int32_t> lens{longest};
    std::vector<uint8_t> bits(longest >> 16, 16);
    cocktail_plan_options opt;
    std::memset(&opt, 0, sizeof(opt));
    check_plan(sh, lens, bits, 2048, opt, rng);
    lens[0] = 1 << 24;
    bits.assign(lens[0] >> 16, 16);
    cocktail_sizes sz;
    REQUIRE(cocktail_plan_ex(&sh, lens.data(), bits.data(), 8, &opt, &sz, nullptr, 0, nullptr, nullptr) == COCKTAIL_EUNSUPPORTED);
  }
  std::printf("planner fuzz: %d random shapes and the extremes passed\n", cases);
  return 0;
}
