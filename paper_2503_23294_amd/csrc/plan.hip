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

constexpr int64_t kCostWeight[kNumClasses] = {1150, 1300, 1100, 530};
// The same for the kernel that serves four query heads per wave: its arithmetic runs on the matrix unit.
constexpr int64_t kQuadCostWeight[kNumClasses] = {1300, 1250, 950, 450};
// Workers per group.  Measured on MI355X: with one query head per kv head 4 to 8 are equal on long
// ranges (8 a hair ahead at 128K), 5 to 6 clearly best on short ones (32K: 33.2 against 35.9 us); the
// grouped-query kernel likes 4.
constexpr int kGroupWorkers = 8, kGroupWorkersShort = 6, kQuadGroupWorkers = 4;
constexpr int kLongRangeBlocks = 24;   // average blocks per worker from which a range counts as long
// The share of a group's cost that goes into its shared pool.
constexpr int kPoolPercent = 25;
constexpr int kPairMode = 0;
constexpr int kLayout = 0;
// Relative speed of a worker of class [self] whose SIMD mate works on class [mate] (INT2, INT4, INT8, FP16), traced
// on MI355X at equal weighted cost: two bandwidth-bound or two ALU-bound waves on a SIMD get in each other's way,
// an INT4 wave next to an FP16 wave runs well ahead.  (INT8 was not traced: neutral.)
constexpr double kPairSpeed[kNumClasses][kNumClasses] = {
    {0.87, 1.0, 1.0, 1.0}, {1.0, 1.17, 1.0, 1.27}, {1.0, 1.0, 1.0, 1.0}, {0.97, 1.06, 1.0, 0.9}};
// A group only gets a pool if its range holds at least this many blocks per worker.
constexpr int kMinBlocksPerWorkerForPool = 4;
// Groups with short ranges (below this many blocks per worker) put a larger share into the pool: there the
// differences between compute units weigh more than the cost of the tickets.
constexpr int kShortRangeBlocks = 16;
constexpr int kShortRangePoolPercent = 40;

// The split parameters.  The defaults are what was measured best on MI355X; the environment variables
// are tuning aids for experiments and are read once per cocktail_plan call.
struct Tuning {
  int64_t weight[kNumClasses] = {kCostWeight[0], kCostWeight[1], kCostWeight[2], kCostWeight[3]};   // COCKTAIL_COST_WEIGHTS="int2,int4,int8,fp16" or "int2,int4,fp16"
  bool weight_set = false;
  int pool_percent = kPoolPercent;      // COCKTAIL_POOL_PERCENT   0..100
  bool pool_percent_set = false;        // the environment fixed the share for every group
  int group_workers = 0;                // COCKTAIL_GROUP_WORKERS  1..1024; 0 = the default for the kernel that will run
  bool pair_speed = true;               // COCKTAIL_PAIR_SPEED     0 | 1
  int layout = kLayout;                 // COCKTAIL_LAYOUT         0 | 1
  int pair_mode = kPairMode;            // COCKTAIL_PAIR_MODE      0 | 2 | 3
  int min_pool_blocks = kMinBlocksPerWorkerForPool;   // COCKTAIL_MIN_POOL_BLOCKS  1..4096
  double pair_table[kNumClasses][kNumClasses];        // COCKTAIL_PAIR_TABLE="16 numbers, row = own class": replaces
  bool pair_table_set = false;                        // kPairSpeed, and switches the correction on for the matrix kernel too
};

static Tuning read_tuning() {
  Tuning t;
  if (const char* e = std::getenv("COCKTAIL_COST_WEIGHTS")) {
    long a = 0, b = 0, c = 0, d = 0;
    const int n = std::sscanf(e, "%ld,%ld,%ld,%ld", &a, &b, &c, &d);
    if (n == 4 && a > 0 && b > 0 && c > 0 && d > 0)
      t.weight[0] = a, t.weight[1] = b, t.weight[2] = c, t.weight[3] = d, t.weight_set = true;
    else if (n == 3 && a > 0 && b > 0 && c > 0)
      t.weight[0] = a, t.weight[1] = b, t.weight[3] = c, t.weight_set = true;
  }
  auto int_knob = [](const char* name, int lo, int hi, int& out) {
    if (const char* e = std::getenv(name)) {
      const int v = std::atoi(e);
      if (v >= lo && v <= hi) out = v;
    }
  };
  for (int a = 0; a < kNumClasses; ++a)
    for (int b = 0; b < kNumClasses; ++b) t.pair_table[a][b] = kPairSpeed[a][b];
  if (const char* e = std::getenv("COCKTAIL_PAIR_TABLE")) {
    double v[16];
    int n = 0;
    const char* q = e;
    while (n < 16) {
      char* end = nullptr;
      const double x = std::strtod(q, &end);
      if (end == q) break;
      v[n++] = x;
      q = end;
      while (*q == ',' || *q == ' ') ++q;
    }
    bool ok = n == 16;
    for (int i = 0; ok && i < 16; ++i) ok = v[i] > 0.25 && v[i] < 4.0;
    if (ok) {
      for (int i = 0; i < 16; ++i) t.pair_table[i / 4][i % 4] = v[i];
      t.pair_table_set = true;
    }
  }
  int ps = 1;
  int_knob("COCKTAIL_POOL_PERCENT", 0, 100, t.pool_percent);
  t.pool_percent_set = std::getenv("COCKTAIL_POOL_PERCENT") != nullptr;
  int_knob("COCKTAIL_GROUP_WORKERS", 1, 1024, t.group_workers);
  int_knob("COCKTAIL_PAIR_SPEED", 0, 1, ps);
  int_knob("COCKTAIL_LAYOUT", 0, 1, t.layout);
  int_knob("COCKTAIL_PAIR_MODE", 0, 3, t.pair_mode);
  int_knob("COCKTAIL_MIN_POOL_BLOCKS", 1, 4096, t.min_pool_blocks);
  t.pair_speed = ps != 0;
  return t;
}

static inline int64_t align16(int64_t x) { return (x + 15) & ~int64_t(15); }

}  // namespace cocktail

using namespace cocktail;

extern "C" const char* cocktail_last_error(void) { return g_err; }
extern "C" int cocktail_version(void) { return (0 << 16) | 5; }

// Reads one field of the plan header by name, so that tools and tests that look inside a plan follow the
// header's real layout instead of a copy of it.
extern "C" int cocktail_plan_field(const void* plan_host, const char* name, int32_t index, int64_t* value) {
  if (!plan_host || !name || !value) return fail(COCKTAIL_EINVAL, "plan_host, name and value must not be NULL");
  const PlanHeader* hd = static_cast<const PlanHeader*>(plan_host);
  if (hd->magic != kPlanMagic || hd->version != kPlanVersion)
    return fail(COCKTAIL_EINVAL, "plan_host is not a plan written by this library version");
#define COCKTAIL_FIELD(f)                                                                            \
  if (std::strcmp(name, #f) == 0) {                                                                  \
    if (index != 0) return fail(COCKTAIL_EINVAL, "plan field %s is not an array", name);             \
    *value = static_cast<int64_t>(hd->f);                                                            \
    return COCKTAIL_OK;                                                                              \
  }
#define COCKTAIL_ARRAY(f)                                                                            \
  if (std::strcmp(name, #f) == 0) {                                                                  \
    if (index < 0 || index >= kNumClasses) return fail(COCKTAIL_EINVAL, "index %d of plan field %s", index, name); \
    *value = static_cast<int64_t>(hd->f[index]);                                                     \
    return COCKTAIL_OK;                                                                              \
  }
  COCKTAIL_FIELD(magic) COCKTAIL_FIELD(version) COCKTAIL_FIELD(batch) COCKTAIL_FIELD(num_q_heads)
  COCKTAIL_FIELD(num_kv_heads) COCKTAIL_FIELD(head_dim) COCKTAIL_FIELD(chunk_size) COCKTAIL_FIELD(group_size)
  COCKTAIL_FIELD(rep) COCKTAIL_FIELD(work_heads) COCKTAIL_FIELD(work_rep) COCKTAIL_FIELD(num_workers) COCKTAIL_FIELD(num_segments) COCKTAIL_FIELD(num_partials)
  COCKTAIL_FIELD(total_gblocks) COCKTAIL_FIELD(v_layout) COCKTAIL_FIELD(total_chunks) COCKTAIL_FIELD(total_tokens)
  COCKTAIL_ARRAY(class_blocks) COCKTAIL_ARRAY(class_bytes) COCKTAIL_ARRAY(block_bytes) COCKTAIL_ARRAY(row_bytes)
  COCKTAIL_FIELD(workspace_bytes) COCKTAIL_FIELD(plan_bytes) COCKTAIL_FIELD(packed_bytes)
  COCKTAIL_FIELD(off_seq_len) COCKTAIL_FIELD(off_cum_tokens) COCKTAIL_FIELD(off_chunk_off) COCKTAIL_FIELD(off_perm)
  COCKTAIL_FIELD(off_class_tokens) COCKTAIL_FIELD(off_class_chunk0) COCKTAIL_FIELD(off_blk_base)
  COCKTAIL_FIELD(off_nblk) COCKTAIL_FIELD(off_run_blocks) COCKTAIL_FIELD(off_segments) COCKTAIL_FIELD(append_capacity)
  COCKTAIL_FIELD(off_worker_rec) COCKTAIL_FIELD(off_group_rec) COCKTAIL_FIELD(off_pool_seg)
  COCKTAIL_FIELD(off_counters) COCKTAIL_FIELD(num_groups) COCKTAIL_FIELD(num_pool_segs)
  COCKTAIL_FIELD(append_blocks) COCKTAIL_FIELD(append_slices) COCKTAIL_FIELD(off_bh_off) COCKTAIL_FIELD(off_rq_items)
  COCKTAIL_FIELD(ws_status_off)
#undef COCKTAIL_FIELD
#undef COCKTAIL_ARRAY
  // constants of the layout that are not stored in the header
  if (std::strcmp(name, "counter_stride_bytes") == 0) return *value = 4 * kCounterStride, COCKTAIL_OK;
  if (std::strcmp(name, "partial_header_floats") == 0) return *value = kPartialFloats, COCKTAIL_OK;
  if (std::strcmp(name, "iter_units") == 0 && index >= 0 && index < kNumClasses) return *value = kIterUnits[index], COCKTAIL_OK;
  if (std::strcmp(name, "sizeof_segment") == 0) return *value = sizeof(Segment), COCKTAIL_OK;
  if (std::strcmp(name, "sizeof_worker_rec") == 0) return *value = sizeof(WorkerRec), COCKTAIL_OK;
  if (std::strcmp(name, "sizeof_group_rec") == 0) return *value = sizeof(GroupRec), COCKTAIL_OK;
  if (std::strcmp(name, "sizeof_pool_seg") == 0) return *value = sizeof(PoolSeg), COCKTAIL_OK;
  if (std::strcmp(name, "sizeof_rq_item") == 0) return *value = sizeof(RQItem), COCKTAIL_OK;
  return fail(COCKTAIL_EINVAL, "unknown plan field %s[%d]", name, index);
}

extern "C" int cocktail_plan(const cocktail_shape* shape, const int32_t* seq_lens, const uint8_t* chunk_bits,
                             int32_t num_workers, cocktail_sizes* sizes, void* plan_host, size_t plan_capacity,
                             int32_t* class_tokens, int32_t* perm) {
  return cocktail_plan_ex(shape, seq_lens, chunk_bits, num_workers, nullptr, sizes, plan_host, plan_capacity,
                          class_tokens, perm);
}

extern "C" int cocktail_plan_ex(const cocktail_shape* shape, const int32_t* seq_lens, const uint8_t* chunk_bits,
                                int32_t num_workers, const cocktail_plan_options* options, cocktail_sizes* sizes,
                                void* plan_host, size_t plan_capacity, int32_t* class_tokens, int32_t* perm) {
  if (int rc = check_shape(shape)) return rc;
  const int32_t append_capacity = options ? options->append_capacity : 0;
  const bool reproducible = options && options->reproducible != 0;
  const bool vector_alu_only = options && options->vector_alu_only != 0;
  const int32_t* max_seq_lens = options ? options->max_seq_lens : nullptr;
  if (options) {
    if (options->reserved0 != 0) return fail(COCKTAIL_EINVAL, "cocktail_plan_options::reserved must be zero");
    for (int32_t v : options->reserved)
      if (v != 0) return fail(COCKTAIL_EINVAL, "cocktail_plan_options::reserved must be zero");
  }
  if (append_capacity < 0 || append_capacity > (1 << 24) - kTB)   // an append run stays below 4 GiB, like a context run
    return fail(COCKTAIL_EINVAL, "append_capacity %d out of range [0, 2^24 - 64]", append_capacity);
  if (!seq_lens || !sizes) return fail(COCKTAIL_EINVAL, "seq_lens and sizes must not be NULL");
  if (num_workers < 1 || num_workers > (1 << 20))
    return fail(COCKTAIL_EINVAL, "num_workers %d out of range [1, 2^20]", num_workers);
  const int B = shape->batch, Hkv = shape->num_kv_heads, D = shape->head_dim, C = shape->chunk_size,
            G = shape->group_size;
  // a wave handles 64 tokens at a time at head_dim 64 and 32 at head_dim 128 (a lane works on 64 channels):
  // the units the pool tickets count in
  const int units_per_block = D == 64 ? 1 : 2;

  int64_t total_chunks = 0, total_tokens = 0;
  for (int b = 0; b < B; ++b) {
    if (seq_lens[b] < 0) return fail(COCKTAIL_EINVAL, "seq_lens[%d] = %d is negative", b, seq_lens[b]);
    if (max_seq_lens && max_seq_lens[b] < seq_lens[b])
      return fail(COCKTAIL_EINVAL, "max_seq_lens[%d] = %d is below seq_lens[%d] = %d", b, max_seq_lens[b], b, seq_lens[b]);
    // the kernels address the blocks of one (b, h, class) run with 32-bit byte offsets and describe it by a
    // buffer resource with a 32-bit size: an all-FP16 run of T tokens has ceil(T / 64) * 64 * 2 D bytes
    const int32_t longest = max_seq_lens ? max_seq_lens[b] : seq_lens[b];   // what the sequence may grow to
    if ((int64_t(longest) + kTB - 1) / kTB * kTB * 2 * D >= (int64_t(1) << 32))
      return fail(COCKTAIL_EUNSUPPORTED, "sequence %d with %d tokens: one (sequence, kv head) run in FP16 would reach 4 GiB "
                  "(at most %lld tokens per sequence at head_dim %d)", b, longest,
                  (long long)(((int64_t(1) << 32) / (2 * D) - 1) / kTB * kTB), D);
    total_chunks += seq_lens[b] / C;
    total_tokens += seq_lens[b];
  }
  if (total_chunks > 0 && !chunk_bits) return fail(COCKTAIL_EINVAL, "chunk_bits is NULL");
  if (total_tokens >= (int64_t(1) << 31)) return fail(COCKTAIL_EINVAL, "more than 2^31 tokens in one call");
  for (int64_t i = 0; i < total_chunks; ++i) {
    const uint8_t v = chunk_bits[i];
    if (v != 2 && v != 4 && v != 8 && v != 16)
      return fail(COCKTAIL_EINVAL, "chunk_bits[%lld] = %d is not one of 2, 4, 8, 16", (long long)i, int(v));
  }

  constexpr int NC = kNumClasses;
  const int* bits_of = kClassBits;
  int32_t row_bytes[NC], block_bytes[NC], algo_row[NC];
  for (int c = 0; c < NC; ++c) {
    const int meta = (c == kFp16Class) ? 0 : 4 * (D / G);
    row_bytes[c] = D * bits_of[c] / 8;
    block_bytes[c] = kTB * (row_bytes[c] + meta);
    algo_row[c] = row_bytes[c] + meta;
  }

  // ---- Alg. 1 prefill loop: class lists in loop order, concatenated INT2 | INT4 | INT8 | FP16 ----
  // v_nblk: blocks per head that hold tokens; v_cap: blocks per head the run is laid out with (more than v_nblk
  // only for FP16 runs with room to grow, cocktail_plan_options::max_seq_lens)
  std::vector<int32_t> v_perm(total_chunks), v_chunk_off(B + 1, 0), v_ct(NC * B), v_cc0(NC * B), v_nblk(NC * B),
      v_cap(NC * B), v_blk_base(NC * (B + 1), 0);
  std::vector<int64_t> v_cum(B + 1, 0);
  int64_t class_tokens_tot[NC] = {};
  int64_t packed = 0;
  for (int b = 0; b < B; ++b) {
    const int n = seq_lens[b] / C;
    const uint8_t* bits = chunk_bits ? chunk_bits + v_chunk_off[b] : nullptr;
    int32_t* pb = v_perm.data() + v_chunk_off[b];
    int pos = 0;
    for (int c = 0; c < NC; ++c) {
      v_cc0[NC * b + c] = pos;
      for (int i = 0; i < n; ++i)
        if (bits[i] == bits_of[c]) pb[pos++] = i;
      int64_t ntok = int64_t(pos - v_cc0[NC * b + c]) * C;
      if (c == kFp16Class) ntok += seq_lens[b] - n * C;  // Sec. III-A: the remainder stays FP16
      v_ct[NC * b + c] = static_cast<int32_t>(ntok);
      v_nblk[NC * b + c] = static_cast<int32_t>((ntok + kTB - 1) / kTB);
      const int64_t room = (c == kFp16Class && max_seq_lens) ? int64_t(max_seq_lens[b]) - seq_lens[b] : 0;
      v_cap[NC * b + c] = static_cast<int32_t>((ntok + room + kTB - 1) / kTB);
      class_tokens_tot[c] += ntok;
      packed += 2 * int64_t(Hkv) * ntok * algo_row[c];
      const int64_t nb = int64_t(v_blk_base[NC * b + c]) + int64_t(Hkv) * v_cap[NC * b + c];
      if (nb >= (int64_t(1) << 31)) return fail(COCKTAIL_EINVAL, "class %d needs more than 2^31 blocks", c);
      v_blk_base[NC * (b + 1) + c] = static_cast<int32_t>(nb);
    }
    v_chunk_off[b + 1] = v_chunk_off[b] + n;
    v_cum[b + 1] = v_cum[b] + seq_lens[b];
  }

  // Relative time per byte of the three classes in the decode kernel (1/64 units).  The FP16 class is
  // a pure stream; the quantised classes also keep the vector ALU busy, so a byte of them takes longer.
  // Measured on MI355X with all three classes running side by side.
  Tuning tune = read_tuning();
  int pool_percent = tune.pool_percent;
  const int rep = shape->num_q_heads / Hkv;
  // 2 to 4 query heads per kv head are served by one wave (token-quad form of V); beyond that the query
  // heads run as two or more waves of one workgroup on the same blocks, where a pool would need a ticket
  // shared by those waves, so those shapes keep the purely static split
  // Up to eight query heads of a kv head are served by one workgroup.  Where more of them share a kv head they are
  // cut into equal sets, and with one wave per query head (the vector-ALU kernel, on request) every head is a set
  // of its own: each set walks the blocks of its kv head as if they were its own.
  const int wrep = work_rep_of(rep, vector_alu_only);   // query heads a workgroup serves
  const int Hw = shape->num_q_heads / wrep;             // heads of the decode work split
  const int share = rep / wrep;                         // work heads that walk the blocks of one kv head
  const bool quads = uses_token_quads(wrep);
  if (quads && !tune.weight_set)
    for (int c = 0; c < NC; ++c) tune.weight[c] = kQuadCostWeight[c];
  const int64_t* weight = tune.weight;
  if ((wrep > 1 && !(quads && quad_waves(wrep) == 1)) || reproducible) pool_percent = 0;

  // ---- physical runs of the class buffers: (class, b, h) order, each a contiguous run of blocks ----
  struct Run {
    int b, h, cls, nb, ntok, blk0;
  };
  std::vector<Run> runs;
  int64_t class_nblk[NC] = {};
  for (int c = 0; c < NC; ++c)
    for (int b = 0; b < B; ++b)
      for (int h = 0; h < Hw; ++h) {
        const int nb = v_nblk[NC * b + c];
        if (nb == 0) continue;
        runs.push_back({b, h, c, nb, v_ct[NC * b + c], v_blk_base[NC * b + c] + (h / share) * v_cap[NC * b + c]});
        class_nblk[c] += nb;
      }
  int64_t tot_blocks = 0;
  for (int c = 0; c < NC; ++c) tot_blocks += class_nblk[c];
  if (tot_blocks >= (int64_t(1) << 31)) return fail(COCKTAIL_EINVAL, "more than 2^31 blocks in one call");
  // `num_workers` is an upper bound: a short context has fewer units of work than the chip has wave slots, and
  // workgroups without work only lengthen the launch (8 heads x 2048 tokens on MI355X: 12.4 us per call with 2048
  // workgroups, 11.5 us with 512).  At most one worker per unit, in multiples of 64.
  const int64_t unit_workers = (tot_blocks * units_per_block + 63) / 64 * 64;
  const int P = static_cast<int>(std::min<int64_t>(num_workers, std::max<int64_t>(unit_workers, 64)));
  const int group_workers = tune.group_workers > 0 ? tune.group_workers
                            : quads                ? kQuadGroupWorkers
                            : tot_blocks >= int64_t(kLongRangeBlocks) * P ? kGroupWorkers : kGroupWorkersShort;

  // ---- global order and segments ----
  // The workers form groups of `group_workers`; group j works on one stripe [cut[c][j], cut[c][j+1]) of
  // the blocks of every class c (blocks in (b, h, block) order).  A segment is the intersection of a
  // stripe with a run; the global order lists the groups one after the other.
  //   layout 0: the class-major order INT2 | INT4 | INT8 | FP16 is cut into NGR parts of equal cost, so a
  //             group works on one class (two where it straddles a class boundary);
  //   layout 1: every group receives the same share of every class (FP16 stripe, then INT2, INT4, INT8).
  const int NGR = (P + group_workers - 1) / group_workers;
  const bool pair_speed_on = tune.pair_speed;
  const int layout = tune.layout;
  const int class_order[NC] = {layout ? 3 : 0, layout ? 0 : 1, layout ? 1 : 2, layout ? 2 : 3};
  std::vector<int64_t> cut[NC];
  {
    int64_t per[NC], tot = 0, start[NC];
    for (int c = 0; c < NC; ++c) {
      per[c] = 2 * int64_t(block_bytes[c]) * weight[c];
      start[c] = tot;
      tot += class_nblk[c] * per[c];
      cut[c].assign(NGR + 1, 0);
    }
    // Share of the total cost in front of every group.  Equal shares per worker to begin with; then,
    // if the workgroups fill the chip twice (workgroup i and i + P/2 share a SIMD), a few rounds that
    // scale every worker's share by the measured relative speed of its class next to its mate's class.
    std::vector<double> wcap(P, 1.0), gfrac(NGR + 1, 0.0);
    const bool pair_speed = pair_speed_on && !layout && P % 2 == 0 && P >= 2 * group_workers &&
                            (wrep == 1 || (tune.pair_table_set && quads && quad_waves(wrep) == 1));
    for (int round = 0; round < (pair_speed ? 4 : 1); ++round) {
      double total_cap = 0.0;
      for (int w = 0; w < P; ++w) total_cap += wcap[w];
      double acc = 0.0;
      for (int j = 0; j < NGR; ++j) {
        gfrac[j] = acc / total_cap;
        for (int w = j * group_workers; w < P && w < (j + 1) * group_workers; ++w) acc += wcap[w];
      }
      gfrac[NGR] = 1.0;
      if (!pair_speed || round == 3) break;
      std::vector<int> wclass(P);
      for (int w = 0; w < P; ++w) {
        const int j = w / group_workers, k = (j + 1) * group_workers <= P ? group_workers : P - j * group_workers;
        const double x = double(tot) * (gfrac[j] + (w - j * group_workers + 0.5) / k * (gfrac[j + 1] - gfrac[j]));
        wclass[w] = x < double(start[1]) ? 0 : x < double(start[2]) ? 1 : x < double(start[3]) ? 2 : 3;
      }
      for (int w = 0; w < P; ++w) wcap[w] = tune.pair_table[wclass[w]][wclass[(w + P / 2) % P]];
    }
    for (int j = 0; j <= NGR; ++j) {
      for (int c = 0; c < NC; ++c) {
        if (layout) {
          const int w_lo = j * group_workers < P ? j * group_workers : P;
          cut[c][j] = class_nblk[c] * w_lo / P;
        } else {
          const int64_t target = static_cast<int64_t>(double(tot) * gfrac[j]);
          int64_t v = (target - start[c] + per[c] / 2) / per[c];
          cut[c][j] = v < 0 ? 0 : (v > class_nblk[c] ? class_nblk[c] : v);
        }
      }
    }
    for (int c = 0; c < NC; ++c) cut[c][0] = 0, cut[c][NGR] = class_nblk[c];
  }
  std::vector<Segment> segs;
  std::vector<int64_t> seg_cost0;   // cumulative cost (weighted bytes of K+V) at the start of each segment
  std::vector<int32_t> group_g0(NGR + 1, 0), group_s0(NGR + 1, 0);
  int64_t gblk = 0, cost = 0;
  {
    std::vector<Run> by_class[NC];
    for (const Run& r : runs) by_class[r.cls].push_back(r);
    size_t cur_run[NC] = {};      // run holding the next block of each class
    int64_t run_first[NC] = {};   // class-local index of that run's first block
    for (int j = 0; j < NGR; ++j) {
      group_g0[j] = static_cast<int32_t>(gblk), group_s0[j] = static_cast<int32_t>(segs.size());
      for (int ci = 0; ci < NC; ++ci) {
        const int c = class_order[ci];
        int64_t lo = cut[c][j];
        const int64_t hi = cut[c][j + 1];
        while (lo < hi) {
          while (run_first[c] + by_class[c][cur_run[c]].nb <= lo) run_first[c] += by_class[c][cur_run[c]++].nb;
          const Run& r = by_class[c][cur_run[c]];
          const int off = static_cast<int>(lo - run_first[c]);
          const int n = static_cast<int>((hi < run_first[c] + r.nb ? hi : run_first[c] + r.nb) - lo);
          Segment sgm;
          sgm.b = r.b, sgm.h = r.h, sgm.cls = c, sgm.ntok = r.ntok - off * kTB;
          sgm.blk0 = r.blk0 + off, sgm.nblk = n;
          sgm.gblk0 = static_cast<int32_t>(gblk);
          sgm.pid0 = 0;
          segs.push_back(sgm);
          seg_cost0.push_back(cost);
          gblk += n;
          cost += int64_t(n) * 2 * block_bytes[c] * weight[c];
          lo += n;
        }
      }
    }
    group_g0[NGR] = static_cast<int32_t>(gblk), group_s0[NGR] = static_cast<int32_t>(segs.size());
  }
  seg_cost0.push_back(cost);
  const int S = static_cast<int>(segs.size());
  const int32_t g_end = static_cast<int32_t>(gblk);
  auto blk_cost = [&](int s) { return 2 * int64_t(block_bytes[segs[s].cls]) * weight[segs[s].cls]; };
  // cumulative cost in front of global block g, which lies in segment s (or g == end of segment s)
  auto cost_at = [&](int32_t g, int s) { return s >= S ? cost : seg_cost0[s] + int64_t(g - segs[s].gblk0) * blk_cost(s); };
  // block boundary whose cumulative cost is nearest to `target`; `s` is a monotone search cursor and
  // returns the segment that holds the boundary block (S at the very end)
  auto block_at = [&](int64_t target, int& s) -> int32_t {
    while (s < S && seg_cost0[s + 1] <= target) ++s;
    if (s >= S) return g_end;
    const int64_t per = blk_cost(s);
    int64_t j = (target - seg_cost0[s] + per / 2) / per;
    if (j < 0) j = 0;
    if (j >= segs[s].nblk) {
      j = 0;
      ++s;
      if (s >= S) return g_end;
    }
    return segs[s].gblk0 + static_cast<int32_t>(j);
  };
  auto seg_of = [&](int32_t g, int s) {   // segment holding block g, searching forward from s
    while (s < S && segs[s].gblk0 + segs[s].nblk <= g) ++s;
    return s;
  };

  // ---- groups of consecutive workers: an equal-cost range each; its tail becomes the shared pool,
  //      the rest is split into one own range per worker ----
  struct Item {
    int32_t g0, g1, seg0, pid0, group, rank;
  };
  std::vector<Item> items(P);
  std::vector<GroupRec> groups;
  std::vector<PoolSeg> psegs;
  {
    for (int w0 = 0, j = 0; w0 < P; w0 += group_workers, ++j) {
      const int w1 = w0 + group_workers < P ? w0 + group_workers : P;
      const int k = w1 - w0;
      const int32_t G0 = group_g0[j], G1 = group_g0[j + 1];
      const int sG0 = group_s0[j], sG1 = group_s0[j + 1];
      const int64_t c0 = cost_at(G0, sG0), c1 = cost_at(G1, sG1);
      GroupRec gr;
      std::memset(&gr, 0, sizeof(gr));
      gr.nworkers = k;
      gr.counter = static_cast<int32_t>(groups.size());
      gr.pseg0 = static_cast<int32_t>(psegs.size());
      int32_t Gp = G1;
      int sGp = sG1;
      if (pool_percent > 0 && int64_t(G1 - G0) >= int64_t(tune.min_pool_blocks) * k) {
        int sc = sG0;
        const int share = int64_t(G1 - G0) < int64_t(kShortRangeBlocks) * k && !tune.pool_percent_set
                              ? kShortRangePoolPercent : pool_percent;
        Gp = block_at(c1 - (c1 - c0) * share / 100, sc);
        sGp = sc;
        if (Gp < G0) Gp = G0, sGp = sG0;
        if (Gp > G1) Gp = G1, sGp = sG1;
        // a pool touches at most kMaxPoolSegments segments: move its start forward if it has to
        int first = seg_of(Gp, sGp);
        const int last = G1 > Gp ? seg_of(G1 - 1, first) : first;
        if (last - first + 1 > kMaxPoolSegments) {
          first = last - kMaxPoolSegments + 1;
          Gp = segs[first].gblk0, sGp = first;
        }
        int32_t gran = 0;
        for (int s = first; s < S && segs[s].gblk0 < G1 && Gp < G1; ++s) {
          const int32_t lo = Gp > segs[s].gblk0 ? Gp : segs[s].gblk0;
          const int32_t hi = G1 < segs[s].gblk0 + segs[s].nblk ? G1 : segs[s].gblk0 + segs[s].nblk;
          if (hi <= lo) continue;
          PoolSeg ps;
          std::memset(&ps, 0, sizeof(ps));
          ps.seg = s;
          ps.unit0 = units_per_block * (lo - segs[s].gblk0);
          ps.nunits = units_per_block * (hi - lo);
          ps.gran0 = gran;
          const int J = kIterUnits[segs[s].cls];
          gran += (ps.nunits + J - 1) / J;
          psegs.push_back(ps);
        }
        gr.ngran = gran;
        gr.nps = static_cast<int32_t>(psegs.size()) - gr.pseg0;
      }
      // own ranges: [G0, Gp) in k parts of equal cost
      const int64_t cp = cost_at(Gp, sGp);
      int sc = sG0;
      int32_t prev = G0;
      int sprev = sG0;
      for (int r = 0; r < k; ++r) {
        int32_t nb;
        int snb;
        if (r == k - 1) {
          nb = Gp, snb = sGp;
        } else {
          nb = block_at(c0 + static_cast<int64_t>((static_cast<__int128>(cp - c0) * (r + 1)) / k), sc);
          snb = sc;
          if (nb > Gp) nb = Gp, snb = sGp;
          if (nb < prev) nb = prev, snb = sprev;
        }
        items[w0 + r] = {prev, nb, seg_of(prev, sprev), 0, gr.counter, r};
        prev = nb, sprev = snb;
      }
      groups.push_back(gr);
    }
  }
  const int NG = static_cast<int>(groups.size());
  const int NPS = static_cast<int>(psegs.size());

  // partial ids.  One per (worker, segment its own range touches) and one per (pool part, rank).  The
  // ids of a (b, kv head) are contiguous, so the merge reads one dense block of the workspace.  A worker
  // enters every segment but its first one at the segment's start, i.e. as its first visitor; so the
  // id of its first piece is stored with the worker and the id of the first visitor with the segment.
  const int BH = B * Hw;
  auto bh_of = [&](const Segment& sg) { return sg.b * Hw + sg.h; };
  std::vector<int32_t> own_cnt(S, 0), bh_off(BH + 1, 0);
  for (int w = 0; w < P; ++w) {
    int sidx = items[w].seg0;
    for (int32_t g = items[w].g0; g < items[w].g1; ++sidx) {
      ++own_cnt[sidx];
      const int32_t end = segs[sidx].gblk0 + segs[sidx].nblk;
      g = end < items[w].g1 ? end : items[w].g1;
    }
  }
  for (int sidx = 0; sidx < S; ++sidx) bh_off[bh_of(segs[sidx]) + 1] += own_cnt[sidx];
  // A pool part needs a partial slot for every rank that can enter its segment from another one.  Own
  // ranges and pool parts both ascend, so these are the leading ranks: those whose own range is empty or
  // ends in an earlier segment.
  for (int g = 0, w0 = 0; g < NG; w0 += groups[g].nworkers, ++g)
    for (int i = 0; i < groups[g].nps; ++i) {
      PoolSeg& ps = psegs[groups[g].pseg0 + i];
      int n = 0;
      for (int r = 0; r < groups[g].nworkers; ++r) {
        const Item& it = items[w0 + r];
        const bool ends_here = it.g0 < it.g1 && seg_of(it.g1 - 1, it.seg0) == ps.seg;
        if (!ends_here) n = r + 1;
      }
      ps.nslots = n;
      bh_off[bh_of(segs[ps.seg]) + 1] += n;
    }
  // the appended tokens: one more partial per slice of the append buffer of a (b, kv head), at the end of its range
  const int append_blocks = (append_capacity + kTB - 1) / kTB;
  const int append_slices = (append_blocks + kAppendSliceBlocks - 1) / kAppendSliceBlocks;
  for (int i = 0; i < BH; ++i) bh_off[i + 1] += append_slices;
  for (int i = 0; i < BH; ++i) bh_off[i + 1] += bh_off[i];
  const int32_t npart = bh_off[BH];
  {
    std::vector<int32_t> cursor(bh_off.begin(), bh_off.end() - 1);
    for (int sidx = 0; sidx < S; ++sidx) {
      segs[sidx].pid0 = cursor[bh_of(segs[sidx])];
      cursor[bh_of(segs[sidx])] += own_cnt[sidx];
    }
    for (int g = 0; g < NG; ++g)
      for (int i = 0; i < groups[g].nps; ++i) {
        PoolSeg& ps = psegs[groups[g].pseg0 + i];
        ps.slot0 = cursor[bh_of(segs[ps.seg])];
        cursor[bh_of(segs[ps.seg])] += ps.nslots;
      }
    std::vector<int32_t> visitors(S, 0);
    for (int w = 0; w < P; ++w) {
      int sidx = items[w].seg0;
      items[w].pid0 = items[w].g0 < items[w].g1 ? segs[sidx].pid0 + visitors[sidx] : 0;
      for (int32_t g = items[w].g0; g < items[w].g1; ++sidx) {
        ++visitors[sidx];
        const int32_t end = segs[sidx].gblk0 + segs[sidx].nblk;
        g = end < items[w].g1 ? end : items[w].g1;
      }
    }
  }

  // ---- reorder+quantize records: one per block of the class buffers ----
  // (blocks of an FP16 run that are only room to grow get a record without valid rows: they are written as zeros)
  std::vector<RQItem> rq_items;
  rq_items.reserve(v_blk_base[NC * B + 0] + v_blk_base[NC * B + 1] + v_blk_base[NC * B + 2] + v_blk_base[NC * B + 3]);
  for (int c = 0; c < NC; ++c)
    for (int b = 0; b < B; ++b) {
      const int nb = v_cap[NC * b + c], ntok = v_ct[NC * b + c];
      if (nb == 0) continue;
      const int n = seq_lens[b] / C;
      const int32_t* pb = v_perm.data() + v_chunk_off[b];
      const int cc0 = v_cc0[NC * b + c];
      const int tail = seq_lens[b] - n * C;
      const int chunk_tokens = c == kFp16Class ? ntok - tail : ntok;
      auto src_token = [&](int r) {   // source token of row r of the class (Alg. 1 order; tail after the FP16 chunks)
        if (r < chunk_tokens) return pb[cc0 + r / C] * C + r % C;
        return n * C + (r - chunk_tokens);
      };
      std::vector<RQItem> head_items(nb);
      for (int j = 0; j < nb; ++j) {
        RQItem& it = head_items[j];
        std::memset(&it, 0, sizeof(it));
        const int r0 = j * kTB;
        const int nvalid = ntok - r0 < kTB ? (ntok > r0 ? ntok - r0 : 0) : kTB;
        it.b = b, it.j = j;
        it.cls_nvalid = c | (nvalid << 8);
        if (nvalid == 0) continue;   // room to grow: t0 = 0, nothing is read
        const int t0 = src_token(r0);
        // rows are consecutive tokens iff the last one is (chunks keep their order, so tokens in between are too)
        it.t0 = src_token(r0 + nvalid - 1) == t0 + nvalid - 1 ? t0 : -1;
      }
      for (int h = 0; h < Hkv; ++h)
        for (int j = 0; j < nb; ++j) {
          RQItem it = head_items[j];
          it.h = h;
          it.ragged_row = (v_cum[b] * Hkv + int64_t(h) * seq_lens[b]) + (it.t0 >= 0 ? it.t0 : 0);
          rq_items.push_back(it);
        }
    }

  // ---- sizes and blob layout ----
  PlanHeader hd;
  std::memset(&hd, 0, sizeof(hd));
  hd.magic = kPlanMagic, hd.version = kPlanVersion;
  hd.batch = B, hd.num_q_heads = shape->num_q_heads, hd.num_kv_heads = Hkv, hd.head_dim = D;
  hd.chunk_size = C, hd.group_size = G, hd.rep = rep, hd.work_heads = Hw, hd.work_rep = wrep;
  hd.num_workers = P, hd.num_segments = S, hd.num_partials = npart;
  hd.num_groups = NG, hd.num_pool_segs = NPS;
  hd.append_capacity = append_capacity, hd.append_blocks = append_blocks, hd.append_slices = append_slices;
  hd.total_gblocks = static_cast<int32_t>(gblk);
  hd.v_layout = quads ? 1 : 0;
  hd.total_chunks = total_chunks, hd.total_tokens = total_tokens, hd.packed_bytes = packed;
  for (int c = 0; c < NC; ++c) {
    hd.class_blocks[c] = v_blk_base[NC * B + c];
    hd.class_bytes[c] = hd.class_blocks[c] * block_bytes[c];
    hd.block_bytes[c] = block_bytes[c];
    hd.row_bytes[c] = row_bytes[c];
  }
  // decode workspace: the partial states, then one status word per (sequence, query head)
  hd.ws_status_off = align16(int64_t(npart > 0 ? npart : 1) * wrep * (D + kPartialFloats) * int64_t(sizeof(float)));
  hd.workspace_bytes = hd.ws_status_off + align16(int64_t(sizeof(int32_t)) * B * shape->num_q_heads);
  int64_t off = align16(sizeof(PlanHeader));
  bool too_large = false;
  auto place = [&](int32_t& field, int64_t bytes) {
    if (off + bytes >= (int64_t(1) << 31)) too_large = true;   // the offsets are 32-bit fields
    field = static_cast<int32_t>(too_large ? 0 : off);
    off = align16(off + bytes);
  };
  place(hd.off_seq_len, 4 * int64_t(B));
  place(hd.off_cum_tokens, 8 * int64_t(B + 1));
  place(hd.off_chunk_off, 4 * int64_t(B + 1));
  place(hd.off_perm, 4 * total_chunks);
  place(hd.off_class_tokens, 4 * NC * int64_t(B));
  place(hd.off_class_chunk0, 4 * NC * int64_t(B));
  place(hd.off_blk_base, 4 * NC * int64_t(B + 1));
  place(hd.off_nblk, 4 * NC * int64_t(B));
  place(hd.off_run_blocks, 4 * NC * int64_t(B));
  place(hd.off_segments, int64_t(sizeof(Segment)) * S);
  place(hd.off_bh_off, 4 * int64_t(BH + 1));
  place(hd.off_worker_rec, int64_t(sizeof(WorkerRec)) * P);
  place(hd.off_group_rec, int64_t(sizeof(GroupRec)) * NG);
  place(hd.off_pool_seg, int64_t(sizeof(PoolSeg)) * NPS);
  place(hd.off_rq_items, int64_t(sizeof(RQItem)) * int64_t(rq_items.size()));
  off = (off + 127) & ~int64_t(127);
  place(hd.off_counters, int64_t(4 * kCounterStride) * NG);
  if (too_large || off >= (int64_t(1) << 31)) return fail(COCKTAIL_EUNSUPPORTED, "plan larger than 2 GiB");
  hd.plan_bytes = off;

  std::memset(sizes, 0, sizeof(*sizes));
  sizes->total_chunks = total_chunks;
  for (int c = 0; c < NC; ++c) {
    sizes->class_tokens[c] = class_tokens_tot[c];
    sizes->class_blocks[c] = hd.class_blocks[c];
    sizes->class_bytes[c] = hd.class_bytes[c];
  }
  sizes->plan_bytes = hd.plan_bytes;
  sizes->workspace_bytes = hd.workspace_bytes;
  sizes->packed_bytes = packed;
  sizes->num_workers = P, sizes->num_partials = npart, sizes->num_segments = S;
  sizes->append_capacity = append_capacity;
  sizes->v_layout = hd.v_layout, sizes->reserved = 0;
  sizes->append_bytes = int64_t(B) * Hkv * hd.append_blocks * kTB * 2 * D;

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
    put(hd.off_class_tokens, v_ct.data(), 4 * NC * size_t(B));
    put(hd.off_class_chunk0, v_cc0.data(), 4 * NC * size_t(B));
    put(hd.off_blk_base, v_blk_base.data(), 4 * NC * size_t(B + 1));
    put(hd.off_nblk, v_nblk.data(), 4 * NC * size_t(B));
    put(hd.off_run_blocks, v_cap.data(), 4 * NC * size_t(B));
    put(hd.off_segments, segs.data(), sizeof(Segment) * size_t(S));
    put(hd.off_bh_off, bh_off.data(), 4 * bh_off.size());
    std::vector<WorkerRec> recs(P);
    std::memset(recs.data(), 0, sizeof(WorkerRec) * recs.size());
    // Which workgroup id runs which range.  Workgroup ids are handed to the compute units in order
    // (round-robin over the XCDs), and when P fills the chip twice, workgroup i shares a SIMD with
    // workgroup i + P/2, which was dispatched later and loses every issue arbitration against it.
    //   mode 0 (default): range w runs as workgroup w.  With the class-major layout the INT2 ranges
    //           get INT4 / FP16 ranges as SIMD mates, the mix that keeps both the vector ALU and the
    //           memory pipeline busy.
    //   mode 2: rank r of group j becomes workgroup (r odd ? P/2 : 0) + j*k/2 + (r/2 + j) mod (k/2):
    //           SIMD mates are neighbouring ranks of one group.  Mode 3: mates are ranks r and r + k/2.
    const int pair_mode = tune.pair_mode;
    const bool spread = pair_mode >= 2 && group_workers % 2 == 0 && P % group_workers == 0;
    for (int w = 0; w < P; ++w) {
      int id = w;
      if (spread) {
        const int hk = group_workers / 2, j = items[w].group, r = items[w].rank;
        id = pair_mode == 2 ? (r & 1) * (P / 2) + j * hk + ((r >> 1) + j) % hk
                            : (r / hk) * (P / 2) + j * hk + (r % hk + j) % hk;
      }
      WorkerRec& rc = recs[id];
      rc.g0 = items[w].g0, rc.g1 = items[w].g1;
      rc.seg0 = items[w].seg0, rc.pid0 = items[w].pid0;
      rc.group = items[w].group;
      rc.rank_nps = items[w].rank | (groups[items[w].group].nps << 16);
      rc.ngran = groups[items[w].group].ngran, rc.pseg0 = groups[items[w].group].pseg0;
      if (items[w].g0 < items[w].g1) rc.first = segs[items[w].seg0];
    }
    put(hd.off_worker_rec, recs.data(), sizeof(WorkerRec) * recs.size());
    put(hd.off_group_rec, groups.data(), sizeof(GroupRec) * groups.size());
    put(hd.off_pool_seg, psegs.data(), sizeof(PoolSeg) * psegs.size());
    put(hd.off_rq_items, rq_items.data(), sizeof(RQItem) * rq_items.size());
  }
  g_err[0] = 0;
  return COCKTAIL_OK;
}
