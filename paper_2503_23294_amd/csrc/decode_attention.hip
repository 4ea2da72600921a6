// Decode side of Alg. 1 (Sec. III-C): single-query attention over the INT2, INT4,
// INT8 and FP16 classes of the packed cache.
//
// Design (gfx950, wave64):
//  * The host planner puts all 64-token blocks of a layer into one global order and cuts it into
//    groups of a few workers.  A worker (workgroup) streams its own block range and then takes
//    pieces of the group's shared pool through an atomic ticket counter, so that the workers of a
//    group finish together; it emits one partial softmax state per (sequence, kv head) segment it
//    touches.
//  * Inside a wave a token is owned by a PAIR of lanes: lane l works on token
//    l % 32 of a 32-token unit and on channels [64*(l/32), 64*(l/32)+64).  The block
//    layout stores the j-th 16-byte piece of all 64 tokens contiguously, so each
//    half-wave reads one contiguous 512-byte run per load instruction, and the q.k
//    dot product needs a single cross-lane add per token.  A lane keeps 64 output
//    accumulators and its half of the query in registers; the kernel stays below
//    256 VGPRs so that two waves share every SIMD and one wave's loads hide behind
//    the other's arithmetic.
//  * Codes are expanded without any conversion: a code field masked out of a
//    half-word IS an fp16 subnormal of value code * 2^(pos-24), which v_dot2_f32_f16
//    and v_fma_mix_f32 consume exactly; the power of two is folded into per-group
//    factors.  Dequantisation is folded too:
//      q.k^      = sum_g scale_g * (q.code)_g + zero_g * sum(q_g)
//      sum p v^  = sum_t (p_t scale_tg) code_t + sum_t p_t zero_tg
//  * Loads go through buffer resources (one VGPR of address per lane) and are
//    software pipelined by hand: J register stages of K units and J of V units are
//    refilled one loop iteration ahead of the arithmetic, with the units of whatever
//    piece comes next (same segment, next segment, or a pool piece).
//  * Softmax is online per lane pair: logits of J units, one lazy rescale when the
//    reference maximum grows by more than 2^8, then the V pass.  (m, l, o[D])
//    partials go to the workspace and a second small kernel merges them exactly
//    (the softmax-weighted sum does not depend on how tokens are grouped, Eq. 4-5).
//  * This kernel serves shapes with one query head per kv head; grouped-query shapes run on the
//    kernel of decode_quads.hip, which shares the pieces, pools and register stages with this one.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdlib>
#include <mutex>
#include <vector>

#include "decode_common.h"

namespace cocktail {

// One lazy-rescale step of a lane's online softmax followed by p_j = 2^(s_j - m).
template <int NGH, int J>
__device__ __forceinline__ void softmax_step(const float (&s)[J], float (&p)[J], LaneState<NGH>& st) {
  float smax = s[0];
#pragma unroll
  for (int jj = 1; jj < J; ++jj) smax = fmaxf(smax, s[jj]);
  // the reference maximum only moves when it is exceeded by more than 2^8, and then for the whole
  // wave at once (to the largest logit any lane has seen): the lanes share one reference, so the
  // number of rescales per state is that of one running maximum, not of 64 independent ones
  const bool grow = smax > st.m + kRescaleThreshold;
  if (__builtin_expect(__builtin_amdgcn_ballot_w64(grow) != 0, 0)) {
    float mnew = fmaxf(smax, st.m);
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) mnew = fmaxf(mnew, __shfl_xor(mnew, o));
    const float alpha = __builtin_amdgcn_exp2f(st.m - mnew);
    st.m = mnew;
    st.l *= alpha;
#pragma unroll
    for (int d = 0; d < DH; ++d) st.acc[d] *= alpha;
#pragma unroll
    for (int g = 0; g < NGH; ++g) st.zacc[g] *= alpha;
  }
#pragma unroll
  for (int jj = 0; jj < J; ++jj) {
    p[jj] = __builtin_amdgcn_exp2f(s[jj] - st.m);
    st.l += p[jj];
  }
}

// Writes this wave's partial state `pid`: (m, l, o[D]) reduced over its lanes, and the number of tokens it covers.
template <int NGH, int GL>
__device__ __forceinline__ void flush_partial(const LaneState<NGH>& st, float* red, int pid, int r, int lane, int tokens) {
  kparams_t prm = kparams();
  const int rep = prm->rep;
  float mw = st.m;
#pragma unroll
  for (int o = 16; o > 0; o >>= 1) mw = fmaxf(mw, __shfl_xor(mw, o));
  const float f = __builtin_amdgcn_exp2f(st.m - mw);
  float lw = st.l * f;
#pragma unroll
  for (int o = 16; o > 0; o >>= 1) lw += __shfl_xor(lw, o);
  float* out = prm->ws + (int64_t(pid) * rep + r) * (D + kPartialFloats);
  if (lane == 0) {
    out[0] = mw;
    out[1] = lw;
    out[2] = __int_as_float(tokens);
  }
  float(*tile)[17] = reinterpret_cast<float(*)[17]>(red + r * 64 * 17);
#pragma unroll
  for (int ch = 0; ch < DH / 16; ++ch) {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int c = 0; c < 16; ++c) {
      const int d = ch * 16 + c;
      tile[lane][c] = (st.acc[d] + st.zacc[d / GL]) * f;
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    // lane (c, quarter) adds 16 rows; quarters 0,1 hold channel half 0 and quarters 2,3 half 1
    const int c = lane & 15, quarter = lane >> 4;
    float sum = 0.f;
#pragma unroll
    for (int row = 0; row < 16; ++row) sum += tile[quarter * 16 + row][c];
    sum += __shfl_xor(sum, 16);
    if ((quarter & 1) == 0) out[kPartialFloats + (quarter >> 1) * DH + ch * 16 + c] = sum;
  }
}

// Zeroes the partial state and loads this lane's half of the query row `qrow`.
template <int NGH, int GL>
__device__ __forceinline__ void begin_state(int qrow, int h, LaneState<NGH>& st, uint32_t (&q)[DH / 2],
                                            float (&qsum)[NGH]) {
#pragma unroll
  for (int i = 0; i < DH; ++i) st.acc[i] = 0.f;
#pragma unroll
  for (int gq = 0; gq < NGH; ++gq) st.zacc[gq] = 0.f;
  st.m = kNegBig;
  st.l = 0.f;
  const u32x4* qp = reinterpret_cast<const u32x4*>(kparams()->q + int64_t(qrow) * (D / 2) + h * (DH / 2));
#pragma unroll
  for (int i = 0; i < DH / 8; ++i) {
    const u32x4 v = qp[i];
    q[4 * i] = v.x, q[4 * i + 1] = v.y, q[4 * i + 2] = v.z, q[4 * i + 3] = v.w;
  }
#pragma unroll
  for (int gq = 0; gq < NGH; ++gq) {
    float a = 0.f;
#pragma unroll
    for (int i = 0; i < GL / 2; ++i) a = dot2(q[gq * (GL / 2) + i], 0x3C003C00u, a);   // (1.0, 1.0)
    qsum[gq] = a;
  }
}

// Consumes the stream while its pieces belong to class CID, starting with `cur` (whose loads have
// not been issued yet); returns with `cur` = the first piece of another class, or the end piece.
//
// J register stages hold the K units and J the V units of the piece being worked on; each stage is
// refilled with the corresponding unit of the NEXT piece as soon as it has been consumed, so the
// loads of a piece are in flight during the arithmetic of the piece before it, across segment and
// pool boundaries alike.  A piece with fewer than J units leaves stages unused, and after the last
// piece of the class nothing is left to fetch: those refills address the first unit past the segment,
// which the buffer resource answers with zeros without touching memory, so the loop body has no
// branches around the loads (the zeros are masked like padding).  The accumulators live and die inside this function, one
// instance per class.
template <class CLS, int CID, int G, int AUX>
__device__ __forceinline__ void run_class(Stream& sm, Piece& cur, float* red, int r, int lane, bool app = false) {
  constexpr int NG = D / G;
  constexpr int NGH = NG >= 2 ? NG / 2 : 1;
  constexpr int GL = G < DH ? G : DH;
  constexpr int J = CLS::J;
  static_assert(J == kIterUnits[CID], "the planner cuts pool pieces to the kernel's iteration size");
  const int t = lane & 31, h = lane >> 5;
  const uint32_t vc = CLS::code_voff(t, h), vm = CLS::meta_voff(t, h);
  const char* const kbase = uni(app ? kparams()->k_app : kparams()->k[CID]);   // app: the append buffers
  const char* const vbase = uni(app ? kparams()->v_app : kparams()->v[CID]);
  const float scale_log2 = kparams()->scale_log2;
  LaneState<NGH> st;
  uint32_t q[DH / 2];
  float qsum[NGH];
  typename CLS::Stage ks[J], vs[J];
  int pid = cur.pid;
  // `cur` is the piece the stream produced last, so the stream's segment fields describe it
  rsrc_t krs = make_rsrc(kbase + int64_t(sm.blk0) * CLS::BLOCKB, uint32_t(sm.nblk) * CLS::BLOCKB);
  rsrc_t vrs = make_rsrc(vbase + int64_t(sm.blk0) * CLS::BLOCKB, uint32_t(sm.nblk) * CLS::BLOCKB);
  int ru = cur.us, rn = cur.nu;   // the piece the stages are (re)filled with
  int roob = 2 * sm.nblk;         // first unit past its segment: a load from there is out of range and costs nothing
#pragma unroll
  for (int jj = 0; jj < J; ++jj) CLS::template load<AUX>(ks[jj], krs, jj < rn ? ru + jj : roob, vc, vm);
#pragma unroll
  for (int jj = 0; jj < J; ++jj) CLS::template load<AUX>(vs[jj], vrs, jj < rn ? ru + jj : roob, vc, vm);
  sched_fence();
  begin_state<NGH, GL>(sm.qrow + r, h, st, q, qsum);   // the query arrives while the first units are on their way
  int valid = cur.valid;
  int covered = 0;   // tokens the current partial state covers (the merge checks the total per sequence)
  Piece nxt = sm.next(lane);
#pragma unroll 1
  while (true) {
    const bool more = nxt.nu > 0 && nxt.cls == CID;
    if (more) {
      krs = make_rsrc(kbase + int64_t(sm.blk0) * CLS::BLOCKB, uint32_t(sm.nblk) * CLS::BLOCKB);
      vrs = make_rsrc(vbase + int64_t(sm.blk0) * CLS::BLOCKB, uint32_t(sm.nblk) * CLS::BLOCKB);
      ru = nxt.us, rn = nxt.nu, roob = 2 * sm.nblk;
    } else {
      rn = 0;   // nothing follows in this class: every refill goes out of range
    }
    covered += valid;
    float s[J], p[J];
#pragma unroll
    for (int jj = 0; jj < J; ++jj) {
      s[jj] = CLS::half_logit(ks[jj], q, qsum);
      sched_fence();
      CLS::template load<AUX>(ks[jj], krs, jj < rn ? ru + jj : roob, vc, vm);
      sched_fence();
    }
#pragma unroll
    for (int jj = 0; jj < J; ++jj) {
      const float full = (s[jj] + __shfl_xor(s[jj], 32)) * scale_log2;   // both halves of the token
      s[jj] = (jj * UT + t < valid) ? full : -INFINITY;
    }
    softmax_step<NGH, J>(s, p, st);
#pragma unroll
    for (int jj = 0; jj < J; ++jj) {
      CLS::accumulate(vs[jj], p[jj], st);
      sched_fence();
      CLS::template load<AUX>(vs[jj], vrs, jj < rn ? ru + jj : roob, vc, vm);
      sched_fence();
    }
    if (!more || nxt.fresh) flush_partial<NGH, GL>(st, red, pid, r, lane, covered);
    if (!more) break;
    if (nxt.fresh) {
      pid = nxt.pid;
      covered = 0;
      begin_state<NGH, GL>(sm.qrow + r, h, st, q, qsum);
    }
    valid = nxt.valid;
    nxt = sm.next(lane);
  }
  cur = nxt;
}

// Workgroups behind the regular workers: workgroup num_workers + bh attends to the tokens appended to
// (sequence, kv head) bh during decoding (Sec. III-A), an FP16 run of num_appended tokens in the
// append buffers, and writes the last partial of bh's range.
template <int G, int AUX>
__device__ __forceinline__ void appended_tokens(int bh, float* red, int r, int lane) {
  kparams_t kp = kparams();
  const int n = kp->num_appended;
  const int pid = uni(kp->bh_off[bh + 1]) - 1;
  if (n <= 0) {
    write_neutral(pid, r, lane);
    return;
  }
  Stream sm;
  sm.init_run(kFp16Class, n, bh * kp->app_blocks, kp->app_blocks,
              (bh / kp->num_kv_heads) * kp->num_q_heads + (bh % kp->num_kv_heads) * kp->rep, pid);
  Piece cur = sm.next(lane);
  if (cur.nu > 0) run_class<HalfClass<G>, kFp16Class, G, AUX>(sm, cur, red, r, lane, true);
}

// One single-wave workgroup per worker (Hq = Hkv: the query head of a kv head is that head).  INT8: the cache
// has an INT8 class; caches without one run a kernel without that code (a third less of it to fetch and
// to allocate registers for, worth 1.5 us on a 32K-token layer).
template <int G, int AUX, bool INT8>
__global__ __launch_bounds__(64) __attribute__((amdgpu_waves_per_eu(2))) void decode_attention_kernel(DecodeParams) {
  __shared__ float red[64 * 17];   // reduction tile of a flush
  const int lane = threadIdx.x;
  constexpr int r = 0;             // query head inside the kv head's group
#ifdef COCKTAIL_TRACE
  const uint64_t t_start = __builtin_amdgcn_s_memrealtime();
#endif
  if (int(blockIdx.x) >= kparams()->num_workers) {
    appended_tokens<G, AUX>(int(blockIdx.x) - kparams()->num_workers, red, r, lane);
    return;
  }
  Stream sm;
  sm.init(load_record(kparams()->recs + blockIdx.x));
  Piece cur = sm.next(lane);
  while (cur.nu > 0) {
    if (cur.cls == 0) {
      run_class<QuantClass<2, G>, 0, G, AUX>(sm, cur, red, r, lane);
    } else if (cur.cls == 1) {
      run_class<QuantClass<4, G>, 1, G, AUX>(sm, cur, red, r, lane);
    } else if (INT8 && cur.cls == 2) {
      if constexpr (INT8) run_class<QuantClass<8, G>, 2, G, AUX>(sm, cur, red, r, lane);
    } else {
      run_class<HalfClass<G>, kFp16Class, G, AUX>(sm, cur, red, r, lane);
    }
  }
  // pool parts this worker never entered still own a partial slot: fill it with the neutral state
  for (int i = 0; i < sm.nps; ++i) {
    if ((sm.used >> i) & 1u) continue;
    const PoolSeg ps = load_record(kparams()->psegs + sm.pseg0 + i);
    if (sm.rank < ps.nslots) write_neutral(ps.slot0 + sm.rank, r, lane);
  }
#ifdef COCKTAIL_TRACE
  if (threadIdx.x == 0) {
    uint64_t* tr = kparams()->trace + blockIdx.x * 4;
    tr[0] = t_start;
    tr[1] = __builtin_amdgcn_s_memrealtime();
    tr[2] = __builtin_amdgcn_s_getreg((4) | (0 << 6) | (31 << 11));    // HW_ID
    tr[3] = __builtin_amdgcn_s_getreg((20) | (0 << 6) | (31 << 11));   // XCC_ID
  }
#endif
}

// Exact merge of the partial states of one (sequence, query head):
//   M = max m_i,  L = sum l_i 2^(m_i - M),  out = sum o_i 2^(m_i - M) / L,  lse = ln2 (M + log2 L).
// The partials of a (sequence, kv head) are a dense block of the workspace.  512 threads: 32 channel
// quads x 16 slices of the block; a slice loads eight partials at a time (128 in flight per workgroup,
// usually the whole block in one round) and folds them with a running maximum, then the sixteen
// slice states are folded through shared memory.  A (sequence, query head) without any partial
// (empty sequence) gets zeros and lse = -inf.
// Every partial also says how many tokens it covers.  Their sum has to be the token count of the
// sequence: the softmax over the concatenation of Alg. 1 attends to every token exactly once.  If it is
// not (ticket counters that were not zero when the call started, calls overlapping on one cache, a
// damaged plan), the row is not a result: out and lse are set to NaN and the difference goes to the
// status array.
constexpr int kMergeSlices = 16;
__global__ __launch_bounds__(32 * kMergeSlices) void decode_merge_kernel(DecodeParams prm) {
  __shared__ float sm_m[kMergeSlices];
  __shared__ float sm_l[kMergeSlices];
  __shared__ int sm_c[kMergeSlices];
  __shared__ float sm_o[kMergeSlices][D];
  const int bhq = blockIdx.x;
  const int rep = prm.rep;
  const int b = bhq / prm.num_q_heads;
  const int hq = bhq - b * prm.num_q_heads;
  const int bh = b * prm.num_kv_heads + hq / rep;
  const int r = hq % rep;
  const int lo = prm.bh_off[bh];
  const int n = prm.bh_off[bh + 1] - lo;
  const int expected = prm.seq_len[b] + prm.num_appended;
  const int tid = threadIdx.x;
  // every worker has drawn its last ticket: put the counters back to zero for the next call
  if (blockIdx.x == 0)
    for (int i = tid; i < prm.num_groups; i += 32 * kMergeSlices) prm.counters[i * kCounterStride] = 0u;
  constexpr int STRIDE = D + kPartialFloats;
  constexpr int U = 8;   // partials in flight per thread
  const int quad = tid & 31, slice = tid >> 5;
  const float* base = prm.ws + (int64_t(lo) * rep + r) * STRIDE;
  float m = -INFINITY, l = 0.f, o0 = 0.f, o1 = 0.f, o2 = 0.f, o3 = 0.f;
  int covered = 0;
  for (int i0 = slice; i0 < n; i0 += kMergeSlices * U) {
    float4 hd[U], va[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int i = i0 + kMergeSlices * u;
      const bool ok = i < n;
      const float* part = base + int64_t(ok ? i : i0) * rep * STRIDE;
      hd[u] = *reinterpret_cast<const float4*>(part);                             // m, l, tokens, unused
      va[u] = *reinterpret_cast<const float4*>(part + kPartialFloats + quad * 4);
      if (!ok) hd[u].x = -INFINITY, hd[u].z = 0.f;
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const float mn = fmaxf(m, hd[u].x);
      // 2^(-inf - -inf) must not occur: a slice that has only seen padding keeps weight 0
      const float a = (m == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(m - mn);
      const float w = (hd[u].x == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(hd[u].x - mn);
      l = l * a + hd[u].y * w;
      o0 = o0 * a + va[u].x * w, o1 = o1 * a + va[u].y * w;
      o2 = o2 * a + va[u].z * w, o3 = o3 * a + va[u].w * w;
      m = mn;
      covered += __float_as_int(hd[u].z);
    }
  }
  sm_o[slice][quad * 4 + 0] = o0, sm_o[slice][quad * 4 + 1] = o1;
  sm_o[slice][quad * 4 + 2] = o2, sm_o[slice][quad * 4 + 3] = o3;
  if (quad == 0) sm_m[slice] = m, sm_l[slice] = l, sm_c[slice] = covered;
  __syncthreads();
  if (tid < D) {
    float mx = sm_m[0];
    int total = sm_c[0];
#pragma unroll
    for (int sidx = 1; sidx < kMergeSlices; ++sidx) mx = fmaxf(mx, sm_m[sidx]), total += sm_c[sidx];
    float big_l = 0.f, o = 0.f;
#pragma unroll
    for (int sidx = 0; sidx < kMergeSlices; ++sidx) {
      const float w = (sm_m[sidx] == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(sm_m[sidx] - mx);
      big_l += sm_l[sidx] * w;
      o += sm_o[sidx][tid] * w;
    }
    const bool empty = !(big_l > 0.f);
    const bool sound = total == expected;
    const float res = empty ? 0.f : o / big_l;
    prm.out[int64_t(bhq) * D + tid] = static_cast<_Float16>(sound ? res : __builtin_nanf(""));
    if (tid == 0) {
      prm.status[bhq] = total - expected;
      if (prm.lse) prm.lse[bhq] = !sound ? __builtin_nanf("") : empty ? -INFINITY : (mx + log2f(big_l)) * 0.6931471805599453f;
    }
  }
}

}  // namespace cocktail

using namespace cocktail;

extern "C" int cocktail_default_workers(const cocktail_shape* shape, int32_t* num_workers) {
  if (int rc = check_shape(shape)) return rc;
  if (!num_workers) return fail(COCKTAIL_EINVAL, "num_workers is NULL");
  int dev = 0;
  hipDeviceProp_t prop;
  if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess) {
    (void)hipGetLastError();
    return fail(COCKTAIL_EHIP, "no HIP device available");
  }
  const int rep = shape->num_q_heads / shape->num_kv_heads;
  const int waves_per_cu = 8;   // two waves per SIMD at <= 256 VGPRs
  int per_cu = waves_per_cu / (uses_token_quads(rep) ? quad_waves(rep) : rep);   // waves per workgroup
  if (per_cu < 1) per_cu = 1;
  *num_workers = prop.multiProcessorCount * per_cu;
  return COCKTAIL_OK;
}

// Scratch of the entry point that allocates nothing: the partial softmax states and the status words of one
// decode call.  In host code this name is only a handle; the device address comes from hipGetSymbolAddress.
constexpr size_t kStaticWorkspaceBytes = size_t(COCKTAIL_STATIC_WORKSPACE_BYTES);
static __device__ __align__(256) unsigned char scratch[kStaticWorkspaceBytes];

namespace {

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};   // per device: address of `scratch` there

// Address of the static workspace on the current device (looked up once per device).
int static_workspace(void** ptr) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) {
    (void)hipGetLastError();
    return fail(COCKTAIL_EHIP, "no current HIP device (or its index is not below %d)", kMaxDevices);
  }
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !p) {
      (void)hipGetLastError();
      return fail(COCKTAIL_EHIP, "hipGetSymbolAddress(static workspace) failed on device %d: %s", dev, hipGetErrorString(e));
    }
    g_scratch_ptr[dev] = p;
  }
  *ptr = g_scratch_ptr[dev];
  return COCKTAIL_OK;
}

int check_plan_matches(const cocktail_shape* shape, const cocktail_cache* cache, const PlanHeader** out) {
  if (int rc = check_shape(shape)) return rc;
  if (!cache || !cache->plan_host || !cache->plan_dev) return fail(COCKTAIL_EINVAL, "cache or its plan is NULL");
  const PlanHeader* hd = static_cast<const PlanHeader*>(cache->plan_host);
  if (hd->magic != kPlanMagic || hd->version != kPlanVersion)
    return fail(COCKTAIL_EINVAL, "plan_host is not a plan written by this library version");
  if (hd->batch != shape->batch || hd->num_kv_heads != shape->num_kv_heads || hd->head_dim != shape->head_dim ||
      hd->chunk_size != shape->chunk_size || hd->group_size != shape->group_size ||
      hd->num_q_heads != shape->num_q_heads)
    return fail(COCKTAIL_EINVAL, "plan was made for a different shape");
  *out = hd;
  return COCKTAIL_OK;
}

// Validates the arguments and enqueues the two kernels; `workspace` holds at least hd->workspace_bytes.
int decode_enqueue(const cocktail_shape* shape, const PlanHeader* hd, const void* q, const cocktail_cache* cache,
                   float sm_scale, void* out, float* lse, void* workspace, void* stream) {
  if (shape->head_dim != D)
    return fail(COCKTAIL_EUNSUPPORTED, "kernels are built for head_dim 128, got %d", shape->head_dim);
  if (hd->rep > COCKTAIL_MAX_Q_PER_KV)
    return fail(COCKTAIL_EUNSUPPORTED, "Hq/Hkv = %d exceeds %d", hd->rep, COCKTAIL_MAX_Q_PER_KV);
  static_assert(COCKTAIL_MAX_Q_PER_KV == kQuadMaxRep, "every ratio above 1 runs on the token-quad kernel");
  if ((reinterpret_cast<uintptr_t>(q) | reinterpret_cast<uintptr_t>(out) | reinterpret_cast<uintptr_t>(workspace) |
       reinterpret_cast<uintptr_t>(cache->plan_dev)) & 15)
    return fail(COCKTAIL_EALIGN, "q, out, workspace and plan_dev must be 16-byte aligned");
  if (lse && (reinterpret_cast<uintptr_t>(lse) & 3)) return fail(COCKTAIL_EALIGN, "lse must be 4-byte aligned");
  DecodeParams p;
  char* pd = static_cast<char*>(cache->plan_dev);
  p.recs = reinterpret_cast<const WorkerRec*>(pd + hd->off_worker_rec);
  p.segs = reinterpret_cast<const Segment*>(pd + hd->off_segments);
  p.psegs = reinterpret_cast<const PoolSeg*>(pd + hd->off_pool_seg);
  p.counters = reinterpret_cast<uint32_t*>(pd + hd->off_counters);
  p.seq_len = reinterpret_cast<const int32_t*>(pd + hd->off_seq_len);
  p.num_groups = hd->num_groups;
  p.num_workers = hd->num_workers;
  p.k_app = p.v_app = nullptr;
  p.num_appended = 0, p.app_blocks = hd->append_blocks;
  if (hd->append_capacity > 0) {
    if (!cache->k_app || !cache->v_app) return fail(COCKTAIL_EINVAL, "the plan has append buffers but k_app or v_app is NULL");
    if ((reinterpret_cast<uintptr_t>(cache->k_app) | reinterpret_cast<uintptr_t>(cache->v_app)) & 15)
      return fail(COCKTAIL_EALIGN, "append buffers must be 16-byte aligned");
    if (cache->num_appended < 0 || cache->num_appended > hd->append_capacity)
      return fail(COCKTAIL_EINVAL, "num_appended %d outside [0, %d]", cache->num_appended, hd->append_capacity);
    p.k_app = static_cast<const char*>(cache->k_app), p.v_app = static_cast<const char*>(cache->v_app);
    p.num_appended = cache->num_appended;
  } else if (cache->num_appended != 0) {
    return fail(COCKTAIL_EINVAL, "num_appended is %d but the plan was made without append buffers", cache->num_appended);
  }
  p.bh_off = reinterpret_cast<const int32_t*>(pd + hd->off_bh_off);
  p.q = static_cast<const uint32_t*>(q);
  for (int c = 0; c < kNumClasses; ++c) {
    if (hd->class_bytes[c] > 0 && (!cache->k[c] || !cache->v[c]))
      return fail(COCKTAIL_EINVAL, "cache buffer of class %d is NULL", c);
    if ((reinterpret_cast<uintptr_t>(cache->k[c]) | reinterpret_cast<uintptr_t>(cache->v[c])) & 15)
      return fail(COCKTAIL_EALIGN, "cache buffers must be 16-byte aligned");
    p.k[c] = static_cast<const char*>(cache->k[c]);
    p.v[c] = static_cast<const char*>(cache->v[c]);
  }
  p.ws = static_cast<float*>(workspace);
  p.status = reinterpret_cast<int32_t*>(static_cast<char*>(workspace) + hd->ws_status_off);
  p.out = static_cast<_Float16*>(out);
  p.lse = lse;
  if (!(sm_scale > 0.f)) sm_scale = 1.0f / std::sqrt(static_cast<float>(shape->head_dim));
  p.scale_log2 = sm_scale * 1.4426950408889634f;
  p.rep = hd->rep, p.num_q_heads = hd->num_q_heads, p.num_kv_heads = hd->num_kv_heads;
#ifdef COCKTAIL_TRACE
  // debugging builds only: the caller provides 32 bytes per worker behind the regular workspace
  p.trace = reinterpret_cast<uint64_t*>(static_cast<char*>(workspace) + ((hd->workspace_bytes + 255) & ~int64_t(255)));
#endif
  hipStream_t st = static_cast<hipStream_t>(stream);
  const int app_groups = hd->append_capacity > 0 ? hd->batch * hd->num_kv_heads : 0;
  if (hd->total_gblocks > 0 || app_groups > 0) {
    const bool quads = hd->v_layout == COCKTAIL_V_TOKEN_QUADS;
    const dim3 grid(hd->num_workers + app_groups, 1, 1), block(64, 1, 1);
    // non-temporal K/V loads when nothing is read twice: one wave per workgroup, and a cache large enough
    // that it cannot stay in the memory-side cache from one call to the next
    static const int nt_override = [] {   // tuning aid, read once: COCKTAIL_NON_TEMPORAL=0 | 1
      const char* e = std::getenv("COCKTAIL_NON_TEMPORAL");
      return e ? (std::atoi(e) != 0 ? 1 : 0) : -1;
    }();
    const bool nt = nt_override >= 0 ? nt_override == 1
                                     : ((hd->rep == 1 || (quads && quad_waves(hd->rep) == 1)) &&
                                        hd->packed_bytes >= kNonTemporalMinBytes);
    const bool int8 = hd->class_blocks[2] > 0;
    if (quads) {
      const hipError_t e = launch_decode_quads(p, shape->group_size, nt, int8, int(grid.x), st);
      if (e != hipSuccess) return fail(COCKTAIL_EHIP, "decode_quads launch failed: %s", hipGetErrorString(e));
    } else {
      void (*kern)(DecodeParams) = nullptr;
#define COCKTAIL_PICK(G)                                                                                              \
  kern = int8 ? (nt ? decode_attention_kernel<G, kAuxNonTemporal, true> : decode_attention_kernel<G, kAuxDefault, true>) \
              : (nt ? decode_attention_kernel<G, kAuxNonTemporal, false> : decode_attention_kernel<G, kAuxDefault, false>)
      switch (shape->group_size) {
        case 32: COCKTAIL_PICK(32); break;
        case 64: COCKTAIL_PICK(64); break;
        default: COCKTAIL_PICK(128); break;
      }
#undef COCKTAIL_PICK
      hipLaunchKernelGGL(kern, grid, block, 0, st, p);
      const hipError_t e = hipGetLastError();
      if (e != hipSuccess) return fail(COCKTAIL_EHIP, "decode_attention launch failed: %s", hipGetErrorString(e));
    }
  }
  hipLaunchKernelGGL(decode_merge_kernel, dim3(shape->batch * shape->num_q_heads), dim3(32 * kMergeSlices), 0, st, p);
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess)
    return fail(COCKTAIL_EHIP, "decode_merge launch failed: %s (the ticket counters in plan_dev were not reset: upload the plan again)",
                hipGetErrorString(e));
  return COCKTAIL_OK;
}

}  // namespace

extern "C" int cocktail_decode_attention(const cocktail_shape* shape, const void* q, const cocktail_cache* cache,
                                         float sm_scale, void* out, float* lse, void* workspace,
                                         size_t workspace_bytes, void* stream) {
  const PlanHeader* hd = nullptr;
  if (int rc = check_plan_matches(shape, cache, &hd)) return rc;
  if (!q || !out || !workspace) return fail(COCKTAIL_EINVAL, "q, out and workspace must not be NULL");
  if (workspace_bytes < static_cast<size_t>(hd->workspace_bytes))
    return fail(COCKTAIL_ENOSPACE, "workspace holds %zu bytes, %lld needed", workspace_bytes,
                (long long)hd->workspace_bytes);
  return decode_enqueue(shape, hd, q, cache, sm_scale, out, lse, workspace, stream);
}

extern "C" int cocktail_decode_attention_static(const cocktail_shape* shape, const void* q, const cocktail_cache* cache,
                                                float sm_scale, void* out, float* lse, void* stream) {
  const PlanHeader* hd = nullptr;
  if (int rc = check_plan_matches(shape, cache, &hd)) return rc;
  if (!q || !out) return fail(COCKTAIL_EINVAL, "q and out must not be NULL");
  if (static_cast<size_t>(hd->workspace_bytes) > kStaticWorkspaceBytes)
    return fail(COCKTAIL_ENOSPACE, "this plan needs a workspace of %lld bytes, the built-in one holds %zu: use "
                "cocktail_decode_attention with a caller-supplied workspace", (long long)hd->workspace_bytes,
                kStaticWorkspaceBytes);
  void* ws = nullptr;
  if (int rc = static_workspace(&ws)) return rc;
  return decode_enqueue(shape, hd, q, cache, sm_scale, out, lse, ws, stream);
}

extern "C" int cocktail_decode_check(const cocktail_shape* shape, const cocktail_cache* cache, const void* workspace,
                                     void* stream) {
  const PlanHeader* hd = nullptr;
  if (int rc = check_plan_matches(shape, cache, &hd)) return rc;
  void* ws = const_cast<void*>(workspace);
  if (!ws) {
    if (static_cast<size_t>(hd->workspace_bytes) > kStaticWorkspaceBytes)
      return fail(COCKTAIL_ENOSPACE, "this plan does not fit the built-in workspace");
    if (int rc = static_workspace(&ws)) return rc;
  }
  const int rows = hd->batch * hd->num_q_heads;
  std::vector<int32_t> status(rows);
  hipError_t e = hipStreamSynchronize(static_cast<hipStream_t>(stream));
  if (e == hipSuccess)
    e = hipMemcpy(status.data(), static_cast<const char*>(ws) + hd->ws_status_off, sizeof(int32_t) * rows, hipMemcpyDeviceToHost);
  if (e != hipSuccess) {
    (void)hipGetLastError();
    return fail(COCKTAIL_EHIP, "reading the status of the last decode call failed: %s", hipGetErrorString(e));
  }
  int bad = 0, first = -1;
  for (int i = 0; i < rows; ++i)
    if (status[i] != 0) {
      if (first < 0) first = i;
      ++bad;
    }
  if (bad)
    return fail(COCKTAIL_ESTATE, "the last decode call covered %d tokens too %s for sequence %d, query head %d (%d of %d rows "
                "affected; their out and lse are NaN): the ticket counters in plan_dev were not zero when the call "
                "started, calls on this cache overlapped, or plan_dev was modified; upload the plan again",
                status[first] < 0 ? -status[first] : status[first], status[first] < 0 ? "few" : "many",
                first / hd->num_q_heads, first % hd->num_q_heads, bad, rows);
  return COCKTAIL_OK;
}
