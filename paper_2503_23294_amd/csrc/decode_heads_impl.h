// Internal: the decode kernel for one query head per kv head (Hq = Hkv), as templates over head_dim; one
// translation unit per head_dim instantiates launch_decode_heads<HD>.
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
#pragma once
#include <hip/hip_runtime.h>

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

// Writes this wave's partial state `pid`: (m, l, o[HD]) reduced over its lanes, and the number of tokens it covers.
template <int HD, int NGH, int GL>
__device__ __forceinline__ void flush_partial(const LaneState<NGH>& st, float* red, int pid, int r, int lane, int tokens) {
  constexpr int UT = Geo<HD>::UT;       // lanes that hold different tokens (the other lanes of a token hold the same m and l)
  kparams_t prm = kparams();
  const int rep = prm->rep;
  float mw = st.m;
#pragma unroll
  for (int o = UT / 2; o > 0; o >>= 1) mw = fmaxf(mw, __shfl_xor(mw, o));
  const float f = __builtin_amdgcn_exp2f(st.m - mw);
  float lw = st.l * f;
#pragma unroll
  for (int o = UT / 2; o > 0; o >>= 1) lw += __shfl_xor(lw, o);
  float* out = prm->ws + (int64_t(pid) * rep + r) * (HD + kPartialFloats);
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
    // lane (c, quarter) adds 16 rows; at head_dim 128 quarters 0,1 hold channel half 0 and quarters 2,3 half 1,
    // at head_dim 64 all four hold the same channels
    const int c = lane & 15, quarter = lane >> 4;
    float sum = 0.f;
#pragma unroll
    for (int row = 0; row < 16; ++row) sum += tile[quarter * 16 + row][c];
    sum += __shfl_xor(sum, 16);
    if constexpr (HD == 64) {
      sum += __shfl_xor(sum, 32);
      if (quarter == 0) out[kPartialFloats + ch * 16 + c] = sum;
    } else {
      if ((quarter & 1) == 0) out[kPartialFloats + (quarter >> 1) * DH + ch * 16 + c] = sum;
    }
  }
}

// Zeroes the partial state and loads this lane's half of the query row `qrow`.
template <int HD, int NGH, int GL>
__device__ __forceinline__ void begin_state(int qrow, int h, LaneState<NGH>& st, uint32_t (&q)[DH / 2],
                                            float (&qsum)[NGH]) {
#pragma unroll
  for (int i = 0; i < DH; ++i) st.acc[i] = 0.f;
#pragma unroll
  for (int gq = 0; gq < NGH; ++gq) st.zacc[gq] = 0.f;
  st.m = kNegBig;
  st.l = 0.f;
  const u32x4* qp = reinterpret_cast<const u32x4*>(kparams()->q + int64_t(qrow) * (HD / 2) + h * (DH / 2));
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
template <int HD, class CLS, int CID, int G, int AUX>
__device__ __forceinline__ void run_class(Stream<HD>& sm, Piece& cur, float* red, int r, int lane, bool app = false) {
  constexpr int NGH = CLS::NGH;
  constexpr int GL = G < DH ? G : DH;
  constexpr int J = CLS::J;
  constexpr int UT = Geo<HD>::UT, UPB = Geo<HD>::UPB;
  static_assert(J == kIterUnits[CID], "the planner cuts pool pieces to the kernel's iteration size");
  const int t = lane % UT, h = lane / UT;
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
  int roob = UPB * sm.nblk;       // first unit past its segment: a load from there is out of range and costs nothing
#pragma unroll
  for (int jj = 0; jj < J; ++jj) CLS::template load<AUX>(ks[jj], krs, jj < rn ? ru + jj : roob, vc, vm);
#pragma unroll
  for (int jj = 0; jj < J; ++jj) CLS::template load<AUX>(vs[jj], vrs, jj < rn ? ru + jj : roob, vc, vm);
  sched_fence();
  begin_state<HD, NGH, GL>(sm.qrow + r, h, st, q, qsum);   // the query arrives while the first units are on their way
  int valid = cur.valid;
  int covered = 0;   // tokens the current partial state covers (the merge checks the total per sequence)
  Piece nxt = sm.next(lane);
#pragma unroll 1
  while (true) {
    const bool more = nxt.nu > 0 && nxt.cls == CID;
    if (more) {
      krs = make_rsrc(kbase + int64_t(sm.blk0) * CLS::BLOCKB, uint32_t(sm.nblk) * CLS::BLOCKB);
      vrs = make_rsrc(vbase + int64_t(sm.blk0) * CLS::BLOCKB, uint32_t(sm.nblk) * CLS::BLOCKB);
      ru = nxt.us, rn = nxt.nu, roob = UPB * sm.nblk;
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
      float full = s[jj];
      if constexpr (HD == 128) full += __shfl_xor(s[jj], 32);   // both halves of the token
      full *= scale_log2;
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
    if (!more || nxt.fresh) flush_partial<HD, NGH, GL>(st, red, pid, r, lane, covered);
    if (!more) break;
    if (nxt.fresh) {
      pid = nxt.pid;
      covered = 0;
      begin_state<HD, NGH, GL>(sm.qrow + r, h, st, q, qsum);
    }
    valid = nxt.valid;
    nxt = sm.next(lane);
  }
  cur = nxt;
}

// Workgroups behind the regular workers attend to the tokens appended during decoding (Sec. III-A): FP16 runs in
// the append buffers, one workgroup per slice of a (sequence, kv head)'s run, each writing one of the last
// partials of that head's range.
template <int HD, int G, int AUX>
__device__ __forceinline__ void appended_tokens(int idx, float* red, int r, int lane) {
  const AppendSlice a = append_slice(idx);
  if (a.tokens <= 0) {
    write_neutral<HD>(a.pid, r, lane);
    return;
  }
  Stream<HD> sm;
  sm.init_run(kFp16Class, a.tokens, a.first_block, a.blocks, a.qrow, a.pid);
  Piece cur = sm.next(lane);
  if (cur.nu > 0) run_class<HD, HalfClass<HD, G>, kFp16Class, G, AUX>(sm, cur, red, r, lane, true);
}

// One single-wave workgroup per worker (Hq = Hkv: the query head of a kv head is that head).  INT8: the cache
// has an INT8 class; caches without one run a kernel without that code (a third less of it to fetch and
// to allocate registers for, worth 1.5 us on a 32K-token layer).
template <int HD, int G, int AUX, bool INT8>
__global__ __launch_bounds__(64) __attribute__((amdgpu_waves_per_eu(2))) void decode_attention_kernel(DecodeParams) {
  __shared__ float red[64 * 17];   // reduction tile of a flush
  const int lane = threadIdx.x;
  constexpr int r = 0;             // query head inside the kv head's group
#ifdef COCKTAIL_TRACE
  const uint64_t t_start = __builtin_amdgcn_s_memrealtime();
#endif
  if (int(blockIdx.x) >= kparams()->num_workers) {
    appended_tokens<HD, G, AUX>(int(blockIdx.x) - kparams()->num_workers, red, r, lane);
    return;
  }
  Stream<HD> sm;
  sm.init(load_record(kparams()->recs + blockIdx.x));
  Piece cur = sm.next(lane);
  while (cur.nu > 0) {
    if (cur.cls == 0) {
      run_class<HD, QuantClass<HD, 2, G>, 0, G, AUX>(sm, cur, red, r, lane);
    } else if (cur.cls == 1) {
      run_class<HD, QuantClass<HD, 4, G>, 1, G, AUX>(sm, cur, red, r, lane);
    } else if (INT8 && cur.cls == 2) {
      if constexpr (INT8) run_class<HD, QuantClass<HD, 8, G>, 2, G, AUX>(sm, cur, red, r, lane);
    } else {
      run_class<HD, HalfClass<HD, G>, kFp16Class, G, AUX>(sm, cur, red, r, lane);
    }
  }
  // pool parts this worker never entered still own a partial slot: fill it with the neutral state
  for (int i = 0; i < sm.nps; ++i) {
    if ((sm.used >> i) & 1u) continue;
    const PoolSeg ps = load_record(kparams()->psegs + sm.pseg0 + i);
    if (sm.rank < ps.nslots) write_neutral<HD>(ps.slot0 + sm.rank, r, lane);
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

// Picks the instance for the group size, the cache policy and the classes present, and launches it.
template <int HD>
hipError_t launch_decode_heads(const DecodeParams& p, int group_size, bool nt, bool int8, int grid, hipStream_t st) {
  void (*kern)(DecodeParams) = nullptr;
#define COCKTAIL_PICK(G)                                                                                                      \
  kern = int8 ? (nt ? decode_attention_kernel<HD, G, kAuxNonTemporal, true> : decode_attention_kernel<HD, G, kAuxDefault, true>) \
              : (nt ? decode_attention_kernel<HD, G, kAuxNonTemporal, false> : decode_attention_kernel<HD, G, kAuxDefault, false>)
  if (group_size == 32) {
    COCKTAIL_PICK(32);
  } else if (group_size == 64) {
    COCKTAIL_PICK(64);
  } else if constexpr (HD >= 128) {
    COCKTAIL_PICK(128);
  }
#undef COCKTAIL_PICK
  if (!kern) return hipErrorInvalidValue;   // a group size larger than head_dim: refused by the shape check before
  hipLaunchKernelGGL(kern, dim3(grid), dim3(64), 0, st, p);
  return hipGetLastError();
}

}  // namespace cocktail
