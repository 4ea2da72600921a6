// Decode side of Alg. 1 (Sec. III-C): single-query attention over the INT2, INT4,
// INT8 and FP16 classes of the packed cache.
//
// This file holds the exact merge of the partial softmax states and the host side of the decode entry points;
// the partial-state kernels are templates (decode_heads_impl.h: one query head per kv head, vector ALU;
// decode_quads_impl.h: grouped-query shapes, 4x4x4 matrix instructions) instantiated per head_dim in their
// own translation units.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdlib>
#include <mutex>
#include <vector>

#include "decode_heads_impl.h"

namespace cocktail {

template hipError_t launch_decode_heads<128>(const DecodeParams&, int, bool, bool, int, hipStream_t);

// Exact merge of the partial states of one (sequence, query head):
//   M = max m_i,  L = sum l_i 2^(m_i - M),  out = sum o_i 2^(m_i - M) / L,  lse = ln2 (M + log2 L).
// The partials of a (sequence, kv head) are a dense block of the workspace.  HD / 4 channel quads x 16
// slices of the block (512 threads at head_dim 128); a slice loads eight partials at a time (128 in flight
// per workgroup, usually the whole block in one round) and folds them with a running maximum, then the
// sixteen slice states are folded through shared memory.  A (sequence, query head) without any partial
// (empty sequence) gets zeros and lse = -inf.
// Every partial also says how many tokens it covers.  Their sum has to be the token count of the
// sequence: the softmax over the concatenation of Alg. 1 attends to every token exactly once.  If it is
// not (ticket counters that were not zero when the call started, calls overlapping on one cache, a
// damaged plan), the row is not a result: out and lse are set to NaN and the difference goes to the
// status array.
constexpr int kMergeSlices = 16;
template <int D>
__global__ __launch_bounds__(D / 4 * kMergeSlices) void decode_merge_kernel(DecodeParams prm) {
  constexpr int QUADS = D / 4;
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
  const int appended = prm.appended ? prm.appended[b] : prm.num_appended;
  const int expected = prm.seq_len[b] + min(max(appended, 0), prm.app_capacity);
  const int tid = threadIdx.x;
  // every worker has drawn its last ticket: put the counters back to zero for the next call
  if (blockIdx.x == 0)
    for (int i = tid; i < prm.num_groups; i += QUADS * kMergeSlices) prm.counters[i * kCounterStride] = 0u;
  constexpr int STRIDE = D + kPartialFloats;
  constexpr int U = 8;   // partials in flight per thread
  const int quad = tid % QUADS, slice = tid / QUADS;
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
  const int wrep = work_rep_of(rep, false);
  // one-wave workgroups: eight per compute unit; two-wave workgroups (which share their K/V units through 32 KB
  // of shared memory each): four
  const int per_cu = uses_token_quads(wrep) ? waves_per_cu / quad_waves(wrep) : waves_per_cu;
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
                   float sm_scale, void* out, float* lse, void* workspace, void* stream, void* event_between = nullptr) {
  if (shape->head_dim != 64 && shape->head_dim != 128)
    return fail(COCKTAIL_EUNSUPPORTED, "kernels are built for head_dim 64 and 128, got %d", shape->head_dim);
  if (hd->rep > COCKTAIL_MAX_Q_PER_KV)
    return fail(COCKTAIL_EUNSUPPORTED, "Hq/Hkv = %d exceeds %d", hd->rep, COCKTAIL_MAX_Q_PER_KV);
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
  p.appended = nullptr, p.app_capacity = hd->append_capacity, p.app_slices = hd->append_slices;
  if (hd->append_capacity > 0) {
    if (!cache->k_app || !cache->v_app) return fail(COCKTAIL_EINVAL, "the plan has append buffers but k_app or v_app is NULL");
    if ((reinterpret_cast<uintptr_t>(cache->k_app) | reinterpret_cast<uintptr_t>(cache->v_app)) & 15)
      return fail(COCKTAIL_EALIGN, "append buffers must be 16-byte aligned");
    if (cache->num_appended < 0 || cache->num_appended > hd->append_capacity)
      return fail(COCKTAIL_EINVAL, "num_appended %d outside [0, %d]", cache->num_appended, hd->append_capacity);
    if (cache->appended_dev && (reinterpret_cast<uintptr_t>(cache->appended_dev) & 3))
      return fail(COCKTAIL_EALIGN, "appended_dev must be 4-byte aligned");
    if (cache->appended_dev && cache->num_appended != 0)
      return fail(COCKTAIL_EINVAL, "num_appended must be 0 when appended_dev holds the per-sequence counts");
    p.k_app = static_cast<const char*>(cache->k_app), p.v_app = static_cast<const char*>(cache->v_app);
    p.num_appended = cache->num_appended;
    p.appended = cache->appended_dev;
  } else if (cache->num_appended != 0 || cache->appended_dev) {
    return fail(COCKTAIL_EINVAL, "num_appended / appended_dev are set but the plan was made without append buffers");
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
  p.rep = hd->work_rep, p.num_q_heads = hd->num_q_heads, p.num_kv_heads = hd->work_heads;
  p.kv_share = hd->work_heads / hd->num_kv_heads;
#ifdef COCKTAIL_TRACE
  // debugging builds only: the caller provides 32 bytes per worker behind the regular workspace
  p.trace = reinterpret_cast<uint64_t*>(static_cast<char*>(workspace) + ((hd->workspace_bytes + 255) & ~int64_t(255)));
#endif
  hipStream_t st = static_cast<hipStream_t>(stream);
  const int app_groups = hd->batch * hd->work_heads * hd->append_slices;   // 0 without append buffers
  if (hd->total_gblocks > 0 || app_groups > 0) {
    const bool quads = hd->v_layout == COCKTAIL_V_TOKEN_QUADS;
    const dim3 grid(hd->num_workers + app_groups, 1, 1);
    // non-temporal K/V loads when nothing is read twice (one workgroup per kv head's blocks: the vector-ALU kernel
    // with one query head per kv head, the matrix kernel with all query heads of a kv head in one workgroup) and the
    // cache is large enough that it cannot stay in the memory-side cache from one call to the next
    static const int nt_override = [] {   // tuning aid, read once: COCKTAIL_NON_TEMPORAL=0 | 1
      const char* e = std::getenv("COCKTAIL_NON_TEMPORAL");
      return e ? (std::atoi(e) != 0 ? 1 : 0) : -1;
    }();
    // (several work heads per kv head - one wave per query head of a grouped-query shape, or sets of eight at
    // ratios above eight - read the same lines from different workgroups: default policy, the L2 serves the repeats)
    const bool nt = nt_override >= 0 ? nt_override == 1
                                     : (hd->work_rep == hd->rep && hd->packed_bytes >= kNonTemporalMinBytes);
    const bool int8 = hd->class_blocks[2] > 0;
    const bool d64 = shape->head_dim == 64;
    const hipError_t e = quads ? (d64 ? launch_decode_quads<64>(p, shape->group_size, nt, int8, int(grid.x), st)
                                      : launch_decode_quads<128>(p, shape->group_size, nt, int8, int(grid.x), st))
                               : (d64 ? launch_decode_heads<64>(p, shape->group_size, nt, int8, int(grid.x), st)
                                      : launch_decode_heads<128>(p, shape->group_size, nt, int8, int(grid.x), st));
    if (e != hipSuccess) return fail(COCKTAIL_EHIP, "decode launch failed: %s", hipGetErrorString(e));
  }
  if (event_between) {   // measurement aid: when the partial-state kernel is done
    const hipError_t ev = hipEventRecord(static_cast<hipEvent_t>(event_between), st);
    if (ev != hipSuccess) return fail(COCKTAIL_EHIP, "recording the event between the two kernels failed: %s", hipGetErrorString(ev));
  }
  if (shape->head_dim == 64)
    hipLaunchKernelGGL(decode_merge_kernel<64>, dim3(shape->batch * shape->num_q_heads), dim3(16 * kMergeSlices), 0, st, p);
  else
    hipLaunchKernelGGL(decode_merge_kernel<128>, dim3(shape->batch * shape->num_q_heads), dim3(32 * kMergeSlices), 0, st, p);
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

extern "C" int cocktail_decode_attention_marked(const cocktail_shape* shape, const void* q, const cocktail_cache* cache,
                                                float sm_scale, void* out, float* lse, void* workspace,
                                                size_t workspace_bytes, void* stream, void* event_between) {
  const PlanHeader* hd = nullptr;
  if (int rc = check_plan_matches(shape, cache, &hd)) return rc;
  if (!q || !out || !workspace || !event_between) return fail(COCKTAIL_EINVAL, "q, out, workspace and event_between must not be NULL");
  if (workspace_bytes < static_cast<size_t>(hd->workspace_bytes))
    return fail(COCKTAIL_ENOSPACE, "workspace holds %zu bytes, %lld needed", workspace_bytes,
                (long long)hd->workspace_bytes);
  return decode_enqueue(shape, hd, q, cache, sm_scale, out, lse, workspace, stream, event_between);
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
