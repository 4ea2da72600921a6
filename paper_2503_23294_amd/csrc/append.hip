// Sec. III-A: the K/V rows of tokens generated during decoding join the cache in FP16, behind the
// context.  They go into the append buffers: per (sequence, kv head) a few 64-token blocks in the
// block layout of the FP16 class (16-byte piece p of token i at (p*64 + i)*16; V in token quads where
// the packed cache stores V that way).
#include <hip/hip_runtime.h>

#include <cstring>

#include "common.h"
#include "plan.h"

namespace cocktail {

// One thread moves one 16-byte piece: thread -> ((b, h), piece); blockIdx.y = 0 for K, 1 for V.
__global__ __launch_bounds__(256) void append_fp16_kernel(const u32x4* __restrict__ k_new,
                                                           const u32x4* __restrict__ v_new, char* __restrict__ k_app,
                                                           char* __restrict__ v_app, int position, int app_blocks,
                                                           int num_bh, int v_quads, int head_dim,
                                                           const int32_t* __restrict__ appended,
                                                           const uint8_t* __restrict__ active, int num_kv_heads,
                                                           int capacity) {
  const int kPieces = 2 * head_dim / 16;       // 16-byte pieces of one fp16 row
  const int idx = blockIdx.x * 256 + threadIdx.x;
  if (idx >= num_bh * kPieces) return;
  const int bh = idx / kPieces, p = idx % kPieces;
  if (appended) {
    // per-sequence positions: the token goes behind what the sequence has appended so far
    const int b = bh / num_kv_heads;
    if (active && !active[b]) return;
    position = appended[b];
    if (position < 0 || position >= capacity) return;   // the append buffer of this sequence is full
  }
  const u32x4* src = blockIdx.y ? v_new : k_new;
  char* dst = blockIdx.y ? v_app : k_app;
  const size_t block = size_t(bh) * app_blocks + position / kTB;
  char* blk = dst + block * size_t(kTB * 2 * head_dim);
  const u32x4 v = src[idx];
  if (blockIdx.y && v_quads) {
    // the piece is channels 8p .. 8p+7 of the token: lane j = p % 4 of its quad, channels e = 8 ((p / 4) % 2) + x
    const int i = position % kTB, h = p >> 3, j = p & 3, e0 = 8 * ((p >> 2) & 1);
#pragma unroll
    for (int x = 0; x < 8; ++x) {
      const uint32_t word = v[x >> 1];
      *reinterpret_cast<uint16_t*>(blk + quad_halfword_offset(8, 1, i, h, j, e0 + x)) =
          uint16_t((x & 1) ? word >> 16 : word);
    }
    return;
  }
  *reinterpret_cast<u32x4*>(blk + (size_t(p) * kTB + position % kTB) * 16) = v;
}

// After the rows are stored: appended[b] += 1 for every active sequence that had room.
__global__ __launch_bounds__(256) void advance_appended_kernel(int32_t* __restrict__ appended,
                                                                const uint8_t* __restrict__ active, int batch, int capacity) {
  for (int b = blockIdx.x * 256 + threadIdx.x; b < batch; b += gridDim.x * 256) {
    const int n = appended[b];
    if ((!active || active[b]) && n >= 0 && n < capacity) appended[b] = n + 1;
  }
}

// Fold (Sec. III-A: generated tokens are context from then on, still FP16): the rows of the append buffers move
// behind the FP16 rows of their (sequence, kv head) in the packed cache.  Sequence b has T1[b] - T0[b] rows to
// move (the context lengths of the new and of the old plan, both on the device); row i goes to token
// n0 + i of the run, n0 = the FP16 tokens the old plan counts.  One thread moves one 16-byte piece of a row
// (V in token quads: its eight half-words one by one, the quad position of a token changes with n0).
// grid: (pieces of `max_count` rows, B * Hkv, 2); blockIdx.z = 0 for K, 1 for V.
__global__ __launch_bounds__(256) void fold_appended_kernel(const char* __restrict__ k_app, const char* __restrict__ v_app,
                                                             char* __restrict__ k_fp16, char* __restrict__ v_fp16,
                                                             const void* __restrict__ old_plan, const void* __restrict__ new_plan,
                                                             int app_blocks, int v_quads, int head_dim, int num_kv_heads) {
  const int kPieces = 2 * head_dim / 16;
  const int idx = blockIdx.x * 256 + threadIdx.x;
  const int i = idx / kPieces, p = idx % kPieces;   // row of the append run, piece of the row
  const int bh = blockIdx.y, b = bh / num_kv_heads, h = bh % num_kv_heads;
  const PlanHeader* h0 = static_cast<const PlanHeader*>(old_plan);
  const PlanHeader* h1 = static_cast<const PlanHeader*>(new_plan);
  const int count = plan_array<int32_t>(new_plan, h1->off_seq_len)[b] - plan_array<int32_t>(old_plan, h0->off_seq_len)[b];
  if (i >= count) return;
  const int n = plan_array<int32_t>(old_plan, h0->off_class_tokens)[kNumClasses * b + kFp16Class] + i;
  const int64_t run0 = plan_array<int32_t>(old_plan, h0->off_blk_base)[kNumClasses * b + kFp16Class] +
                       int64_t(h) * plan_array<int32_t>(old_plan, h0->off_run_blocks)[kNumClasses * b + kFp16Class];
  const size_t block_bytes = size_t(kTB) * 2 * head_dim;
  const char* sblk = (blockIdx.z ? v_app : k_app) + (size_t(bh) * app_blocks + i / kTB) * block_bytes;
  char* dblk = (blockIdx.z ? v_fp16 : k_fp16) + size_t(run0 + n / kTB) * block_bytes;
  if (blockIdx.z && v_quads) {
    const int hh = p >> 3, j = p & 3, e0 = 8 * ((p >> 2) & 1);
#pragma unroll
    for (int x = 0; x < 8; ++x)
      *reinterpret_cast<uint16_t*>(dblk + quad_halfword_offset(8, 1, n % kTB, hh, j, e0 + x)) =
          *reinterpret_cast<const uint16_t*>(sblk + quad_halfword_offset(8, 1, i % kTB, hh, j, e0 + x));
    return;
  }
  *reinterpret_cast<u32x4*>(dblk + (size_t(p) * kTB + n % kTB) * 16) =
      *reinterpret_cast<const u32x4*>(sblk + (size_t(p) * kTB + i % kTB) * 16);
}

// After a fold nothing is appended any more.
__global__ __launch_bounds__(256) void clear_appended_kernel(int32_t* __restrict__ appended, int batch) {
  for (int b = blockIdx.x * 256 + threadIdx.x; b < batch; b += gridDim.x * 256) appended[b] = 0;
}

}  // namespace cocktail

using namespace cocktail;

namespace {

int check_append(const cocktail_shape* shape, const void* k_new, const void* v_new, const cocktail_cache* cache,
                 const PlanHeader** out) {
  if (int rc = check_shape(shape)) return rc;
  if (!cache || !cache->plan_host) return fail(COCKTAIL_EINVAL, "cache or its plan is NULL");
  const PlanHeader* hd = static_cast<const PlanHeader*>(cache->plan_host);
  if (hd->magic != kPlanMagic || hd->version != kPlanVersion)
    return fail(COCKTAIL_EINVAL, "plan_host is not a plan written by this library version");
  if (hd->batch != shape->batch || hd->num_kv_heads != shape->num_kv_heads || hd->head_dim != shape->head_dim ||
      hd->chunk_size != shape->chunk_size || hd->group_size != shape->group_size ||
      hd->num_q_heads != shape->num_q_heads)
    return fail(COCKTAIL_EINVAL, "plan was made for a different shape");
  if (shape->head_dim != 64 && shape->head_dim != 128)
    return fail(COCKTAIL_EUNSUPPORTED, "kernels are built for head_dim 64 and 128, got %d", shape->head_dim);
  if (hd->append_capacity <= 0) return fail(COCKTAIL_EINVAL, "the plan was made without append buffers");
  if (!k_new || !v_new || !cache->k_app || !cache->v_app)
    return fail(COCKTAIL_EINVAL, "k_new, v_new and the append buffers must not be NULL");
  if ((reinterpret_cast<uintptr_t>(k_new) | reinterpret_cast<uintptr_t>(v_new) |
       reinterpret_cast<uintptr_t>(cache->k_app) | reinterpret_cast<uintptr_t>(cache->v_app)) & 15)
    return fail(COCKTAIL_EALIGN, "k_new, v_new and the append buffers must be 16-byte aligned");
  *out = hd;
  return COCKTAIL_OK;
}

}  // namespace

extern "C" int cocktail_append_fp16_ragged(const cocktail_shape* shape, const void* k_new, const void* v_new,
                                           const cocktail_cache* cache, const uint8_t* active_dev, void* stream) {
  const PlanHeader* hd = nullptr;
  if (int rc = check_append(shape, k_new, v_new, cache, &hd)) return rc;
  if (!cache->appended_dev) return fail(COCKTAIL_EINVAL, "appended_dev is NULL: the per-sequence counts live there");
  if (reinterpret_cast<uintptr_t>(cache->appended_dev) & 3) return fail(COCKTAIL_EALIGN, "appended_dev must be 4-byte aligned");
  const int num_bh = hd->batch * hd->num_kv_heads;
  const dim3 grid((num_bh * (shape->head_dim / 8) + 255) / 256, 2, 1);
  hipStream_t st = static_cast<hipStream_t>(stream);
  hipLaunchKernelGGL(append_fp16_kernel, grid, dim3(256), 0, st, static_cast<const u32x4*>(k_new),
                     static_cast<const u32x4*>(v_new), static_cast<char*>(cache->k_app), static_cast<char*>(cache->v_app), 0,
                     hd->append_blocks, num_bh, hd->v_layout, shape->head_dim, cache->appended_dev, active_dev,
                     hd->num_kv_heads, hd->append_capacity);
  hipLaunchKernelGGL(advance_appended_kernel, dim3((hd->batch + 255) / 256 < 64 ? (hd->batch + 255) / 256 : 64), dim3(256), 0, st,
                     cache->appended_dev, active_dev, hd->batch, hd->append_capacity);
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(COCKTAIL_EHIP, "append launch failed: %s", hipGetErrorString(e));
  return COCKTAIL_OK;
}

extern "C" int cocktail_append_fp16(const cocktail_shape* shape, const void* k_new, const void* v_new,
                                    const cocktail_cache* cache, int32_t position, void* stream) {
  const PlanHeader* hd = nullptr;
  if (int rc = check_append(shape, k_new, v_new, cache, &hd)) return rc;
  if (position < 0 || position >= hd->append_capacity)
    return fail(COCKTAIL_EINVAL, "position %d outside the append capacity %d", position, hd->append_capacity);
  const int num_bh = hd->batch * hd->num_kv_heads;
  const dim3 grid((num_bh * (shape->head_dim / 8) + 255) / 256, 2, 1);
  hipLaunchKernelGGL(append_fp16_kernel, grid, dim3(256), 0, static_cast<hipStream_t>(stream),
                     static_cast<const u32x4*>(k_new), static_cast<const u32x4*>(v_new),
                     static_cast<char*>(cache->k_app), static_cast<char*>(cache->v_app), position, hd->append_blocks,
                     num_bh, hd->v_layout, shape->head_dim, static_cast<const int32_t*>(nullptr),
                     static_cast<const uint8_t*>(nullptr), hd->num_kv_heads, hd->append_capacity);
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(COCKTAIL_EHIP, "append launch failed: %s", hipGetErrorString(e));
  return COCKTAIL_OK;
}

extern "C" int cocktail_fold_appended(const cocktail_shape* shape, const cocktail_cache* cache, const void* new_plan_host,
                                      const void* new_plan_dev, void* stream) {
  if (int rc = check_shape(shape)) return rc;
  if (!cache || !cache->plan_host || !cache->plan_dev) return fail(COCKTAIL_EINVAL, "cache or its plan is NULL");
  if (!new_plan_host || !new_plan_dev) return fail(COCKTAIL_EINVAL, "new_plan_host and new_plan_dev must not be NULL");
  const PlanHeader* h0 = static_cast<const PlanHeader*>(cache->plan_host);
  const PlanHeader* h1 = static_cast<const PlanHeader*>(new_plan_host);
  if (h0->magic != kPlanMagic || h0->version != kPlanVersion || h1->magic != kPlanMagic || h1->version != kPlanVersion)
    return fail(COCKTAIL_EINVAL, "plan_host or new_plan_host is not a plan written by this library version");
  for (const PlanHeader* hd : {h0, h1})
    if (hd->batch != shape->batch || hd->num_kv_heads != shape->num_kv_heads || hd->head_dim != shape->head_dim ||
        hd->chunk_size != shape->chunk_size || hd->group_size != shape->group_size || hd->num_q_heads != shape->num_q_heads)
      return fail(COCKTAIL_EINVAL, "plan was made for a different shape");
  if (shape->head_dim != 64 && shape->head_dim != 128)
    return fail(COCKTAIL_EUNSUPPORTED, "kernels are built for head_dim 64 and 128, got %d", shape->head_dim);
  if (h0->append_capacity <= 0) return fail(COCKTAIL_EINVAL, "the plan was made without append buffers");
  if (h0->v_layout != h1->v_layout) return fail(COCKTAIL_EINVAL, "the two plans store V in different forms");
  if ((reinterpret_cast<uintptr_t>(cache->plan_dev) | reinterpret_cast<uintptr_t>(new_plan_dev)) & 15)
    return fail(COCKTAIL_EALIGN, "plan_dev and new_plan_dev must be 16-byte aligned");
  // the new plan has to describe the same buffers: every run where it was, with the blocks it had, and nothing but
  // FP16 tokens added
  const int B = shape->batch;
  constexpr int NC = kNumClasses;
  const int32_t* t0 = plan_array<int32_t>(h0, h0->off_seq_len);
  const int32_t* t1 = plan_array<int32_t>(h1, h1->off_seq_len);
  const int32_t* ct0 = plan_array<int32_t>(h0, h0->off_class_tokens);
  const int32_t* ct1 = plan_array<int32_t>(h1, h1->off_class_tokens);
  if (std::memcmp(plan_array<int32_t>(h0, h0->off_blk_base), plan_array<int32_t>(h1, h1->off_blk_base), sizeof(int32_t) * NC * (B + 1)) != 0 ||
      std::memcmp(plan_array<int32_t>(h0, h0->off_run_blocks), plan_array<int32_t>(h1, h1->off_run_blocks), sizeof(int32_t) * NC * B) != 0)
    return fail(COCKTAIL_EINVAL, "the new plan lays the cache out differently (plan both with the same max_seq_lens)");
  int max_count = 0;
  for (int b = 0; b < B; ++b) {
    const int count = t1[b] - t0[b];
    if (count < 0 || count > h0->append_capacity)
      return fail(COCKTAIL_EINVAL, "sequence %d: %d tokens to fold, the append buffers hold 0 to %d", b, count, h0->append_capacity);
    for (int c = 0; c < NC; ++c)
      if (ct1[NC * b + c] - ct0[NC * b + c] != (c == kFp16Class ? count : 0))
        return fail(COCKTAIL_EINVAL, "sequence %d: the new plan differs from the old one in more than FP16 tokens at the end", b);
    if (cache->appended_dev == nullptr && count != cache->num_appended)
      return fail(COCKTAIL_EINVAL, "sequence %d: the new plan has %d tokens more, %d are appended", b, count, cache->num_appended);
    max_count = count > max_count ? count : max_count;
  }
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (max_count > 0) {
    if (!cache->k_app || !cache->v_app || !cache->k[kFp16Class] || !cache->v[kFp16Class])
      return fail(COCKTAIL_EINVAL, "the append buffers and the FP16 class buffers must not be NULL");
    if ((reinterpret_cast<uintptr_t>(cache->k_app) | reinterpret_cast<uintptr_t>(cache->v_app) |
         reinterpret_cast<uintptr_t>(cache->k[kFp16Class]) | reinterpret_cast<uintptr_t>(cache->v[kFp16Class])) & 15)
      return fail(COCKTAIL_EALIGN, "the append buffers and the FP16 class buffers must be 16-byte aligned");
    const int pieces = shape->head_dim / 8;
    const dim3 grid(static_cast<unsigned>((int64_t(max_count) * pieces + 255) / 256), static_cast<unsigned>(B * shape->num_kv_heads), 2);
    if (grid.y > 65535u) return fail(COCKTAIL_EUNSUPPORTED, "more than 65535 (sequence, kv head) pairs in one fold");
    hipLaunchKernelGGL(fold_appended_kernel, grid, dim3(256), 0, st, static_cast<const char*>(cache->k_app),
                       static_cast<const char*>(cache->v_app), static_cast<char*>(cache->k[kFp16Class]),
                       static_cast<char*>(cache->v[kFp16Class]), cache->plan_dev, new_plan_dev, h0->append_blocks, h0->v_layout,
                       shape->head_dim, shape->num_kv_heads);
  }
  if (cache->appended_dev)
    hipLaunchKernelGGL(clear_appended_kernel, dim3((B + 255) / 256 < 64 ? (B + 255) / 256 : 64), dim3(256), 0, st,
                       cache->appended_dev, B);
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(COCKTAIL_EHIP, "fold launch failed: %s", hipGetErrorString(e));
  return COCKTAIL_OK;
}
