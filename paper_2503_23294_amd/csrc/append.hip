// Sec. III-A: the K/V rows of tokens generated during decoding join the cache in FP16, behind the
// context.  They go into the append buffers: per (sequence, kv head) a few 64-token blocks in the
// block layout of the FP16 class (16-byte piece p of token i at (p*64 + i)*16; V in token quads where
// the packed cache stores V that way).
#include <hip/hip_runtime.h>

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
