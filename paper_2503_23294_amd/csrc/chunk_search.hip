// Chunk-level quantization search (Sec. III-B): Eq. 1 cosine similarity of the query embedding with
// every context-chunk embedding, Eq. 2-3 thresholds from the extreme scores of the sequence, and the
// bitwidth of every chunk by the comparisons of Alg. 1's prefill loop.
//
// Floating point decides an integer here, so the arithmetic is fixed: dot products and norms are
// accumulated in binary64 (the products of binary32 inputs are exact there), the score is rounded
// once to binary32, and the thresholds are three unfused binary32 operations each.
#include <hip/hip_runtime.h>

#include <cmath>

#include "common.h"

namespace cocktail {

// One wave per chunk: q.c, c.c and q.q in binary64, butterfly-reduced over the lanes.
__global__ __launch_bounds__(256) void similarity_kernel(const float* __restrict__ q_emb,
                                                          const float* __restrict__ c_emb,
                                                          const int32_t* __restrict__ chunk_off, int batch,
                                                          int embed_dim, int total, float* __restrict__ scores) {
  const int lane = threadIdx.x & 63;
  const int i = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (i >= total) return;
  int lo = 0, hi = batch;   // sequence b with chunk_off[b] <= i < chunk_off[b+1]
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (chunk_off[mid] <= i) lo = mid; else hi = mid;
  }
  const float* q = q_emb + size_t(lo) * embed_dim;
  const float* c = c_emb + size_t(i) * embed_dim;
  double qc = 0.0, cc = 0.0, qq = 0.0;
  for (int e = lane; e < embed_dim; e += 64) {
    const double a = q[e], b = c[e];
    qc += a * b, cc += b * b, qq += a * a;
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    qc += __shfl_xor(qc, o), cc += __shfl_xor(cc, o), qq += __shfl_xor(qq, o);
  }
  if (lane == 0) {
    const double denom = sqrt(qq) * sqrt(cc);
    scores[i] = denom > 0.0 ? static_cast<float>(qc / denom) : 0.0f;   // a zero vector has no direction
  }
}

// One workgroup per sequence: s_min, s_max, the two thresholds, then one comparison pair per chunk.
__global__ __launch_bounds__(256) void assign_bitwidth_kernel(const float* __restrict__ scores,
                                                               const int32_t* __restrict__ chunk_off, float alpha,
                                                               float beta, uint8_t* __restrict__ bits) {
#pragma clang fp contract(off)
  __shared__ float sm_min[4], sm_max[4];
  const int b = blockIdx.x;
  const int i0 = chunk_off[b], i1 = chunk_off[b + 1];
  if (i1 <= i0) return;
  float mn = INFINITY, mx = -INFINITY;
  for (int i = i0 + threadIdx.x; i < i1; i += 256) {
    const float s = scores[i];
    mn = fminf(mn, s), mx = fmaxf(mx, s);
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) mn = fminf(mn, __shfl_xor(mn, o)), mx = fmaxf(mx, __shfl_xor(mx, o));
  if ((threadIdx.x & 63) == 0) sm_min[threadIdx.x >> 6] = mn, sm_max[threadIdx.x >> 6] = mx;
  __syncthreads();
  mn = fminf(fminf(sm_min[0], sm_min[1]), fminf(sm_min[2], sm_min[3]));
  mx = fmaxf(fmaxf(sm_max[0], sm_max[1]), fmaxf(sm_max[2], sm_max[3]));
  const float d = mx - mn;
  const float t_low = mn + d * alpha;     // Eq. 2
  const float t_high = mx - d * beta;     // Eq. 3
  for (int i = i0 + threadIdx.x; i < i1; i += 256) {
    const float s = scores[i];
    bits[i] = s < t_low ? 2 : (s > t_high ? 16 : 4);   // order of Alg. 1's prefill loop
  }
}

}  // namespace cocktail

using namespace cocktail;

extern "C" int cocktail_chunk_bitwidths(int32_t batch, int32_t embed_dim, int32_t total_chunks,
                                        const int32_t* chunk_off, const float* query_emb, const float* chunk_emb,
                                        float alpha, float beta, float* scores, uint8_t* chunk_bits, void* stream) {
  if (batch < 1 || embed_dim < 1 || total_chunks < 0)
    return fail(COCKTAIL_EINVAL, "batch and embed_dim must be >= 1, total_chunks >= 0");
  if (!(alpha >= 0.f && alpha <= 1.f) || !(beta >= 0.f && beta <= 1.f))
    return fail(COCKTAIL_EINVAL, "alpha %g and beta %g must lie in [0, 1]", double(alpha), double(beta));
  if (!chunk_off || !query_emb) return fail(COCKTAIL_EINVAL, "chunk_off and query_emb must not be NULL");
  if (total_chunks > 0 && (!chunk_emb || !scores || !chunk_bits))
    return fail(COCKTAIL_EINVAL, "chunk_emb, scores and chunk_bits must not be NULL");
  if ((reinterpret_cast<uintptr_t>(chunk_off) | reinterpret_cast<uintptr_t>(query_emb) |
       reinterpret_cast<uintptr_t>(chunk_emb) | reinterpret_cast<uintptr_t>(scores)) & 3)
    return fail(COCKTAIL_EALIGN, "chunk_off, query_emb, chunk_emb and scores must be 4-byte aligned");
  if (total_chunks == 0) return COCKTAIL_OK;
  hipStream_t st = static_cast<hipStream_t>(stream);
  hipLaunchKernelGGL(similarity_kernel, dim3((total_chunks + 3) / 4), dim3(256), 0, st, query_emb, chunk_emb, chunk_off,
                     batch, embed_dim, total_chunks, scores);
  hipLaunchKernelGGL(assign_bitwidth_kernel, dim3(batch), dim3(256), 0, st, scores, chunk_off, alpha, beta,
                     chunk_bits);
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(COCKTAIL_EHIP, "chunk_bitwidths launch failed: %s", hipGetErrorString(e));
  return COCKTAIL_OK;
}
