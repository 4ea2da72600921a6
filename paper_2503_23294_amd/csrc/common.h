// Internal helpers shared by the translation units of libcocktail.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/cocktail.h"

namespace cocktail {

// Records a message for cocktail_last_error() and returns `code`.
int fail(int code, const char* fmt, ...) __attribute__((format(printf, 2, 3)));

// Validates the geometry common to all entry points.
int check_shape(const cocktail_shape* s);

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef _Float16 h2 __attribute__((ext_vector_type(2)));

// Reinterpret a dword as two halves.  Always goes through a by-value scalar:
// __builtin_bit_cast applied directly to a vector element expression (v[i], v.x)
// reads element 0 with this compiler.
__host__ __device__ inline h2 as_h2(uint32_t u) { return __builtin_bit_cast(h2, u); }
__host__ __device__ inline uint32_t as_u32(h2 v) { return __builtin_bit_cast(uint32_t, v); }

#ifdef __HIPCC__
// Reads a plan record through the scalar data path: the records are written by the host only, and
// every wave reads them at a wave-uniform address, so they can go straight into scalar registers.
template <class T>
__device__ __forceinline__ T load_record(const T* p) {
  static_assert(sizeof(T) % 4 == 0, "records are made of 32-bit fields");
  struct Words {
    int32_t w[sizeof(T) / 4];
  } tmp;
  const auto* src = reinterpret_cast<const __attribute__((address_space(4))) int32_t*>(reinterpret_cast<uint64_t>(p));
#pragma unroll
  for (size_t i = 0; i < sizeof(T) / 4; ++i) tmp.w[i] = src[i];
  return __builtin_bit_cast(T, tmp);
}
#endif

}  // namespace cocktail
