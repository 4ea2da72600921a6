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

}  // namespace cocktail
