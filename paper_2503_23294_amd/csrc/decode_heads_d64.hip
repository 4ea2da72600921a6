// The one-query-head-per-kv-head decode kernel at head_dim 64 (see decode_heads_impl.h).
#include "decode_heads_impl.h"

namespace cocktail {
template hipError_t launch_decode_heads<64>(const DecodeParams&, int, bool, bool, int, hipStream_t);
}
