// The grouped-query decode kernel at head_dim 64 (see decode_quads_impl.h).
#include "decode_quads_impl.h"

namespace cocktail {
template hipError_t launch_decode_quads<64>(const DecodeParams&, int, bool, bool, int, hipStream_t);
}
