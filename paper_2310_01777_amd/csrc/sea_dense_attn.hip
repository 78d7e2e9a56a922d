// Dense (quadratic) softmax attention baseline, tile by tile with no T x T buffer.
#include "sea_internal.h"

namespace sea {

hipError_t launch_dense_attn(const Shape&, sea_dtype, const void*, const void*, const void*, void*,
                             hipStream_t) {
  return hipErrorNotSupported;
}

}  // namespace sea
