// 2-bit V2a (shared library of codebooks) instantiation of the small-batch matrix-core kernel.
#include "xfp_decode_batch.inc.h"

namespace xfp {

hipError_t launch_batch_lib2(const DecodeArgs &a, int M, bool y_f32, float *part, const void *xt, const void *xb,
                             hipStream_t s)
{
    return launch_batch_bits<2, 1>(a, M, y_f32, part, xt, xb, s);
}

}  // namespace xfp
