// Streaming kernel for V2a tensors with a scale and a mid-point per group (paper section 3.4): the plain
// variant instantiated in MODE 2, in a translation unit of its own so that the build stays parallel.
#include "xfp_decode_stream.inc.h"

namespace xfp {

hipError_t launch_stream_affine(int bits, bool y_f32, const DecodeArgs &a, int slots, hipStream_t s)
{
    if (!a.gscale || !a.gmid || a.fuse_half || a.k_slices) return hipErrorInvalidValue;
    return launch_stream_aff(bits, y_f32, a, slots, s);
}

}  // namespace xfp
