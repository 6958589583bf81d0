// Split-K variant of the streaming kernel (grid z = slice of K, fp32 partial sums).
#include "xfp_decode_stream.inc.h"

namespace xfp {

hipError_t launch_stream_split(int bits, int mode, bool y_f32, const DecodeArgs &a, int slots, hipStream_t s)
{
    return launch_stream_variant<1>(bits, mode, y_f32, a, slots, s);
}

}  // namespace xfp
