// Gate/up variant of the streaming kernel: SiLU(gate) * up applied in the store.
#include "xfp_decode_stream.inc.h"

namespace xfp {

hipError_t launch_stream_fused(int bits, int mode, bool y_f32, const DecodeArgs &a, int slots, hipStream_t s)
{
    return launch_stream_variant<2>(bits, mode, y_f32, a, slots, s);
}

}  // namespace xfp
