// Instantiates the decode kernels of one loop nest (Algorithm 1) for teams of up to 4
// utterances, packed weights stored as bf16.
#include "decode_impl.h"

namespace rnnt {
hipError_t launch_decode_f1b(const DecodeParams &p, int rgj, hipStream_t stream)
{
    return launch_variant<1, kFrameLooping, kWeightBf16>(p, rgj, stream);
}
}  // namespace rnnt
