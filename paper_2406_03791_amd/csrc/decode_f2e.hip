// Instantiates the decode kernels of one loop nest (Algorithm 1) for teams of up to 8
// utterances, packed weights stored as e4m3.
#include "decode_impl.h"

namespace rnnt {
hipError_t launch_decode_f2e(const DecodeParams &p, int rgj, hipStream_t stream)
{
    return launch_variant<2, kFrameLooping, kWeightFp8>(p, rgj, stream);
}
}  // namespace rnnt
