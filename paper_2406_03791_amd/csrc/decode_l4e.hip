// Instantiates the decode kernels of one loop nest (label looping and TDT) for teams of up to 16
// utterances, packed weights stored as e4m3.
#include "decode_impl.h"

namespace rnnt {
hipError_t launch_decode_l4e(const DecodeParams &p, int rgj, hipStream_t stream)
{
    return launch_variant<4, kLabelLooping, kWeightFp8>(p, rgj, stream);
}
}  // namespace rnnt
