// Instantiates the decode kernels of one loop nest (label looping and TDT) for teams of up to 8
// utterances, packed weights stored as fp32.
#include "decode_impl.h"

namespace rnnt {
hipError_t launch_decode_l2(const DecodeParams &p, int rgj, hipStream_t stream)
{
    return launch_variant<2, kLabelLooping, kWeightF32>(p, rgj, stream);
}
}  // namespace rnnt
