// One instantiation unit of the persistent decode kernel (decode_impl.h).  The build compiles
// this file once per (loop nest, prediction row groups, weight storage) with
//   -DRNNT_INST_NEST=f|l|s   Algorithm 1 (frame looping), label looping / TDT, or Algorithm 1 for
//                            teams of one utterance (row groups 1 only)
//   -DRNNT_INST_RG=1|2|4     row groups (of 4 utterances) of a team in the prediction stages
//   -DRNNT_INST_WT=f32|bf16|fp8|bf16a|fp8a|fp4a   storage of the packed weights (bf16a: the bfloat16 mode;
//                            fp8a / fp4a: the bfloat16 mode with e4m3- / e2m1-stored weights)
// so that the instances compile in parallel; decode.hip declares the launch functions and
// picks one per call.
#include "decode_impl.h"

#define RNNT_CAT5_(a, b, c, d, e) a##b##c##d##e
#define RNNT_CAT5(a, b, c, d, e) RNNT_CAT5_(a, b, c, d, e)
#define RNNT_NEST_f kFrameLooping
#define RNNT_NEST_l kLabelLooping
#define RNNT_NEST_s kFrameLoopingSingle
#define RNNT_WT_f32 kWeightF32
#define RNNT_WT_bf16 kWeightBf16
#define RNNT_WT_fp8 kWeightFp8
#define RNNT_WT_bf16a kWeightBf16Arith
#define RNNT_WT_fp8a kWeightFp8Bf16Arith
#define RNNT_WT_fp4a kWeightFp4Bf16Arith
#define RNNT_CAT2_(a, b) a##b
#define RNNT_CAT2(a, b) RNNT_CAT2_(a, b)

namespace rnnt {
hipError_t RNNT_CAT5(launch_decode_, RNNT_INST_NEST, RNNT_INST_RG, _, RNNT_INST_WT)(
    const DecodeParams &p, int rgj, hipStream_t stream)
{
    return launch_variant<RNNT_INST_RG, RNNT_CAT2(RNNT_NEST_, RNNT_INST_NEST),
                          RNNT_CAT2(RNNT_WT_, RNNT_INST_WT)>(p, rgj, stream);
}
}  // namespace rnnt
