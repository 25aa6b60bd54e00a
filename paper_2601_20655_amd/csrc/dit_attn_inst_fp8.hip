// Instantiations of the pipelined kernel with 8-bit (e4m3) score operands: self-attention of one
// sequence per batch entry and packed requests, 32 query rows per wavefront.
#include "dit_attn_fwd_pipe.h"

namespace dit {

hipError_t launch_attn_pipe_fp8(const AttnArgs& a, int D, int pv_op, int nw, hipStream_t s) {
#define DIT_FP8_CASE(DD, PV)                                                                   \
    if (D == DD && pv_op == PV)                                                                 \
        return nw == 8 ? launch_attn_pipe_inst<DD, 1, OP_FP8, PV, 8, false>(a, s)               \
                       : launch_attn_pipe_inst<DD, 1, OP_FP8, PV, 4, false>(a, s);
    DIT_FP8_CASE(128, OP_F16)
    DIT_FP8_CASE(128, OP_BF16)
    DIT_FP8_CASE(64, OP_F16)
    DIT_FP8_CASE(64, OP_BF16)
#undef DIT_FP8_CASE
    return hipErrorInvalidValue;
}

hipError_t launch_attn_pipe_varlen_fp8(const AttnArgs& a, const VarlenTable& vt, int D, int pv_op, int nw,
                                       hipStream_t s) {
#define DIT_FP8_CASE(DD, PV)                                                                   \
    if (D == DD && pv_op == PV)                                                                 \
        return nw == 8 ? launch_attn_pipe_varlen_inst<DD, OP_FP8, PV, 8>(a, vt, s)              \
                       : launch_attn_pipe_varlen_inst<DD, OP_FP8, PV, 4>(a, vt, s);
    DIT_FP8_CASE(128, OP_F16)
    DIT_FP8_CASE(128, OP_BF16)
    DIT_FP8_CASE(64, OP_F16)
    DIT_FP8_CASE(64, OP_BF16)
#undef DIT_FP8_CASE
    return hipErrorInvalidValue;
}

}  // namespace dit
