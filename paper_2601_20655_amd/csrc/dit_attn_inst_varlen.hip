// Instantiations of the pipelined kernel for packed requests of different lengths.
#include "dit_attn_fwd_pipe.h"

namespace dit {

hipError_t launch_attn_pipe_varlen(const AttnArgs& a, const VarlenTable& vt, int D, int qk_op, int pv_op, int nw,
                                   hipStream_t s) {
#define DIT_VARLEN_CASE(DD, QK, PV)                                                          \
    if (D == DD && qk_op == QK && pv_op == PV)                                                \
        return nw == 8 ? launch_attn_pipe_varlen_inst<DD, QK, PV, 8>(a, vt, s)                \
                       : launch_attn_pipe_varlen_inst<DD, QK, PV, 4>(a, vt, s);
    DIT_VARLEN_CASE(128, OP_F16, OP_F16)
    DIT_VARLEN_CASE(128, OP_F16, OP_BF16)
    DIT_VARLEN_CASE(128, OP_BF16, OP_F16)
    DIT_VARLEN_CASE(128, OP_BF16, OP_BF16)
    DIT_VARLEN_CASE(64, OP_F16, OP_F16)
    DIT_VARLEN_CASE(64, OP_F16, OP_BF16)
    DIT_VARLEN_CASE(64, OP_BF16, OP_F16)
    DIT_VARLEN_CASE(64, OP_BF16, OP_BF16)
#undef DIT_VARLEN_CASE
    return hipErrorInvalidValue;
}

}  // namespace dit
