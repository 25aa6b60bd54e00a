// Instantiations of the pipelined self-attention kernel on 16x16x32 MFMAs: one sequence per batch entry and
// packed requests.
#include "dit_attn_fwd_pipe16.h"

namespace dit {

#define DIT_PIPE16_CASES(X) \
    X(128, OP_F16, OP_F16)   \
    X(128, OP_F16, OP_BF16)  \
    X(128, OP_BF16, OP_F16)  \
    X(128, OP_BF16, OP_BF16) \
    X(64, OP_F16, OP_F16)    \
    X(64, OP_F16, OP_BF16)   \
    X(64, OP_BF16, OP_F16)   \
    X(64, OP_BF16, OP_BF16)

hipError_t launch_attn_pipe16(const AttnArgs& a, int D, int qk_op, int pv_op, int nw, hipStream_t s) {
#define DIT_CASE(DD, QK, PV)                                                \
    if (D == DD && qk_op == QK && pv_op == PV)                               \
        return nw == 8 ? launch_attn_pipe16_inst<DD, QK, PV, 8>(a, s) : launch_attn_pipe16_inst<DD, QK, PV, 4>(a, s);
    DIT_PIPE16_CASES(DIT_CASE)
#undef DIT_CASE
    return hipErrorInvalidValue;
}

hipError_t launch_attn_pipe16_chain(const AttnArgs& a, int D, int qk_op, int pv_op, int nw, hipStream_t s) {
#define DIT_CASE(DD, QK, PV)                                 \
    if (D == DD && qk_op == QK && pv_op == PV)                \
        return nw == 8 ? launch_attn_pipe16_chain_inst<DD, QK, PV, 8>(a, s) \
                       : launch_attn_pipe16_chain_inst<DD, QK, PV, 4>(a, s);
    DIT_PIPE16_CASES(DIT_CASE)
#undef DIT_CASE
    return hipErrorInvalidValue;
}

hipError_t launch_attn_pipe16_varlen(const AttnArgs& a, const VarlenTable& vt, int D, int qk_op, int pv_op, int nw,
                                     hipStream_t s) {
#define DIT_CASE(DD, QK, PV)                                                            \
    if (D == DD && qk_op == QK && pv_op == PV)                                           \
        return nw == 8 ? launch_attn_pipe16_varlen_inst<DD, QK, PV, 8>(a, vt, s)         \
                       : launch_attn_pipe16_varlen_inst<DD, QK, PV, 4>(a, vt, s);
    DIT_PIPE16_CASES(DIT_CASE)
#undef DIT_CASE
    return hipErrorInvalidValue;
}

}  // namespace dit
