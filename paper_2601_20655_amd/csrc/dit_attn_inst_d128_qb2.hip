// Instantiations of the attention kernel for head_dim 128, 2 query block(s) per wavefront.
#include "dit_attn_fwd_pipe.h"

namespace dit {

hipError_t launch_attn_d128_qb2(const AttnArgs& a, int qk_op, int pv_op, bool fused, hipStream_t s) {
    if (!fused) {
        if (qk_op == OP_F16 && pv_op == OP_F16) return launch_attn_inst<128, 2, OP_F16, OP_F16, false>(a, s);
        if (qk_op == OP_F16 && pv_op == OP_BF16) return launch_attn_inst<128, 2, OP_F16, OP_BF16, false>(a, s);
        if (qk_op == OP_BF16 && pv_op == OP_F16) return launch_attn_inst<128, 2, OP_BF16, OP_F16, false>(a, s);
        if (qk_op == OP_BF16 && pv_op == OP_BF16) return launch_attn_inst<128, 2, OP_BF16, OP_BF16, false>(a, s);
    }
    if (fused && pv_op == OP_BF16) {
        if (qk_op == OP_F16) return launch_attn_inst<128, 2, OP_F16, OP_BF16, true>(a, s);
        if (qk_op == OP_BF16) return launch_attn_inst<128, 2, OP_BF16, OP_BF16, true>(a, s);
    }
    return hipErrorInvalidValue;
}

hipError_t launch_attn_pipe_d128_qb2(const AttnArgs& a, int qk_op, int pv_op, int nw, hipStream_t s) {
    const bool listed = a.tile_mask != nullptr;
#define DIT_PIPE_CASE(QK, PV)                                                                       \
    if (qk_op == QK && pv_op == PV) {                                                                \
        if (listed)                                                                                  \
            return nw == 8 ? launch_attn_pipe_inst<128, 2, QK, PV, 8, true>(a, s)                     \
                           : launch_attn_pipe_inst<128, 2, QK, PV, 4, true>(a, s);                    \
        return nw == 8 ? launch_attn_pipe_inst<128, 2, QK, PV, 8, false>(a, s)                        \
                       : launch_attn_pipe_inst<128, 2, QK, PV, 4, false>(a, s);                       \
    }
    DIT_PIPE_CASE(OP_F16, OP_F16)
    DIT_PIPE_CASE(OP_F16, OP_BF16)
    DIT_PIPE_CASE(OP_BF16, OP_F16)
    DIT_PIPE_CASE(OP_BF16, OP_BF16)
#undef DIT_PIPE_CASE
    return hipErrorInvalidValue;
}

}  // namespace dit
