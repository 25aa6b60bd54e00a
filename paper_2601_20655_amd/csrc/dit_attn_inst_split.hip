// Instantiations of the plain attention kernel in its decoupled (two-softmax) cross-attention form.
#include "dit_attn_fwd.h"

namespace dit {

hipError_t launch_attn_split(const AttnArgs& a, int D, int qk_op, int pv_op, hipStream_t s) {
#define DIT_SPLIT_CASE(DD, QK, PV) \
    if (D == DD && qk_op == QK && pv_op == PV) return launch_attn_inst<DD, 1, QK, PV, false, true>(a, s);
    DIT_SPLIT_CASE(128, OP_F16, OP_F16)
    DIT_SPLIT_CASE(128, OP_F16, OP_BF16)
    DIT_SPLIT_CASE(128, OP_BF16, OP_F16)
    DIT_SPLIT_CASE(128, OP_BF16, OP_BF16)
    DIT_SPLIT_CASE(64, OP_F16, OP_F16)
    DIT_SPLIT_CASE(64, OP_F16, OP_BF16)
    DIT_SPLIT_CASE(64, OP_BF16, OP_F16)
    DIT_SPLIT_CASE(64, OP_BF16, OP_BF16)
#undef DIT_SPLIT_CASE
    return hipErrorInvalidValue;
}

}  // namespace dit
