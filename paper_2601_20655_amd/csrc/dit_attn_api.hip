// C ABI of the library: argument validation, workspace carving, kernel sequencing.
// Every argument check happens before the first launch: a call that returns anything but DIT_ERR_HIP has had
// no effect; DIT_ERR_HIP (a launch failed) may leave workspace and output partly written.
#include <math.h>
#include <stdio.h>
#include <string.h>

#include "../../include/dit_attn.h"
#include "dit_attn_internal.h"

namespace dit {
hipError_t launch_attn_d128_qb1(const AttnArgs&, int, int, bool, hipStream_t);
hipError_t launch_attn_d128_qb2(const AttnArgs&, int, int, bool, hipStream_t);
hipError_t launch_attn_d64_qb1(const AttnArgs&, int, int, bool, hipStream_t);
hipError_t launch_attn_d64_qb2(const AttnArgs&, int, int, bool, hipStream_t);

hipError_t launch_attn_pipe_d128_qb1(const AttnArgs&, int, int, int, hipStream_t);
hipError_t launch_attn_pipe_d128_qb2(const AttnArgs&, int, int, int, hipStream_t);
hipError_t launch_attn_pipe_d64_qb1(const AttnArgs&, int, int, int, hipStream_t);
hipError_t launch_attn_pipe_d64_qb2(const AttnArgs&, int, int, int, hipStream_t);
hipError_t launch_attn_pipe_fp8(const AttnArgs&, int D, int pv_op, int nw, hipStream_t);
hipError_t launch_attn_pipe_varlen_fp8(const AttnArgs&, const VarlenTable&, int D, int pv_op, int nw, hipStream_t);

// Software-pipelined kernel: pre-packed tiles, no key mask beyond the ragged tail.
hipError_t launch_attn_pipe(const AttnArgs& a, int D, int qb, int qk_op, int pv_op, int nw, hipStream_t s) {
    if (qk_op == OP_FP8) return qb == 1 ? launch_attn_pipe_fp8(a, D, pv_op, nw, s) : hipErrorInvalidValue;
    if (D == 128 && qb == 1) return launch_attn_pipe_d128_qb1(a, qk_op, pv_op, nw, s);
    if (D == 128 && qb == 2) return launch_attn_pipe_d128_qb2(a, qk_op, pv_op, nw, s);
    if (D == 64 && qb == 1) return launch_attn_pipe_d64_qb1(a, qk_op, pv_op, nw, s);
    if (D == 64 && qb == 2) return launch_attn_pipe_d64_qb2(a, qk_op, pv_op, nw, s);
    return hipErrorInvalidValue;
}

hipError_t launch_attn(const AttnArgs& a, int D, int qb, int qk_op, int pv_op, bool fused, hipStream_t s) {
    if (D == 128 && qb == 1) return launch_attn_d128_qb1(a, qk_op, pv_op, fused, s);
    if (D == 128 && qb == 2) return launch_attn_d128_qb2(a, qk_op, pv_op, fused, s);
    if (D == 64 && qb == 1) return launch_attn_d64_qb1(a, qk_op, pv_op, fused, s);
    if (D == 64 && qb == 2) return launch_attn_d64_qb2(a, qk_op, pv_op, fused, s);
    return hipErrorInvalidValue;
}
}  // namespace dit

namespace {

static_assert(DIT_MAX_REQUESTS == dit::kMaxRequests, "request limit of the ABI and of the kernel table");

thread_local char g_hip_error[256] = "";
thread_local hipEvent_t g_ev_before = nullptr, g_ev_after = nullptr;

dit_status hip_fail(hipError_t e, const char* where) {
    snprintf(g_hip_error, sizeof(g_hip_error), "%s: %s", where, hipGetErrorString(e));
    return DIT_ERR_HIP;
}

}  // namespace

int dit::report_hip_error(hipError_t e, const char* where) { return hip_fail(e, where); }

namespace {

constexpr size_t kAlign = 256;
size_t round_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

struct Flags {
    int qk_op, pv_op, qb, nw;
    bool fused, simple, pipelined, resident, mfma32;
};

// Resolve flag bits into operand types and staging mode.
dit_status parse_flags(uint32_t f, Flags* out) {
    const uint32_t known = DIT_FLAG_QK_BF16 | DIT_FLAG_QK_F16 | DIT_FLAG_PV_BF16 | DIT_FLAG_PV_F16 |
                           DIT_FLAG_KV_PREPACK | DIT_FLAG_KV_FUSED | DIT_FLAG_WIDE_QTILE |
                           DIT_FLAG_SIMPLE_SCHEDULE | DIT_FLAG_BIG_WORKGROUP | DIT_FLAG_SMALL_WORKGROUP |
                           DIT_FLAG_PIPELINED_SCHEDULE | DIT_FLAG_KV_RESIDENT | DIT_FLAG_QK_FP8 |
                           DIT_FLAG_MFMA_32X32;
    if (f & ~known) return DIT_ERR_INVALID_ARG;
    if ((f & DIT_FLAG_QK_BF16) && (f & DIT_FLAG_QK_F16)) return DIT_ERR_INVALID_ARG;
    if ((f & DIT_FLAG_PV_BF16) && (f & DIT_FLAG_PV_F16)) return DIT_ERR_INVALID_ARG;
    if ((f & DIT_FLAG_KV_PREPACK) && (f & DIT_FLAG_KV_FUSED)) return DIT_ERR_INVALID_ARG;
    if ((f & DIT_FLAG_QK_FP8) && (f & (DIT_FLAG_QK_BF16 | DIT_FLAG_QK_F16))) return DIT_ERR_INVALID_ARG;
    out->qk_op = (f & DIT_FLAG_QK_FP8) ? dit::OP_FP8 : (f & DIT_FLAG_QK_BF16) ? dit::OP_BF16 : dit::OP_F16;
    out->pv_op = (f & DIT_FLAG_PV_BF16) ? dit::OP_BF16 : dit::OP_F16;
    out->fused = (f & DIT_FLAG_KV_FUSED) != 0;
    out->resident = (f & DIT_FLAG_KV_RESIDENT) != 0;
    out->mfma32 = (f & DIT_FLAG_MFMA_32X32) != 0;
    if (out->resident && out->fused) return DIT_ERR_INVALID_ARG;  // FUSED keeps nothing to reuse
    out->qb = (f & DIT_FLAG_WIDE_QTILE) ? 2 : 1;
    if ((f & DIT_FLAG_SIMPLE_SCHEDULE) && (f & DIT_FLAG_PIPELINED_SCHEDULE)) return DIT_ERR_INVALID_ARG;
    out->simple = (f & DIT_FLAG_SIMPLE_SCHEDULE) != 0;
    out->pipelined = (f & DIT_FLAG_PIPELINED_SCHEDULE) != 0;
    if ((f & DIT_FLAG_BIG_WORKGROUP) && (f & DIT_FLAG_SMALL_WORKGROUP)) return DIT_ERR_INVALID_ARG;
    out->nw = (f & DIT_FLAG_BIG_WORKGROUP) ? 8 : (f & DIT_FLAG_SMALL_WORKGROUP) ? 4 : 0;  // 0 = choose by size
    return DIT_OK;
}

// Self-attention (one sequence per batch entry or packed requests) runs the pipelined kernel on 16x16x32 MFMAs
// unless a flag asks for a form that only exists on 32x32x16 MFMAs (8-bit scores, 64 rows per wavefront, the
// plain and fused schedules) or for the 32x32x16 kernel itself.  The V^T tiles are packed in the matching key order.
bool self_attn_uses_mfma16(const Flags& fl) {
    return !fl.fused && !fl.simple && fl.qb == 1 && fl.qk_op != dit::OP_FP8 && !fl.mfma32;
}

// Attention kernel launch, bracketed by the caller's timing events when the hook is set.
dit_status run_attn(const dit::AttnArgs& aa, int D, const Flags& fl, bool fused, bool mfma16, hipStream_t s,
                    bool chain16 = false) {
    const bool timed = g_ev_before && g_ev_after;
    hipError_t e;
    if (timed && (e = hipEventRecord(g_ev_before, s)) != hipSuccess) return hip_fail(e, "hipEventRecord");
    if (aa.tile_count_a) {
        e = dit::launch_attn_split(aa, D, fl.qk_op, fl.pv_op, s);
    } else if (chain16) {
        e = dit::launch_attn_pipe16_chain(aa, D, fl.qk_op, fl.pv_op, fl.nw, s);
    } else if (mfma16) {
        e = dit::launch_attn_pipe16(aa, D, fl.qk_op, fl.pv_op, fl.nw, s);
    } else if (!fused && !fl.simple) {
        e = dit::launch_attn_pipe(aa, D, fl.qb, fl.qk_op, fl.pv_op, fl.nw, s);
    } else {
        e = dit::launch_attn(aa, D, fl.qb, fl.qk_op, fl.pv_op, fused, s);
    }
    if (e != hipSuccess) return hip_fail(e, "attention kernel");
    if (timed && (e = hipEventRecord(g_ev_after, s)) != hipSuccess) return hip_fail(e, "hipEventRecord");
    return DIT_OK;
}

bool dtype_ok(int32_t d) { return d == DIT_BF16 || d == DIT_F32; }

// Rows must start on 16-byte boundaries: base pointer and every stride.
bool aligned16(const void* p, const dit_strides& s, int32_t dtype) {
    const int64_t per16 = dtype == DIT_F32 ? 4 : 8;
    if (reinterpret_cast<uintptr_t>(p) & 15u) return false;
    return s.batch % per16 == 0 && s.token % per16 == 0 && s.head % per16 == 0;
}

// Rows of D contiguous channels may not overlap: a token's and a head's rows are at least D apart, and of the
// two strides the larger one clears all the rows the smaller one steps over ([B,L,H,D]: token >= H*head;
// [B,H,L,D]: head >= L*token).  L = 0 skips the second half (packed requests check their own total).
bool strides_ok(const dit_strides& s, int32_t B, int32_t H, int32_t D, int64_t L) {
    if (s.token < D || s.head < D) return false;
    if (B > 1 && s.batch < D) return false;
    if (s.batch < 0) return false;
    if (H > 1 && L > 1) {
        const bool token_major = s.token >= (int64_t)H * s.head;
        const bool head_major = s.head >= L * s.token;
        if (!token_major && !head_major) return false;
    }
    return true;
}

// eps >= 0, a known mode; the channel weights are read as float4
dit_status norm_ok(const dit_qk_norm& n) {
    if (n.mode != DIT_NORM_NONE && n.mode != DIT_NORM_HEAD && n.mode != DIT_NORM_TOKEN) return DIT_ERR_INVALID_ARG;
    if (n.mode == DIT_NORM_NONE) return DIT_OK;
    if (!(n.eps >= 0.f) || !isfinite(n.eps)) return DIT_ERR_INVALID_ARG;
    if ((reinterpret_cast<uintptr_t>(n.q_gamma) | reinterpret_cast<uintptr_t>(n.k_gamma)) & 15u)
        return DIT_ERR_ALIGNMENT;
    return DIT_OK;
}

// Workspace tail for the per-token multipliers of q and k rows (TOKEN mode only).
size_t rstd_bytes(const dit_qk_norm& n, int64_t q_rows, int64_t k_rows) {
    if (n.mode != DIT_NORM_TOKEN) return 0;
    return round_up((size_t)q_rows * sizeof(float), kAlign) + round_up((size_t)k_rows * sizeof(float), kAlign);
}

// Fills the normalisation arguments of both kernels; in TOKEN mode launches the two statistics passes.
dit_status setup_norm(const dit_qk_norm& n, const void* q, const void* k, const dit_strides& sq, const dit_strides& sk,
                      int B, int Lq, int Lk, int H, int D, int in_f32, uint8_t* rstd_ws, dit::NormArgs* qn,
                      dit::NormArgs* kn, bool k_resident, hipStream_t s) {
    memset(qn, 0, sizeof(*qn));
    memset(kn, 0, sizeof(*kn));
    if (n.mode == DIT_NORM_NONE) return DIT_OK;
    qn->mode = kn->mode = n.mode;
    qn->eps = kn->eps = n.eps;
    qn->gamma = n.q_gamma;
    kn->gamma = n.k_gamma;
    if (n.mode == DIT_NORM_TOKEN) {
        float* rq = reinterpret_cast<float*>(rstd_ws);
        float* rk = reinterpret_cast<float*>(rstd_ws + round_up((size_t)B * Lq * sizeof(float), kAlign));
        dit::RstdArgs ra;
        ra.x = q; ra.rstd = rq; ra.s_b = sq.batch; ra.s_t = sq.token; ra.s_h = sq.head;
        ra.B = B; ra.L = Lq; ra.H = H; ra.D = D; ra.in_f32 = in_f32; ra.eps = n.eps;
        hipError_t e = dit::launch_token_rstd(ra, s);
        if (e != hipSuccess) return hip_fail(e, "token_rstd_kernel");
        if (!k_resident) {  // the key rows' factors only feed the pre-pack pass
            ra.x = k; ra.rstd = rk; ra.s_b = sk.batch; ra.s_t = sk.token; ra.s_h = sk.head; ra.L = Lk;
            e = dit::launch_token_rstd(ra, s);
            if (e != hipSuccess) return hip_fail(e, "token_rstd_kernel");
        }
        qn->rstd = rq;
        kn->rstd = rk;
    }
    return DIT_OK;
}

struct SelfPlan {
    Flags fl;
    int64_t L;
    int nKT, nQT;
    int table_entries;
    size_t tab_off, tiles_off, rstd_off, total;
};

dit_status plan_self(const dit_self_attn_params* p, SelfPlan* pl) {
    if (!p) return DIT_ERR_INVALID_ARG;
    if (p->B < 1 || p->H < 1 || p->D < 1 || p->T < 1 || p->Hg < 1 || p->Wg < 1) return DIT_ERR_INVALID_ARG;
    if (p->D != 64 && p->D != 128) return DIT_ERR_UNSUPPORTED;
    if (p->d_t < 0 || p->d_h < 0 || p->d_w < 0 || ((p->d_t | p->d_h | p->d_w) & 1) ||
        p->d_t + p->d_h + p->d_w != p->D)
        return DIT_ERR_INVALID_ARG;
    if (!(p->rope_base > 0.f) || !isfinite(p->rope_base) || !isfinite(p->scale)) return DIT_ERR_INVALID_ARG;
    if (!dtype_ok(p->in_dtype) || !dtype_ok(p->out_dtype)) return DIT_ERR_INVALID_ARG;
    dit_status st = parse_flags(p->flags, &pl->fl);
    if (st != DIT_OK) return st;
    if ((st = norm_ok(p->norm)) != DIT_OK) return st;
    if (pl->fl.fused && p->norm.mode != DIT_NORM_NONE) return DIT_ERR_UNSUPPORTED;
    const int64_t L = (int64_t)p->T * p->Hg * p->Wg;
    if (L > (1 << 24)) return DIT_ERR_UNSUPPORTED;  // token indices are 32-bit with room for tile padding
    if ((int64_t)p->B * p->H > (1 << 20)) return DIT_ERR_UNSUPPORTED;
    if (pl->fl.fused) {
        // fused staging keeps V in bf16 and is built for head_dim 128 with bf16 inputs only
        if (p->in_dtype != DIT_BF16 || p->D != 128 || pl->fl.pv_op != dit::OP_BF16 ||
            !(p->flags & DIT_FLAG_PV_BF16))
            return DIT_ERR_UNSUPPORTED;
    }
    if (!strides_ok(p->sq, p->B, p->H, p->D, L) || !strides_ok(p->sk, p->B, p->H, p->D, L) ||
        !strides_ok(p->sv, p->B, p->H, p->D, L) || !strides_ok(p->so, p->B, p->H, p->D, L))
        return DIT_ERR_INVALID_ARG;
    pl->L = L;
    pl->nKT = (int)((L + dit::kBK - 1) / dit::kBK);
    if (pl->fl.nw == 8 && pl->fl.qb == 2) return DIT_ERR_UNSUPPORTED;  // would need 512 registers x 512 lanes
    // 8-bit score operands exist in the pipelined 32-rows-per-wavefront kernel only
    if (pl->fl.qk_op == dit::OP_FP8 && (pl->fl.fused || pl->fl.simple || pl->fl.qb == 2)) return DIT_ERR_UNSUPPORTED;
    if (pl->fl.fused || pl->fl.simple || pl->fl.qb == 2) {
        pl->fl.nw = 4;  // only the pipelined 32-rows-per-wavefront kernel has the 8-wavefront form
    } else if (pl->fl.nw == 0) {
        // 8 wavefronts when 256-row workgroups still cover the 256 CUs at least twice over
        pl->fl.nw = ((L + 255) / 256) * p->B * p->H >= 512 ? 8 : 4;
    }
    const int bq = 32 * pl->fl.nw * pl->fl.qb;
    pl->nQT = (int)((L + bq - 1) / bq);
    if ((int64_t)pl->nQT * p->B * p->H > 0x7fffffffLL) return DIT_ERR_UNSUPPORTED;
    if ((int64_t)pl->nKT * p->B * p->H > 0x7fffffffLL) return DIT_ERR_UNSUPPORTED;  // one pre-pack workgroup each
    pl->table_entries = p->T * (p->d_t / 2) + p->Hg * (p->d_h / 2) + p->Wg * (p->d_w / 2);
    pl->tab_off = 0;
    pl->tiles_off = round_up((size_t)pl->table_entries * sizeof(float2), kAlign);
    size_t tiles = pl->fl.fused ? 0 : (size_t)p->B * p->H * pl->nKT * dit::tile_bytes(p->D);
    pl->rstd_off = pl->tiles_off + round_up(tiles, kAlign);
    pl->total = pl->rstd_off + rstd_bytes(p->norm, (int64_t)p->B * L, (int64_t)p->B * L);
    if (pl->total == 0) pl->total = kAlign;
    return DIT_OK;
}

struct VarlenPlan {
    Flags fl;
    dit::VarlenTable vt;
    int maxT, maxHg, maxWg;
    int table_entries;
    size_t tab_off, tiles_off, rstd_off, total;
};

dit_status plan_varlen(const dit_varlen_attn_params* p, VarlenPlan* pl) {
    if (!p || !p->grids) return DIT_ERR_INVALID_ARG;
    if (p->n_requests < 1 || p->H < 1 || p->D < 1) return DIT_ERR_INVALID_ARG;
    if (p->n_requests > DIT_MAX_REQUESTS) return DIT_ERR_UNSUPPORTED;
    if (p->D != 64 && p->D != 128) return DIT_ERR_UNSUPPORTED;
    if (p->d_t < 0 || p->d_h < 0 || p->d_w < 0 || ((p->d_t | p->d_h | p->d_w) & 1) ||
        p->d_t + p->d_h + p->d_w != p->D)
        return DIT_ERR_INVALID_ARG;
    if (!(p->rope_base > 0.f) || !isfinite(p->rope_base) || !isfinite(p->scale)) return DIT_ERR_INVALID_ARG;
    if (!dtype_ok(p->in_dtype) || !dtype_ok(p->out_dtype)) return DIT_ERR_INVALID_ARG;
    dit_status st = parse_flags(p->flags, &pl->fl);
    if (st != DIT_OK) return st;
    if ((st = norm_ok(p->norm)) != DIT_OK) return st;
    // only the pipelined kernel with pre-packed tiles and 32 rows per wavefront has this form
    if (pl->fl.fused || pl->fl.simple || pl->fl.qb == 2) return DIT_ERR_UNSUPPORTED;
    if (p->H > (1 << 16)) return DIT_ERR_UNSUPPORTED;
    if (!strides_ok(p->sq, 1, p->H, p->D, 0) || !strides_ok(p->sk, 1, p->H, p->D, 0) ||
        !strides_ok(p->sv, 1, p->H, p->D, 0) || !strides_ok(p->so, 1, p->H, p->D, 0))
        return DIT_ERR_INVALID_ARG;

    const int n = p->n_requests;
    int64_t Ls[DIT_MAX_REQUESTS], tok0[DIT_MAX_REQUESTS];
    int order[DIT_MAX_REQUESTS];
    int64_t total = 0, big_blocks = 0;
    pl->maxT = pl->maxHg = pl->maxWg = 0;
    for (int i = 0; i < n; ++i) {
        const dit_grid& g = p->grids[i];
        if (g.T < 1 || g.Hg < 1 || g.Wg < 1) return DIT_ERR_INVALID_ARG;
        Ls[i] = (int64_t)g.T * g.Hg * g.Wg;
        if (Ls[i] > (1 << 24)) return DIT_ERR_UNSUPPORTED;
        tok0[i] = total;
        total += Ls[i];
        big_blocks += (Ls[i] + 255) / 256 * p->H;
        if (g.T > pl->maxT) pl->maxT = g.T;
        if (g.Hg > pl->maxHg) pl->maxHg = g.Hg;
        if (g.Wg > pl->maxWg) pl->maxWg = g.Wg;
        order[i] = i;
    }
    if (total > (1 << 24)) return DIT_ERR_UNSUPPORTED;  // token indices are 32-bit with room for tile padding
    if (pl->fl.nw == 0) pl->fl.nw = big_blocks >= 512 ? 8 : 4;
    const int bq = 32 * pl->fl.nw;
    // longest request first (stable, so equal lengths keep the caller's order)
    for (int i = 1; i < n; ++i) {
        const int o = order[i];
        int j = i;
        for (; j > 0 && Ls[order[j - 1]] < Ls[o]; --j) order[j] = order[j - 1];
        order[j] = o;
    }
    dit::VarlenTable& vt = pl->vt;
    memset(&vt, 0, sizeof(vt));
    vt.n = n;
    vt.total_tokens = (int)total;
    int tile0 = 0;
    int64_t queue[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    for (int r = 0; r < n; ++r) {
        const int i = order[r];
        dit::ReqDesc& d = vt.r[r];
        d.tok0 = (int)tok0[i];
        d.L = (int)Ls[i];
        d.Hg = p->grids[i].Hg;
        d.Wg = p->grids[i].Wg;
        d.nKT = (int)((Ls[i] + dit::kBK - 1) / dit::kBK);
        d.nQT = (int)((Ls[i] + bq - 1) / bq);
        d.tile0 = tile0;
        tile0 += d.nKT;
        // the kernel's rule: XCD x takes heads h with (r*H + h) % 8 == x
        for (int x = 0; x < 8; ++x) {
            const int h_first = (x - r * p->H) & 7;
            const int heads = h_first < p->H ? (p->H - h_first + 7) >> 3 : 0;
            queue[x] += (int64_t)heads * d.nQT;
        }
    }
    vt.total_tiles = tile0;
    int64_t qmax = 0;
    for (int x = 0; x < 8; ++x) qmax = queue[x] > qmax ? queue[x] : qmax;
    if (8 * qmax > 0x7fffffffLL || (int64_t)tile0 * p->H > 0x7fffffffLL) return DIT_ERR_UNSUPPORTED;
    vt.queue_len = (int)qmax;

    pl->table_entries = pl->maxT * (p->d_t / 2) + pl->maxHg * (p->d_h / 2) + pl->maxWg * (p->d_w / 2);
    pl->tab_off = 0;
    pl->tiles_off = round_up((size_t)pl->table_entries * sizeof(float2), kAlign);
    pl->rstd_off = pl->tiles_off + round_up((size_t)tile0 * p->H * dit::tile_bytes(p->D), kAlign);
    pl->total = pl->rstd_off + rstd_bytes(p->norm, total, total);
    return DIT_OK;
}

struct CrossPlan {
    Flags fl;
    bool chain16;  // the chained 16x16x32 kernel (joint softmax, default)
    int nKT, nQT;
    int split, nTA;  // decoupled form: first key of the second sequence, tiles of the first (0, 0: joint)
    size_t mask_off, list_off, count_off, count_a_off, keysrc_off, tiles_off, rstd_off, total;
};

dit_status plan_cross(const dit_cross_attn_params* p, CrossPlan* pl) {
    if (!p) return DIT_ERR_INVALID_ARG;
    if (p->B < 1 || p->H < 1 || p->D < 1 || p->Lq < 1 || p->Lk < 1) return DIT_ERR_INVALID_ARG;
    if (p->D != 64 && p->D != 128) return DIT_ERR_UNSUPPORTED;
    if (!isfinite(p->scale)) return DIT_ERR_INVALID_ARG;
    if (!dtype_ok(p->in_dtype) || !dtype_ok(p->out_dtype)) return DIT_ERR_INVALID_ARG;
    dit_status st = parse_flags(p->flags, &pl->fl);
    if (st != DIT_OK) return st;
    if (pl->fl.fused) return DIT_ERR_UNSUPPORTED;
    if ((st = norm_ok(p->norm)) != DIT_OK) return st;
    if (p->Lq > (1 << 24) || p->Lk > (1 << 24) || (int64_t)p->B * p->H > (1 << 20)) return DIT_ERR_UNSUPPORTED;
    if (!strides_ok(p->sq, p->B, p->H, p->D, p->Lq) || !strides_ok(p->sk, p->B, p->H, p->D, p->Lk) ||
        !strides_ok(p->sv, p->B, p->H, p->D, p->Lk) || !strides_ok(p->so, p->B, p->H, p->D, p->Lq))
        return DIT_ERR_INVALID_ARG;
    if (p->Lk_split < 0 || p->Lk_split > p->Lk) return DIT_ERR_INVALID_ARG;
    pl->split = (p->Lk_split == p->Lk) ? 0 : p->Lk_split;  // a split at either end is the joint softmax
    pl->nTA = (pl->split + dit::kBK - 1) / dit::kBK;
    pl->nKT = pl->nTA + (p->Lk - pl->split + dit::kBK - 1) / dit::kBK;
    if (pl->fl.qk_op == dit::OP_FP8) return DIT_ERR_UNSUPPORTED;  // self-attention only
    if (pl->split > 0 && (pl->fl.pipelined || pl->fl.qb == 2)) return DIT_ERR_UNSUPPORTED;
    if (pl->fl.nw == 8 && pl->fl.qb == 2) return DIT_ERR_UNSUPPORTED;
    // the pipelined kernel keeps the list of non-empty tiles in the 64 lanes of a wavefront
    if (pl->fl.pipelined && pl->nKT > 64) return DIT_ERR_UNSUPPORTED;
    // Default for one joint softmax: the pipelined 16x16x32 kernel, each workgroup chaining several query tiles.
    // The plain kernel serves the decoupled form and DIT_FLAG_SIMPLE_SCHEDULE (also with DIT_FLAG_MFMA_32X32
    // or 64 rows per wavefront); DIT_FLAG_PIPELINED_SCHEDULE asks for the listed 32x32x16 pipelined kernel.
    // (the chained kernel takes 16-bit query rows, normalised or not: fp32 rows go to the plain kernel)
    pl->chain16 = pl->split == 0 && !pl->fl.simple && !pl->fl.pipelined && !pl->fl.mfma32 && pl->fl.qb == 1 &&
                  p->in_dtype == DIT_BF16;
    if (!pl->fl.pipelined && !pl->chain16) pl->fl.simple = true;
    if (pl->chain16) {
        if (pl->fl.nw == 0) pl->fl.nw = (int64_t)((p->Lq + 255) / 256) * p->B * p->H >= 512 ? 8 : 4;
    } else if (pl->fl.simple || pl->fl.qb == 2) {
        pl->fl.nw = 4;
    } else if (pl->fl.nw == 0) {
        // few key tiles per query tile: two small workgroups per CU overlap each other's
        // prologue and epilogue better than one large workgroup saves on tile traffic (measured)
        pl->fl.nw = 4;
    }
    const int bq = 32 * pl->fl.nw * pl->fl.qb;
    pl->nQT = (p->Lq + bq - 1) / bq;
    if ((int64_t)pl->nQT * p->B * p->H > 0x7fffffffLL) return DIT_ERR_UNSUPPORTED;
    if ((int64_t)pl->nKT * p->B * p->H > 0x7fffffffLL) return DIT_ERR_UNSUPPORTED;
    // workspace: per-tile key masks, compacted list of non-empty tiles, their count, the source key of
    // every tile slot, tile images
    pl->mask_off = 0;
    pl->list_off = round_up((size_t)p->B * pl->nKT * sizeof(uint64_t), kAlign);
    pl->count_off = pl->list_off + round_up((size_t)p->B * pl->nKT * sizeof(int), kAlign);
    pl->count_a_off = pl->count_off + round_up((size_t)p->B * sizeof(int), kAlign);
    pl->keysrc_off = pl->count_a_off + round_up((size_t)p->B * sizeof(int), kAlign);
    pl->tiles_off = pl->keysrc_off + round_up((size_t)p->B * pl->nKT * dit::kBK * sizeof(int), kAlign);
    pl->rstd_off = pl->tiles_off + round_up((size_t)p->B * p->H * pl->nKT * dit::tile_bytes(p->D), kAlign);
    pl->total = pl->rstd_off + rstd_bytes(p->norm, (int64_t)p->B * p->Lq, (int64_t)p->B * p->Lk);
    return DIT_OK;
}

}  // namespace

extern "C" {

size_t dit_attn_workspace_bytes(const dit_self_attn_params* p) {
    SelfPlan pl;
    return plan_self(p, &pl) == DIT_OK ? pl.total : 0;
}

size_t dit_cross_attn_workspace_bytes(const dit_cross_attn_params* p) {
    CrossPlan pl;
    return plan_cross(p, &pl) == DIT_OK ? pl.total : 0;
}

dit_status dit_attn_forward(const void* q, const void* k, const void* v, void* out, float* lse,
                            const dit_self_attn_params* p, void* workspace, size_t workspace_bytes,
                            void* stream) {
    SelfPlan pl;
    dit_status st = plan_self(p, &pl);
    if (st != DIT_OK) return st;
    if (!q || !out) return DIT_ERR_INVALID_ARG;
    if (!pl.fl.resident && (!k || !v)) return DIT_ERR_INVALID_ARG;
    if (!aligned16(q, p->sq, p->in_dtype) || !aligned16(out, p->so, p->out_dtype)) return DIT_ERR_ALIGNMENT;
    if (!pl.fl.resident && (!aligned16(k, p->sk, p->in_dtype) || !aligned16(v, p->sv, p->in_dtype)))
        return DIT_ERR_ALIGNMENT;
    if (lse && (reinterpret_cast<uintptr_t>(lse) & 3u)) return DIT_ERR_ALIGNMENT;
    if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & (kAlign - 1)) || workspace_bytes < pl.total)
        return DIT_ERR_WORKSPACE;

    hipStream_t s = static_cast<hipStream_t>(stream);
    uint8_t* ws = static_cast<uint8_t*>(workspace);

    dit::RopeGeom rg;
    rg.hd[0] = p->d_t / 2; rg.hd[1] = p->d_h / 2; rg.hd[2] = p->d_w / 2;
    rg.off[0] = 0; rg.off[1] = p->T * rg.hd[0]; rg.off[2] = rg.off[1] + p->Hg * rg.hd[1];
    rg.Hg = p->Hg; rg.Wg = p->Wg;

    dit::TableArgs ta;
    ta.tab = reinterpret_cast<float2*>(ws + pl.tab_off);
    ta.n[0] = p->T; ta.n[1] = p->Hg; ta.n[2] = p->Wg;
    ta.origin[0] = p->t0; ta.origin[1] = p->h0; ta.origin[2] = p->w0;
    ta.rg = rg;
    ta.base = (double)p->rope_base;
    ta.total = pl.table_entries;
    hipError_t e = hipSuccess;
    if (!pl.fl.resident) {
        e = dit::launch_rope_table(ta, s);
        if (e != hipSuccess) return hip_fail(e, "rope_table_kernel");
    }

    const float scale = p->scale > 0.f ? p->scale : 1.0f / sqrtf((float)p->D);

    dit::NormArgs qn, kn;
    st = setup_norm(p->norm, q, k, p->sq, p->sk, p->B, (int)pl.L, (int)pl.L, p->H, p->D, p->in_dtype == DIT_F32,
                    ws + pl.rstd_off, &qn, &kn, pl.fl.resident, s);
    if (st != DIT_OK) return st;

    if (!pl.fl.fused && !pl.fl.resident) {
        dit::PackArgs pa;
        memset(&pa, 0, sizeof(pa));
        pa.kn = kn;
        pa.k = k; pa.v = v; pa.valid = nullptr;
        pa.tiles = ws + pl.tiles_off;
        pa.tile_mask = nullptr;
        pa.tab = ta.tab;
        pa.B = p->B; pa.H = p->H; pa.Lk = (int)pl.L; pa.nKT = pl.nKT;
        pa.in_f32 = p->in_dtype == DIT_F32;
        pa.v_layout = self_attn_uses_mfma16(pl.fl) ? 1 : 0;
        pa.sk_b = p->sk.batch; pa.sk_t = p->sk.token; pa.sk_h = p->sk.head;
        pa.sv_b = p->sv.batch; pa.sv_t = p->sv.token; pa.sv_h = p->sv.head;
        pa.rg = rg;
        e = dit::launch_prepack(pa, p->D, pl.fl.qk_op, pl.fl.pv_op, s);
        if (e != hipSuccess) return hip_fail(e, "kv_prepack_kernel");
    }

    dit::AttnArgs aa;
    memset(&aa, 0, sizeof(aa));
    aa.q = q; aa.out = out; aa.lse = lse;
    aa.tiles = pl.fl.fused ? nullptr : ws + pl.tiles_off;
    aa.tile_mask = nullptr;
    aa.tab = ta.tab;
    aa.k = k; aa.v = v;
    aa.sk_b = p->sk.batch; aa.sk_t = p->sk.token; aa.sk_h = p->sk.head;
    aa.sv_b = p->sv.batch; aa.sv_t = p->sv.token; aa.sv_h = p->sv.head;
    aa.B = p->B; aa.H = p->H; aa.Lq = (int)pl.L; aa.Lk = (int)pl.L; aa.nKT = pl.nKT; aa.nQT = pl.nQT;
    aa.in_f32 = p->in_dtype == DIT_F32; aa.out_f32 = p->out_dtype == DIT_F32;
    aa.sq_b = p->sq.batch; aa.sq_t = p->sq.token; aa.sq_h = p->sq.head;
    aa.so_b = p->so.batch; aa.so_t = p->so.token; aa.so_h = p->so.head;
    aa.rg = rg;
    aa.qscale = scale * dit::kLog2e;
    aa.qn = qn;
    return run_attn(aa, p->D, pl.fl, pl.fl.fused, self_attn_uses_mfma16(pl.fl), s);
}

}  // extern "C"

namespace {

// Both cross-attention entry points: which keys attend comes as a byte mask (kv_valid, nullable) or as two counts
// per request (kv_len with second_start; use_len).
dit_status cross_forward(const void* q, const void* k, const void* v, const uint8_t* kv_valid, bool use_len,
                         const int32_t* kv_len, int32_t second_start, void* out, float* lse,
                         const dit_cross_attn_params* p, void* workspace, size_t workspace_bytes, void* stream) {
    CrossPlan pl;
    dit_status st = plan_cross(p, &pl);
    if (st != DIT_OK) return st;
    if (use_len) {
        if (second_start < 0 || second_start > p->Lk) return DIT_ERR_INVALID_ARG;
        if (pl.split > 0 && second_start != pl.split) return DIT_ERR_INVALID_ARG;
        if (!pl.fl.resident && !kv_len) return DIT_ERR_INVALID_ARG;
        if (kv_len && (reinterpret_cast<uintptr_t>(kv_len) & 3u)) return DIT_ERR_ALIGNMENT;
    }
    if (!q || !out) return DIT_ERR_INVALID_ARG;
    if (!pl.fl.resident && (!k || !v)) return DIT_ERR_INVALID_ARG;
    if (!aligned16(q, p->sq, p->in_dtype) || !aligned16(out, p->so, p->out_dtype)) return DIT_ERR_ALIGNMENT;
    if (!pl.fl.resident && (!aligned16(k, p->sk, p->in_dtype) || !aligned16(v, p->sv, p->in_dtype)))
        return DIT_ERR_ALIGNMENT;
    if (lse && (reinterpret_cast<uintptr_t>(lse) & 3u)) return DIT_ERR_ALIGNMENT;
    if (lse && pl.split > 0) return DIT_ERR_UNSUPPORTED;  // two softmaxes have no single log-sum-exp
    if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & (kAlign - 1)) || workspace_bytes < pl.total)
        return DIT_ERR_WORKSPACE;

    hipStream_t s = static_cast<hipStream_t>(stream);
    uint8_t* ws = static_cast<uint8_t*>(workspace);
    const float scale = p->scale > 0.f ? p->scale : 1.0f / sqrtf((float)p->D);

    dit::NormArgs qn, kn;
    st = setup_norm(p->norm, q, k, p->sq, p->sk, p->B, p->Lq, p->Lk, p->H, p->D, p->in_dtype == DIT_F32,
                    ws + pl.rstd_off, &qn, &kn, pl.fl.resident, s);
    if (st != DIT_OK) return st;

    dit::PackArgs pa;
    memset(&pa, 0, sizeof(pa));
    pa.kn = kn;
    pa.k = k; pa.v = v; pa.valid = kv_valid;
    pa.tiles = ws + pl.tiles_off;
    pa.tile_mask = reinterpret_cast<uint64_t*>(ws + pl.mask_off);
    pa.tile_list = reinterpret_cast<int*>(ws + pl.list_off);
    pa.tile_count = reinterpret_cast<int*>(ws + pl.count_off);
    pa.tile_count_a = pl.split > 0 ? reinterpret_cast<int*>(ws + pl.count_a_off) : nullptr;
    pa.key_src = kv_valid ? reinterpret_cast<int*>(ws + pl.keysrc_off) : nullptr;
    pa.kv_len = use_len ? kv_len : nullptr;
    pa.second_start = second_start;
    pa.split = pl.split;
    pa.nTA = pl.nTA;
    pa.tab = nullptr;
    pa.v_layout = pl.chain16 ? 1 : 0;
    pa.B = p->B; pa.H = p->H; pa.Lk = p->Lk; pa.nKT = pl.nKT;
    pa.in_f32 = p->in_dtype == DIT_F32;
    pa.sk_b = p->sk.batch; pa.sk_t = p->sk.token; pa.sk_h = p->sk.head;
    pa.sv_b = p->sv.batch; pa.sv_t = p->sv.token; pa.sv_h = p->sv.head;
    if (!pl.fl.resident) {
        hipError_t e = hipSuccess;
        if (pa.key_src && (e = dit::launch_key_compact(pa, s)) != hipSuccess) return hip_fail(e, "key_compact_kernel");
        e = dit::launch_prepack(pa, p->D, pl.fl.qk_op, pl.fl.pv_op, s);
        if (e != hipSuccess) return hip_fail(e, "kv_prepack_kernel");
        if (!pa.kv_len) {  // (with key counts the pre-pack writes the tile list itself)
            e = dit::launch_tile_compact(pa, s);
            if (e != hipSuccess) return hip_fail(e, "tile_compact_kernel");
        }
    }

    dit::AttnArgs aa;
    memset(&aa, 0, sizeof(aa));
    aa.q = q; aa.out = out; aa.lse = lse;
    aa.tiles = pa.tiles;
    aa.tile_mask = pa.tile_mask;
    aa.tile_list = pa.tile_list;
    aa.tile_count = pa.tile_count;
    aa.tile_count_a = pa.tile_count_a;
    aa.tab = nullptr;
    aa.B = p->B; aa.H = p->H; aa.Lq = p->Lq; aa.Lk = p->Lk; aa.nKT = pl.nKT; aa.nQT = pl.nQT;
    aa.in_f32 = p->in_dtype == DIT_F32; aa.out_f32 = p->out_dtype == DIT_F32;
    aa.sq_b = p->sq.batch; aa.sq_t = p->sq.token; aa.sq_h = p->sq.head;
    aa.so_b = p->so.batch; aa.so_t = p->so.token; aa.so_h = p->so.head;
    aa.qscale = scale * dit::kLog2e;
    aa.qn = qn;
    return run_attn(aa, p->D, pl.fl, false, false, s, pl.chain16);
}

}  // namespace

extern "C" {

dit_status dit_cross_attn_forward(const void* q, const void* k, const void* v, const uint8_t* kv_valid,
                                  void* out, float* lse, const dit_cross_attn_params* p, void* workspace,
                                  size_t workspace_bytes, void* stream) {
    return cross_forward(q, k, v, kv_valid, false, nullptr, 0, out, lse, p, workspace, workspace_bytes, stream);
}

dit_status dit_cross_attn_forward_lengths(const void* q, const void* k, const void* v, const int32_t* kv_len,
                                          int32_t second_start, void* out, float* lse,
                                          const dit_cross_attn_params* p, void* workspace, size_t workspace_bytes,
                                          void* stream) {
    return cross_forward(q, k, v, nullptr, true, kv_len, second_start, out, lse, p, workspace, workspace_bytes,
                         stream);
}

size_t dit_attn_varlen_workspace_bytes(const dit_varlen_attn_params* p) {
    VarlenPlan pl;
    return plan_varlen(p, &pl) == DIT_OK ? pl.total : 0;
}

dit_status dit_attn_varlen_forward(const void* q, const void* k, const void* v, void* out, float* lse,
                                   const dit_varlen_attn_params* p, void* workspace, size_t workspace_bytes,
                                   void* stream) {
    VarlenPlan pl;
    dit_status st = plan_varlen(p, &pl);
    if (st != DIT_OK) return st;
    if (!q || !out) return DIT_ERR_INVALID_ARG;
    if (!pl.fl.resident && (!k || !v)) return DIT_ERR_INVALID_ARG;
    if (!aligned16(q, p->sq, p->in_dtype) || !aligned16(out, p->so, p->out_dtype)) return DIT_ERR_ALIGNMENT;
    if (!pl.fl.resident && (!aligned16(k, p->sk, p->in_dtype) || !aligned16(v, p->sv, p->in_dtype)))
        return DIT_ERR_ALIGNMENT;
    if (lse && (reinterpret_cast<uintptr_t>(lse) & 3u)) return DIT_ERR_ALIGNMENT;
    if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & (kAlign - 1)) || workspace_bytes < pl.total)
        return DIT_ERR_WORKSPACE;

    hipStream_t s = static_cast<hipStream_t>(stream);
    uint8_t* ws = static_cast<uint8_t*>(workspace);

    // one table for all requests, long enough for the largest extent on each axis
    dit::RopeGeom rg;
    rg.hd[0] = p->d_t / 2; rg.hd[1] = p->d_h / 2; rg.hd[2] = p->d_w / 2;
    rg.off[0] = 0; rg.off[1] = pl.maxT * rg.hd[0]; rg.off[2] = rg.off[1] + pl.maxHg * rg.hd[1];
    rg.Hg = pl.maxHg; rg.Wg = pl.maxWg;  // replaced per request inside the kernels

    dit::TableArgs ta;
    ta.tab = reinterpret_cast<float2*>(ws + pl.tab_off);
    ta.n[0] = pl.maxT; ta.n[1] = pl.maxHg; ta.n[2] = pl.maxWg;
    ta.origin[0] = p->t0; ta.origin[1] = p->h0; ta.origin[2] = p->w0;
    ta.rg = rg;
    ta.base = (double)p->rope_base;
    ta.total = pl.table_entries;
    hipError_t e = hipSuccess;
    if (!pl.fl.resident) {
        e = dit::launch_rope_table(ta, s);
        if (e != hipSuccess) return hip_fail(e, "rope_table_kernel");
    }

    const float scale = p->scale > 0.f ? p->scale : 1.0f / sqrtf((float)p->D);

    dit::NormArgs qn, kn;
    dit_strides sq1 = p->sq, sk1 = p->sk;
    sq1.batch = sk1.batch = 0;
    st = setup_norm(p->norm, q, k, sq1, sk1, 1, pl.vt.total_tokens, pl.vt.total_tokens, p->H, p->D,
                    p->in_dtype == DIT_F32, ws + pl.rstd_off, &qn, &kn, pl.fl.resident, s);
    if (st != DIT_OK) return st;

    dit::PackArgs pa;
    memset(&pa, 0, sizeof(pa));
    pa.kn = kn;
    pa.k = k; pa.v = v;
    pa.tiles = ws + pl.tiles_off;
    pa.tab = ta.tab;
    pa.B = 1; pa.H = p->H; pa.Lk = pl.vt.total_tokens; pa.nKT = pl.vt.total_tiles;
    pa.in_f32 = p->in_dtype == DIT_F32;
    pa.v_layout = self_attn_uses_mfma16(pl.fl) ? 1 : 0;
    pa.sk_t = p->sk.token; pa.sk_h = p->sk.head;
    pa.sv_t = p->sv.token; pa.sv_h = p->sv.head;
    pa.rg = rg;
    if (!pl.fl.resident) {
        e = dit::launch_prepack_varlen(pa, pl.vt, p->D, pl.fl.qk_op, pl.fl.pv_op, s);
        if (e != hipSuccess) return hip_fail(e, "kv_prepack_varlen_kernel");
    }

    dit::AttnArgs aa;
    memset(&aa, 0, sizeof(aa));
    aa.q = q; aa.out = out; aa.lse = lse;
    aa.tiles = pa.tiles;
    aa.tab = ta.tab;
    aa.B = 1; aa.H = p->H; aa.Lq = pl.vt.total_tokens; aa.Lk = pl.vt.total_tokens;
    aa.nKT = pl.vt.total_tiles; aa.nQT = 0;
    aa.in_f32 = p->in_dtype == DIT_F32; aa.out_f32 = p->out_dtype == DIT_F32;
    aa.sq_t = p->sq.token; aa.sq_h = p->sq.head;
    aa.so_t = p->so.token; aa.so_h = p->so.head;
    aa.rg = rg;
    aa.qscale = scale * dit::kLog2e;
    aa.qn = qn;

    const bool timed = g_ev_before && g_ev_after;
    if (timed && (e = hipEventRecord(g_ev_before, s)) != hipSuccess) return hip_fail(e, "hipEventRecord");
    e = pl.fl.qk_op == dit::OP_FP8
            ? dit::launch_attn_pipe_varlen_fp8(aa, pl.vt, p->D, pl.fl.pv_op, pl.fl.nw, s)
            : self_attn_uses_mfma16(pl.fl)
                  ? dit::launch_attn_pipe16_varlen(aa, pl.vt, p->D, pl.fl.qk_op, pl.fl.pv_op, pl.fl.nw, s)
                  : dit::launch_attn_pipe_varlen(aa, pl.vt, p->D, pl.fl.qk_op, pl.fl.pv_op, pl.fl.nw, s);
    if (e != hipSuccess) return hip_fail(e, "attention kernel");
    if (timed && (e = hipEventRecord(g_ev_after, s)) != hipSuccess) return hip_fail(e, "hipEventRecord");
    return DIT_OK;
}

dit_status dit_linear_forward(const void* x, const void* w, const void* bias, void* y, const dit_linear_params* p,
                              void* stream) {
    if (!x || !w || !y || !p) return DIT_ERR_INVALID_ARG;
    if (p->M < 1 || p->N < 1 || p->K < 1 || p->flags != 0) return DIT_ERR_INVALID_ARG;
    if (p->ldx < p->K || p->ldw < p->K || p->ldy < p->N) return DIT_ERR_INVALID_ARG;
    if (p->out_dtype != DIT_BF16 && p->out_dtype != DIT_F32) return DIT_ERR_INVALID_ARG;
    if (p->K % dit::kLinBK != 0 || p->N % 8 != 0) return DIT_ERR_UNSUPPORTED;
    // the kernel addresses the rows of one 256-row tile with 32-bit byte offsets
    if (p->ldx > (int64_t)1 << 22 || p->ldw > (int64_t)1 << 22) return DIT_ERR_UNSUPPORTED;
    const size_t ye = p->out_dtype == DIT_F32 ? 4 : 2;
    if ((uintptr_t)x % 16 || (uintptr_t)w % 16 || (uintptr_t)y % 16 || (p->ldx * 2) % 16 || (p->ldw * 2) % 16 ||
        (p->ldy * ye) % 16 || (uintptr_t)bias % 8)
        return DIT_ERR_ALIGNMENT;
    dit::LinearArgs a{};
    a.x = static_cast<const uint16_t*>(x);
    a.w = static_cast<const uint16_t*>(w);
    a.bias = static_cast<const uint16_t*>(bias);
    a.y = y;
    a.M = p->M;
    a.N = p->N;
    a.K = p->K;
    a.ldx = p->ldx;
    a.ldw = p->ldw;
    a.ldy = p->ldy;
    a.nTM = (p->M + dit::kLinBM - 1) / dit::kLinBM;
    a.nTN = (p->N + dit::kLinBN - 1) / dit::kLinBN;
    a.out_f32 = p->out_dtype == DIT_F32;
    if ((int64_t)a.nTM * a.nTN > 0x7fffffff) return DIT_ERR_UNSUPPORTED;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const bool timed = g_ev_before && g_ev_after;
    hipError_t e;
    if (timed && (e = hipEventRecord(g_ev_before, s)) != hipSuccess) return hip_fail(e, "hipEventRecord");
    e = dit::launch_linear(a, s);
    if (e != hipSuccess) return hip_fail(e, "linear_kernel");
    if (timed && (e = hipEventRecord(g_ev_after, s)) != hipSuccess) return hip_fail(e, "hipEventRecord");
    return DIT_OK;
}

dit_status dit_qkv_proj_forward(const void* x, const void* w, const void* bias, void* q_out,
                                const dit_linear_params* lp, const dit_self_attn_params* ap, void* workspace,
                                size_t workspace_bytes, void* stream) {
    if (!x || !w || !q_out || !lp || !ap) return DIT_ERR_INVALID_ARG;
    SelfPlan pl;
    dit_status st = plan_self(ap, &pl);
    if (st != DIT_OK) return st;
    // what the fused form covers: one sequence, head_dim 128, an even number of heads (a 256-feature tile is two
    // heads of one of q, k, v), 16-bit rows, the default attention kernel's tile images.  Of the q/k normalisations
    // the per-head one is done in the epilogue (a head's channels are inside a tile); the per-token one takes a second
    // pass over the K' images, because a token-wide mean spans every tile of the k part.
    if (ap->B != 1 || ap->D != 128 || (ap->H & 1) || ap->in_dtype != DIT_BF16 || !self_attn_uses_mfma16(pl.fl) ||
        pl.fl.resident)
        return DIT_ERR_UNSUPPORTED;
    if (lp->flags != 0 || lp->out_dtype != DIT_BF16) return DIT_ERR_INVALID_ARG;
    if (lp->M != pl.L || lp->N != 3 * (int64_t)ap->H * ap->D || lp->K < 1) return DIT_ERR_INVALID_ARG;
    if (lp->ldx < lp->K || lp->ldw < lp->K) return DIT_ERR_INVALID_ARG;
    if (lp->K % dit::kLinBK != 0) return DIT_ERR_UNSUPPORTED;
    if (lp->ldx > (int64_t)1 << 22 || lp->ldw > (int64_t)1 << 22) return DIT_ERR_UNSUPPORTED;
    if ((uintptr_t)x % 16 || (uintptr_t)w % 16 || (lp->ldx * 2) % 16 || (lp->ldw * 2) % 16 || (uintptr_t)bias % 8)
        return DIT_ERR_ALIGNMENT;
    if (!aligned16(q_out, ap->sq, DIT_BF16)) return DIT_ERR_ALIGNMENT;
    if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & (kAlign - 1)) || workspace_bytes < pl.total)
        return DIT_ERR_WORKSPACE;

    hipStream_t s = static_cast<hipStream_t>(stream);
    uint8_t* ws = static_cast<uint8_t*>(workspace);
    dit::RopeGeom rg;
    rg.hd[0] = ap->d_t / 2; rg.hd[1] = ap->d_h / 2; rg.hd[2] = ap->d_w / 2;
    rg.off[0] = 0; rg.off[1] = ap->T * rg.hd[0]; rg.off[2] = rg.off[1] + ap->Hg * rg.hd[1];
    rg.Hg = ap->Hg; rg.Wg = ap->Wg;
    dit::TableArgs ta;
    ta.tab = reinterpret_cast<float2*>(ws + pl.tab_off);
    ta.n[0] = ap->T; ta.n[1] = ap->Hg; ta.n[2] = ap->Wg;
    ta.origin[0] = ap->t0; ta.origin[1] = ap->h0; ta.origin[2] = ap->w0;
    ta.rg = rg;
    ta.base = (double)ap->rope_base;
    ta.total = pl.table_entries;
    hipError_t e = dit::launch_rope_table(ta, s);
    if (e != hipSuccess) return hip_fail(e, "rope_table_kernel");

    dit::LinearArgs a{};
    a.x = static_cast<const uint16_t*>(x);
    a.w = static_cast<const uint16_t*>(w);
    a.bias = static_cast<const uint16_t*>(bias);
    a.y = q_out;
    a.M = lp->M;
    a.N = lp->N;
    a.K = lp->K;
    a.ldx = lp->ldx;
    a.ldw = lp->ldw;
    a.ldy = 0;
    a.nTM = (lp->M + dit::kLinBM - 1) / dit::kLinBM;
    a.nTN = lp->N / dit::kLinBN;
    a.out_f32 = 0;
    a.qkv = 1;
    a.qkv_H = ap->H;
    a.qkv_nKT = pl.nKT;
    a.qkv_tiles = ws + pl.tiles_off;
    a.qkv_tab = ta.tab;
    a.qkv_rg = rg;
    a.qkv_sq_t = ap->sq.token;
    a.qkv_sq_h = ap->sq.head;
    a.qkv_qk_f16 = pl.fl.qk_op == dit::OP_F16;
    a.qkv_pv_f16 = pl.fl.pv_op == dit::OP_F16;
    a.qkv_norm = ap->norm.mode == DIT_NORM_HEAD ? 1 : ap->norm.mode == DIT_NORM_TOKEN ? 2 : 0;
    a.qkv_eps = ap->norm.eps;
    a.qkv_kgamma = ap->norm.k_gamma;
    if ((int64_t)a.nTM * a.nTN > 0x7fffffff) return DIT_ERR_UNSUPPORTED;
    const bool timed = g_ev_before && g_ev_after;
    if (timed && (e = hipEventRecord(g_ev_before, s)) != hipSuccess) return hip_fail(e, "hipEventRecord");
    e = dit::launch_linear(a, s);
    if (e != hipSuccess) return hip_fail(e, "linear_kernel");
    if (timed && (e = hipEventRecord(g_ev_after, s)) != hipSuccess) return hip_fail(e, "hipEventRecord");
    if (ap->norm.mode == DIT_NORM_TOKEN) {
        dit::KRescaleArgs ra;
        ra.tiles = a.qkv_tiles;
        ra.H = ap->H;
        ra.nKT = pl.nKT;
        ra.L = (int)pl.L;
        ra.eps = ap->norm.eps;
        ra.qk_f16 = a.qkv_qk_f16;
        e = dit::launch_k_rescale(ra, s);
        if (e != hipSuccess) return hip_fail(e, "k_rescale_kernel");
    }
    return DIT_OK;
}

void dit_attn_set_timing_events(void* before, void* after) {
    g_ev_before = static_cast<hipEvent_t>(before);
    g_ev_after = static_cast<hipEvent_t>(after);
}

const char* dit_strerror(dit_status s) {
    switch (s) {
        case DIT_OK: return "ok";
        case DIT_ERR_INVALID_ARG: return "invalid argument";
        case DIT_ERR_UNSUPPORTED: return "unsupported shape or flag combination";
        case DIT_ERR_ALIGNMENT: return "pointer or stride breaks 16-byte row alignment";
        case DIT_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
        case DIT_ERR_HIP: return "HIP runtime error";
    }
    return "unknown status";
}

const char* dit_last_hip_error(void) { return g_hip_error; }

int dit_attn_version(void) { return 10500; }  // 1.5.0

}  // extern "C"
