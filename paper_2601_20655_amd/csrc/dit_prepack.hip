// Memory-bound helper kernels that run before the attention kernel on the same stream:
//  * rope_table_kernel: (cos, sin) of every (axis, position, pair) angle, evaluated in fp64
//    and stored as fp32, so that the rotation itself never calls a transcendental.
//  * kv_prepack_kernel: rotates K, rounds K' and V once to the MFMA operand types (16-bit, or for
//    K' 8-bit E4M3 with one power-of-two factor per row) and writes each 64-key tile as the exact
//    byte image the attention kernel keeps in LDS (K' rows, then V^T rows with keys permuted into
//    the order the PV product consumes).
#include "dit_attn_device.h"

namespace dit {

__global__ void __launch_bounds__(256) rope_table_kernel(const TableArgs a) {
    const int idx = blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= a.total) return;
    int ax = 0;
    if (idx >= a.rg.off[2]) ax = 2;
    else if (idx >= a.rg.off[1]) ax = 1;
    const int local = idx - a.rg.off[ax];
    const int hd = a.rg.hd[ax];
    const int p = local / hd, i = local - p * hd;
    // angle = position * base^(-2i/d_a) with d_a = 2*hd
    const double omega = pow(a.base, -(double)i / (double)hd);
    const double phi = (double)(a.origin[ax] + p) * omega;
    a.tab[idx] = make_float2((float)cos(phi), (float)sin(phi));
}

hipError_t launch_rope_table(const TableArgs& a, hipStream_t s) {
    if (a.total <= 0) return hipSuccess;
    hipLaunchKernelGGL(rope_table_kernel, dim3((a.total + 255) / 256), dim3(256), 0, s, a);
    return hipGetLastError();
}

// One workgroup per token: 1/sqrt(mean of x^2 over all H*D channels + eps).
__global__ void __launch_bounds__(256) token_rstd_kernel(const RstdArgs a) {
    __shared__ float part[4];
    const int64_t row = blockIdx.x;
    const int b = (int)(row / a.L), n = (int)(row - (int64_t)b * a.L);
    const int cpr = a.D / 8, chunks = a.H * cpr;
    const int64_t base = (int64_t)b * a.s_b + (int64_t)n * a.s_t;
    float ss = 0.f;
    for (int i = threadIdx.x; i < chunks; i += 256) {
        const int h = i / cpr, c = i - h * cpr;
        float x[8];
        load8(a.x, base + (int64_t)h * a.s_h + 8 * c, a.in_f32, x);
#pragma unroll
        for (int e = 0; e < 8; ++e) ss = fmaf(x[e], x[e], ss);
    }
#pragma unroll
    for (int m = 1; m < 64; m <<= 1) ss += __shfl_xor(ss, m);
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = ss;
    __syncthreads();
    if (threadIdx.x == 0) {
        const float tot = (part[0] + part[1]) + (part[2] + part[3]);
        a.rstd[row] = 1.0f / sqrtf(tot / (float)(a.H * a.D) + a.eps);
    }
}

hipError_t launch_token_rstd(const RstdArgs& a, hipStream_t s) {
    hipLaunchKernelGGL(token_rstd_kernel, dim3((unsigned)((int64_t)a.B * a.L)), dim3(256), 0, s, a);
    return hipGetLastError();
}

// One workgroup per (tile, group of up to kRescaleHeads heads): four lanes a key row.  The lanes of a row first add
// up the heads' shares of the row's sum of squares, each lane every fourth head and then the four partial sums in a
// fixed order, so that every workgroup -- whichever heads it then scales -- arrives at the same factor for a token.
constexpr int kRescaleHeads = 8;
__global__ void __launch_bounds__(256) k_rescale_kernel(const KRescaleArgs a) {
    using G = TileGeom<128>;
    const int groups = (a.H + kRescaleHeads - 1) / kRescaleHeads;
    const int hg = blockIdx.x % groups, j = blockIdx.x / groups;
    const int r = threadIdx.x >> 2, part = threadIdx.x & 3;
    const int tok = j * kBK + r;
    const bool live = tok < a.L;  // slots past the sequence hold zeros and stay as they are
    float ssq = 0.f;
    for (int hh = part; hh < a.H; hh += 4)
        ssq += reinterpret_cast<const float*>(a.tiles + ((size_t)hh * a.nKT + j) * G::TILE_BYTES + kBK * G::KROW)[r];
    ssq += __shfl_xor(ssq, 1);
    ssq += __shfl_xor(ssq, 2);
    const float rs = 1.0f / sqrtf(ssq / (float)(a.H * 128) + a.eps);
    if (!live) return;
    const int h_end = (hg + 1) * kRescaleHeads < a.H ? (hg + 1) * kRescaleHeads : a.H;
    for (int h = hg * kRescaleHeads; h < h_end; ++h) {
        // chunk 4 c + part: the four lanes of a row move 64 contiguous bytes per instruction
        uint8_t* const row = a.tiles + ((size_t)h * a.nKT + j) * G::TILE_BYTES + r * G::KROW + part * 16;
        u32x4 v[4];
#pragma unroll
        for (int c = 0; c < 4; ++c) v[c] = *reinterpret_cast<const u32x4*>(row + c * 64);
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            float x[8];
            if (a.qk_f16) {
                const uint32_t w[4] = {v[c].x, v[c].y, v[c].z, v[c].w};
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const f16x2 p = __builtin_bit_cast(f16x2, w[e]);
                    x[2 * e] = (float)p.x;
                    x[2 * e + 1] = (float)p.y;
                }
            } else {
                widen8(v[c], x);
            }
#pragma unroll
            for (int e = 0; e < 8; ++e) x[e] *= rs;
            *reinterpret_cast<u32x4*>(row + c * 64) = a.qk_f16 ? pack8<OP_F16>(x) : pack8<OP_BF16>(x);
        }
        // the pad behind the row too, so that the pass leaves no sector partly written (see pack_tile)
        if (part == 3) *reinterpret_cast<u32x4*>(row + 256 - 48) = mk4(0u, 0u, 0u, 0u);
    }
}

hipError_t launch_k_rescale(const KRescaleArgs& a, hipStream_t s) {
    const int groups = (a.H + kRescaleHeads - 1) / kRescaleHeads;
    hipLaunchKernelGGL(k_rescale_kernel, dim3((unsigned)(groups * a.nKT)), dim3(256), 0, s, a);
    return hipGetLastError();
}

// What one workgroup packs: 64 keys of one (batch or request, head).
struct PackTile {
    uint8_t* dst;        // tile image
    int64_t k_off, v_off;  // element offset of key 0 of this sequence for this head
    int key0, key_end;   // keys [key0, key0 + 64) clipped to key_end
    const int* key_src;  // if set: slot r holds key key_src[r] (-1: empty) instead of key0 + r
    // ranges (key counts instead of a mask): slot i = slot0 + r of the tile sequence holds key sa + i if i < la,
    // key sb + (i - la) if i - la < lb, else nothing
    bool ranges;
    int slot0, la, sa, lb, sb;
    RopeGeom rg;         // with this sequence's grid
    int h;               // head (channel weights of the normalisation)
    int64_t stat_off;    // index of key 0 in the per-token normalisation table
};

template <int D, int QK_OP, int PV_OP>
__device__ __forceinline__ void pack_tile(const PackArgs& a, const PackTile& t, uint16_t* vs) {
    using G = TileGeom<D>;
    constexpr int CPR = D / 8;
    constexpr int ROWS_PER_PASS = kThreads / CPR;
    constexpr int NI = kBK / ROWS_PER_PASS;
    constexpr int VS = D + 2;  // padded row of the transposition buffer, in 16-bit elements
    const int tid = threadIdx.x;
    const int c = tid % CPR;

#pragma unroll
    for (int i = 0; i < NI; ++i) {
        const int r = tid / CPR + i * ROWS_PER_PASS;
        int key;
        bool ok;
        if (t.ranges) {
            const int i_ = t.slot0 + r;
            key = i_ < t.la ? t.sa + i_ : (i_ - t.la < t.lb ? t.sb + (i_ - t.la) : -1);
            ok = key >= 0;
        } else {
            key = t.key_src ? t.key_src[r] : t.key0 + r;
            ok = t.key_src ? key >= 0 : key < t.key_end;
        }
        float xk[8], xv[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) xk[e] = xv[e] = 0.f;
        if (ok) {
            load8(a.k, t.k_off + (int64_t)key * a.sk_t + 8 * c, a.in_f32, xk);
            load8(a.v, t.v_off + (int64_t)key * a.sv_t + 8 * c, a.in_f32, xv);
        }
        if (a.kn.mode) {  // the CPR neighbouring lanes that share a row add up its squares
            float rs;
            if (a.kn.mode == 2) {
                rs = ok ? a.kn.rstd[t.stat_off + key] : 0.f;
            } else {
                float ss = 0.f;
#pragma unroll
                for (int e = 0; e < 8; ++e) ss = fmaf(xk[e], xk[e], ss);
#pragma unroll
                for (int m = 1; m < CPR; m <<= 1) ss += __shfl_xor(ss, m);
                rs = 1.0f / sqrtf(ss * (1.0f / D) + a.kn.eps);
            }
            if (ok) norm8(xk, a.kn, rs, t.h, D, c);
        }
        if (ok) {
            if (a.tab) {
                int pt, ph, pw;
                token_pos(key, t.rg, pt, ph, pw);
                rope8(xk, c, t.rg, a.tab, pt, ph, pw);
            }
        }
        if constexpr (QK_OP == OP_FP8) {
            // one power-of-two factor per key row brings its largest magnitude into [128, 256)
            float am = 0.f;
#pragma unroll
            for (int e = 0; e < 8; ++e) am = fmaxf(am, fabsf(xk[e]));
#pragma unroll
            for (int m = 1; m < CPR; m <<= 1) am = fmaxf(am, __shfl_xor(am, m));
            const int ex = fp8_row_exponent(am);
            const float sc = pow2i(ex);
#pragma unroll
            for (int e = 0; e < 8; ++e) xk[e] *= sc;
            // chunk c = channels [8c, 8c+8) goes where the lane that multiplies it against the same
            // channels of q' finds it: contraction step c / 8, lane half c % 2, slot (c / 2) % 4
            const int off = (c >> 3) * 64 + (c & 1) * 32 + ((c >> 1) & 3) * 8;
            *reinterpret_cast<uint2*>(t.dst + r * G::KROW8 + off) = pack8_fp8(xk);
            if (c == CPR - 1) *reinterpret_cast<u32x4*>(t.dst + r * G::KROW8 + D) = mk4(0u, 0u, 0u, 0u);  // the pad, see below
            if (c == 0) t.dst[G::KSCALE_OFF + r] = (uint8_t)(127 - ex);
        } else {
            // (layout 1: rows 4..11 of every 16 keep their 16-byte chunks in swapped pairs, see below)
            const int cs = a.v_layout ? c ^ (((r >> 2) ^ (r >> 3)) & 1) : c;
            *reinterpret_cast<u32x4*>(t.dst + r * G::KROW + cs * 16) = pack8<QK_OP>(xk);
            // the 16 pad bytes behind the row are written too (zeros): a part is then a run of fully written
            // 32-byte sectors, and none of them has to be read back from memory to be completed
            if (c == CPR - 1) *reinterpret_cast<u32x4*>(t.dst + r * G::KROW + D * 2) = mk4(0u, 0u, 0u, 0u);
        }
        const u32x4 pv = pack8<PV_OP>(xv);
        uint32_t* row = reinterpret_cast<uint32_t*>(vs + r * VS + 8 * c);
        row[0] = pv.x; row[1] = pv.y; row[2] = pv.z; row[3] = pv.w;
    }
    __syncthreads();

    // V^T chunk (d, kc) = eight key slots, in the order the attention kernel's PV operand wants its keys:
    //  32x32x16 MFMAs (v_layout 0): slot 4g+e holds key 16*(kc/2) + 8g + 4*(kc%2) + e of the tile;
    //  16x16x32 MFMAs (v_layout 1): slot 4g+e holds key 32*(kc/4) + 16g + 4*(kc%4) + e.
#pragma unroll
    for (int i = 0; i < D / 32; ++i) {
        const int d = (tid >> 3) + 32 * i;
        const int kc = tid & 7;
        const int k0 = a.v_layout ? 32 * (kc >> 2) + 4 * (kc & 3) : 16 * (kc >> 1) + 4 * (kc & 1);
        const int kstep = a.v_layout ? 16 : 8;
        uint32_t w[4];
#pragma unroll
        for (int g = 0; g < 2; ++g)
#pragma unroll
            for (int e2 = 0; e2 < 2; ++e2) {
                const int ka = k0 + kstep * g + 2 * e2;
                w[2 * g + e2] = (uint32_t)vs[ka * VS + d] | ((uint32_t)vs[(ka + 1) * VS + d] << 16);
            }
        // Layout 1, both parts: in rows 4..11 of every 16, neighbouring chunks 2n and 2n+1 change places.  A
        // 16x16x32 operand read has lane 16 g + i fetch chunk g of row i, and the LDS serves the 64 lanes of a
        // 128-bit read in four cycles of four lane quads each: quads {0,3,5,6}, {1,2,4,7}, {8,11,13,14},
        // {9,10,12,15} (found by letting two lanes at a time read one bank and watching the conflict counter).
        // With plain rows two lanes of every cycle meet in one bank (every operand read then takes 8 LDS cycles
        // instead of 4); with the swap each cycle's 16 lanes cover the 16 bank groups once.
        const int kcs = a.v_layout ? kc ^ (((d >> 2) ^ (d >> 3)) & 1) : kc;
        *reinterpret_cast<u32x4*>(t.dst + G::K_BYTES + d * G::VROW + kcs * 16) = mk4(w[0], w[1], w[2], w[3]);
        if (kc == 7) *reinterpret_cast<u32x4*>(t.dst + G::K_BYTES + d * G::VROW + kBK * 2) = mk4(0u, 0u, 0u, 0u);
    }
}

// One workgroup per (tile, head, batch).
template <int D, int QK_OP, int PV_OP>
__global__ void __launch_bounds__(kThreads) kv_prepack_kernel(const PackArgs a) {
    using G = TileGeom<D>;
    __shared__ __attribute__((aligned(16))) uint16_t vs[kBK * (D + 2)];
    const int tid = threadIdx.x;
    // heads vary fastest: neighbouring workgroups read neighbouring 256-byte pieces of the same 64 tokens
    const int h = blockIdx.x % a.H, jb = blockIdx.x / a.H, j = jb % a.nKT, b = jb / a.nKT;
    PackTile t;
    t.dst = a.tiles + ((size_t)(b * a.H + h) * a.nKT + j) * G::TILE_BYTES;
    t.k_off = (int64_t)b * a.sk_b + (int64_t)h * a.sk_h;
    t.v_off = (int64_t)b * a.sv_b + (int64_t)h * a.sv_h;
    // keys of this tile: [key0, key0 + 64) clipped to key_end (two key groups when split > 0)
    const bool second = a.split > 0 && j >= a.nTA;
    t.key0 = second ? a.split + (j - a.nTA) * kBK : j * kBK;
    t.key_end = (a.split > 0 && !second) ? a.split : a.Lk;
    t.key_src = a.key_src ? a.key_src + ((size_t)b * a.nKT + j) * kBK : nullptr;
    t.ranges = a.kv_len != nullptr;
    t.slot0 = t.la = t.sa = t.lb = t.sb = 0;
    int ca = 0, cb = 0;  // ranges: tiles that hold a key, first and second key group (decoupled) or all (joint: ca)
    if (t.ranges) {
        // counts are clamped to the ranges they count in: whatever the caller wrote, every key index stays inside k, v
        const int end0 = a.split > 0 ? a.split : a.second_start;
        int len0 = a.kv_len[2 * b], len1 = a.kv_len[2 * b + 1];
        len0 = len0 < 0 ? 0 : (len0 > end0 ? end0 : len0);
        len1 = len1 < 0 ? 0 : (len1 > a.Lk - a.second_start ? a.Lk - a.second_start : len1);
        if (a.split > 0) {  // two key groups, each in tiles of its own
            t.slot0 = (second ? j - a.nTA : j) * kBK;
            t.la = second ? len1 : len0;
            t.sa = second ? a.split : 0;
            ca = (len0 + kBK - 1) / kBK;
            cb = (len1 + kBK - 1) / kBK;
        } else {  // one softmax: the second range follows the first densely
            t.slot0 = j * kBK;
            t.la = len0; t.sa = 0; t.lb = len1; t.sb = a.second_start;
            ca = (len0 + len1 + kBK - 1) / kBK;
        }
    }
    t.rg = a.rg;
    t.h = h;
    t.stat_off = (int64_t)b * a.Lk;
    pack_tile<D, QK_OP, PV_OP>(a, t, vs);

    if (a.tile_mask && h == 0 && tid < 64) {
        bool ok;
        if (t.ranges) ok = t.slot0 + tid < t.la + t.lb;
        else ok = t.key_src ? t.key_src[tid] >= 0 : t.key0 + tid < t.key_end;
        const uint64_t m = __ballot(ok);
        if (tid == 0) {
            a.tile_mask[(size_t)b * a.nKT + j] = m;
            if (t.ranges) {
                // the list of tiles that hold a key and its counts, which tile_compact_kernel otherwise derives from the masks
                const int jj = second ? j - a.nTA : j;
                if (m != 0ull) a.tile_list[(size_t)b * a.nKT + (second ? ca + jj : jj)] = j;
                if (j == 0) {
                    a.tile_count[b] = ca + cb;
                    if (a.tile_count_a) a.tile_count_a[b] = ca;
                }
            }
        }
    }
}

// Packed requests: one workgroup per (tile of any request, head).
template <int D, int QK_OP, int PV_OP>
__global__ void __launch_bounds__(kThreads) kv_prepack_varlen_kernel(const PackArgs a, const VarlenTable vt) {
    using G = TileGeom<D>;
    __shared__ __attribute__((aligned(16))) uint16_t vs[kBK * (D + 2)];
    const int h = blockIdx.x % a.H, gj = blockIdx.x / a.H;
    int r = 0;
    while (r + 1 < vt.n && gj >= vt.r[r + 1].tile0) ++r;
    const ReqDesc& q = vt.r[r];
    const int j = gj - q.tile0;
    PackTile t;
    t.dst = a.tiles + ((size_t)q.tile0 * a.H + (size_t)h * q.nKT + j) * G::TILE_BYTES;
    t.k_off = (int64_t)q.tok0 * a.sk_t + (int64_t)h * a.sk_h;
    t.v_off = (int64_t)q.tok0 * a.sv_t + (int64_t)h * a.sv_h;
    t.key0 = j * kBK;
    t.key_end = q.L;
    t.key_src = nullptr;
    t.ranges = false;
    t.rg = a.rg;
    t.rg.Hg = q.Hg;
    t.rg.Wg = q.Wg;
    t.h = h;
    t.stat_off = q.tok0;
    pack_tile<D, QK_OP, PV_OP>(a, t, vs);
}

// Key padding masks: one wavefront per (batch entry, key group) writes the group's valid keys, in
// ascending order, densely into the slots of the group's tiles; the slots left over get -1.  Attention
// does not depend on the order of the keys, so the padded keys cost no tile: a request keeps
// ceil(valid keys / 64) tiles per group whatever the positions of its padding.
__global__ void __launch_bounds__(64) key_compact_kernel(const uint8_t* valid, int* key_src, int Lk, int nKT,
                                                         int split, int nTA) {
    const int b = blockIdx.x, g = blockIdx.y, lane = threadIdx.x;
    const int k0 = g == 0 ? 0 : split, k1 = (g == 0 && split > 0) ? split : Lk;
    const int t0 = g == 0 ? 0 : nTA, t1 = (g == 0 && split > 0) ? nTA : nKT;
    int* out = key_src + ((size_t)b * nKT + t0) * kBK;
    int count = 0;
    for (int base = k0; base < k1; base += 64) {
        const int key = base + lane;
        const bool ok = key < k1 && valid[(size_t)b * Lk + key] != 0;
        const uint64_t m = __ballot(ok);
        if (ok) out[count + __popcll(m & ((1ull << lane) - 1ull))] = key;
        count += __popcll(m);
    }
    for (int i = count + lane; i < (t1 - t0) * kBK; i += 64) out[i] = -1;
}

hipError_t launch_key_compact(const PackArgs& a, hipStream_t s) {
    hipLaunchKernelGGL(key_compact_kernel, dim3(a.B, a.split > 0 ? 2 : 1), dim3(64), 0, s, a.valid, a.key_src, a.Lk,
                       a.nKT, a.split, a.nTA);
    return hipGetLastError();
}

// One wavefront per batch entry: tile_list[b] = ascending indices of tiles whose key mask is not empty.
__global__ void __launch_bounds__(64) tile_compact_kernel(const uint64_t* tile_mask, int* tile_list,
                                                          int* tile_count, int* tile_count_a, int nKT, int nTA) {
    const int b = blockIdx.x, lane = threadIdx.x;
    const uint64_t* m = tile_mask + (size_t)b * nKT;
    int* out = tile_list + (size_t)b * nKT;
    int count = 0, count_a = 0;
    for (int base = 0; base < nKT; base += 64) {
        const int t = base + lane;
        const bool keep = t < nKT && m[t] != 0ull;
        const uint64_t votes = __ballot(keep);
        if (keep) out[count + __popcll(votes & ((1ull << lane) - 1ull))] = t;
        count += __popcll(votes);
        count_a += __popcll(__ballot(keep && t < nTA));
    }
    if (lane == 0) {
        tile_count[b] = count;
        if (tile_count_a) tile_count_a[b] = count_a;
    }
}

hipError_t launch_tile_compact(const PackArgs& a, hipStream_t s) {
    hipLaunchKernelGGL(tile_compact_kernel, dim3(a.B), dim3(64), 0, s, a.tile_mask, a.tile_list, a.tile_count,
                       a.tile_count_a, a.nKT, a.nTA);
    return hipGetLastError();
}

template <int D, int QK_OP, int PV_OP>
static hipError_t launch_prepack_inst(const PackArgs& a, hipStream_t s) {
    hipLaunchKernelGGL((kv_prepack_kernel<D, QK_OP, PV_OP>), dim3((unsigned)((int64_t)a.H * a.nKT * a.B)), dim3(kThreads), 0, s, a);
    return hipGetLastError();
}

hipError_t launch_prepack_varlen(const PackArgs& a, const VarlenTable& vt, int D, int qk_op, int pv_op, hipStream_t s) {
#define DIT_PACKV_CASE(DD, QK, PV)                                                                        \
    if (D == DD && qk_op == QK && pv_op == PV) {                                                           \
        hipLaunchKernelGGL((kv_prepack_varlen_kernel<DD, QK, PV>), dim3((unsigned)((int64_t)a.H * vt.total_tiles)), dim3(kThreads), 0, \
                           s, a, vt);                                                                      \
        return hipGetLastError();                                                                          \
    }
    DIT_PACKV_CASE(128, OP_F16, OP_F16)
    DIT_PACKV_CASE(128, OP_F16, OP_BF16)
    DIT_PACKV_CASE(128, OP_BF16, OP_F16)
    DIT_PACKV_CASE(128, OP_BF16, OP_BF16)
    DIT_PACKV_CASE(64, OP_F16, OP_F16)
    DIT_PACKV_CASE(64, OP_F16, OP_BF16)
    DIT_PACKV_CASE(64, OP_BF16, OP_F16)
    DIT_PACKV_CASE(64, OP_BF16, OP_BF16)
    DIT_PACKV_CASE(128, OP_FP8, OP_F16)
    DIT_PACKV_CASE(128, OP_FP8, OP_BF16)
    DIT_PACKV_CASE(64, OP_FP8, OP_F16)
    DIT_PACKV_CASE(64, OP_FP8, OP_BF16)
#undef DIT_PACKV_CASE
    return hipErrorInvalidValue;
}

hipError_t launch_prepack(const PackArgs& a, int D, int qk_op, int pv_op, hipStream_t s) {
#define DIT_PACK_CASE(DD, QK, PV) \
    if (D == DD && qk_op == QK && pv_op == PV) return launch_prepack_inst<DD, QK, PV>(a, s);
    DIT_PACK_CASE(128, OP_F16, OP_F16)
    DIT_PACK_CASE(128, OP_F16, OP_BF16)
    DIT_PACK_CASE(128, OP_BF16, OP_F16)
    DIT_PACK_CASE(128, OP_BF16, OP_BF16)
    DIT_PACK_CASE(64, OP_F16, OP_F16)
    DIT_PACK_CASE(64, OP_F16, OP_BF16)
    DIT_PACK_CASE(64, OP_BF16, OP_F16)
    DIT_PACK_CASE(64, OP_BF16, OP_BF16)
    DIT_PACK_CASE(128, OP_FP8, OP_F16)
    DIT_PACK_CASE(128, OP_FP8, OP_BF16)
    DIT_PACK_CASE(64, OP_FP8, OP_F16)
    DIT_PACK_CASE(64, OP_FP8, OP_BF16)
#undef DIT_PACK_CASE
    return hipErrorInvalidValue;
}

}  // namespace dit
