// Flash-style attention forward for gfx950: S^T = K' Q'^T and O^T = V^T P^T on 32x32x16 MFMA
// with fp32 accumulation, online softmax in the base-2 domain, K/V tiles double-buffered in LDS.
//
// Work split: a workgroup of four wavefronts owns 4*QB*32 query rows of one (batch, head);
// each wavefront owns QB blocks of 32 rows and walks all key tiles of 64 keys.
//
// Keys sit on the M axis of the score product, so a lane holds 16 scores of ONE query per
// 32x32 block: the row maximum is an in-lane reduction plus one exchange with lane^32, and the
// probabilities, rounded to 16 bit, are already laid out as the B operand of the PV product.
// V^T is staged with its keys permuted to the same order (see kv_prepack / stage_v_fused).
#pragma once
#include "dit_attn_device.h"

namespace dit {

// The running maximum is only raised when a row's tile maximum exceeds it by more than this
// (base-2 exponent): probabilities then stay below 2^8, exact in the final normalisation,
// and the accumulator rescale is skipped on most tiles.
constexpr float kRescaleThr = 8.0f;

// SPLIT: decoupled cross-attention.  The first tile_count_a[b] listed tiles form one softmax, the
// rest a second one; when the loop crosses over, the first result is normalised, parked in
// registers as fp16 and added back in the epilogue.
template <int D, int QB, int QK_OP, int PV_OP, bool FUSED, bool SPLIT = false>
__global__ void __launch_bounds__(kThreads, QB == 1 ? 2 : 1) attn_fwd_kernel(const AttnArgs a) {
    using G = TileGeom<D>;
    constexpr int NKS = D / 16;           // contraction steps of the score product
    constexpr int NDB = D / 32;           // 32-channel blocks of the output
    constexpr int BQ = 4 * QB * 32;       // query rows per workgroup
    constexpr int CPR = D / 8;            // 16-byte chunks per K' row
    constexpr int KROWS_PER_PASS = kThreads / CPR;
    constexpr int NI_K = kBK / KROWS_PER_PASS;
    constexpr int NI_V = D / 32;          // V^T: 8 chunks per row, 32 rows per pass
    static_assert(!FUSED || (PV_OP == OP_BF16 && D == 128), "fused staging keeps V in bf16, D = 128");
    static_assert(!SPLIT || !FUSED, "the decoupled form works on pre-packed tiles");

    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, half = lane >> 5;

    // Workgroups are dealt round-robin to the 8 XCDs; renumber them so that each XCD gets a
    // contiguous range, i.e. the query tiles of the same head share one L2.
    int logical;
    {
        const int nblk = gridDim.x, bid = blockIdx.x;
        const int xcd = bid & 7, idx = bid >> 3;
        const int chunk = nblk >> 3, rem = nblk & 7;
        logical = xcd * chunk + (xcd < rem ? xcd : rem) + idx;
    }
    // Self-attention: consecutive workgroups are the query tiles of one (batch, head).  With per-request
    // key lists (cross-attention) requests differ in length, so they are interleaved instead: every
    // XCD gets the same share of every request (contiguous ranges would leave the XCDs unequal work),
    // and the workgroups that share a CU are of different lengths and drift out of lock step.
    int qt, b, h;
    if (a.tile_mask) {
        b = logical % a.B;
        const int rest = logical / a.B;
        qt = rest % a.nQT;
        h = rest / a.nQT;
    } else {
        qt = logical % a.nQT;
        const int bh_ = logical / a.nQT;
        b = bh_ / a.H;
        h = bh_ - b * a.H;
    }
    const int bh = b * a.H + h;

    // ---- staging of K/V tiles ----
    const int kchunk_off = (tid / CPR) * G::KROW + (tid % CPR) * 16;
    const int vchunk_off = G::K_BYTES + (tid >> 3) * G::VROW + (tid & 7) * 16;
    const uint8_t* tiles = FUSED ? nullptr : a.tiles + (size_t)bh * a.nKT * G::TILE_BYTES;
    u32x4 preK[NI_K];
    u32x4 preV[NI_V];       // pre-packed path: V^T chunks
    uint32_t preW[16];      // fused path: two units of 8 keys x 2 channels

    // fused path: raw K rows (rotated when written to LDS) and raw V as 8 keys x 2 channels
    const int64_t kbase = (int64_t)b * a.sk_b + (int64_t)h * a.sk_h;
    const int64_t vbase = (int64_t)b * a.sv_b + (int64_t)h * a.sv_h;

    auto issue_loads = [&](int j) {
        if constexpr (!FUSED) {
            const uint8_t* src = tiles + (size_t)j * G::TILE_BYTES;
#pragma unroll
            for (int i = 0; i < NI_K; ++i)
                preK[i] = *reinterpret_cast<const u32x4*>(src + kchunk_off + i * KROWS_PER_PASS * G::KROW);
#pragma unroll
            for (int i = 0; i < NI_V; ++i)
                preV[i] = *reinterpret_cast<const u32x4*>(src + vchunk_off + i * 32 * G::VROW);
        } else {
#pragma unroll
            for (int i = 0; i < NI_K; ++i) {
                const int key = j * kBK + tid / CPR + i * KROWS_PER_PASS;
                preK[i] = mk4(0, 0, 0, 0);
                if (key < a.Lk)
                    preK[i] = *reinterpret_cast<const u32x4*>(static_cast<const uint16_t*>(a.k) + kbase +
                                                             (int64_t)key * a.sk_t + 8 * (tid % CPR));
            }
            // unit u = wave + 4*i2 names the key set (kg = u / 2, hf = u % 2); lane = channel pair
#pragma unroll
            for (int i2 = 0; i2 < 2; ++i2) {
                const int u = wave + 4 * i2;
#pragma unroll
                for (int s = 0; s < 8; ++s) {
                    const int key = j * kBK + 16 * (u >> 1) + 8 * (s >> 2) + 4 * (u & 1) + (s & 3);
                    preW[i2 * 8 + s] = 0;
                    if (key < a.Lk)
                        preW[i2 * 8 + s] = *reinterpret_cast<const uint32_t*>(
                            static_cast<const uint16_t*>(a.v) + vbase + (int64_t)key * a.sv_t + 2 * lane);
                }
            }
        }
    };

    auto write_lds = [&](int j, int buf) {
        uint8_t* dst = smem + buf * G::TILE_BYTES;
        if constexpr (!FUSED) {
#pragma unroll
            for (int i = 0; i < NI_K; ++i)
                *reinterpret_cast<u32x4*>(dst + kchunk_off + i * KROWS_PER_PASS * G::KROW) = preK[i];
#pragma unroll
            for (int i = 0; i < NI_V; ++i)
                *reinterpret_cast<u32x4*>(dst + vchunk_off + i * 32 * G::VROW) = preV[i];
        } else {
#pragma unroll
            for (int i = 0; i < NI_K; ++i) {
                const int key = j * kBK + tid / CPR + i * KROWS_PER_PASS;
                const int kc = key < a.Lk ? key : a.Lk - 1;
                float x[8];
                widen8(preK[i], x);
                int pt, ph, pw;
                token_pos(kc, a.rg, pt, ph, pw);
                rope8(x, tid % CPR, a.rg, a.tab, pt, ph, pw);
                *reinterpret_cast<u32x4*>(dst + kchunk_off + i * KROWS_PER_PASS * G::KROW) = pack8<QK_OP>(x);
            }
#pragma unroll
            for (int i2 = 0; i2 < 2; ++i2) {
                const int u = wave + 4 * i2;
                uint32_t w[8];
#pragma unroll
                for (int s = 0; s < 8; ++s) w[s] = preW[i2 * 8 + s];
                u32x4 lo, hi;  // channel 2*lane and 2*lane+1, eight keys each
                lo.x = __builtin_amdgcn_perm(w[1], w[0], 0x05040100u);
                lo.y = __builtin_amdgcn_perm(w[3], w[2], 0x05040100u);
                lo.z = __builtin_amdgcn_perm(w[5], w[4], 0x05040100u);
                lo.w = __builtin_amdgcn_perm(w[7], w[6], 0x05040100u);
                hi.x = __builtin_amdgcn_perm(w[1], w[0], 0x07060302u);
                hi.y = __builtin_amdgcn_perm(w[3], w[2], 0x07060302u);
                hi.z = __builtin_amdgcn_perm(w[5], w[4], 0x07060302u);
                hi.w = __builtin_amdgcn_perm(w[7], w[6], 0x07060302u);
                uint8_t* vd = dst + G::K_BYTES + u * 16;
                *reinterpret_cast<u32x4*>(vd + (2 * lane) * G::VROW) = lo;
                *reinterpret_cast<u32x4*>(vd + (2 * lane + 1) * G::VROW) = hi;
            }
        }
    };

    // ---- running state ----
    f32x16 O[NDB][QB];
    // negm: every element = -(running maximum), or 0 while the row has seen no valid key.  A score
    // MFMA chain starts from it, so the scores come out relative to the running maximum and the common
    // case (no row tops it by more than the threshold) needs no subtraction in front of exp2.
    f32x16 negm[QB];
    float m_run[QB], l_run[QB];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        m_run[qb] = -INFINITY;
        l_run[qb] = 0.f;
#pragma unroll
        for (int r = 0; r < 16; ++r) negm[qb][r] = 0.f;
#pragma unroll
        for (int db = 0; db < NDB; ++db)
#pragma unroll
            for (int r = 0; r < 16; ++r) O[db][qb][r] = 0.f;
    }

    const int kread_off = l32 * G::KROW + half * 16;
    const int vread_off = G::K_BYTES + l32 * G::VROW + half * 16;
    // With key masks (cross-attention) the loop runs over the compacted list of tiles that hold a
    // valid key; otherwise over all tiles, of which only the last can be ragged.
    const uint64_t* tmask = a.tile_mask ? a.tile_mask + (size_t)b * a.nKT : nullptr;
    const int* tlist = a.tile_mask ? a.tile_list + (size_t)b * a.nKT : nullptr;
    const int n_steps = a.tile_mask ? a.tile_count[b] : a.nKT;
    const int tail = a.Lk - (a.nKT - 1) * kBK;  // valid keys of the last tile (1..64)
    auto tile_of = [&](int j) -> int { return tlist ? tlist[j] : j; };

    // ---- Q rows are requested first (16-bit inputs: raw, converted below): they come from HBM and
    // need nothing but the workgroup's coordinates, while the first tile needs the tile list ----
    u32x4 Qf[QB][NKS];
    u32x4 qraw[QB][NKS];
    int qrow[QB];
    int64_t qbase[QB];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        qrow[qb] = qt * BQ + wave * (32 * QB) + qb * 32 + l32;
        const int qr = qrow[qb] < a.Lq ? qrow[qb] : a.Lq - 1;
        qbase[qb] = (int64_t)b * a.sq_b + (int64_t)qr * a.sq_t + (int64_t)h * a.sq_h;
        if (!a.in_f32) {
#pragma unroll
            for (int ks = 0; ks < NKS; ++ks)
                qraw[qb][ks] = *reinterpret_cast<const u32x4*>(static_cast<const uint16_t*>(a.q) + qbase[qb] +
                                                              8 * (2 * ks + half));
        }
    }

    // the first tile is on its way while the Q prologue waits for its own loads
    int tile = 0;
    if (n_steps > 0) {
        tile = tile_of(0);
        issue_loads(tile);
    }

    // ---- Q prologue: rotate, fold scale*log2(e), round once, keep as B operands ----
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        const int qr = qrow[qb] < a.Lq ? qrow[qb] : a.Lq - 1;
        const int64_t base = qbase[qb];
        int pt = 0, ph = 0, pw = 0;
        if (a.tab) token_pos(qr, a.rg, pt, ph, pw);
        float rs = 1.f;
        if (a.qn.mode) rs = q_row_rstd<D>(a.qn, a.q, base, a.in_f32, half, (int64_t)b * a.Lq + qr);
#pragma unroll
        for (int ks = 0; ks < NKS; ++ks) {
            const int c = 2 * ks + half;
            float x[8];
            if (a.in_f32) load8(a.q, base + 8 * c, 1, x);
            else widen8(qraw[qb][ks], x);
            if (a.qn.mode) norm8(x, a.qn, rs, h, D, c);
            if (a.tab) rope8(x, c, a.rg, a.tab, pt, ph, pw);
#pragma unroll
            for (int e = 0; e < 8; ++e) x[e] *= a.qscale;
            Qf[qb][ks] = pack8<QK_OP>(x);
        }
    }

    if (n_steps > 0) {
        write_lds(tile, 0);
        __syncthreads();
    }

    // first softmax's output, fp16 pairs in the accumulator's lane layout (zero until the switch)
    uint32_t first[SPLIT ? QB : 1][SPLIT ? NDB * 8 : 1];
    const int n_first = SPLIT ? a.tile_count_a[b] : -1;
    if constexpr (SPLIT) {
#pragma unroll
        for (int qb = 0; qb < QB; ++qb)
#pragma unroll
            for (int i = 0; i < NDB * 8; ++i) first[qb][i] = 0u;
    }

    for (int j = 0; j < n_steps; ++j) {
        const int buf = j & 1;
        if constexpr (SPLIT) {
            if (j == n_first) {  // wave-uniform: the second conditioning sequence starts here
#pragma unroll
                for (int qb = 0; qb < QB; ++qb) {
                    const float l = l_run[qb] + __shfl_xor(l_run[qb], 32);
                    const float inv = l > 0.f ? 1.0f / l : 0.f;
#pragma unroll
                    for (int db = 0; db < NDB; ++db)
#pragma unroll
                        for (int r = 0; r < 16; r += 2) {
                            first[qb][db * 8 + r / 2] = pack2<OP_F16>(O[db][qb][r] * inv, O[db][qb][r + 1] * inv);
                            O[db][qb][r] = 0.f;
                            O[db][qb][r + 1] = 0.f;
                        }
                    m_run[qb] = -INFINITY;
                    l_run[qb] = 0.f;
#pragma unroll
                    for (int r = 0; r < 16; ++r) negm[qb][r] = 0.f;
                }
            }
        }
        const int next_tile = j + 1 < n_steps ? tile_of(j + 1) : 0;
        if (j + 1 < n_steps) issue_loads(next_tile);

        uint64_t mask;
        if (tmask) {
            mask = tmask[tile];
        } else {
            mask = (tile == a.nKT - 1 && tail < kBK) ? ((1ull << tail) - 1ull) : ~0ull;
        }

        {
            const uint8_t* kt = smem + buf * G::TILE_BYTES + kread_off;
            const uint8_t* vt = smem + buf * G::TILE_BYTES + vread_off;

            // S^T[key][query] for two 32-key blocks
            f32x16 S[2][QB];
#pragma unroll
            for (int ks = 0; ks < NKS; ++ks) {
#pragma unroll
                for (int kb = 0; kb < 2; ++kb) {
                    const u32x4 ka = *reinterpret_cast<const u32x4*>(kt + kb * 32 * G::KROW + ks * 32);
#pragma unroll
                    for (int qb = 0; qb < QB; ++qb)
                        S[kb][qb] = mfma32<QK_OP>(ka, Qf[qb][ks], ks == 0 ? negm[qb] : S[kb][qb]);
                }
            }

            if (mask != ~0ull) {
                // register r of block kb is key 32*kb + 8*(r/4) + 4*half + r%4 of the tile
                const uint64_t mlane = mask >> (4 * half);
#pragma unroll
                for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const bool ok = (mlane >> (32 * kb + 8 * (r >> 2) + (r & 3))) & 1ull;
#pragma unroll
                        for (int qb = 0; qb < QB; ++qb) S[kb][qb][r] = ok ? S[kb][qb][r] : -INFINITY;
                    }
            }

            u32x4 P[4][QB];
#pragma unroll
            for (int qb = 0; qb < QB; ++qb) {
                float mx = S[0][qb][0];
#pragma unroll
                for (int r = 1; r < 16; ++r) mx = fmaxf(mx, S[0][qb][r]);
#pragma unroll
                for (int r = 0; r < 16; ++r) mx = fmaxf(mx, S[1][qb][r]);
                mx = fmaxf(mx, __shfl_xor(mx, 32));
                // mx is relative to the base the chain started from: the running maximum, or 0 for a row
                // that has seen no valid key yet (which takes the update as soon as it sees one)
                const bool fresh = m_run[qb] == -INFINITY;
                const bool need = fresh ? mx > -INFINITY : mx > kRescaleThr;
                if (__any(need)) {
                    const float m_new = (fresh ? 0.f : m_run[qb]) + mx;
                    const float alpha = need ? __builtin_amdgcn_exp2f(m_run[qb] - m_new) : 1.0f;
                    const float shift = need ? mx : 0.f;
                    m_run[qb] = need ? m_new : m_run[qb];
                    l_run[qb] *= alpha;
#pragma unroll
                    for (int db = 0; db < NDB; ++db)
#pragma unroll
                        for (int r = 0; r < 16; ++r) O[db][qb][r] *= alpha;
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        negm[qb][r] = m_run[qb] == -INFINITY ? 0.f : -m_run[qb];
                        S[0][qb][r] -= shift;
                        S[1][qb][r] -= shift;
                    }
                }
#pragma unroll
                for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                    for (int r = 0; r < 16; ++r) S[kb][qb][r] = __builtin_amdgcn_exp2f(S[kb][qb][r]);
                // fp16 P: the row sum is taken in fp32 over the unrounded probabilities, four chains of
                // plain additions: the dot-product instruction that would sum the packed pairs does
                // not overlap with a running MFMA (measured: about 8 clocks each, unhidden), additions
                // do.  Numerator and denominator then differ by at most 2^-11 relative.
                float lsum4[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int kg = 0; kg < 4; ++kg) {
                    const int o = 8 * (kg & 1);
                    const f32x16& s = S[kg >> 1][qb];
                    P[kg][qb] = mk4(pack2<PV_OP>(s[o + 0], s[o + 1]), pack2<PV_OP>(s[o + 2], s[o + 3]),
                                    pack2<PV_OP>(s[o + 4], s[o + 5]), pack2<PV_OP>(s[o + 6], s[o + 7]));
                    if constexpr (PV_OP == OP_F16) {
#pragma unroll
                        for (int e = 0; e < 8; ++e) lsum4[e & 3] += s[o + e];
                    } else {  // bf16 P: sum the rounded values, which cancels their (8-bit) rounding error
                        lsum4[0] = sum2<PV_OP>(P[kg][qb].x, lsum4[0]);
                        lsum4[1] = sum2<PV_OP>(P[kg][qb].y, lsum4[1]);
                        lsum4[2] = sum2<PV_OP>(P[kg][qb].z, lsum4[2]);
                        lsum4[3] = sum2<PV_OP>(P[kg][qb].w, lsum4[3]);
                    }
                }
                const float lsum = (lsum4[0] + lsum4[1]) + (lsum4[2] + lsum4[3]);
                l_run[qb] += lsum;
            }

            // O^T[channel][query] += V^T[channel][key] P^T[key][query]
#pragma unroll
            for (int kg = 0; kg < 4; ++kg) {
#pragma unroll
                for (int db = 0; db < NDB; ++db) {
                    const u32x4 va = *reinterpret_cast<const u32x4*>(vt + db * 32 * G::VROW + kg * 32);
#pragma unroll
                    for (int qb = 0; qb < QB; ++qb) O[db][qb] = mfma32<PV_OP>(va, P[kg][qb], O[db][qb]);
                }
            }
        }

        if (j + 1 < n_steps) write_lds(next_tile, buf ^ 1);
        __syncthreads();
        tile = next_tile;
    }

    // ---- epilogue: normalise and store; lane holds channels 32*db + 8*g + 4*half + e ----
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        const float l = l_run[qb] + __shfl_xor(l_run[qb], 32);
        const float inv = l > 0.f ? 1.0f / l : 0.f;
        if (qrow[qb] < a.Lq) {
            const int64_t obase = (int64_t)b * a.so_b + (int64_t)qrow[qb] * a.so_t + (int64_t)h * a.so_h;
#pragma unroll
            for (int db = 0; db < NDB; ++db)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const int d0 = 32 * db + 8 * g + 4 * half;
                    float o0 = O[db][qb][4 * g + 0] * inv, o1 = O[db][qb][4 * g + 1] * inv;
                    float o2 = O[db][qb][4 * g + 2] * inv, o3 = O[db][qb][4 * g + 3] * inv;
                    if constexpr (SPLIT) {
                        const f16x2 f01 = __builtin_bit_cast(f16x2, first[qb][db * 8 + 2 * g]);
                        const f16x2 f23 = __builtin_bit_cast(f16x2, first[qb][db * 8 + 2 * g + 1]);
                        o0 += (float)f01[0]; o1 += (float)f01[1];
                        o2 += (float)f23[0]; o3 += (float)f23[1];
                    }
                    if (a.out_f32) {
                        *reinterpret_cast<float4*>(static_cast<float*>(a.out) + obase + d0) =
                            make_float4(o0, o1, o2, o3);
                    } else {
                        *reinterpret_cast<uint2*>(static_cast<uint16_t*>(a.out) + obase + d0) =
                            make_uint2(pack2<OP_BF16>(o0, o1), pack2<OP_BF16>(o2, o3));
                    }
                }
            if (a.lse && half == 0) {
                const float v = l > 0.f ? (m_run[qb] + __builtin_amdgcn_logf(l)) * 0.6931471805599453f : -INFINITY;
                a.lse[((int64_t)b * a.H + h) * a.Lq + qrow[qb]] = v;
            }
        }
    }
}

template <int D, int QB, int QK_OP, int PV_OP, bool FUSED, bool SPLIT = false>
hipError_t launch_attn_inst(const AttnArgs& a, hipStream_t s) {
    auto kern = attn_fwd_kernel<D, QB, QK_OP, PV_OP, FUSED, SPLIT>;
    constexpr int smem = 2 * TileGeom<D>::TILE_BYTES;
    static std::atomic<uint64_t> attr_set{0};
    hipError_t e = allow_dynamic_lds(kern, smem, attr_set);
    if (e != hipSuccess) return e;
    const dim3 grid((unsigned)((int64_t)a.nQT * a.B * a.H));
    hipLaunchKernelGGL(kern, grid, dim3(kThreads), smem, s, a);
    return hipGetLastError();
}

}  // namespace dit
