// Software-pipelined self-attention forward on 16x16x32 MFMAs (gfx950), the default self-attention kernel.
//
// Same pipeline as attn_pipe_body (dit_attn_fwd_pipe.h): scores of tile j+1 on the matrix cores while tile
// j's softmax runs on the vector ALU, PV of tile j while the maxima of tile j+1 are taken, K'/V^T tile images
// streamed global -> LDS directly, 8 wavefronts in two staggered halves.  What differs is the shape of the
// matrix instruction.  On this chip the board's power limit, not instruction issue, bounds a kernel that keeps
// the matrix cores busy with real data, and v_mfma_f32_16x16x32 delivers 14 % more flops per joule than
// v_mfma_f32_32x32x16 (an MFMA-only loop on random fp16 operands sustains 1,790 against 1,560 TFLOP/s on the
// same board): its dot products are 32 long, so each accumulator element is read and written half as often per
// flop.  The price is twice as many instructions and two query blocks per wavefront that share every K'/V^T
// fragment read from LDS (so the LDS traffic is unchanged).
//
// Layout of v_mfma_f32_16x16x32 (D(16x16) += A(16x32) B(32x16)), lane l = 16 g + i:
//   A: row i, contraction indices 8g .. 8g+7;  B: column i, contraction indices 8g .. 8g+7;
//   C/D: column i, rows 4g .. 4g+3.
// Scores: S^T(key, query) = K' Q'^T with keys on the rows: a lane holds, for each of its two queries
// (16 qb + i), the scores of keys 16 kb + 4g + r (kb = 0..3, r = 0..3) of a 64-key tile: 16 per query.
// The rounded probabilities of key blocks 2m and 2m+1 (8 values) are, in that order, the lane's B operand for the
// 32-key group m of O^T += V^T P^T, and the V^T tile image stores its keys in exactly that order
// (kv_prepack_kernel, V16 layout), so P never moves between lanes.
#pragma once
#include "dit_attn_fwd_pipe.h"

namespace dit {

// The 16x16 results are kept four to a 16-register block (the scores of a query block: quarter kb = key block;
// the output: quarter = channel block within a group of four) and the MFMA works on one quarter of the block.
// Element-wise changes on the rare paths are then sub-register writes of one wide value, which the register
// allocator keeps in place (as separate 4-register values it copied all of them around every branch).
template <int OP>
__device__ __forceinline__ f32x16 mfma16_q(u32x4 a, u32x4 b, f32x16 c, int q) {
    f32x4 x = {c[4 * q], c[4 * q + 1], c[4 * q + 2], c[4 * q + 3]};
    x = mfma16<OP>(a, b, x);
#pragma unroll
    for (int i = 0; i < 4; ++i) c[4 * q + i] = x[i];
    return c;
}
// the same with the accumulator quarter starting from `init`
template <int OP>
__device__ __forceinline__ f32x16 mfma16_q_init(u32x4 a, u32x4 b, f32x4 init, f32x16 c, int q) {
    const f32x4 x = mfma16<OP>(a, b, init);
#pragma unroll
    for (int i = 0; i < 4; ++i) c[4 * q + i] = x[i];
    return c;
}

// Lane (i, g) keeps max over the four lanes (i, 0..3): one swap of neighbouring 16-lane rows, one of the halves.
__device__ __forceinline__ float max_across_rows16(float x) {
    const auto r = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return max_across_halves(fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1])));
}

// The same for a sum (x of (i, g) + x of (i, g ^ 1), then the two halves): no trip through the LDS crossbar.
__device__ __forceinline__ float sum_across_rows16(float x) {
    const auto r = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    const float s = __uint_as_float(r[0]) + __uint_as_float(r[1]);
    const auto h = __builtin_amdgcn_permlane32_swap(__float_as_uint(s), __float_as_uint(s), false, false);
    return __uint_as_float(h[0]) + __uint_as_float(h[1]);
}

// Multiplier 1/sqrt(mean(x^2) + eps) of one q row whose D channels are read by the four lanes (i, 0..3), lane
// row g taking the 16-byte chunks 4 ks + g.
template <int D>
__device__ __forceinline__ float q_row_rstd16(const NormArgs& n, const void* q, int64_t base, int in_f32, int g,
                                              int64_t stat) {
    if (n.mode == 2) return n.rstd[stat];
    float ss = 0.f;
#pragma unroll
    for (int ks = 0; ks < D / 32; ++ks) {
        float x[8];
        load8(q, base + 8 * (4 * ks + g), in_f32, x);
#pragma unroll
        for (int e = 0; e < 8; ++e) ss = fmaf(x[e], x[e], ss);
    }
    ss += __shfl_xor(ss, 16);
    ss += __shfl_xor(ss, 32);
    return 1.0f / sqrtf(ss * (1.0f / D) + n.eps);
}

// NW = wavefronts per workgroup (4 or 8); a wavefront owns 32 query rows (two blocks of 16), the workgroup's
// NW * 32 rows share every K/V tile in LDS.
// The chained form keeps, behind the tile buffers, one area per wavefront the size of its 32 query rows in 16
// bits.  The rows of the NEXT query tile are copied into it (global -> LDS) while the current one is in its loop;
// at the boundary they are converted into operand registers, and the area then serves as the staging area of the
// output rows (below) before the rows after next are requested.  Held in registers across the store instead, the
// raw rows pushed the operand registers into scratch memory, eight reloads waited for one by one per query tile.
template <int D>
constexpr int chain_stage_bytes() { return 32 * D * 2; }
template <int D, int NW>
constexpr int chain_lds_bytes() { return 4 * TileGeom<D>::PART_KIB * 1024 + NW * chain_stage_bytes<D>(); }

// CHAIN: the workgroup takes pv.qt_count consecutive query tiles of its (sequence, head), one after the other,
// against ONE stream of key tiles that wraps around at the end of the sequence: the tiles of the next query
// tile's first steps arrive during the last steps of the one before, and between two query tiles there is
// only the store of the output, the conversion of the next query rows (requested before the store) and the
// first score tile.  For sequences of a few key tiles (cross-attention: 8 to 13) the start-up of a workgroup
// -- query rows and first tiles from memory, one after the other -- is otherwise as long as its loop.  The
// chained form keeps every wavefront on the same side of the barrier (no stagger).
template <int D, int QK_OP, int PV_OP, int NW, bool CHAIN = false>
__device__ __forceinline__ void attn_pipe16_body(const AttnArgs& a, const PipeView& pv) {
    using G = TileGeom<D>;
    constexpr int NKS = D / 32;        // MFMAs of one score chain
    constexpr int NCB = D / 16;        // 16-channel blocks of the output
    constexpr int NKF = 4 * NKS;       // K' fragments of a tile: (ks, kb), each feeds the two query blocks
    constexpr int NVF = 2 * NCB;       // V^T fragments of a tile: (m, cb)
    constexpr int BQ = NW * 32;
    constexpr int NI = G::PART_KIB / NW;  // full rounds of wavefront-wide 1 KiB loads per tile part
    static_assert(G::PART_KIB - NW * NI == 2, "two odd pieces per tile part");
    static_assert(QK_OP != OP_FP8, "16-bit score operands only");

    constexpr bool STAG = pipe_staggered<NW>() && !CHAIN;
    constexpr int VST = STAG ? 3 : 2;  // V^T buffers
    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];
    uint8_t* const kbuf = smem;  // K buffers 0/1, then the V buffers
    uint8_t* const vbuf = smem + 2 * G::K_BYTES;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int i16 = lane & 15, g4 = lane >> 4;
    int qt = pv.qt;
    RopeGeom rg = a.rg;
    rg.Hg = pv.Hg;
    rg.Wg = pv.Wg;

    // Query rows (16-bit inputs) are requested before anything else; they are converted after the first
    // tiles have been requested.
    u32x4 Qf[2][NKS];
    u32x4 qraw[2][NKS];
    int qrow[2];
    uint8_t* const qarea = smem + 4 * G::K_BYTES + wave * chain_stage_bytes<D>();  // chained form only
    constexpr int QPR = D / 8;  // 16-byte pieces per 16-bit query row
    // chained form: this wavefront's 32 rows of query tile `qtile` -> its area, piece p of row r in slot
    // p ^ (r % QPR) (the copy fills LDS in lane order, so the swizzle is in which piece a lane fetches)
    // (In the three pieces of code that run once per query tile of a chain -- this copy, the conversion and the
    // store -- every per-lane offset is worked out from a lane number the compiler cannot see through: left to
    // itself it works them all out ahead of the chain, cannot keep them in registers through the key loop, and
    // reloads some seventy of them from scratch memory at every query tile.)
    auto opaque_lane = [&]() {
        int l = lane;
        asm volatile("" : "+v"(l));
        return l;
    };
    auto request_q_lds = [&](int qtile) {
        const int ln = opaque_lane();
#pragma unroll
        for (int k = 0; k < 32 * QPR / 64; ++k) {
            const int r = k * (64 / QPR) + ln / QPR, slot = ln % QPR;
            const int row = qtile * BQ + wave * 32 + r;
            const int qr = row < pv.Lq ? row : pv.Lq - 1;
            const uint16_t* src = static_cast<const uint16_t*>(a.q) + pv.q_off + (int64_t)qr * a.sq_t +
                                  8 * (slot ^ (r & (QPR - 1)));
            __builtin_amdgcn_global_load_lds((gptr_t)src, (lptr_t)(qarea + k * 1024), 16, 0, 0);
        }
    };
    auto request_q = [&](int qtile) {
        if constexpr (CHAIN) {
            request_q_lds(qtile);
        } else if (!a.in_f32) {
#pragma unroll
            for (int qb = 0; qb < 2; ++qb) {
                const int row = qtile * BQ + wave * 32 + qb * 16 + i16;
                const int qr = row < pv.Lq ? row : pv.Lq - 1;
                const int64_t base = pv.q_off + (int64_t)qr * a.sq_t;
#pragma unroll
                for (int ks = 0; ks < NKS; ++ks)
                    qraw[qb][ks] = *reinterpret_cast<const u32x4*>(static_cast<const uint16_t*>(a.q) + base +
                                                                  8 * (4 * ks + g4));
            }
        }
    };
    request_q(qt);

    // ---- tile streaming (as in attn_pipe_body): a tile part is PART_KIB pieces of 1 KiB; wavefront w moves
    // pieces w, w+NW, ... of both parts; the two odd pieces of the K part go to wavefronts 0 and 1, those of
    // the V part to wavefronts 2 and 3.
    const uint8_t* const tiles = pv.tiles;  // wavefront-uniform
    const int n_steps = pv.nKT;
    const int last = n_steps - 1;
    const int tail = pv.Lk - (pv.nKT - 1) * kBK;  // valid keys of the last tile (1..64)
    // past the end: the last tile again; chained: the stream wraps around to the sequence's first tiles
    auto tile_of = [&](int j) -> int {
        if constexpr (CHAIN) {
            j = j >= n_steps ? j - n_steps : j;
            return j >= n_steps ? j - n_steps : j;  // j <= n_steps + 1, and a sequence may have one tile
        } else {
            return j < last ? j : last;
        }
    };
    auto mask_of = [&](int j) -> uint64_t {
        if constexpr (CHAIN) return j == last ? pv.last_mask : ~0ull;
        else return (j == last && tail < kBK) ? ((1ull << tail) - 1ull) : ~0ull;
    };
    constexpr int NDMA = 2 * NI + 1;
    auto dma_piece = [&](int i, int tk, int kb_, int tv, int vb_) {
        const uint8_t* ksrc = tiles + (size_t)tk * G::TILE_BYTES;
        const uint8_t* vsrc = tiles + (size_t)tv * G::TILE_BYTES + G::K_BYTES;
        uint8_t* kdst = kbuf + kb_ * G::K_BYTES;
        uint8_t* vdst = vbuf + vb_ * G::V_BYTES;
        // (chained form: the empty statement keeps the compiler from carrying per-lane 64-bit addresses through
        // the loop, two registers each, which it spilled there; uniform base + 32-bit lane offset instead)
        uint32_t lane_off = lane * 16;
        if constexpr (CHAIN) asm volatile("" : "+v"(lane_off));
        if (i < 2 * NI) {
            const int c = (wave + NW * (i >> 1)) * 1024;
            if ((i & 1) == 0) {
                __builtin_amdgcn_global_load_lds((gptr_t)(ksrc + c + lane_off), (lptr_t)(kdst + c), 16, 0, 0);
            } else {
                __builtin_amdgcn_global_load_lds((gptr_t)(vsrc + c + lane_off), (lptr_t)(vdst + c), 16, 0, 0);
            }
        } else if (NW == 4 || wave < 4) {
            const int c = (NW * NI + (wave & 1)) * 1024;
            const uint8_t* osrc = wave < 2 ? ksrc : vsrc;
            uint8_t* odst = wave < 2 ? kdst : vdst;
            __builtin_amdgcn_global_load_lds((gptr_t)(osrc + c + lane_off), (lptr_t)(odst + c), 16, 0, 0);
        }
    };
    auto dma_tiles = [&](int tk, int kb_, int tv, int vb_) {
#pragma unroll
        for (int i = 0; i < NDMA; ++i) dma_piece(i, tk, kb_, tv, vb_);
    };
    auto dma_wait_and_sync = [&]() {
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
    };

    // ---- running state ----
    constexpr int NOG = NCB / 4;  // output blocks of 64 channels: quarter cb % 4 of O[cb / 4]
    f32x16 O[NOG][2];
    f32x4 negm[2];  // every element = -m_run: the accumulator a score MFMA chain starts from
    float m_run[2], l_run[2];
    auto reset_state = [&]() {
#pragma unroll
        for (int qb = 0; qb < 2; ++qb) {
            m_run[qb] = 0.f;
            l_run[qb] = 0.f;
#pragma unroll
            for (int og = 0; og < NOG; ++og)
#pragma unroll
                for (int r = 0; r < 16; ++r) O[og][qb][r] = 0.f;
        }
    };
    reset_state();

    // Rows 4..11 of every 16 hold neighbouring 16-byte chunks in swapped pairs (pack_tile, layout 1): with that,
    // the lanes the LDS serves in one cycle of a 128-bit read fall into distinct banks (plain rows gave two-way
    // conflicts on every operand read).
    const int gsw = g4 ^ (((i16 >> 2) ^ (i16 >> 3)) & 1);
    const int kread_off = i16 * G::KROW + gsw * 16;
    const int vread_off = i16 * G::VROW + gsw * 16;
    // K' fragment f = 4 ks + kb: keys 16 kb .. +15, channels 32 ks .. +31 (the lane: key i, channels 8g .. +7)
    auto k_operand = [&](const uint8_t* kt, int f) {
        return *reinterpret_cast<const u32x4*>(kt + (f & 3) * 16 * G::KROW + (f >> 2) * 64);
    };
    // V^T fragment v = NCB m + cb: channels 16 cb .. +15, key slots 32 m .. +31 (the lane: channel i, slots 8g .. +7)
    auto v_operand = [&](const uint8_t* vt, int v) {
        return *reinterpret_cast<const u32x4*>(vt + (v % NCB) * 16 * G::VROW + (v / NCB) * 64);
    };

    // S^T of one tile from zero (first tile only): S[qb][4 kb + r] = score of key 16 kb + 4 g + r
    auto qk_tile = [&](f32x16 (&S)[2], int buf) {
        const uint8_t* kt = kbuf + buf * G::K_BYTES + kread_off;
#pragma unroll
        for (int qb = 0; qb < 2; ++qb)
#pragma unroll
            for (int r = 0; r < 16; ++r) S[qb][r] = 0.f;
#pragma unroll
        for (int f = 0; f < NKF; ++f) {
            const u32x4 ka = k_operand(kt, f);
#pragma unroll
            for (int qb = 0; qb < 2; ++qb) S[qb] = mfma16_q<QK_OP>(ka, Qf[qb][f >> 2], S[qb], f & 3);
        }
    };

    // keys whose mask bit is clear leave the softmax; element 4 kb + r is key 16 kb + 4 g + r of the tile
    auto mask_apply = [&](f32x16 (&S)[2], uint64_t mask) {
        const uint64_t mlane = mask >> (4 * g4);
#pragma unroll
        for (int kb = 0; kb < 4; ++kb)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const bool ok = (mlane >> (16 * kb + r)) & 1ull;
#pragma unroll
                for (int qb = 0; qb < 2; ++qb) S[qb][4 * kb + r] = ok ? S[qb][4 * kb + r] : -INFINITY;
            }
    };

    // Row maxima of a score tile (relative to m_run once the loop runs), over all four lanes of a row.
    float mx_new[2];
    auto row_max = [&](const f32x16 (&S)[2]) {
#pragma unroll
        for (int qb = 0; qb < 2; ++qb) {
            float mx = S[qb][0];
#pragma unroll
            for (int r = 1; r < 16; ++r) mx = fmaxf(mx, S[qb][r]);
            mx_new[qb] = max_across_rows16(mx);
        }
    };
    // Raise the running maximum of the rows whose pending tile S (relative scores) tops the threshold:
    // m += shift, and everything expressed relative to m moves with it.  mx_new holds full row maxima.
    // The scores and the chain seed are moved ON THE MATRIX CORES: S -= shift is one more accumulation step
    // S += 1 * (-shift) per key block, with an all-ones A operand and a B operand that holds -shift of the
    // lane's query in its first two contraction slots (shift = hi + lo in the operand type, exact for every
    // shift that matters) and zeros elsewhere.  Every definition of S in the loop is then an MFMA that
    // accumulates in place; vector-ALU subtractions here made the register allocator give the changed scores
    // new registers and copy all 32 of them on the common path that changes none.
    auto shift_rows = [&](f32x16 (&S)[2]) {
        constexpr uint32_t kOnes = QK_OP == OP_F16 ? 0x3c003c00u : 0x3f803f80u;
        const u32x4 ones = mk4(kOnes, kOnes, kOnes, kOnes);
#pragma unroll
        for (int qb = 0; qb < 2; ++qb) {
            const float want = mx_new[qb] > kRescaleThr ? mx_new[qb] : 0.f;
            // hi + lo in the score operand type; what is applied is their exact fp32 sum
            const uint32_t hi_bits = pack2<QK_OP>(want, 0.f) & 0xffffu;
            const float hi = QK_OP == OP_F16 ? (float)__builtin_bit_cast(f16x2, hi_bits)[0] : bf16_lo(hi_bits);
            const uint32_t lo_bits = pack2<QK_OP>(want - hi, 0.f) & 0xffffu;
            const float lo = QK_OP == OP_F16 ? (float)__builtin_bit_cast(f16x2, lo_bits)[0] : bf16_lo(lo_bits);
            const float shift = hi + lo;
            const float alpha = __builtin_amdgcn_exp2f(-shift);
            m_run[qb] += shift;
            l_run[qb] *= alpha;
            // B operand: contraction slots 0 and 1 (lanes of row g = 0) = -hi, -lo
            const uint32_t neg = ((hi_bits | (lo_bits << 16)) ^ 0x80008000u);
            const u32x4 bsh = mk4(g4 == 0 ? neg : 0u, 0u, 0u, 0u);
            negm[qb] = mfma16<QK_OP>(ones, bsh, negm[qb]);
#pragma unroll
            for (int kb = 0; kb < 4; ++kb) S[qb] = mfma16_q<QK_OP>(ones, bsh, S[qb], kb);
#pragma unroll
            for (int og = 0; og < NOG; ++og)
#pragma unroll
                for (int r = 0; r < 16; ++r) O[og][qb][r] *= alpha;
        }
    };

#ifndef DIT_PIPE16_LA
#define DIT_PIPE16_LA 6
#endif
    // LDS fragment reads issued this many fragments ahead of their MFMAs (chained form: one fewer, which is what
    // keeps its loop free of spilled registers)
#ifndef DIT_CHAIN_LA
#define DIT_CHAIN_LA (DIT_PIPE16_LA - 1)
#endif
    constexpr int LA = CHAIN ? DIT_CHAIN_LA : DIT_PIPE16_LA;
    constexpr int NCH = 16;            // softmax slices: two scores -> one dword of P
    constexpr int CPA = NCH / NKF;     // slices per K' fragment (pair of score MFMAs): 1 at d128, 2 at d64
    constexpr int CPB = NCH / NVF;     // maxima slices per V^T fragment
#ifndef DIT_PIPE16_PRE
#define DIT_PIPE16_PRE 3
#endif
    // exp2 of a softmax slice runs this many slices ahead of its pack (at least one fragment's worth)
    constexpr int PRE = DIT_PIPE16_PRE < CPA ? CPA : DIT_PIPE16_PRE;
    static_assert(CPA * NKF == NCH && CPB * NVF == NCH, "slices must divide evenly over fragments");
    static_assert(LA <= NKF && LA <= NVF, "lookahead too deep");

    const bool late = STAG && wave >= NW / 2;
    auto next_vslot = [](int s) { return s + 1 == VST ? 0 : s + 1; };
    // chained: parity of the number of key-tile steps taken before this query tile (the K' buffers alternate
    // along the whole stream, not per query tile)
    int par = 0;
    auto kslot = [&](int j) -> int {
        if constexpr (CHAIN) return (j + par) & 1;
        else return j & 1;
    };
    auto dma_interval = [&](int j, int vs) { dma_tiles(tile_of(j + 2), kslot(j), tile_of(j + 1), next_vslot(vs)); };

    // One pipelined iteration: Sc holds the relative scores of tile j (all <= threshold), Sn receives those of
    // tile j + 1.  vs = j % VST, the buffer V^T(j) sits in.  LATE (compile-time) selects where the barrier sits.
    // MASKED (compile-time): tile j + 1 may be the ragged last tile, or lie past the end.  The loop proper runs
    // the unmasked form; the last iterations of a sequence are separate copies, so that the steady state holds
    // no conditional change of the pending scores at all.
    auto iteration = [&](auto late_tag, auto masked_tag, f32x16 (&Sc)[2], f32x16 (&Sn)[2], int j, int vs) {
        constexpr bool LATE = decltype(late_tag)::value;
        constexpr bool MASKED = decltype(masked_tag)::value;
        const uint8_t* kt = kbuf + kslot(j + 1) * G::K_BYTES + kread_off;
        const uint8_t* vt = vbuf + vs * G::V_BYTES + vread_off;

        if constexpr (STAG && DIT_PIPE_PRIO == 1) __builtin_amdgcn_s_setprio(1);
        if constexpr (STAG && DIT_PIPE_PRIO == 2) __builtin_amdgcn_s_setprio(0);
        // ---- part A: S(j+1) on MFMA, P(j) and row sums on VALU ----
        u32x4 kf[NKF];
        u32x4 vf[NVF];
#pragma unroll
        for (int f = 0; f < LA; ++f) kf[f] = k_operand(kt, f);
        if constexpr (!LATE) dma_interval(j, vs);

        // slice c = (m, qb, w): dword w of the B operand of key group m for query block qb;
        // w < 2: scores 2w, 2w+1 of key block 2m; w >= 2: scores 2(w-2), 2(w-2)+1 of key block 2m+1
        uint32_t Pd[2][2][4];
        float ls[2][2];
        constexpr bool PKSUM = PV_OP == OP_F16;  // row sums over the rounded pairs, packed fp16 (see attn_pipe_body)
        f16x2 lsp[2][2];
#pragma unroll
        for (int qb = 0; qb < 2; ++qb) {
            ls[qb][0] = ls[qb][1] = 0.f;
            lsp[qb][0] = lsp[qb][1] = f16x2{(_Float16)0.f, (_Float16)0.f};
        }
        auto exp_slice = [&](int c) {
            const int m = c / 8, qb = (c % 8) / 4, w = c % 4, e = 4 * (2 * m + (w >> 1)) + 2 * (w & 1);
            Sc[qb][e] = __builtin_amdgcn_exp2f(Sc[qb][e]);
            Sc[qb][e + 1] = __builtin_amdgcn_exp2f(Sc[qb][e + 1]);
        };
        auto pack_slice = [&](int c) {
            const int m = c / 8, qb = (c % 8) / 4, w = c % 4, e = 4 * (2 * m + (w >> 1)) + 2 * (w & 1);
            const float e0 = Sc[qb][e], e1 = Sc[qb][e + 1];
            Pd[qb][m][w] = pack2<PV_OP>(e0, e1);
            if constexpr (PKSUM) {
                lsp[qb][w & 1] += __builtin_bit_cast(f16x2, Pd[qb][m][w]);
            } else {
                ls[qb][0] += e0;
                ls[qb][1] += e1;
            }
        };
#pragma unroll
        for (int c = 0; c < PRE; ++c) exp_slice(c);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int f = 0; f < NKF; ++f) {
            const int ks = f >> 2, kb = f & 3;
            if (f + LA < NKF) kf[f + LA] = k_operand(kt, f + LA);
            // the last fragments of part A fetch the first V^T fragments of part B
            if (f >= NKF - LA) vf[f - (NKF - LA)] = v_operand(vt, f - (NKF - LA));
            Sn[0] = ks == 0 ? mfma16_q_init<QK_OP>(kf[f], Qf[0][ks], negm[0], Sn[0], kb)
                            : mfma16_q<QK_OP>(kf[f], Qf[0][ks], Sn[0], kb);
#pragma unroll
            for (int cc = 0; cc < CPA; ++cc)
                if (f * CPA + cc + PRE < NCH) exp_slice(f * CPA + cc + PRE);
            __builtin_amdgcn_sched_barrier(0);
            Sn[1] = ks == 0 ? mfma16_q_init<QK_OP>(kf[f], Qf[1][ks], negm[1], Sn[1], kb)
                            : mfma16_q<QK_OP>(kf[f], Qf[1][ks], Sn[1], kb);
#pragma unroll
            for (int cc = 0; cc < CPA; ++cc) pack_slice(f * CPA + cc);
            __builtin_amdgcn_sched_barrier(0);
        }

        if constexpr (LATE) {  // the late half's barrier; its loads for the next interval follow at once
            dma_wait_and_sync();
            dma_interval(j + 1, next_vslot(vs));
            __builtin_amdgcn_sched_barrier(0);
        }

        if constexpr (STAG && DIT_PIPE_PRIO == 1) __builtin_amdgcn_s_setprio(0);
        if constexpr (STAG && DIT_PIPE_PRIO == 2) __builtin_amdgcn_s_setprio(1);
        // ---- part B: O += V^T(j) P(j) on MFMA, maxima of S(j+1) on VALU ----
        float pm[4] = {-INFINITY, -INFINITY, -INFINITY, -INFINITY};
        // slice c of the maxima: the two scores (kb, qb, r..r+1) with c = 8 kb + 4 qb + r / 2 ... any order will do
        auto max_slice = [&](int c) {
            const int kb = c / 4, qb = (c % 4) / 2, e = 4 * kb + 2 * (c % 2);
            pm[c & 3] = max3(pm[c & 3], Sn[qb][e], Sn[qb][e + 1]);
        };
#pragma unroll
        for (int v = 0; v < NVF; ++v) {
            const int m = v / NCB, cb = v % NCB;
            if (v + LA < NVF) vf[v + LA] = v_operand(vt, v + LA);
            const u32x4 pb0 = mk4(Pd[0][m][0], Pd[0][m][1], Pd[0][m][2], Pd[0][m][3]);
            const u32x4 pb1 = mk4(Pd[1][m][0], Pd[1][m][1], Pd[1][m][2], Pd[1][m][3]);
            O[cb / 4][0] = mfma16_q<PV_OP>(vf[v], pb0, O[cb / 4][0], cb % 4);
            // the first fragment leaves the last score MFMAs time to retire
            if (v >= 1) {
#pragma unroll
                for (int cc = 0; cc < CPB; ++cc) max_slice((v - 1) * CPB + cc);
            }
            __builtin_amdgcn_sched_barrier(0);
            O[cb / 4][1] = mfma16_q<PV_OP>(vf[v], pb1, O[cb / 4][1], cb % 4);
            __builtin_amdgcn_sched_barrier(0);
        }
#pragma unroll
        for (int c = (NVF - 1) * CPB; c < NCH; ++c) max_slice(c);
#pragma unroll
        for (int qb = 0; qb < 2; ++qb) {
            if constexpr (PKSUM) {
                const f16x2 t2 = lsp[qb][0] + lsp[qb][1];
                l_run[qb] += (float)t2[0] + (float)t2[1];
            } else {
                l_run[qb] += ls[qb][0] + ls[qb][1];
            }
            asm volatile("" : "+v"(l_run[qb]));  // keeps the row-sum chain here (it would sink past the barrier)
        }
        // Common case: no score of the pending tile tops the threshold in ANY lane, which needs no exchange
        // between lanes at all; the full row maxima are only formed on the rare paths below.
        bool need = __any(fmaxf(fmaxf(pm[0], pm[1]), fmaxf(pm[2], pm[3])) > kRescaleThr);
        if constexpr (!LATE) dma_wait_and_sync();
        if constexpr (MASKED) {
            const uint64_t mnext = mask_of(j + 1);
            // A ragged tile takes the rescale path whatever its maxima say.  It need not (the maxima above were
            // taken before the mask: they can only call for a shift that is not needed, never miss one, and a masked
            // score is -inf, which every path below takes as it is), and the chained form, where the ragged tile is
            // one in eight, does not; the other forms keep the assignment: without it the compiler lays their key
            // loop out differently, instruction for instruction the same and 8 % slower on all-zero inputs.
            if (mnext != ~0ull) {
                mask_apply(Sn, mnext);
                if constexpr (!CHAIN) need = true;
            }
            // after the last tile these are scores of a stale buffer: never let them touch the state
            need = need && j < last;
        }
        // (rows whose maximum stays under the threshold are shifted by zero)
        if (need) {
            row_max(Sn);
            shift_rows(Sn);
        }
    };

    // ---- prologue: tiles 0 (K, V) and 1 (K) start streaming, then Q is converted while they fly ----
    if (n_steps > 0) {
        const int t1 = last > 0 ? 1 : 0;
        dma_tiles(0, 0, 0, 0);
        dma_tiles(t1, 1, 0, 1);  // K'(1); its V part lands in a buffer iteration 0 refills anyway
    }

    int vs_run = 0;  // chained: the V^T buffer of the stream's current step
    const int n_qt = CHAIN ? pv.qt_count : 1;
    // chained form: the rows of query tile `qtile` in this wavefront's area -> operand registers.  It takes 16-bit
    // query rows (the host sends fp32 rows and rotations to the other kernels): widen, normalise if asked to, scale,
    // round.  A row's four lanes (i, 0..3) hold its channels; the per-head statistic is their sum, the per-token one
    // comes from the table.
    auto convert_q_area = [&](int qtile) {
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // the copy into the area (long done, except at the start)
        const int ln = opaque_lane();
        auto chunk = [&](int qb, int ks, float x[8]) {
            const int r = 16 * qb + (ln & 15);
            widen8(*reinterpret_cast<const u32x4*>(qarea + r * (D * 2) + (((4 * ks + (ln >> 4)) ^ (r & (QPR - 1))) << 4)), x);
        };
        float rs[2] = {1.f, 1.f};
        if (a.qn.mode == 2) {
#pragma unroll
            for (int qb = 0; qb < 2; ++qb) {
                const int row = qtile * BQ + wave * 32 + 16 * qb + (ln & 15);
                rs[qb] = a.qn.rstd[pv.stat_off + (row < pv.Lq ? row : pv.Lq - 1)];
            }
        } else if (a.qn.mode == 1) {
#pragma unroll
            for (int qb = 0; qb < 2; ++qb) {
                float ss = 0.f;
#pragma unroll
                for (int ks = 0; ks < NKS; ++ks) {
                    float x[8];
                    chunk(qb, ks, x);
#pragma unroll
                    for (int e = 0; e < 8; ++e) ss = fmaf(x[e], x[e], ss);
                }
                rs[qb] = 1.0f / sqrtf(sum_across_rows16(ss) * (1.0f / D) + a.qn.eps);
            }
        }
#pragma unroll
        for (int qb = 0; qb < 2; ++qb)
#pragma unroll
            for (int ks = 0; ks < NKS; ++ks) {
                float x[8];
                chunk(qb, ks, x);
                if (a.qn.mode) norm8(x, a.qn, rs[qb], pv.h, D, 4 * ks + (ln >> 4));
#pragma unroll
                for (int e = 0; e < 8; ++e) x[e] *= a.qscale;
                Qf[qb][ks] = pack8<QK_OP>(x);
            }
    };
    for (int it = 0; it < n_qt; ++it) {  // one pass unless chained
    if constexpr (CHAIN) {
        // the operands of this query tile were converted at the end of the one before; its area is free for
        // the rows of the next one, which arrive while this one is in its loop
        if (it == 0) convert_q_area(qt);
        else reset_state();
        if (it + 1 < n_qt) request_q(qt + 1);
    }
    // ---- Q: rotate, fold scale*log2(e), round once, keep as B operands ----
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
        qrow[qb] = qt * BQ + wave * 32 + qb * 16 + i16;
        const int qr = qrow[qb] < pv.Lq ? qrow[qb] : pv.Lq - 1;
        const int64_t base = pv.q_off + (int64_t)qr * a.sq_t;
        if constexpr (!CHAIN) {
            int pt = 0, ph = 0, pw = 0;
            if (a.tab) token_pos(qr, rg, pt, ph, pw);
            float rs = 1.f;
            if (a.qn.mode) rs = q_row_rstd16<D>(a.qn, a.q, base, a.in_f32, g4, pv.stat_off + qr);
#pragma unroll
            for (int ks = 0; ks < NKS; ++ks) {
                const int c = 4 * ks + g4;
                float x[8];
                if (a.in_f32) load8(a.q, base + 8 * c, 1, x);
                else widen8(qraw[qb][ks], x);
                if (a.qn.mode) norm8(x, a.qn, rs, pv.h, D, c);
                if (a.tab) rope8(x, c, rg, a.tab, pt, ph, pw);
#pragma unroll
                for (int e = 0; e < 8; ++e) x[e] *= a.qscale;
                Qf[qb][ks] = pack8<QK_OP>(x);
            }
        }
    }

    if (n_steps > 0) {
        // scores of tile 0 become the first running maximum
        // (chained, later query tiles: the tiles are there, and the barrier that ended the step before has been passed)
        if (!CHAIN || it == 0) dma_wait_and_sync();
        f32x16 S0[2], S1[2];
        qk_tile(S0, kslot(0));
        __syncthreads();  // every wavefront has read K'(0) before iteration 0 streams K'(2) over it
        if constexpr (STAG) {
            if (late) dma_interval(0, 0);
        }
        if (mask_of(0) != ~0ull) mask_apply(S0, mask_of(0));
        row_max(S0);  // finite: a sequence has at least one key
#pragma unroll
        for (int qb = 0; qb < 2; ++qb) {
            m_run[qb] = mx_new[qb];
#pragma unroll
            for (int r = 0; r < 4; ++r) negm[qb][r] = -m_run[qb];
#pragma unroll
            for (int r = 0; r < 16; ++r) S0[qb][r] -= m_run[qb];
        }

        auto key_loop = [&](auto late_tag) {
            int j = 0, vs = CHAIN ? vs_run : 0;
            // iteration j produces the scores of tile j + 1: unmasked while j + 1 < last
            for (; j + 3 < n_steps; j += 2) {
                iteration(late_tag, std::false_type{}, S0, S1, j, vs);
                vs = next_vslot(vs);
                iteration(late_tag, std::false_type{}, S1, S0, j + 1, vs);
                vs = next_vslot(vs);
            }
            // the last one to three iterations
            if (j < n_steps) {
                iteration(late_tag, std::true_type{}, S0, S1, j, vs);
                vs = next_vslot(vs);
                ++j;
            }
            if (j < n_steps) {
                iteration(late_tag, std::true_type{}, S1, S0, j, vs);
                vs = next_vslot(vs);
                ++j;
            }
            if (j < n_steps) {
                iteration(late_tag, std::true_type{}, S0, S1, j, vs);
                vs = next_vslot(vs);
            }
            if constexpr (CHAIN) vs_run = vs;
        };
        if (late) {
            key_loop(std::true_type{});
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        } else {
            key_loop(std::false_type{});
        }
    }

    // ---- epilogue: the lane holds channels 16 cb + 4 g + r of its two queries ----
    if constexpr (CHAIN) {
        // Stored from the accumulators a wavefront instruction writes sixteen 32-byte pieces of sixteen rows; with
        // an output as large as the input and a loop of eight steps that was a third of a query tile's time.  The
        // wavefront passes its 32 rows through a staging area of its own behind the tile buffers, STG bytes at a
        // time, and stores whole rows, 16 bytes a lane (pieces of a staged row swizzled with the row number).
        constexpr int STG = chain_stage_bytes<D>();
        uint8_t* const region = qarea;
        const int ln = opaque_lane();
        const int li = ln & 15, lg = ln >> 4;
        float inv[2];
#pragma unroll
        for (int qb = 0; qb < 2; ++qb) {
            const float l = sum_across_rows16(l_run[qb]);
            inv[qb] = l > 0.f ? 1.0f / l : 0.f;
            const int row = qt * BQ + wave * 32 + qb * 16 + li;
            if (a.lse && lg == 0 && row < pv.Lq) {
                const float v = l > 0.f ? (m_run[qb] + __builtin_amdgcn_logf(l)) * 0.6931471805599453f : -INFINITY;
                a.lse[pv.lse_off + row] = v;
            }
        }
        auto stage_and_store = [&](auto es_tag) {
            constexpr int ES = decltype(es_tag)::value;  // bytes per output element
            constexpr int RB = D * ES;                   // bytes per staged row
            constexpr int PR = RB / 16;                  // 16-byte pieces per row
            constexpr int RPP = STG / RB < 16 ? STG / RB : 16;  // rows per pass: at most one 16-row block
            static_assert(RPP >= 1 && 16 % RPP == 0 && PR <= 64 && 64 % PR == 0 && (RPP * RB) % 1024 == 0,
                          "staging geometry");
            const int row0 = qt * BQ + wave * 32;
            const bool full = row0 + 32 <= pv.Lq;  // wavefront-uniform
#pragma unroll
            for (int pass = 0; pass < 32 / RPP; ++pass) {
                const int qb = pass * RPP / 16;
                const int rr = li - (pass * RPP) % 16;  // this lane's row within the pass, if it has one
                if (rr >= 0 && rr < RPP) {
#pragma unroll
                    for (int cb = 0; cb < NCB; ++cb) {
                        const int e = 4 * (cb % 4);
                        const float o0 = O[cb / 4][qb][e] * inv[qb], o1 = O[cb / 4][qb][e + 1] * inv[qb];
                        const float o2 = O[cb / 4][qb][e + 2] * inv[qb], o3 = O[cb / 4][qb][e + 3] * inv[qb];
                        const int col = (16 * cb + 4 * lg) * ES;
                        uint8_t* const dst = region + rr * RB + (((col >> 4) ^ (rr & (PR - 1))) << 4) + (col & 15);
                        if constexpr (ES == 4) *reinterpret_cast<float4*>(dst) = make_float4(o0, o1, o2, o3);
                        else *reinterpret_cast<uint2*>(dst) = make_uint2(pack2<OP_BF16>(o0, o1), pack2<OP_BF16>(o2, o3));
                    }
                }
                // all of a pass's pieces are read back before the first is stored, and a tile that lies inside the
                // sequence stores without a row test: with a test per store each read sat in a branch of its own
                // and was waited for there, sixteen LDS round trips one after the other per query tile
                constexpr int NK = RPP * RB / 1024;
                static_assert(NK == 2 || NK % 4 == 0, "pieces are read back two or four at a time");
                u32x4 v[NK];
#pragma unroll
                for (int k = 0; k < NK; ++k) {
                    const int r = k * (64 / PR) + ln / PR, pc = ln % PR;
                    v[k] = *reinterpret_cast<const u32x4*>(region + r * RB + ((pc ^ (r & (PR - 1))) << 4));
                }
                // (four values the compiler must hold at once: left alone it sinks each read to its store)
                if constexpr (NK == 2) {
                    asm volatile("" : "+v"(v[0]), "+v"(v[1])::"memory");
                } else {
#pragma unroll
                    for (int k = 0; k < NK; k += 4)
                        asm volatile("" : "+v"(v[k]), "+v"(v[k + 1]), "+v"(v[k + 2]), "+v"(v[k + 3])::"memory");
                }
                uint8_t* const obase = static_cast<uint8_t*>(a.out) +
                                       (pv.o_off + (int64_t)(row0 + pass * RPP + ln / PR) * a.so_t) * ES + (ln % PR) * 16;
                const int64_t kstride = (int64_t)(64 / PR) * a.so_t * ES;
                if (full) {
#pragma unroll
                    for (int k = 0; k < NK; ++k) *reinterpret_cast<u32x4*>(obase + k * kstride) = v[k];
                } else {
#pragma unroll
                    for (int k = 0; k < NK; ++k)
                        if (row0 + pass * RPP + k * (64 / PR) + ln / PR < pv.Lq)
                            *reinterpret_cast<u32x4*>(obase + k * kstride) = v[k];
                }
            }
        };
        // the next query tile's operands out of the area, then the area is the staging area
        if (it + 1 < n_qt) convert_q_area(qt + 1);
        if (a.out_f32) stage_and_store(std::integral_constant<int, 4>());
        else stage_and_store(std::integral_constant<int, 2>());
    } else {
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
        float l = l_run[qb];
        l += __shfl_xor(l, 16);
        l += __shfl_xor(l, 32);
        const float inv = l > 0.f ? 1.0f / l : 0.f;
        if (qrow[qb] < pv.Lq) {
            const int64_t obase = pv.o_off + (int64_t)qrow[qb] * a.so_t;
#pragma unroll
            for (int cb = 0; cb < NCB; ++cb) {
                const int d0 = 16 * cb + 4 * g4;
                const int e = 4 * (cb % 4);
                const float o0 = O[cb / 4][qb][e] * inv, o1 = O[cb / 4][qb][e + 1] * inv;
                const float o2 = O[cb / 4][qb][e + 2] * inv, o3 = O[cb / 4][qb][e + 3] * inv;
                if (a.out_f32) {
                    *reinterpret_cast<float4*>(static_cast<float*>(a.out) + obase + d0) = make_float4(o0, o1, o2, o3);
                } else {
                    *reinterpret_cast<uint2*>(static_cast<uint16_t*>(a.out) + obase + d0) =
                        make_uint2(pack2<OP_BF16>(o0, o1), pack2<OP_BF16>(o2, o3));
                }
            }
            if (a.lse && g4 == 0) {
                const float v = l > 0.f ? (m_run[qb] + __builtin_amdgcn_logf(l)) * 0.6931471805599453f : -INFINITY;
                a.lse[pv.lse_off + qrow[qb]] = v;
            }
        }
    }
    }
    if constexpr (CHAIN) {
        ++qt;
        par ^= n_steps & 1;
    }
    }  // query tiles
}

// One sequence per batch entry, all of the same length.
template <int D, int QK_OP, int PV_OP, int NW>
__global__ void __launch_bounds__(64 * NW, 2) attn_fwd_pipe16_kernel(const AttnArgs a) {
    const int logical = xcd_contiguous_block();
    PipeView pv;
    const int bh = logical / a.nQT;
    pv.qt = logical % a.nQT;
    pv.b = bh / a.H;
    pv.h = bh - pv.b * a.H;
    pv.Lq = a.Lq;
    pv.Lk = a.Lk;
    pv.nKT = a.nKT;
    pv.tiles = a.tiles + (size_t)bh * a.nKT * TileGeom<D>::TILE_BYTES;
    pv.q_off = (int64_t)pv.b * a.sq_b + (int64_t)pv.h * a.sq_h;
    pv.o_off = (int64_t)pv.b * a.so_b + (int64_t)pv.h * a.so_h;
    pv.lse_off = ((int64_t)pv.b * a.H + pv.h) * a.Lq;
    pv.stat_off = (int64_t)pv.b * a.Lq;
    pv.Hg = a.rg.Hg;
    pv.Wg = a.rg.Wg;
    attn_pipe16_body<D, QK_OP, PV_OP, NW>(a, pv);
}

// Packed requests of different lengths: work distribution as attn_fwd_pipe_varlen_kernel.
template <int D, int QK_OP, int PV_OP, int NW>
__global__ void __launch_bounds__(64 * NW, 2) attn_fwd_pipe16_varlen_kernel(const AttnArgs a, const VarlenTable vt) {
    const int xcd = blockIdx.x & 7;
    int idx = blockIdx.x >> 3;
    int r = 0, h_first = 0;
    for (; r < vt.n; ++r) {
        h_first = (xcd - r * a.H) & 7;
        const int heads = h_first < a.H ? (a.H - h_first + 7) >> 3 : 0;
        const int nblk = heads * vt.r[r].nQT;
        if (idx < nblk) break;
        idx -= nblk;
    }
    if (r == vt.n) return;  // uniform over the workgroup, before any barrier
    const ReqDesc& rq = vt.r[r];
    PipeView pv;
    pv.qt = idx % rq.nQT;
    pv.h = h_first + 8 * (idx / rq.nQT);
    pv.b = 0;
    pv.Lq = rq.L;
    pv.Lk = rq.L;
    pv.nKT = rq.nKT;
    pv.tiles = a.tiles + ((size_t)rq.tile0 * a.H + (size_t)pv.h * rq.nKT) * TileGeom<D>::TILE_BYTES;
    pv.q_off = (int64_t)rq.tok0 * a.sq_t + (int64_t)pv.h * a.sq_h;
    pv.o_off = (int64_t)rq.tok0 * a.so_t + (int64_t)pv.h * a.so_h;
    pv.lse_off = (int64_t)pv.h * vt.total_tokens + rq.tok0;
    pv.stat_off = rq.tok0;
    pv.Hg = rq.Hg;
    pv.Wg = rq.Wg;
    attn_pipe16_body<D, QK_OP, PV_OP, NW>(a, pv);
}

// Cross-attention with one joint softmax per request: workgroups chain `qch` query tiles of one (request, head).
// The pre-pack leaves a request's attending keys densely in its tiles 0 .. count-1 (key_compact_kernel; without a
// byte mask all keys attend), so only the last of them is partial; count and that tile's mask come from the
// workspace.  Workgroup order: request fastest, then chunk, then head, so that the workgroups an XCD holds at a
// time share a handful of (request, head) tile sets in its L2 and requests of different lengths are interleaved.
template <int D, int QK_OP, int PV_OP, int NW>
__global__ void __launch_bounds__(64 * NW, 2) attn_fwd_pipe16_chain_kernel(const AttnArgs a, int qch) {
    const int logical = xcd_contiguous_block();
    const int nch = (a.nQT + qch - 1) / qch;
    PipeView pv;
    pv.b = logical % a.B;
    const int rest = logical / a.B;
    const int ch = rest % nch;
    pv.h = rest / nch;
    pv.qt = ch * qch;
    pv.qt_count = a.nQT - pv.qt < qch ? a.nQT - pv.qt : qch;
    const int bh = pv.b * a.H + pv.h;
    const int count = a.tile_count[pv.b];
    pv.Lq = a.Lq;
    pv.Lk = a.Lk;
    pv.nKT = count;
    pv.last_mask = count > 0 ? a.tile_mask[(size_t)pv.b * a.nKT + count - 1] : 0ull;
    pv.tiles = a.tiles + (size_t)bh * a.nKT * TileGeom<D>::TILE_BYTES;
    pv.q_off = (int64_t)pv.b * a.sq_b + (int64_t)pv.h * a.sq_h;
    pv.o_off = (int64_t)pv.b * a.so_b + (int64_t)pv.h * a.so_h;
    pv.lse_off = ((int64_t)pv.b * a.H + pv.h) * a.Lq;
    pv.stat_off = (int64_t)pv.b * a.Lq;
    pv.Hg = a.rg.Hg;
    pv.Wg = a.rg.Wg;
    attn_pipe16_body<D, QK_OP, PV_OP, NW, true>(a, pv);
}

template <int D, int QK_OP, int PV_OP, int NW>
hipError_t launch_attn_pipe16_chain_inst(const AttnArgs& a, hipStream_t s) {
    auto kern = attn_fwd_pipe16_chain_kernel<D, QK_OP, PV_OP, NW>;
    constexpr int smem = chain_lds_bytes<D, NW>();
    static std::atomic<uint64_t> attr_set{0};
    hipError_t e = allow_dynamic_lds(kern, smem, attr_set);
    if (e != hipSuccess) return e;
    // query tiles per workgroup: long enough chains that a workgroup's start-up is a small part of its life,
    // enough workgroups (about five per compute unit) that requests of different lengths even out
    int dev = 0, cus = 0;
    e = hipGetDevice(&dev);
    if (e == hipSuccess) e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
    if (e != hipSuccess) return e;
    const int64_t total_qt = (int64_t)a.nQT * a.B * a.H;
#ifndef DIT_CHAIN_PER_CU
#define DIT_CHAIN_PER_CU 5
#endif
#ifndef DIT_CHAIN_MAX
#define DIT_CHAIN_MAX 16
#endif
    int64_t qch = total_qt / (DIT_CHAIN_PER_CU * (int64_t)(cus > 0 ? cus : 1));
    qch = qch < 1 ? 1 : (qch > DIT_CHAIN_MAX ? DIT_CHAIN_MAX : qch);
    const int64_t nch = (a.nQT + qch - 1) / qch;
    hipLaunchKernelGGL(kern, dim3((unsigned)(nch * a.B * a.H)), dim3(64 * NW), smem, s, a, (int)qch);
    return hipGetLastError();
}

template <int D, int QK_OP, int PV_OP, int NW>
hipError_t launch_attn_pipe16_inst(const AttnArgs& a, hipStream_t s) {
    auto kern = attn_fwd_pipe16_kernel<D, QK_OP, PV_OP, NW>;
    constexpr int smem = pipe_lds_bytes<D, NW>();
    static std::atomic<uint64_t> attr_set{0};
    hipError_t e = allow_dynamic_lds(kern, smem, attr_set);
    if (e != hipSuccess) return e;
    const dim3 grid((unsigned)((int64_t)a.nQT * a.B * a.H));
    hipLaunchKernelGGL(kern, grid, dim3(64 * NW), smem, s, a);
    return hipGetLastError();
}

template <int D, int QK_OP, int PV_OP, int NW>
hipError_t launch_attn_pipe16_varlen_inst(const AttnArgs& a, const VarlenTable& vt, hipStream_t s) {
    auto kern = attn_fwd_pipe16_varlen_kernel<D, QK_OP, PV_OP, NW>;
    constexpr int smem = pipe_lds_bytes<D, NW>();
    static std::atomic<uint64_t> attr_set{0};
    hipError_t e = allow_dynamic_lds(kern, smem, attr_set);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, dim3((unsigned)(8 * vt.queue_len)), dim3(64 * NW), smem, s, a, vt);
    return hipGetLastError();
}

}  // namespace dit
