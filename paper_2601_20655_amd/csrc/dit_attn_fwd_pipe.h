// Software-pipelined attention forward for gfx950 (pre-packed K'/V^T tiles; LISTED = false: every
// tile attends and only the ragged tail is masked; LISTED = true: per-tile 64-bit key masks and a
// compacted list of the non-empty tiles, the cross-attention form).  Same math and operand layouts as attn_fwd_kernel; what changes is
// the schedule inside a wavefront, so that the matrix pipe and the vector ALU work at the same
// time instead of taking turns:
//
//   iteration j, part A:  S(j+1)^T = K'(j+1) Q'^T  on MFMA   ||  P(j) = exp2(S(j) - m), row sums on VALU
//   iteration j, part B:  O^T += V^T(j) P(j)^T     on MFMA   ||  row maxima of S(j+1), rescale test on VALU
//
// K/V tiles reach LDS by direct global->LDS loads (no staging registers): while iteration j runs,
// K'(j+2) and V^T(j+1) stream into the buffers iteration j-1 has finished with.
//
// Scores are kept RELATIVE to the running maximum: the score MFMA chain starts from an
// accumulator filled with -m instead of zero, so exp2 applies to the MFMA result directly and the
// per-score subtraction disappears from the vector ALU.  When a row's maximum has to move (rare,
// thresholded), the accumulator, the row sum and the pending score tile are shifted together.
//
// QK_OP = OP_FP8 swaps the score product for the 8-bit MFMA (64 channels per instruction, row factors
// applied by the instruction); everything after the scores is the same code.
#pragma once
#include <type_traits>

#include "dit_attn_fwd.h"

// Schedule constants of the pipelined kernel (overridable at build time for tuning sweeps).
#ifndef DIT_PIPE_LA
#define DIT_PIPE_LA 6   // LDS fragment reads are issued this many fragments ahead of their MFMA
#endif
#ifndef DIT_PIPE_PRE
#define DIT_PIPE_PRE 2  // exp2 of a softmax slice runs this many slices ahead of its pack (and before the first MFMA)
#endif

#ifndef DIT_PIPE_STAGGER
#define DIT_PIPE_STAGGER 1  // 8-wavefront workgroups: wavefronts 4-7 run half an iteration behind wavefronts 0-3
#endif
#ifndef DIT_PIPE_PRIO
#define DIT_PIPE_PRIO 1  // staggered form: wavefront priority raised during part A (1), part B (2), never (0)
#endif
namespace dit {

typedef const __attribute__((address_space(1))) void* gptr_t;
typedef __attribute__((address_space(3))) void* lptr_t;

// Lane l keeps max(x[l % 32], x[32 + l % 32]): one swap of the two 32-lane halves, no LDS trip.
__device__ __forceinline__ float max_across_halves(float x) {
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}

// max(a, b, c) in one instruction (scores are never NaN, so no canonicalisation is needed)
__device__ __forceinline__ float max3(float a, float b, float c) {
    float r;
    asm("v_max3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
    return r;
}

// Staggered form (8 wavefronts, one workgroup per CU): the two wavefronts of a SIMD run half an
// iteration apart, so one of them has matrix work while the other goes through the scalar end of
// its iteration; a V^T tile is then read in two consecutive barrier intervals and needs three
// buffers.
template <int NW>
constexpr bool pipe_staggered() { return NW == 8 && DIT_PIPE_STAGGER; }
template <int D, int NW>
constexpr int pipe_lds_bytes() {
    return (2 + (pipe_staggered<NW>() ? 3 : 2)) * TileGeom<D>::PART_KIB * 1024;
}

// The sequence one workgroup works on: which query tile of which (sequence, head), and where that
// sequence's rows and tiles start.
struct PipeView {
    int qt, h, b;          // query tile, head, batch entry (b indexes the tile lists, LISTED only)
    int Lq, Lk, nKT;
    const uint8_t* tiles;  // tile images of this (sequence, head)
    int64_t q_off, o_off;  // element offsets of row 0 of this (sequence, head) in q / out
    int64_t lse_off;       // index of row 0 in lse
    int64_t stat_off;      // index of row 0 in the per-token normalisation table
    int Hg, Wg;            // latent grid of this sequence
    int qt_count;          // chained form (attn_pipe16_body<.., CHAIN>): consecutive query tiles taken, from qt
    uint64_t last_mask;    // chained form: key mask of the sequence's last tile
};

// NW = wavefronts per workgroup (4 or 8); the workgroup owns NW*QB*32 query rows that share every
// K/V tile in LDS.
template <int D, int QB, int QK_OP, int PV_OP, int NW, bool LISTED>
__device__ __forceinline__ void attn_pipe_body(const AttnArgs& a, const PipeView& pv) {
    using G = TileGeom<D>;
    // FP8: the score product runs on 8-bit (e4m3) operands, 64 channels per MFMA instead of 16, with one
    // power-of-two factor per q' row and per k' row that the MFMA applies itself
    constexpr bool FP8 = QK_OP == OP_FP8;
    constexpr int NKS = FP8 ? D / 64 : D / 16;  // MFMAs of one score chain
    constexpr int NQC = D / 16;                 // 16-byte chunks of a q row each lane of a pair reads
    constexpr int NDB = D / 32;
    constexpr int BQ = NW * QB * 32;
    static_assert(!FP8 || QB == 1, "8-bit score operands: 32 rows per wavefront only");
    using QFrag = std::conditional_t<FP8, i32x8, u32x4>;
    constexpr int NI = G::PART_KIB / NW;  // full rounds of wavefront-wide 1 KiB loads per tile part
    static_assert(G::PART_KIB - NW * NI == 2, "two odd pieces per tile part");

    constexpr bool STAG = pipe_staggered<NW>();
    constexpr int VST = STAG ? 3 : 2;  // V^T buffers
    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];
    // LDS map: K buffers 0/1, then the V buffers
    uint8_t* const kbuf = smem;
    uint8_t* const vbuf = smem + 2 * G::K_BYTES;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l32 = lane & 31, half = lane >> 5;
    const int qt = pv.qt, b = pv.b;
    RopeGeom rg = a.rg;
    rg.Hg = pv.Hg;
    rg.Wg = pv.Wg;

    // Query rows (16-bit inputs) are requested before anything else: they come from HBM and need
    // only the workgroup's coordinates, while the first tiles wait for the tile list.  They are
    // converted into Qf after the first tiles have been requested.
    QFrag Qf[QB][NKS];
    int q_code[QB];  // FP8: 8-bit scale code of the lane's q' row
    u32x4 qraw[QB][NQC];
    int qrow[QB];
    if (!a.in_f32) {
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) {
            const int row = qt * BQ + wave * (32 * QB) + qb * 32 + l32;
            const int qr = row < pv.Lq ? row : pv.Lq - 1;
            const int64_t base = pv.q_off + (int64_t)qr * a.sq_t;
#pragma unroll
            for (int ks = 0; ks < NQC; ++ks)
                qraw[qb][ks] = *reinterpret_cast<const u32x4*>(static_cast<const uint16_t*>(a.q) + base +
                                                              8 * (2 * ks + half));
        }
    }

    // ---- tile streaming.  A tile part is PART_KIB pieces of 1 KiB (64 lanes x 16 bytes).  Wavefront
    // w moves pieces w, w+NW, ... of both parts; the two odd pieces of the K part go to wavefronts
    // 0 and 1, those of the V part to wavefronts 2 and 3.
    const uint8_t* const tiles = pv.tiles;  // wavefront-uniform
    const uint32_t lane_off = lane * 16;
    // The loop runs over "steps"; step j works on tile tile_of(j).  Without a list that is tile j.
    // With a list (at most 64 tiles, checked by the host), lane i of every wavefront keeps list entry i
    // and the key mask of tile i in registers and a step reads them with v_readlane: no memory operation in
    // the loop, whose waits on LDS operand reads would otherwise have to drain scalar loads too.
    const int n_steps = LISTED ? a.tile_count[b] : pv.nKT;
    const int last = n_steps - 1;
    const int tail = pv.Lk - (pv.nKT - 1) * kBK;  // valid keys of the last tile (1..64)
    int v_tile = 0;  // filled in the prologue, after the first tiles have been requested
    uint32_t v_mask_lo = ~0u, v_mask_hi = ~0u;
    auto tile_of = [&](int j) -> int {
        j = j < last ? j : last;  // past the end: the last tile again (fetched into a buffer nobody reads)
        if constexpr (LISTED) return __builtin_amdgcn_readlane(v_tile, j);
        return j;
    };
    auto mask_of = [&](int j) -> uint64_t {
        if (j > last) return ~0ull;
        if constexpr (LISTED) {
            const int t = __builtin_amdgcn_readlane(v_tile, j);
            return ((uint64_t)(uint32_t)__builtin_amdgcn_readlane((int)v_mask_hi, t) << 32) |
                   (uint32_t)__builtin_amdgcn_readlane((int)v_mask_lo, t);
        }
        return (j == last && tail < kBK) ? ((1ull << tail) - 1ull) : ~0ull;
    };
    // One tile pair = NDMA loads per wavefront: pieces 2i (K part) and 2i+1 (V part) for i < NI, then
    // the odd piece.  They go out together right after a barrier: spreading them over part A, or
    // letting the two halves of the workgroup take turns, measured within 1 %.
    constexpr int NDMA = 2 * NI + 1;
    // (tk, tv: tile numbers, already looked up)
    auto dma_piece = [&](int i, int tk, int kb_, int tv, int vb_) {
        const uint8_t* ksrc = tiles + (size_t)tk * G::TILE_BYTES;
        const uint8_t* vsrc = tiles + (size_t)tv * G::TILE_BYTES + G::K_BYTES;
        uint8_t* kdst = kbuf + kb_ * G::K_BYTES;
        uint8_t* vdst = vbuf + vb_ * G::V_BYTES;
        if (i < 2 * NI) {
            const int r = i >> 1;
            const int c = (wave + NW * r) * 1024;
            if ((i & 1) == 0) {
                // FP8: the 8-bit K' rows and their scale codes fill pieces 0..9 of the K part; whole
                // rounds move pieces 0..7, the odd load below pieces 8 and 9, the rest stays behind
                if (!FP8 || (r + 1) * NW <= 8)
                    __builtin_amdgcn_global_load_lds((gptr_t)(ksrc + c + lane_off), (lptr_t)(kdst + c), 16, 0, 0);
            } else {
                __builtin_amdgcn_global_load_lds((gptr_t)(vsrc + c + lane_off), (lptr_t)(vdst + c), 16, 0, 0);
            }
        } else if (NW == 4 || wave < 4) {
            const int c = (NW * NI + (wave & 1)) * 1024;
            if constexpr (FP8) {
                const int ck = (8 + (wave & 1)) * 1024;
                const uint8_t* osrc = wave < 2 ? ksrc + ck : vsrc + c;
                uint8_t* odst = wave < 2 ? kdst + ck : vdst + c;
                __builtin_amdgcn_global_load_lds((gptr_t)(osrc + lane_off), (lptr_t)odst, 16, 0, 0);
            } else {
                const uint8_t* osrc = wave < 2 ? ksrc : vsrc;
                uint8_t* odst = wave < 2 ? kdst : vdst;
                __builtin_amdgcn_global_load_lds((gptr_t)(osrc + c + lane_off), (lptr_t)(odst + c), 16, 0, 0);
            }
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
    f32x16 O[NDB][QB];
    f32x16 negm[QB];  // every element = -m_run: the accumulator a score MFMA chain starts from
    float m_run[QB], l_run[QB];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        m_run[qb] = 0.f;
        l_run[qb] = 0.f;
#pragma unroll
        for (int db = 0; db < NDB; ++db)
#pragma unroll
            for (int r = 0; r < 16; ++r) O[db][qb][r] = 0.f;
    }

    const int kread_off = FP8 ? l32 * G::KROW8 + half * 32 : l32 * G::KROW + half * 16;
    const int vread_off = l32 * G::VROW + half * 16;
    // A operand of score MFMA f (key block f & 1, contraction step f >> 1) of the tile at kt
    auto k_operand = [&](const uint8_t* kt, int f) {
        if constexpr (FP8) {
            const uint8_t* p = kt + (f & 1) * 32 * G::KROW8 + (f >> 1) * 64;
            const u32x4 lo = *reinterpret_cast<const u32x4*>(p), hi = *reinterpret_cast<const u32x4*>(p + 16);
            const i32x8 r = {(int)lo.x, (int)lo.y, (int)lo.z, (int)lo.w, (int)hi.x, (int)hi.y, (int)hi.z, (int)hi.w};
            return r;
        } else {
            return *reinterpret_cast<const u32x4*>(kt + (f & 1) * 32 * G::KROW + (f >> 1) * 32);
        }
    };
    // FP8: scale code of the lane's key row in key block kb of the tile in K buffer buf
    auto k_code = [&](int buf, int kb) -> int { return kbuf[buf * G::K_BYTES + G::KSCALE_OFF + kb * 32 + l32]; };
    auto score_mfma = [&](const auto& ka, const QFrag& qf, const f32x16& acc, int kcode, int qcode) {
        if constexpr (FP8) return mfma32_fp8(ka, qf, acc, kcode, qcode);
        else return mfma32<QK_OP>(ka, qf, acc);
    };
    // S^T of one tile: two 32-key blocks per query block
    auto qk_tile = [&](f32x16 (&S)[2][QB], int buf) {
        const uint8_t* kt = kbuf + buf * G::K_BYTES + kread_off;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int qb = 0; qb < QB; ++qb)
#pragma unroll
                for (int r = 0; r < 16; ++r) S[kb][qb][r] = 0.f;
        int kc[2] = {0, 0};
        if constexpr (FP8) {
            kc[0] = k_code(buf, 0);
            kc[1] = k_code(buf, 1);
        }
#pragma unroll
        for (int ks = 0; ks < NKS; ++ks) {
#pragma unroll
            for (int kb = 0; kb < 2; ++kb) {
                const auto ka = k_operand(kt, 2 * ks + kb);
#pragma unroll
                for (int qb = 0; qb < QB; ++qb) S[kb][qb] = score_mfma(ka, Qf[qb][ks], S[kb][qb], kc[kb], q_code[qb]);
            }
        }
    };

    // keys whose mask bit is clear leave the softmax
    auto mask_apply = [&](f32x16 (&S)[2][QB], uint64_t mask) {
        const uint64_t mlane = mask >> (4 * half);
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const bool ok = (mlane >> (32 * kb + 8 * (r >> 2) + (r & 3))) & 1ull;
#pragma unroll
                for (int qb = 0; qb < QB; ++qb) S[kb][qb][r] = ok ? S[kb][qb][r] : -INFINITY;
            }
    };

    // Row maxima of a score tile (relative to m_run once the loop runs); mx_new receives them.
    float mx_new[QB];
    auto row_max = [&](const f32x16 (&S)[2][QB]) {
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) {
            float mx = S[0][qb][0];
#pragma unroll
            for (int r = 1; r < 16; ++r) mx = fmaxf(mx, S[0][qb][r]);
#pragma unroll
            for (int r = 0; r < 16; ++r) mx = fmaxf(mx, S[1][qb][r]);
            mx_new[qb] = max_across_halves(mx);
        }
    };
    auto any_row_needs_shift = [&]() -> bool {
        bool need = false;
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) need |= mx_new[qb] > kRescaleThr;
        return __any(need);
    };
    // Raise the running maximum of the rows whose pending tile S (relative scores) tops the
    // threshold: m += shift, and everything expressed relative to m moves with it.
    auto shift_rows = [&](f32x16 (&S)[2][QB]) {
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) {
            const float shift = mx_new[qb] > kRescaleThr ? mx_new[qb] : 0.f;
            const float alpha = __builtin_amdgcn_exp2f(-shift);
            m_run[qb] += shift;
            l_run[qb] *= alpha;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                negm[qb][r] = -m_run[qb];
                S[0][qb][r] -= shift;
                S[1][qb][r] -= shift;
            }
#pragma unroll
            for (int db = 0; db < NDB; ++db)
#pragma unroll
                for (int r = 0; r < 16; ++r) O[db][qb][r] *= alpha;
        }
    };

    // One pipelined iteration: Sc holds the relative scores of tile j (all <= threshold), Sn
    // receives those of tile j + 1.  Both parts are written as MFMA steps with a slice of vector
    // work attached to each, and the compiler is told not to move anything across step
    // boundaries, so the instruction stream alternates matrix and vector instructions.
    constexpr int LA = DIT_PIPE_LA;          // LDS fragment reads issued this many fragments ahead
    constexpr int NCH = 16 * QB;             // vector slices: two scores of one query block each
    constexpr int NA = 2 * NKS * QB;         // MFMA steps of part A
    constexpr int NB = 4 * NDB * QB;         // MFMA steps of part B
    constexpr int CPA = NCH / NA, CPB = NCH / NB;
    constexpr int PRE = DIT_PIPE_PRE;        // exp slices issued before the first MFMA, covering LDS latency
    static_assert(CPA * NA == NCH && CPB * NB == NCH, "slices must divide evenly over MFMA steps");
    constexpr int LAK = FP8 ? 2 * NKS : LA;  // FP8: a tile's few (32-byte) K' operands are all read up front
    static_assert(LAK <= 2 * NKS && LA <= 4 * NDB && LAK * QB <= NA, "lookahead too deep");
    // All softmax slices of tile j run in part A, under the score MFMAs of tile j + 1, while the SIMD's
    // other wavefront is in its part B (PV MFMAs and the cheap maxima).  Spreading the slices over both
    // parts paid while each slice carried a v_dot2c; since the row sums are plain additions it measures
    // 2.7 % slower than this.
    // (FP8: all softmax slices stay in part A, whose four long MFMA steps leave the vector ALU to them,
    // while the other wavefront of the SIMD is in its MFMA-heavy part B; moving half of the slices into
    // part B measured 8 % slower.)
    constexpr bool COPY = QB == 2;

    // Wavefronts of the late half (staggered form) pass the workgroup barrier between the two parts
    // of an iteration, the others at its end; both issue their tile loads right after their barrier.
    const bool late = STAG && wave >= NW / 2;
    auto next_vslot = [](int s) { return s + 1 == VST ? 0 : s + 1; };
    // loads of barrier interval j: K'(j + 2) over K'(j), V^T(j + 1) into the buffer after V^T(j)'s
    auto dma_interval = [&](int j, int vs) { dma_tiles(tile_of(j + 2), j & 1, tile_of(j + 1), next_vslot(vs)); };

    // vs = j % VST, the buffer V^T(j) sits in
    // LATE (a compile-time tag) selects where the barrier sits; each half runs its own copy of the
    // loop so that an iteration stays one straight-line block.
    auto iteration = [&](auto late_tag, f32x16 (&Sc)[2][QB], f32x16 (&Sn)[2][QB], int j, int vs) {
        constexpr bool LATE = decltype(late_tag)::value;
        const uint8_t* kt = kbuf + ((j + 1) & 1) * G::K_BYTES + kread_off;
        const uint8_t* vt = vbuf + vs * G::V_BYTES + vread_off;
        auto kfrag = [&](int f) { return k_operand(kt, f); };
        auto vfrag = [&](int g) { return *reinterpret_cast<const u32x4*>(vt + (g % NDB) * 32 * G::VROW + (g / NDB) * 32); };

        // The two wavefronts of a SIMD are in different parts at any time (staggered form); the
        // issue arbiter otherwise favours the older wavefront throughout, which then idles at the
        // barrier while the younger one finishes alone.  Raising the priority in one part makes
        // the preference alternate.
        if constexpr (STAG && DIT_PIPE_PRIO == 1) __builtin_amdgcn_s_setprio(1);
        if constexpr (STAG && DIT_PIPE_PRIO == 2) __builtin_amdgcn_s_setprio(0);
        // ---- part A: S(j+1) on MFMA, P(j) and row sums on VALU ----
        decltype(k_operand(kt, 0)) kf[2 * NKS];
        u32x4 vf[4 * NDB];
#pragma unroll
        for (int f = 0; f < LAK; ++f) kf[f] = kfrag(f);
        int kc[2] = {0, 0};
        if constexpr (FP8) {
            kc[0] = k_code((j + 1) & 1, 0);
            kc[1] = k_code((j + 1) & 1, 1);
        }
        if constexpr (!LATE) dma_interval(j, vs);

        uint32_t Pd[QB][16];
        float ls[QB][2];
        // fp16 P: the tile's row sum is taken over the ROUNDED pairs with packed fp16 additions (half the
        // instructions of two fp32 chains; a tile's 16 values per chain stay below 2^12 and lose at most 2^-11
        // relative per addition, errors that are independent from tile to tile and average out over the row).
        constexpr bool PKSUM = PV_OP == OP_F16;
        f16x2 lsp[QB][2];
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) {
            ls[qb][0] = ls[qb][1] = 0.f;
            lsp[qb][0] = lsp[qb][1] = f16x2{(_Float16)0.f, (_Float16)0.f};
        }
        // slice c = (query block c / 16, dword i = c % 16): scores 2i, 2i+1 of that block
        auto exp_slice = [&](int c) {
            const int qv = c / 16, i = c % 16;
            Sc[i / 8][qv][(2 * i) % 16] = __builtin_amdgcn_exp2f(Sc[i / 8][qv][(2 * i) % 16]);
            Sc[i / 8][qv][(2 * i + 1) % 16] = __builtin_amdgcn_exp2f(Sc[i / 8][qv][(2 * i + 1) % 16]);
        };
        // Row sums: fp16 P -- packed fp16 additions of the rounded pairs (see PKSUM above); bf16 P -- two fp32 chains
        // over the unrounded values.  The dot-product instruction that would sum a packed pair in fp32 does not
        // overlap with a running MFMA (about 8 clocks each, unhidden); additions, maxima and exp2 hide completely.
        auto pack_slice = [&](int c) {
            const int qv = c / 16, i = c % 16;
            const float e0 = Sc[i / 8][qv][(2 * i) % 16], e1 = Sc[i / 8][qv][(2 * i + 1) % 16];
            Pd[qv][i] = pack2<PV_OP>(e0, e1);
            if constexpr (PKSUM) {
                lsp[qv][i & 1] += __builtin_bit_cast(f16x2, Pd[qv][i]);
            } else {
                ls[qv][0] += e0;
                ls[qv][1] += e1;
            }
        };
#pragma unroll
        for (int c = 0; c < PRE; ++c) exp_slice(c);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int t = 0; t < NA; ++t) {
            const int f = t / QB, qb = t % QB, ks = f >> 1, kb = f & 1;
            if (qb == 0 && f + LAK < 2 * NKS) kf[f + LAK] = kfrag(f + LAK);
            // the last steps of part A fetch the first V^T fragments of part B
            if constexpr (FP8) {  // (fewer steps than fragments: spread evenly)
#pragma unroll
                for (int g = t * LA / NA; g < (t + 1) * LA / NA; ++g) vf[g] = vfrag(g);
            } else {
                if (t >= NA - LA) vf[t - (NA - LA)] = vfrag(t - (NA - LA));
            }
            Sn[kb][qb] = score_mfma(kf[f], Qf[qb][ks], ks == 0 ? negm[qb] : Sn[kb][qb], kc[kb], q_code[qb]);
#pragma unroll
            for (int cc = 0; cc < CPA; ++cc) {
                const int c = t * CPA + cc;
                if (c + PRE < NCH) exp_slice(c + PRE);
                pack_slice(c);
            }
            __builtin_amdgcn_sched_barrier(0);
        }

        if constexpr (LATE) {  // the late half's barrier; its loads for the next interval follow at once
            dma_wait_and_sync();
            // (unconditional, to keep the iteration one block: past the end the last tile is
            // fetched again into buffers nobody reads, and awaited before the wavefront leaves)
            dma_interval(j + 1, next_vslot(vs));
            __builtin_amdgcn_sched_barrier(0);
        }

        if constexpr (STAG && DIT_PIPE_PRIO == 1) __builtin_amdgcn_s_setprio(0);
        if constexpr (STAG && DIT_PIPE_PRIO == 2) __builtin_amdgcn_s_setprio(1);
        // ---- part B: O += V^T(j) P(j) on MFMA, row maxima of S(j+1) on VALU ----
        float pm[QB][4];
#pragma unroll
        for (int qb = 0; qb < QB; ++qb)
#pragma unroll
            for (int e = 0; e < 4; ++e) pm[qb][e] = -INFINITY;
        // COPY (64 rows per wavefront): the score MFMAs always write Sn, which then sits in the
        // accumulation registers; the maxima are taken while the values are copied into Sc, the
        // vector-ALU side's buffer, whose previous contents part A has consumed by now.
        auto max_slice = [&](int c) {
            const int qv = c / 16, i = c % 16;
            const float s0 = Sn[i / 8][qv][(2 * i) % 16], s1 = Sn[i / 8][qv][(2 * i + 1) % 16];
            if constexpr (COPY) {
                Sc[i / 8][qv][(2 * i) % 16] = s0;
                Sc[i / 8][qv][(2 * i + 1) % 16] = s1;
            }
            pm[qv][i & 3] = max3(pm[qv][i & 3], s0, s1);
        };
#pragma unroll
        for (int u = 0; u < NB; ++u) {
            const int g = u / QB, qb = u % QB, kg = g / NDB, db = g % NDB;
            if (qb == 0 && g + LA < 4 * NDB) vf[g + LA] = vfrag(g + LA);
            const u32x4 pb = mk4(Pd[qb][4 * kg], Pd[qb][4 * kg + 1], Pd[qb][4 * kg + 2], Pd[qb][4 * kg + 3]);
            O[db][qb] = mfma32<PV_OP>(vf[g], pb, O[db][qb]);
            // the first two steps leave the last score MFMAs time to retire
            if (u >= 2) {
#pragma unroll
                for (int cc = 0; cc < CPB; ++cc) max_slice((u - 2) * CPB + cc);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
#pragma unroll
        for (int c = (NB - 2) * CPB; c < NCH; ++c) max_slice(c);
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) {
            if constexpr (PKSUM) {
                const f16x2 t2 = lsp[qb][0] + lsp[qb][1];
                l_run[qb] += (float)t2[0] + (float)t2[1];
            } else {
                l_run[qb] += ls[qb][0] + ls[qb][1];
            }
            asm volatile("" : "+v"(l_run[qb]));  // keeps the row-sum chain here (it would sink past the barrier)
        }
#pragma unroll
        for (int qb = 0; qb < QB; ++qb)
            mx_new[qb] = max_across_halves(fmaxf(max3(pm[qb][0], pm[qb][1], pm[qb][2]), pm[qb][3]));
        bool need = any_row_needs_shift();
        if constexpr (!LATE) dma_wait_and_sync();
        // rare paths, outside the pipelined block
        f32x16 (&Sp)[2][QB] = COPY ? Sc : Sn;  // the pending scores of tile j + 1
        const uint64_t mnext = mask_of(j + 1);
        if (mnext != ~0ull) {
            mask_apply(Sp, mnext);
            row_max(Sp);
            need = any_row_needs_shift();
        }
        // after the last tile these are scores of a stale buffer: never let them touch the state
        if (need && j < last) shift_rows(Sp);
    };

    // ---- prologue: tiles 0 (K, V) and 1 (K) start streaming, then Q is loaded while they fly ----
    if (n_steps > 0) {
        // the first two tile numbers come by scalar loads, which do not queue behind the query rows
        int t0 = 0, t1 = last > 0 ? 1 : 0;
        if constexpr (LISTED) {
            const int* tl = a.tile_list + (size_t)b * pv.nKT;
            t0 = tl[0];
            t1 = tl[t1];
        }
        dma_tiles(t0, 0, t0, 0);
        dma_tiles(t1, 1, t0, 1);  // K'(1); its V part lands in a buffer iteration 0 refills anyway
    }
    if constexpr (LISTED) {
        // lane i: list entry i, and the key mask of TILE i (looked up by tile number, so that the
        // two loads do not depend on each other)
        if (lane < n_steps) v_tile = a.tile_list[(size_t)b * pv.nKT + lane];
        if (lane < pv.nKT) {
            const uint64_t m = a.tile_mask[(size_t)b * pv.nKT + lane];
            v_mask_lo = (uint32_t)m;
            v_mask_hi = (uint32_t)(m >> 32);
        }
    }

    // ---- Q: rotate, fold scale*log2(e), round once, keep as B operands ----
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        qrow[qb] = qt * BQ + wave * (32 * QB) + qb * 32 + l32;
        const int qr = qrow[qb] < pv.Lq ? qrow[qb] : pv.Lq - 1;
        const int64_t base = pv.q_off + (int64_t)qr * a.sq_t;
        int pt = 0, ph = 0, pw = 0;
        if (a.tab) token_pos(qr, rg, pt, ph, pw);
        float rs = 1.f;
        if (a.qn.mode) rs = q_row_rstd<D>(a.qn, a.q, base, a.in_f32, half, pv.stat_off + qr);
        float xq[FP8 ? NQC : 1][8];  // FP8: the whole row is needed before its factor is known
        float am = 0.f;
#pragma unroll
        for (int ks = 0; ks < NQC; ++ks) {
            const int c = 2 * ks + half;
            float x[8];
            if (a.in_f32) load8(a.q, base + 8 * c, 1, x);
            else widen8(qraw[qb][ks], x);
            if (a.qn.mode) norm8(x, a.qn, rs, pv.h, D, c);
            if (a.tab) rope8(x, c, rg, a.tab, pt, ph, pw);
#pragma unroll
            for (int e = 0; e < 8; ++e) x[e] *= a.qscale;
            if constexpr (FP8) {
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    xq[ks][e] = x[e];
                    am = fmaxf(am, fabsf(x[e]));
                }
            } else {
                Qf[qb][ks] = pack8<QK_OP>(x);
            }
        }
        q_code[qb] = 0;
        if constexpr (FP8) {
            am = fmaxf(am, __shfl_xor(am, 32));
            const int ex = fp8_row_exponent(am);
            const float sc = pow2i(ex);
            q_code[qb] = 127 - ex;
            // chunk 2*ks + half of the row -> contraction step ks / 4, bytes 8*(ks % 4).. of the lane's 32
#pragma unroll
            for (int ks = 0; ks < NQC; ++ks) {
#pragma unroll
                for (int e = 0; e < 8; ++e) xq[ks][e] *= sc;
                const uint2 w = pack8_fp8(xq[ks]);
                Qf[qb][ks / 4][2 * (ks % 4)] = (int)w.x;
                Qf[qb][ks / 4][2 * (ks % 4) + 1] = (int)w.y;
            }
        }
    }

    if (n_steps > 0) {  // (a request with no valid key skips to the epilogue: zeros, lse = -inf)
    // scores of tile 0 become the first running maximum
    dma_wait_and_sync();
    f32x16 S0[2][QB], S1[2][QB];
    qk_tile(S0, 0);
    __syncthreads();  // every wavefront has read K'(0) before iteration 0 streams K'(2) over it
    if constexpr (STAG) {
        if (late) dma_interval(0, 0);
    }
    if (mask_of(0) != ~0ull) mask_apply(S0, mask_of(0));
    row_max(S0);  // finite: every listed tile holds at least one valid key
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        m_run[qb] = mx_new[qb];
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            negm[qb][r] = -m_run[qb];
            S0[0][qb][r] -= m_run[qb];
            S0[1][qb][r] -= m_run[qb];
        }
    }

    auto key_loop = [&](auto late_tag) {
        int j = 0, vs = 0;
        if constexpr (COPY) {
            for (; j < n_steps; ++j) {
                iteration(late_tag, S0, S1, j, vs);
                vs = next_vslot(vs);
            }
        } else {
            for (; j + 1 < n_steps; j += 2) {
                iteration(late_tag, S0, S1, j, vs);
                vs = next_vslot(vs);
                iteration(late_tag, S1, S0, j + 1, vs);
                vs = next_vslot(vs);
            }
            if (j < n_steps) iteration(late_tag, S0, S1, j, vs);
        }
    };
    if (late) {
        key_loop(std::true_type{});
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    } else {
        key_loop(std::false_type{});
    }
    }

    // ---- epilogue ----
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        const float l = l_run[qb] + __shfl_xor(l_run[qb], 32);
        const float inv = l > 0.f ? 1.0f / l : 0.f;
        if (qrow[qb] < pv.Lq) {
            const int64_t obase = pv.o_off + (int64_t)qrow[qb] * a.so_t;
#pragma unroll
            for (int db = 0; db < NDB; ++db)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const int d0 = 32 * db + 8 * g + 4 * half;
                    const float o0 = O[db][qb][4 * g + 0] * inv, o1 = O[db][qb][4 * g + 1] * inv;
                    const float o2 = O[db][qb][4 * g + 2] * inv, o3 = O[db][qb][4 * g + 3] * inv;
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
                a.lse[pv.lse_off + qrow[qb]] = v;
            }
        }
    }
}

// blockIdx -> logical workgroup such that each XCD (workgroups are dealt to the 8 XCDs round-robin)
// works through one contiguous range of logical workgroups: neighbours share K/V tiles in its L2.
__device__ __forceinline__ int xcd_contiguous_block() {
    const int nblk = gridDim.x, bid = blockIdx.x;
    const int xcd = bid & 7, idx = bid >> 3;
    const int chunk = nblk >> 3, rem = nblk & 7;
    return xcd * chunk + (xcd < rem ? xcd : rem) + idx;
}

// One sequence per batch entry, all of the same length.
template <int D, int QB, int QK_OP, int PV_OP, int NW, bool LISTED>
__global__ void __launch_bounds__(64 * NW, QB == 1 ? 2 : 1) attn_fwd_pipe_kernel(const AttnArgs a) {
    const int logical = xcd_contiguous_block();
    PipeView pv;
    if constexpr (LISTED) {  // requests of different lengths: interleaved (see attn_fwd_kernel)
        pv.b = logical % a.B;
        const int rest = logical / a.B;
        pv.qt = rest % a.nQT;
        pv.h = rest / a.nQT;
    } else {
        const int bh_ = logical / a.nQT;
        pv.qt = logical % a.nQT;
        pv.b = bh_ / a.H;
        pv.h = bh_ - pv.b * a.H;
    }
    const int bh = pv.b * a.H + pv.h;
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
    attn_pipe_body<D, QB, QK_OP, PV_OP, NW, LISTED>(a, pv);
}

// Packed requests of different lengths (self-attention, no lists).  XCD x owns the (request, head)
// pairs with (table index * H + head) % 8 == x and walks them in table order, so every XCD gets
// a near-equal share of every request and meets the longest ones first.  Workgroups past the end
// of their XCD's queue leave at once.
template <int D, int QK_OP, int PV_OP, int NW>
__global__ void __launch_bounds__(64 * NW, 2) attn_fwd_pipe_varlen_kernel(const AttnArgs a, const VarlenTable vt) {
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
    attn_pipe_body<D, 1, QK_OP, PV_OP, NW, false>(a, pv);
}

template <int D, int QB, int QK_OP, int PV_OP, int NW, bool LISTED>
hipError_t launch_attn_pipe_inst(const AttnArgs& a, hipStream_t s) {
    auto kern = attn_fwd_pipe_kernel<D, QB, QK_OP, PV_OP, NW, LISTED>;
    constexpr int smem = pipe_lds_bytes<D, NW>();
    static std::atomic<uint64_t> attr_set{0};
    hipError_t e = allow_dynamic_lds(kern, smem, attr_set);
    if (e != hipSuccess) return e;
    const dim3 grid((unsigned)((int64_t)a.nQT * a.B * a.H));
    hipLaunchKernelGGL(kern, grid, dim3(64 * NW), smem, s, a);
    return hipGetLastError();
}

template <int D, int QK_OP, int PV_OP, int NW>
hipError_t launch_attn_pipe_varlen_inst(const AttnArgs& a, const VarlenTable& vt, hipStream_t s) {
    auto kern = attn_fwd_pipe_varlen_kernel<D, QK_OP, PV_OP, NW>;
    constexpr int smem = pipe_lds_bytes<D, NW>();
    static std::atomic<uint64_t> attr_set{0};
    hipError_t e = allow_dynamic_lds(kern, smem, attr_set);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, dim3((unsigned)(8 * vt.queue_len)), dim3(64 * NW), smem, s, a, vt);
    return hipGetLastError();
}

}  // namespace dit
