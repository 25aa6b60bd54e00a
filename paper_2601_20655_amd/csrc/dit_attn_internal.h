// Internal declarations shared by the host dispatch and the gfx950 kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>

namespace dit {

constexpr int kBK = 64;         // keys per K/V tile
constexpr int kThreads = 256;   // four wavefronts per workgroup
constexpr float kLog2e = 1.4426950408889634f;

enum OperandType { OP_BF16 = 0, OP_F16 = 1, OP_FP8 = 2 };  // OP_FP8 (e4m3): score operands only

// One K/V tile as it sits in LDS (and, pre-packed, in workspace): 64 rows of K' followed by
// D rows of V^T.  Rows carry 16 bytes of padding so that the 16-byte operand reads of 16
// consecutive rows fall into distinct LDS banks and every address is lane_base + immediate.
// Each part is padded to 4*n + 2 KiB so that four wavefronts can stream it with n
// wavefront-wide 16-byte loads each plus one more load on two of them.
template <int D>
struct TileGeom {
    static constexpr int KROW = D * 2 + 16;      // bytes per K' row (one key, D channels)
    static constexpr int VROW = kBK * 2 + 16;    // bytes per V^T row (one channel, 64 keys)
    static constexpr int PART_KIB = D == 128 ? 18 : 10;
    static constexpr int K_BYTES = PART_KIB * 1024;  // >= 64 * KROW
    static constexpr int V_BYTES = PART_KIB * 1024;  // >= D * VROW
    static constexpr int TILE_BYTES = K_BYTES + V_BYTES;
    static_assert(kBK * KROW <= K_BYTES && D * VROW <= V_BYTES && PART_KIB % 4 == 2, "tile part sizes");
    // 8-bit (e4m3) score operands: the K part starts with 64 rows of D bytes (same padding rule)
    // followed by one byte per key, 127 - e, where the row was multiplied by 2^e before rounding;
    // the rest of the part is unused.
    static constexpr int KROW8 = D + 16;
    static constexpr int KSCALE_OFF = kBK * KROW8;
    static_assert(KSCALE_OFF + kBK <= K_BYTES, "8-bit K' rows and their scales fit the K part");
};

inline size_t tile_bytes(int D) { return D == 128 ? TileGeom<128>::TILE_BYTES : TileGeom<64>::TILE_BYTES; }

// Rotary tables: float2 (cos, sin) per (axis, position index, pair).  Entry of axis a is
// tab[off[a] + p * hd[a] + i], position index p counted from the grid origin.
struct RopeGeom {
    int hd[3];   // pairs per axis (d_a / 2)
    int off[3];  // first table entry of each axis
    int Hg, Wg;  // latent grid height and width (token -> (t,h,w) decode)
};

// RMS normalisation of q or k rows ahead of the rotation: y = x * gamma / sqrt(mean(x^2) + eps).
struct NormArgs {
    int mode;            // 0 off; 1 mean over the D channels of the head; 2 over all H*D channels of the token
    float eps;
    const float* gamma;  // nullable [H*D]
    const float* rstd;   // mode 2: 1/sqrt(mean + eps) per token row, filled by launch_token_rstd
};

// per-token 1/sqrt(mean over H*D channels + eps)
struct RstdArgs {
    const void* x;
    float* rstd;  // [B*L]
    int64_t s_b, s_t, s_h;
    int B, L, H, D;
    int in_f32;
    float eps;
};

struct TableArgs {
    float2* tab;
    int n[3];       // positions per axis (T, Hg, Wg)
    int origin[3];  // t0, h0, w0
    RopeGeom rg;
    double base;
    int total;
};

struct PackArgs {
    const void* k;
    const void* v;
    const uint8_t* valid;  // nullable [B, Lk]
    int* key_src;          // with valid: [B, nKT, 64] source key of every tile slot, -1 = empty (launch_key_compact)
    const int* kv_len;     // nullable [B, 2] (instead of valid): the keys that attend are the first kv_len[b][0] of
                           // [0, ...) and the first kv_len[b][1] of [second_start, Lk); the pre-pack works out every
                           // slot's source key, the tile masks, the tile list and its counts from the two numbers
    int second_start;      // with kv_len: first key of the second range (decoupled form: = split)
    uint8_t* tiles;        // [B*H, nKT, TILE_BYTES]
    uint64_t* tile_mask;   // nullable [B, nKT]
    int* tile_list;        // nullable [B, nKT], filled by launch_tile_compact
    int* tile_count;       // nullable [B]
    int* tile_count_a;     // nullable [B]: listed tiles that belong to the first key group
    int split, nTA;        // split > 0: keys [0, split) fill tiles [0, nTA), keys [split, Lk) the rest
    const float2* tab;     // nullable (no rotation)
    int B, H, Lk, nKT;
    int in_f32;
    int v_layout;  // tile layout: 0 for kernels on 32x32x16 MFMAs, 1 for 16x16x32 (key order in V^T rows, chunk swizzle; see pack_tile)
    int64_t sk_b, sk_t, sk_h, sv_b, sv_t, sv_h;
    RopeGeom rg;
    NormArgs kn;  // normalisation of k rows (rstd indexed by b*Lk + key, packed requests: by token)
};

struct AttnArgs {
    const void* q;
    void* out;
    float* lse;                 // nullable
    const uint8_t* tiles;       // pre-packed K'/V^T tiles
    const uint64_t* tile_mask;  // nullable [B, nKT]; bit = key of the tile attends
    const int* tile_list;       // with tile_mask: [B, nKT] indices of the tiles with any valid key, ascending
    const int* tile_count;      // with tile_mask: [B] how many entries of tile_list are used
    const int* tile_count_a;    // decoupled cross-attention: [B] how many of them form the first softmax
    const float2* tab;          // nullable: no rotation of q
    // raw K/V for the fused staging path
    const void* k;
    const void* v;
    int64_t sk_b, sk_t, sk_h, sv_b, sv_t, sv_h;
    int B, H, Lq, Lk, nKT, nQT;
    int in_f32, out_f32;
    int64_t sq_b, sq_t, sq_h, so_b, so_t, so_h;
    RopeGeom rg;
    float qscale;  // softmax scale * log2(e), folded into q'
    NormArgs qn;   // normalisation of q rows (rstd indexed by b*Lq + row, packed requests: by token)
};

// Several requests with their own latent grids packed back to back along the token axis
// (batched serving): one descriptor per request, passed to the kernels by value.
constexpr int kMaxRequests = 64;
struct ReqDesc {
    int tok0;    // first token of the request in the packed tensors
    int L;       // its tokens = T * Hg * Wg
    int Hg, Wg;  // grid height and width (token -> position decode)
    int nKT;     // key tiles
    int nQT;     // query tiles
    int tile0;   // key tiles of all earlier table entries (per head)
    int pad_;
};
// Table order is the order workgroups are handed out in (longest request first), not token order.
struct VarlenTable {
    int n;             // requests
    int total_tokens;  // sum of L
    int total_tiles;   // sum of nKT
    int queue_len;     // workgroups per XCD queue; the grid is 8 * queue_len
    ReqDesc r[kMaxRequests];
};

// Kernels that need more than the default 64 KiB of dynamic LDS: the attribute is set once per kernel
// instantiation and device (`done` is that instantiation's bit set of devices), not on every launch.
template <typename K>
inline hipError_t allow_dynamic_lds(K kern, int bytes, std::atomic<uint64_t>& done) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    const uint64_t bit = 1ull << (dev & 63);
    if (done.load(std::memory_order_acquire) & bit) return hipSuccess;
    e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    if (e == hipSuccess) done.fetch_or(bit, std::memory_order_release);
    return e;
}

// Records "<where>: <HIP error text>" for dit_last_hip_error() of the calling thread; returns DIT_ERR_HIP.
int report_hip_error(hipError_t e, const char* where);

hipError_t launch_rope_table(const TableArgs& a, hipStream_t s);
hipError_t launch_token_rstd(const RstdArgs& a, hipStream_t s);
hipError_t launch_prepack_varlen(const PackArgs& a, const VarlenTable& vt, int D, int qk_op, int pv_op, hipStream_t s);
hipError_t launch_attn_pipe_varlen(const AttnArgs& a, const VarlenTable& vt, int D, int qk_op, int pv_op, int nw,
                                   hipStream_t s);
hipError_t launch_prepack(const PackArgs& a, int D, int qk_op, int pv_op, hipStream_t s);
// pipelined self-attention on 16x16x32 MFMAs (16-bit operands, 32 rows per wavefront, tiles packed with v_layout 1)
hipError_t launch_attn_pipe16(const AttnArgs& a, int D, int qk_op, int pv_op, int nw, hipStream_t s);
hipError_t launch_attn_pipe16_varlen(const AttnArgs& a, const VarlenTable& vt, int D, int qk_op, int pv_op, int nw,
                                     hipStream_t s);
hipError_t launch_attn_pipe16_chain(const AttnArgs& a, int D, int qk_op, int pv_op, int nw, hipStream_t s);
// before launch_prepack when a.valid is set: the valid keys of every batch entry (of each key group) in
// ascending order, densely over the tile slots
hipError_t launch_key_compact(const PackArgs& a, hipStream_t s);
// after launch_prepack: compact the non-empty tiles of every batch entry into tile_list / tile_count
hipError_t launch_tile_compact(const PackArgs& a, hipStream_t s);
// qb = 32-row query blocks per wavefront (1 or 2)
hipError_t launch_attn(const AttnArgs& a, int D, int qb, int qk_op, int pv_op, bool fused,
                       hipStream_t s);
// plain kernel, two softmaxes (AttnArgs::tile_count_a set), 32 rows per wavefront
hipError_t launch_attn_split(const AttnArgs& a, int D, int qk_op, int pv_op, hipStream_t s);

// ---- dense projection y = x w^T + bias ----
constexpr int kLinBM = 256;  // tokens per workgroup tile
constexpr int kLinBN = 256;  // output features per workgroup tile
constexpr int kLinBK = 64;   // contraction indices per step
struct LinearArgs {
    const uint16_t* x;     // [M, K] bf16, row stride ldx
    const uint16_t* w;     // [N, K] bf16, row stride ldw
    const uint16_t* bias;  // [N] bf16, nullable
    void* y;               // [M, N] bf16 or fp32, row stride ldy
    int M, N, K;           // K a multiple of kLinBK, N a multiple of 8
    int64_t ldx, ldw, ldy;
    int nTM, nTN;          // tiles along M and N
    int out_f32;
    // Fused q/k/v form (qkv != 0; N = 3 H D, head_dim 128, the M tokens are ONE sequence): features [0, HD) are q
    // rows and go to y as [token, head, channel] with the strides below; features [HD, 2 HD) are k rows, which are
    // rotated, rounded to the score operand type and written as the K' parts of the attention kernel's tile images;
    // features [2 HD, 3 HD) are v rows, rounded to the PV operand type and written transposed as the V^T parts.
    int qkv;
    int qkv_H, qkv_nKT;          // heads; key tiles = ceil(M / 64)
    uint8_t* qkv_tiles;          // [H, nKT, TILE_BYTES], layout of the 16x16x32 kernels (PackArgs::v_layout 1)
    const float2* qkv_tab;       // rotation table
    RopeGeom qkv_rg;
    int64_t qkv_sq_t, qkv_sq_h;  // element strides of the q rows in y
    int qkv_qk_f16, qkv_pv_f16;  // operand types of the two tile parts: fp16 (saturating) or bf16
    int qkv_norm;                // 1: k rows are RMS-normalised over the head's channels before the rotation;
                                 // 2: over all heads of the token -- the weights here, the factor in k_rescale_kernel
    float qkv_eps;
    const float* qkv_kgamma;     // nullable [H*128]
};
hipError_t launch_linear(const LinearArgs& a, hipStream_t s);

// Second half of the per-token normalisation of the fused q/k/v projection: the projection's epilogue left, in the
// spare bytes behind the K' rows of every tile image, one float per key slot = the sum of squares of that token's k
// row over the head's channels; this pass adds the heads' shares, and multiplies the token's K' rows of all heads by
// 1/sqrt(sum / (H*D) + eps).
struct KRescaleArgs {
    uint8_t* tiles;  // [H, nKT, TILE_BYTES], head_dim 128
    int H, nKT, L;   // heads, key tiles, tokens
    float eps;
    int qk_f16;      // K' rows hold fp16 (else bf16)
};
hipError_t launch_k_rescale(const KRescaleArgs& a, hipStream_t s);

}  // namespace dit
