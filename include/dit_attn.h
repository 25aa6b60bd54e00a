/*
 * dit_attn.h -- C ABI of the MI355X (gfx950) DiT attention library.
 *
 * The library computes the attention of the Diffusion stage of a Wan2.1-class video
 * diffusion transformer -- the stage that does the generating in the image-to-video workflow
 * the OnePiece paper serves (Sec. 2.4, the AIGC workflow) -- as the user function a
 * TaskWorker runs on tensors that already sit in GPU memory (Sec. 4.4, TaskWorker).
 * The paper names this workload but gives no mathematics for it; what is computed is
 * defined here, and a CPU fp64 statement of the same definition lives in oracle/.
 *
 * Common rules for every entry point
 *  - All tensor pointers are DEVICE pointers owned by the caller.  The library never
 *    allocates, frees or synchronises: kernels are enqueued on `stream` (a hipStream_t
 *    passed as void*, NULL = the default stream) and the call returns at once.
 *  - Tensors are addressed as  base + b*stride.batch + n*stride.token + h*stride.head + c
 *    (strides in ELEMENTS, channel stride 1).  [B,L,H,D] and [B,H,L,D] both fit.
 *    Every row start must be 16-byte aligned, else DIT_ERR_ALIGNMENT.
 *  - `workspace` is caller-owned device scratch of at least *_workspace_bytes(params)
 *    bytes, 256-byte aligned.  Its contents are overwritten by each call; two calls that
 *    share one workspace must be ordered on one stream.
 *  - Arguments are validated before anything is launched: a call that returns any error but
 *    DIT_ERR_HIP has had no effect.  DIT_ERR_HIP means a HIP launch or event call failed part-way
 *    through the call's kernel sequence; the workspace and the output may then be partly
 *    written.  No exception crosses the ABI.
 *  - Rows may not overlap: every token and head stride is at least D, and the larger of the two
 *    clears all rows the smaller one steps over (token >= H*head or head >= L*token); with
 *    B > 1 the batch stride is at least D.  Else DIT_ERR_INVALID_ARG.
 *  - Arithmetic: inputs bf16 (or fp32), q and k rotated and scaled in fp32, then rounded
 *    once (nearest-even) to the 16-bit MFMA operand type chosen by `flags`; scores,
 *    softmax statistics and the output accumulator are fp32; output bf16 or fp32.
 */
#ifndef DIT_ATTN_H
#define DIT_ATTN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    DIT_OK = 0,
    DIT_ERR_INVALID_ARG = -1, /* NULL pointer, non-positive size, bad RoPE split, bad enum */
    DIT_ERR_UNSUPPORTED = -2, /* head_dim other than 64/128, or a flag combination not built */
    DIT_ERR_ALIGNMENT = -3,   /* a base pointer or stride breaks 16-byte row alignment */
    DIT_ERR_WORKSPACE = -4,   /* workspace NULL, misaligned or too small */
    DIT_ERR_HIP = -5          /* a HIP runtime call failed; see dit_last_hip_error() */
} dit_status;

typedef enum { DIT_BF16 = 0, DIT_F32 = 1 } dit_dtype;

/*
 * flags: precision of the 16-bit MFMA operands and the K/V staging strategy.
 * 0 selects the defaults: fp16 operands for both products, K/V pre-packed.
 *
 * fp16 operands (11 significant bits) keep max|err| near 2e-3 x output RMS against the
 * fp64 definition at 32,760 tokens; bf16 operands (8 bits) give about 2e-2.  Both run at
 * the same MFMA rate.  fp16 operands SATURATE: where |scale*log2(e)*q'|, |k'| or |v| exceeds 65504, the
 * largest finite fp16 number, the operand becomes +-65504 (bf16 inputs can hold such values; the result is
 * then that of the clamped operands: finite and deterministic, but not the definition's).  A caller whose
 * activations can be that large opts out with DIT_FLAG_QK_BF16 | DIT_FLAG_PV_BF16, which keep the full
 * bf16 range at bf16 precision.
 */
enum {
    DIT_FLAG_QK_BF16 = 1u << 0, /* round q', k' to bf16 */
    DIT_FLAG_QK_F16 = 1u << 1,  /* round q', k' to fp16 (default) */
    DIT_FLAG_PV_BF16 = 1u << 2, /* round P to bf16, V stays bf16 */
    DIT_FLAG_PV_F16 = 1u << 3,  /* round P to fp16, V widened bf16 -> fp16 (default) */
    /* K/V staging for dit_attn_forward:
     *  PREPACK (default): one memory-bound pass rotates K and lays K', V^T out in workspace
     *  as ready-to-copy LDS tile images; the attention kernel then only copies tiles.
     *  FUSED: no K/V workspace; each K tile is rotated while it is staged into LDS and
     *  each V tile is transposed in registers.  Requires bf16 inputs and PV_BF16. */
    DIT_FLAG_KV_PREPACK = 1u << 4,
    DIT_FLAG_KV_FUSED = 1u << 5,
    /* 256 query rows per workgroup (64 per wavefront, one workgroup per CU) instead of
     * 128 (32 per wavefront, two workgroups per CU). */
    DIT_FLAG_WIDE_QTILE = 1u << 6,
    /* Self-attention with pre-packed K/V normally runs a software-pipelined kernel (scores of
     * tile j+1 on the matrix pipe while tile j's softmax runs on the vector ALU, tiles streamed
     * global->LDS directly).  This flag selects the plain one-tile-at-a-time kernel instead
     * (the one cross-attention and FUSED always use); same results up to rounding order. */
    DIT_FLAG_SIMPLE_SCHEDULE = 1u << 7,
    /* Workgroup size of the pipelined self-attention kernel.  BIG: 8 wavefronts, 256 query rows
     * share each K/V tile in LDS (half the L2 -> LDS tile traffic).  SMALL: 4 wavefronts, 128
     * rows, two workgroups per CU.  Neither flag: BIG when that still gives every CU at least
     * two workgroups, else SMALL. */
    DIT_FLAG_BIG_WORKGROUP = 1u << 8,
    DIT_FLAG_SMALL_WORKGROUP = 1u << 9,
    /* Cross-attention runs the plain kernel by default: with a dozen key tiles per query tile its
     * shorter prologue beats the pipelined kernel's better steady state (measured).  This flag
     * selects the pipelined kernel there too (at most 64 key tiles, i.e. Lk <= 4096 for the joint
     * form, else DIT_ERR_UNSUPPORTED).  No effect on self-attention. */
    DIT_FLAG_PIPELINED_SCHEDULE = 1u << 10,
    /* The workspace still holds the rotated, pre-packed K'/V^T tile images (and the rotation table,
     * the key tile lists and masks) that an earlier forward call of the SAME entry point wrote for the
     * same k, v, kv_valid, shapes, grid(s), origin, rope_base, norm (mode, eps, k_gamma), key split,
     * operand-type flags and, for self-attention, the flags that choose the matrix-instruction shape the
     * tiles are laid out for (MFMA_32X32, WIDE_QTILE, SIMPLE_SCHEDULE, QK_FP8); that call must precede
     * this one in stream order.  The key-side passes are skipped: k, v and kv_valid are not read and may
     * be NULL.  q, scale, q_gamma, the output and the workgroup-size flags may differ from call to call.
     * This is the K/V cache of a denoising loop: the conditioning keys and values of cross-attention are
     * the same at every step, and a caller that evaluates several query sets against one K, V pays for
     * one pre-pack.  Nothing records what the workspace holds: the caller vouches for it.  Not with
     * DIT_FLAG_KV_FUSED (DIT_ERR_INVALID_ARG). */
    DIT_FLAG_KV_RESIDENT = 1u << 11,
    /* Score product on 8-bit operands: q' and k' are rounded to e4m3 (4 significant bits), each row
     * with its own power-of-two factor that the matrix instruction applies; P and V keep their 16-bit
     * types and everything else stays fp32.  The matrix pipe runs this product at twice the 16-bit
     * rate and reads half the K' bytes.  THE ERROR IS TEN TIMES THAT OF THE 16-BIT PATH and does not
     * meet its contract: with unit-variance inputs expect an RMS error near 3e-2 x output RMS and a
     * largest error near 0.2 x output RMS.  Self-attention entry points only (dit_attn_forward with the
     * pipelined 32-rows-per-wavefront kernel, dit_attn_varlen_forward); excludes QK_BF16 / QK_F16
     * (DIT_ERR_INVALID_ARG) and KV_FUSED, SIMPLE_SCHEDULE, WIDE_QTILE, cross-attention
     * (DIT_ERR_UNSUPPORTED).  Never selected by default. */
    DIT_FLAG_QK_FP8 = 1u << 12,
    /* Self-attention entry points (dit_attn_forward with the pipelined 32-rows-per-wavefront kernel,
     * dit_attn_varlen_forward) run on 16x16x32 matrix instructions by default: under the board's power limit
     * they deliver more flops per joule than 32x32x16 ones (measured: the kernel is 8 % faster on N(0,1) inputs).
     * This flag selects the 32x32x16 form of the same pipeline instead; same results up to rounding order.  It
     * decides the key order inside the pre-packed V^T tiles, so it belongs to the flags that may not change
     * between the calls that share tiles under DIT_FLAG_KV_RESIDENT.  No effect on cross-attention and on the
     * forms that only exist on 32x32x16 instructions (QK_FP8, WIDE_QTILE, SIMPLE_SCHEDULE, KV_FUSED). */
    DIT_FLAG_MFMA_32X32 = 1u << 13
};

typedef struct {
    int64_t batch, token, head; /* element strides; the channel stride is 1 */
} dit_strides;

/*
 * Optional RMS normalisation of the q and k rows, applied in fp32 before the rotation (the
 * per-block q/k normalisation of the DiT, fused so that normalised q and k never travel through
 * memory):   y[c] = x[c] * gamma[c] / sqrt(mean(x^2) + eps).
 * DIT_NORM_HEAD: the mean runs over the D channels of each head.
 * DIT_NORM_TOKEN: over all H*D channels of the token (one more memory-bound pass over q and k
 * computes the per-token factor into workspace).
 * q_gamma, k_gamma: DEVICE fp32 arrays of H*D weights, head-major, 16-byte aligned; NULL = all 1.
 * eps >= 0.  A zero-initialised struct switches the normalisation off.  Not available with
 * DIT_FLAG_KV_FUSED (DIT_ERR_UNSUPPORTED).
 */
typedef enum { DIT_NORM_NONE = 0, DIT_NORM_HEAD = 1, DIT_NORM_TOKEN = 2 } dit_norm_mode;

typedef struct {
    int32_t mode; /* dit_norm_mode */
    float eps;
    const float *q_gamma;
    const float *k_gamma;
} dit_qk_norm;

/*
 * Self-attention over the L = T*Hg*Wg tokens of a latent grid, no mask.
 * Token n (row-major, w fastest) sits at integer position
 *     (t, h, w) = (t0 + n / (Hg*Wg), h0 + (n / Wg) % Hg, w0 + n % Wg).
 * 3-axis rotary embedding on q and k: the D channels are three contiguous sections
 * (t, h, w) of sizes d_t, d_h, d_w (each even, 0 allowed, sum D).  In section a at
 * channel offset o_a, pair i is channels (o_a+2i, o_a+2i+1); with
 * phi = pos_a * rope_base^(-2i/d_a):
 *     x'[2i] = x[2i] cos(phi) - x[2i+1] sin(phi),  x'[2i+1] = x[2i] sin(phi) + x[2i+1] cos(phi).
 * out[n] = sum_m softmax_m(scale * <q'_n, k'_m>) v_m over all L keys.
 */
typedef struct {
    int32_t B, H, D;       /* batch, heads, head_dim (64 or 128) */
    int32_t T, Hg, Wg;     /* latent grid */
    int32_t t0, h0, w0;    /* position origin */
    int32_t d_t, d_h, d_w; /* RoPE split */
    float rope_base;       /* e.g. 10000 */
    float scale;           /* <= 0 selects 1/sqrt(D) */
    int32_t in_dtype;      /* dit_dtype of q, k, v */
    int32_t out_dtype;     /* dit_dtype of out */
    uint32_t flags;        /* DIT_FLAG_* */
    dit_strides sq, sk, sv, so;
    dit_qk_norm norm;      /* zero = off */
} dit_self_attn_params;

/* Bytes of workspace dit_attn_forward needs for these params (0 on invalid params). */
size_t dit_attn_workspace_bytes(const dit_self_attn_params *p);

/*
 * The spatiotemporal self-attention of one transformer block of the Diffusion stage (Sec. 2.4),
 * run as a TaskWorker's user function on device-resident tensors (Sec. 4.4); the definition is the
 * comment on dit_self_attn_params.
 * q, k, v: [B, L, H, D] by strides, in_dtype.  out: same logical shape, out_dtype.
 * lse (nullable): fp32 [B, H, L] dense, natural-log sum of exp(scale * score) per row.
 */
dit_status dit_attn_forward(const void *q, const void *k, const void *v, void *out, float *lse,
                            const dit_self_attn_params *p, void *workspace,
                            size_t workspace_bytes, void *stream);

/*
 * Cross-attention of Lq query tokens over Lk conditioning tokens (text then image
 * embeddings, concatenated by the caller), no positional rotation.
 * Lk_split = 0 (or Lk): ONE joint softmax over the Lk keys.
 * 0 < Lk_split < Lk: decoupled form -- keys [0, Lk_split) and [Lk_split, Lk) are two
 * conditioning sequences with a softmax each, and the two attention outputs are added:
 *     out = softmax(scale q k_A^T) v_A + softmax(scale q k_B^T) v_B;
 * a sequence without a valid key contributes zero.  The first partial result is held in fp16
 * while the second is accumulated.  lse must be NULL and PIPELINED_SCHEDULE / WIDE_QTILE are
 * not available in this form (DIT_ERR_UNSUPPORTED).  kv_valid (nullable): uint8 [B, Lk] dense, 1 = key attends, 0 = padding.
 * A request with no valid key yields out = 0 and lse = -inf.
 * Flags: QK_*, PV_*, WIDE_QTILE, PIPELINED_SCHEDULE and (with it) the workgroup-size flags apply; K/V are
 * always pre-packed.  With kv_valid, the valid keys of a request (of each sequence in the decoupled form)
 * are packed densely, in ascending order, into 64-key tiles: a request costs ceil(valid keys / 64)
 * tiles per sequence wherever its padding sits, and only the last of them is partly filled.
 */
typedef struct {
    int32_t B, H, D;
    int32_t Lq, Lk;
    float scale;      /* <= 0 selects 1/sqrt(D) */
    int32_t in_dtype; /* dit_dtype of q, k, v */
    int32_t out_dtype;
    uint32_t flags;
    int32_t Lk_split; /* 0: joint softmax; else first key of the second conditioning sequence */
    dit_strides sq, sk, sv, so;
    dit_qk_norm norm; /* zero = off */
} dit_cross_attn_params;

size_t dit_cross_attn_workspace_bytes(const dit_cross_attn_params *p);

/* The text/image cross-attention of the same block (Sec. 2.4: the Diffusion stage is conditioned on the
 * text and image encoders' outputs); the definition is the comment on dit_cross_attn_params. */
dit_status dit_cross_attn_forward(const void *q, const void *k, const void *v,
                                  const uint8_t *kv_valid, void *out, float *lse,
                                  const dit_cross_attn_params *p, void *workspace,
                                  size_t workspace_bytes, void *stream);

/* The same computation for batched requests whose conditioning sequences differ in LENGTH (Sec. 4.3: in
 * Individual Mode the requests of a queue are handed to a worker as one batch; Sec. 2.4: a text sequence
 * padded to a fixed length followed by an image sequence), with the lengths themselves instead of a byte
 * mask: the keys that attend in request b are the first kv_len[2b] keys of [0, second_start) and the first
 * kv_len[2b + 1] keys of [second_start, Lk).
 *   kv_len        DEVICE pointer, int32 [B, 2], 4-byte aligned, read by the pre-pack pass on `stream`; counts
 *                 outside their range are clamped to it (negative: 0).  May be NULL with
 *                 DIT_FLAG_KV_RESIDENT (the tiles of an earlier call are reused and nothing key-side is read).
 *   second_start  0 .. Lk; with p->Lk_split in (0, Lk) (one softmax per sequence) it must equal Lk_split,
 *                 else DIT_ERR_INVALID_ARG.
 * Everything else -- q, k, v, out, lse, params, flags, workspace (same size: dit_cross_attn_workspace_bytes),
 * errors -- as dit_cross_attn_forward.  No mask is read and no key list is built: the pre-pack pass places each
 * key from the two counts, so two small passes of the mask form (key compaction, tile list) do not run.
 * A request with both counts 0 gets out = 0 and lse = -inf.  Ownership: the caller keeps kv_len alive and
 * unchanged until the work enqueued on `stream` has finished. */
dit_status dit_cross_attn_forward_lengths(const void *q, const void *k, const void *v,
                                          const int32_t *kv_len, int32_t second_start, void *out,
                                          float *lse, const dit_cross_attn_params *p, void *workspace,
                                          size_t workspace_bytes, void *stream);

/*
 * dit_cross_attn_forward for callers that cannot allocate device memory or take a workspace from
 * an allocator: code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.
 * Same arguments, results, flags and errors as dit_cross_attn_forward, minus the workspace: the
 * scratch is a device array of DIT_STATIC_WORKSPACE_BYTES bytes that is part of the library image
 * (every GPU the library runs on holds its own copy until the process ends).  The call makes no
 * hipMalloc / hipFree and calls no allocating routine; it works on the device that is current.
 *  - DIT_ERR_WORKSPACE if dit_cross_attn_workspace_bytes(p) exceeds DIT_STATIC_WORKSPACE_BYTES
 *    (the batched 14B-class case -- 4 requests x 40 heads x 769 keys, d128 -- needs 73.2 MiB).
 *  - The first call on a device looks the array's address up (hipGetSymbolAddress; this may load
 *    the library's code object on that device): make one call before capturing a graph.
 *  - All calls on one GPU share the one array: calls that overlap on a GPU (two streams, two
 *    threads) race, and the caller must order them.  The array keeps what the last call left, and
 *    nothing in it has to start at zero: every call writes each mask, list, count and tile before
 *    it reads it.  With DIT_FLAG_KV_RESIDENT the tiles of the last call ON THIS ENTRY POINT AND GPU
 *    are reused, under that flag's rules.
 */
#define DIT_STATIC_WORKSPACE_BYTES (96u << 20)

dit_status dit_cross_attn_forward_static(const void *q, const void *k, const void *v,
                                         const uint8_t *kv_valid, void *out, float *lse,
                                         const dit_cross_attn_params *p, void *stream);

/*
 * Self-attention of several requests in one call (batched serving: the Diffusion stage works on
 * a batch of Tasks whose videos differ in resolution and length, Sec. 4.4 "TaskWorker").
 * Request i has its own latent grid grids[i] = (T, Hg, Wg) and L_i = T*Hg*Wg tokens; the requests
 * are packed back to back along the token axis, request i occupying rows
 * [sum_{j<i} L_j, sum_{j<=i} L_j) of q, k, v and out, each addressed as
 * base + n*stride.token + h*stride.head + c (stride.batch is ignored).  A token attends to the
 * tokens of its own request only; positions, rotation and softmax are those of dit_attn_forward
 * applied per request, with one origin, RoPE split, base and scale for all.
 * `grids` is a HOST array of n_requests entries, read during the call only.  At most
 * DIT_MAX_REQUESTS requests and 2^24 tokens in total (DIT_ERR_UNSUPPORTED beyond).
 * Flags: QK_*, PV_*, BIG_WORKGROUP / SMALL_WORKGROUP; KV_FUSED, WIDE_QTILE and SIMPLE_SCHEDULE are
 * not available (DIT_ERR_UNSUPPORTED).
 * lse (nullable): fp32 [H, total tokens] dense.
 */
#define DIT_MAX_REQUESTS 64

typedef struct {
    int32_t T, Hg, Wg;
} dit_grid;

typedef struct {
    int32_t n_requests, H, D;
    const dit_grid *grids; /* host pointer */
    int32_t t0, h0, w0;    /* position origin of every request */
    int32_t d_t, d_h, d_w; /* RoPE split */
    float rope_base;
    float scale;           /* <= 0 selects 1/sqrt(D) */
    int32_t in_dtype, out_dtype;
    uint32_t flags;
    dit_strides sq, sk, sv, so;
    dit_qk_norm norm; /* zero = off */
} dit_varlen_attn_params;

size_t dit_attn_varlen_workspace_bytes(const dit_varlen_attn_params *p);

dit_status dit_attn_varlen_forward(const void *q, const void *k, const void *v, void *out,
                                   float *lse, const dit_varlen_attn_params *p, void *workspace,
                                   size_t workspace_bytes, void *stream);

/*
 * Dense projection of token rows: y[m, n] = sum_k x[m, k] * w[n, k] + bias[n] -- the query, key,
 * value and output projections either side of attention in a transformer block of the Diffusion
 * stage (Sec. 2.4); weights are stored [out features, in features] as the model's linear layers
 * keep them, so the fused q/k/v projection is one call on the three weights stacked along n.
 * x: [M, K] bf16, w: [N, K] bf16, bias: [N] bf16 or NULL, y: [M, N] bf16 or fp32 (out_dtype); all
 * DEVICE pointers, row strides ldx, ldw, ldy in ELEMENTS (>= the row length), element stride 1.
 * Products are exact in fp32, sums are accumulated in fp32 on the matrix cores (contraction
 * order unspecified), the bias is added in fp32, the result is rounded once (nearest-even) if bf16.
 * x and w may not overlap y.  No workspace.
 * Errors: NULL x/w/y/p, M, N or K < 1, a stride shorter than its row, bad out_dtype or nonzero
 * flags -> DIT_ERR_INVALID_ARG; K not a multiple of 64, N not a multiple of 8, or ldx or ldw above
 * 2^22 elements -> DIT_ERR_UNSUPPORTED; a base pointer or row stride that breaks 16-byte row alignment (8 bytes for
 * bias) -> DIT_ERR_ALIGNMENT.
 */
typedef struct {
    int32_t M, N, K;
    int64_t ldx, ldw, ldy;
    int32_t out_dtype; /* DIT_BF16 or DIT_F32 */
    uint32_t flags;    /* reserved, must be 0 */
} dit_linear_params;

dit_status dit_linear_forward(const void *x, const void *w, const void *bias, void *y,
                              const dit_linear_params *p, void *stream);

/*
 * Timing hook for benchmarks and profilers (not part of the attention definition): while
 * both handles are non-NULL, every forward call made by the calling thread records the
 * hipEvent_t `before` on the stream just before the attention kernel and `after` just after
 * it, so the dominant kernel can be timed apart from the table and pre-pack kernels.
 * The events are the caller's; pass NULL, NULL to switch the hook off.
 */
void dit_attn_set_timing_events(void *before, void *after);

/*
 * Measurement utility for benchmarks (not part of the attention definition): enqueues one kernel in which
 * every SIMD of the current device runs two wavefronts that issue 32x32x16 MFMAs back to back from
 * registers -- no memory traffic, no LDS, no vector arithmetic -- so that the rate the matrix cores sustain
 * on this board can be set beside the published peak.  operand_dtype: DIT_PROBE_F16 or DIT_PROBE_BF16.
 * bits_a, bits_b: what the A and B operands hold.  0: the constant 0.5 (the rate is then bound by issue and
 * clock); n > 0: random signs, exponents in [-3, 0] and random significands of n significant bits, leading one
 * included (11 = all of fp16, 8 = all of bf16; with fewer the low stored bits are zero; larger values are
 * clamped to the format) -- the data-dependent switching of real inputs, under which the board meets its
 * power limit, and which grows with the number of bits the data carries.
 * Each wavefront issues mfma_per_wavefront MFMAs, rounded up to a multiple of 16.
 * sink: DEVICE buffer of at least 2 * compute units * 256 floats that receives one value per lane (it only
 * keeps the work alive).  *flops (HOST) receives the multiply-add flops the kernel performs; the caller
 * times the kernel on `stream`.  Errors: DIT_ERR_INVALID_ARG (NULL, bad dtype, a negative count),
 * DIT_ERR_ALIGNMENT, DIT_ERR_WORKSPACE (sink too small), DIT_ERR_HIP.
 */
enum { DIT_PROBE_BF16 = 0, DIT_PROBE_F16 = 1 };

dit_status dit_mfma_probe(int32_t operand_dtype, int32_t bits_a, int32_t bits_b, int64_t mfma_per_wavefront,
                          float *sink, size_t sink_bytes, double *flops, void *stream);

/* The fused q/k/v projection in front of self-attention (Sec. 2.4: a transformer block of the Diffusion stage projects
 * its token rows to queries, keys and values and attends): y = x w^T + bias with the rows of w ordered [q; k; v],
 * H*D rows each (N = 3*H*D).  The q rows are stored to q_out as they come out (bf16, strides ap->sq); the k and v
 * values are rounded to bf16 as the rows of dit_linear_forward would be, the k values then rotated (the RoPE of
 * dit_attn_forward for ap's grid, sections, origin and base) and rounded to the score operand type, the v values
 * rounded to the PV operand type and transposed, and both written as the K'/V^T tile images that dit_attn_forward
 * keeps in its workspace.  A following
 *     dit_attn_forward(q_out, NULL, NULL, out, lse, ap' = ap with flags | DIT_FLAG_KV_RESIDENT, workspace, ...)
 * on the same workspace then needs no pre-pack pass, k and v never exist as rows in memory, and (without a
 * normalisation) its result is bit for bit that of dit_linear_forward with bf16 output followed by
 * dit_attn_forward on the q, k, v columns of that output.
 *   x [M, K] bf16 (row stride lp->ldx), w [3*H*D, K] bf16 (lp->ldw), bias [3*H*D] bf16 or NULL: DEVICE pointers.
 *   lp: M = T*Hg*Wg of ap, N = 3*H*D, K a multiple of 64, out_dtype DIT_BF16, flags 0; ldy is ignored.
 *   ap: the parameters of the attention call that follows, without DIT_FLAG_KV_RESIDENT.  Covered: B = 1,
 *       D = 128, an even H, in_dtype DIT_BF16, flags that select the default attention kernel (operand-type
 *       flags are honoured); anything else DIT_ERR_UNSUPPORTED.  sk, sv are ignored.  With a q/k normalisation the
 *       k rows are normalised here, in fp32 on the bf16-rounded values (norm.eps, norm.k_gamma), before the rotation;
 *       the q rows are stored as they are and the attention call, given the same norm, normalises them as it reads
 *       them.  DIT_NORM_HEAD is done in the projection's epilogue.  DIT_NORM_TOKEN, whose mean runs over all heads
 *       of a token and so over every output tile of the k part, takes a second, memory-bound pass over the K' images
 *       (k_rescale_kernel): the epilogue applies the weights and leaves each head's sum of squares in the spare
 *       bytes of the tile images, the pass multiplies each token's K' rows by its factor (K' is rounded twice).
 *   workspace: dit_attn_workspace_bytes(ap) bytes, 256-byte aligned; written: rotation table and every tile image.
 * Errors as dit_linear_forward and dit_attn_forward; nothing is enqueued unless all checks pass. */
dit_status dit_qkv_proj_forward(const void *x, const void *w, const void *bias, void *q_out,
                                const dit_linear_params *lp, const dit_self_attn_params *ap,
                                void *workspace, size_t workspace_bytes, void *stream);

/* Static strings; never NULL. */
const char *dit_strerror(dit_status s);
/* Text of the last HIP error seen by the calling thread ("" if none). */
const char *dit_last_hip_error(void);
/* major*10000 + minor*100 + patch */
int dit_attn_version(void);

#ifdef __cplusplus
}
#endif
#endif /* DIT_ATTN_H */
