/*
 * libtaq — Trigger-Aware Quantized (TAQ) cross-attention for AMD MI355X (gfx950).
 *
 * C ABI of the library. It implements the quantized UNet cross-attention block of
 * PersonalQ, Section III-B ("Trigger-Aware Quantization"):
 *
 *   K~ = M_KV*K + (1-M_KV)*Q_a(K),  V~ likewise,  Q~ = Q_a(Q)          (Eq. 2)
 *   A  = softmax(Q~ K~^T / sqrt(d))                                     (attention definition)
 *   A^ = M_A*A + (1-M_A)*Q_a(A)                                         (Eq. 3)
 *   out = to_out(A^ V~)
 *
 * where the masks are 1 on the trigger-token rows of K/V (and the same columns
 * of A). Details the paper leaves open are fixed as follows:
 *   - Q_a on signed data is the symmetric quantizer  code = clamp(rint(x*qmax/amax)),
 *     scale = amax/qmax, qmax = 2^(b-1)-1, all in IEEE float32, rint half-to-even;
 *   - rows: K/V per (head, text token); Q per (image token, head); hidden states and
 *     the attention output per image token; weights per output channel (8 bit);
 *   - Q_a on probabilities is the fixed grid code = rint(pmax*A), A^ = code/pmax, pmax = 2^b - 1 (255 or 15);
 *     shape->prob_grid selects a power-of-two grid or the row's own range instead;
 *   - to_q, to_out and the K/V projections of unprotected tokens are W8A8 integer
 *     contractions; protected K/V rows are computed from the unquantized fp16 context
 *     row (with the 8-bit weight codes) and stored as fp16.
 *
 * General rules
 *   - Every data pointer is DEVICE memory owned by the caller, 16-byte aligned, unless
 *     said otherwise. The library allocates nothing and keeps no state between calls
 *     (apart from remembering, per kernel and device, that a launch attribute was set).
 *   - Calls enqueue work on `hip_stream` (a hipStream_t passed as void*, NULL = the
 *     default stream) and return without waiting; the caller synchronises.
 *   - Return value: TAQ_OK (0) or a negative taq_status. On error nothing is launched.
 *     Inputs are assumed finite; NaN/Inf give unspecified results.
 *   - Shapes: B batch elements, N image (query) tokens, C = H*d channels, T text
 *     tokens, Cc text-context channels. Supported: T <= 96, d % 8 == 0, d <= 160,
 *     C % 32 == 0, Cc % 32 == 0, H <= 64.
 */
#ifndef TAQ_H
#define TAQ_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum taq_status {
    TAQ_OK = 0,
    TAQ_ERR_INVALID_ARG = -1,      /* NULL pointer, non-positive size, inconsistent arguments */
    TAQ_ERR_UNSUPPORTED_BITS = -2, /* a bit width outside what this build implements        */
    TAQ_ERR_BAD_SHAPE = -3,        /* shape outside the supported set listed above          */
    TAQ_ERR_MISALIGNED = -4,       /* a pointer is not 16-byte aligned                      */
    TAQ_ERR_HIP = -5,              /* the HIP runtime reported an error at launch           */
    TAQ_ERR_SCRATCH_TOO_SMALL = -6 /* taq_cross_attn_static: shape needs more scratch than the library's array */
} taq_status;

/* Problem description shared by all calls. */
typedef struct taq_shape {
    int B, N, C, H, T, Cc;   /* d = C / H                                                   */
    int bits_kv;             /* 4 | 8 : width of unprotected K/V rows; 16 : keep every row fp16 */
    int bits_prob;           /* 8 | 4 : probabilities on the 1/255 or 1/15 grid outside trigger columns;
                                16 : A^ = A (Eq. 3 switched off)                                */
    int bits_q;              /* 8 | 4 : Q~ = Q_a(Q), qmax = 127 or 7 (codes stay one per byte); 16 : Q~ = Q  */
    int bits_proj;           /* 8 : W8A8 projections; 16 : unquantized projections, Wk / Wv / Wq / Wo are then the
                                fp16 matrices themselves in every call (see taq_cross_attn).
                                Any 16 among bits_prob / bits_q / bits_proj selects plain float32 kernels, one per
                                stage: reference runs (Eq. 1's "everything else in full precision"), not speed.  */
    float softmax_scale;     /* 0 => 1/sqrt(d)                                               */
    int w_layout;            /* layout of the Wq / Wo buffers given to taq_cross_attn:
                                0 : i8 [C, C] row-major codes only
                                1 : buffers written by taq_pack_weight (row-major codes followed by a copy
                                    in matrix-core operand order, which the single-kernel path reads with
                                    fully coalesced loads)                                      */
    int prob_grid;           /* grid of Q_a on the probabilities in Eq. (3):
                                TAQ_PROB_LINEAR (0) : code = rint(pmax*A), A^ = code/pmax
                                TAQ_PROB_LOG2   (1) : code = clip(rint(-log2 A), 0, 2^bits_prob - 1),
                                                      A^ = 2^-code (the "Logarithmic" quantizer of the
                                                      trigger-separation ablation, Section IV)
                                TAQ_PROB_ROWMAX (2) : the affine quantizer with the row's own range:
                                                      amax = largest unprotected A of the (token, head) row,
                                                      code = rint(pmax*A/amax), A^ = code*amax/pmax     */
    int tok_tile;            /* image tokens per workgroup of the single-kernel and head-group paths: 0 = the library
                                picks (16 when 32-token tiles would fill at most half of the GPU's compute units;
                                head-group path: when they would give at most four workgroups per compute unit);
                                32 or 16 forces one (tests and tuning). Results do not depend on it.              */
} taq_shape;

enum { TAQ_PROB_LINEAR = 0, TAQ_PROB_LOG2 = 1, TAQ_PROB_ROWMAX = 2 };

/* Optional taps for tests and profiling (all pointers device memory or NULL). */
typedef struct taq_debug {
    int8_t* h_code;  /* i8  [B,N,C]  per-token codes of `hidden`                             */
    float*  s_h;     /* f32 [B,N]                                                            */
    int8_t* q_code;  /* i8  [B,N,C]  Q~ codes                                                */
    float*  s_Q;     /* f32 [B,N,H]                                                          */
    float*  O;       /* f32 [B,N,C]  A^ V~ before its quantization                           */
    int8_t* o_code;  /* i8  [B,N,C]                                                          */
    float*  s_o;     /* f32 [B,N]                                                            */
    uint8_t* p_code; /* u8  [B,N,H,T] codes of Q_a(A) in Eq. (3) (on the log2 grid: the exponent code);
                        entries of protected columns are unspecified                         */
    unsigned stage_mask; /* 0 = whole block; else OR of TAQ_STAGE_* to run only those stages
                            (they then read what earlier calls left in `workspace`)          */
} taq_debug;

#define TAQ_STAGE_HIDDEN_QUANT 1u  /* per-token int8 codes of hidden            */
#define TAQ_STAGE_TO_Q         2u  /* to_q integer GEMM + dequantisation         */
#define TAQ_STAGE_Q_QUANT      4u  /* Q~ = Q_a(Q), Eq. (2) third line            */
#define TAQ_STAGE_ATTN_CORE    8u  /* scores, softmax, Eq. (3), A^ V~            */
#define TAQ_STAGE_O_QUANT      16u /* per-token int8 codes of the attention out  */
#define TAQ_STAGE_TO_OUT       32u /* to_out integer GEMM + bias, fp16 store     */

/* One request of a batched call: the arguments of taq_cross_attn, per request. */
typedef struct taq_request {
    const void*    hidden;
    const void*    qkv_packed;
    const int8_t*  Wq;
    const int8_t*  Wo;
    const float*   scales;
    const uint8_t* trigger_mask;
    void*          out;
} taq_request;

/* Bytes the caller must allocate for `qkv_packed` (the mixed-precision K~/V~ of
 * Eq. 2 for every batch element) and for `workspace` (scratch of either call) at
 * this shape. Host-only; no GPU work. */
int taq_kv_packed_bytes(const taq_shape* shape, size_t* bytes);
int taq_workspace_bytes(const taq_shape* shape, size_t* bytes);

/* Per-output-channel symmetric int8 codes of an fp16 weight matrix
 * (8-bit weights as in every setting of the paper's Table 1; round-to-nearest).
 *   W_f16  : f16 [rows, cols] row-major (rows = output channels), cols % 8 == 0
 *   codes  : i8  [rows, cols]  out
 *   scales : f32 [rows]        out */
int taq_quantize_weight(const void* W_f16, int rows, int cols, int8_t* codes, float* scales,
                        void* hip_stream);

/* (Helpers of this build, not operations of the paper: the paper prescribes no memory layout.)
 * Optional re-layout of a [C, C] weight-code matrix for taq_cross_attn (shape->w_layout = 1): `out` receives
 * the row-major codes followed by a copy ordered the way the matrix cores read them for this shape's head
 * dimension. The method is unchanged (the paper does not prescribe a memory layout); only load efficiency is.
 *   codes : i8 [C, C] row-major (as written by taq_quantize_weight); may be the start of `out` itself
 *   out   : taq_weight_bytes() bytes
 * shape->N is ignored. */
int taq_weight_bytes(const taq_shape* shape, size_t* bytes);
int taq_pack_weight(const int8_t* codes, const taq_shape* shape, int8_t* out, void* hip_stream);

/* Eq. (2), K and V lines: project the text context and build K~, V~.
 *   context      : f16 [B, T, Cc]
 *   trigger_mask : u8  [B, T], non-zero = trigger token (protected row). Read on the
 *                  device; any number of rows, contiguous or not, may be set.
 *   Wk, Wv       : f16 [C, Cc] row-major (out x in)
 *   bits         : must equal shape->bits_kv (4, 8 or 16)
 *   qkv_packed   : out, taq_kv_packed_bytes() bytes. Holds, per batch element: the
 *                  protected-token list, per-(head,token) scales, int8 or packed int4
 *                  codes (element 2j in the low nibble of byte j) of unprotected rows,
 *                  and the fp16 protected rows. Opaque to the caller; see taq_unpack_kv.
 *   workspace    : taq_workspace_bytes() bytes of scratch, contents undefined after.
 * shape->N is ignored. */
int taq_quantize_kv(const void* context, const uint8_t* trigger_mask, const void* Wk,
                    const void* Wv, int bits, const taq_shape* shape, void* qkv_packed,
                    void* workspace, void* hip_stream);

/* Same as taq_quantize_kv with the 8-bit weight codes of to_k / to_v formed beforehand (they depend
 * only on the checkpoint, the context on the prompt: Section III-B keeps one K~/V~ per prompt, and a
 * serving process keeps one set of weight codes per checkpoint):
 *   Wkv_code : i8  [2*C, Cc] row-major, the codes of Wk (rows 0..C-1) then of Wv (rows C..2C-1),
 *              as written by taq_quantize_weight on each matrix
 *   s_wkv    : f32 [2*C]     their per-output-channel scales, in the same order
 * Results are bit-identical to taq_quantize_kv on the fp16 matrices. Both buffers device memory,
 * 16-byte aligned, read only. */
int taq_quantize_kv_w8(const void* context, const uint8_t* trigger_mask, const int8_t* Wkv_code,
                       const float* s_wkv, int bits, const taq_shape* shape, void* qkv_packed,
                       void* workspace, void* hip_stream);

/* Eq. (2) third line, the attention definition and Eq. (3): the block for image tokens.
 *   hidden       : f16 [B, N, C]
 *   qkv_packed   : as written by taq_quantize_kv for the same B, T, C, H, bits_kv
 *   Wq, Wo       : i8  [C, C] row-major (out x in) weight codes (taq_quantize_weight), or, with
 *                  shape->w_layout = 1, the buffers written by taq_pack_weight; with shape->bits_proj = 16
 *                  the unquantized f16 [C, C] matrices (passed through the same pointers)
 *   scales       : f32 [3*C] = s_wq[C] | s_wo[C] | bias_o[C] (bias of to_out; zeros if none); with
 *                  bits_proj = 16 only the bias part is read
 *   trigger_mask : u8 [B, T] or NULL. The protected-token list recorded in qkv_packed is
 *                  what the kernels use; this argument is accepted for symmetry only.
 *   out          : f16 [B, N, C]
 *   workspace    : taq_workspace_bytes() bytes of scratch */
int taq_cross_attn(const void* hidden, const void* qkv_packed, const int8_t* Wq, const int8_t* Wo,
                   const float* scales, const uint8_t* trigger_mask, const taq_shape* shape,
                   void* out, void* workspace, void* hip_stream);

/* Same as taq_cross_attn with optional taps on the intermediate codes and scales
 * (dbg may be NULL). Taps are copied out of the workspace on the same stream. */
int taq_cross_attn_ex(const void* hidden, const void* qkv_packed, const int8_t* Wq,
                      const int8_t* Wo, const float* scales, const uint8_t* trigger_mask,
                      const taq_shape* shape, void* out, void* workspace, void* hip_stream,
                      const taq_debug* dbg);

/* taq_cross_attn for callers that cannot hand over (or allocate) a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid allocation. Same arguments minus `workspace`;
 * the scratch memory is a fixed array of TAQ_STATIC_SCRATCH_BYTES inside the library, one copy per
 * GPU, held until the process ends. The call allocates and frees nothing.
 *   - A shape whose kernels need more scratch than the array holds is rejected with
 *     TAQ_ERR_SCRATCH_TOO_SMALL and nothing is launched (shapes that run as one kernel need none
 *     and are never rejected for size; the others need about 11 * B * N * C bytes).
 *   - All calls on one GPU share that GPU's array: calls that may overlap on one GPU (different
 *     streams, several host threads) race; serialise them or use taq_cross_attn with own workspaces.
 *   - Results are bit-identical to taq_cross_attn. */
#define TAQ_STATIC_SCRATCH_BYTES (16u << 20)
int taq_cross_attn_static(const void* hidden, const void* qkv_packed, const int8_t* Wq, const int8_t* Wo,
                          const float* scales, const uint8_t* trigger_mask, const taq_shape* shape,
                          void* out, void* hip_stream);

/* The same block (Section III-B: Eq. 2 third line, the attention definition, Eq. 3) for R independent requests of
 * one shape, each with its own weights, K~/V~ and hidden states: the serving setting the paper motivates (Section I:
 * many personalised checkpoints of one backbone behind one service; one quantized checkpoint and one K~/V~ per
 * request). `table` is HOST memory, R entries, read before the call returns. `workspace` must hold R times
 * taq_workspace_bytes(). Requests of the single-kernel shapes go out as grouped launches of up to 16. */
int taq_cross_attn_batched(int R, const taq_request* table, const taq_shape* shape,
                           void* workspace, void* hip_stream);

/* Mean squared difference of two fp16 arrays of n elements, as a float64 in device memory: the loss L of the
 * token-sensitivity experiment (Section III-B, Eq. 1) on block outputs. x, y, out device memory; out 8-byte aligned. */
int taq_mse_f16(const void* x_f16, const void* y_f16, size_t n, double* out, void* hip_stream);

/* Expand qkv_packed into plain arrays (for tests). Any output may be NULL.
 *   k_codes, v_codes : i8  [B, T, C]  (int4 codes sign-extended; zeros on protected rows)
 *   k_scales,v_scales: f32 [B, H, T]  (zeros on protected rows)
 *   k_trig, v_trig   : f16 [B, T, C]  (protected rows in place, zeros elsewhere) */
int taq_unpack_kv(const void* qkv_packed, const taq_shape* shape, int8_t* k_codes, int8_t* v_codes,
                  float* k_scales, float* v_scales, void* k_trig_f16, void* v_trig_f16,
                  void* hip_stream);

/* Where the plain code sections sit inside qkv_packed, for tools that read the codes themselves: byte offsets of
 * the K and the V section, each u8 [B][T][row_bytes]; row_bytes = C with 8-bit rows, C/2 with 4-bit rows (two's
 * complement nibbles, element 2j in the low nibble of byte j, as Eq. (2)'s codes are packed), 0 with bits_kv = 16
 * (no code sections). Protected rows hold zeros. Host-only; no GPU work. */
int taq_kv_code_layout(const taq_shape* shape, size_t* k_code_offset, size_t* v_code_offset, size_t* row_bytes);

/* Static, human-readable name of a status code. */
const char* taq_status_string(int status);

#ifdef __cplusplus
}
#endif
#endif /* TAQ_H */
