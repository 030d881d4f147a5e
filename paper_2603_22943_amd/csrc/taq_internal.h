// Internal declarations shared by the libtaq translation units (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include <stddef.h>
#include <stdint.h>

#include <atomic>

#include "taq.h"

#define TAQ_MAX_T 96        // text tokens the attention core holds in LDS (3 tiles of 32)
#define TAQ_MAX_D 160       // largest head dimension (5 steps of 32)
#define TAQ_MAX_H 64

namespace taq {

static inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// Layout of qkv_packed: fixed by the shape alone, every section 256-byte aligned.
struct KvLayout {
    size_t ntrig;     // i32 [B]        number of protected tokens
    size_t trig_idx;  // i32 [B][T]     token index of protected slot s (first ntrig valid)
    size_t slot_of;   // i32 [B][T]     slot of token t, or -1 if unprotected
    size_t s_k;       // f32 [B][H][T]  0 on protected tokens
    size_t s_v;       // f32 [B][H][T]
    size_t k_code;    // u8  [B][T][Cb] Cb = C (8 bit) | C/2 (4 bit) | 0 (16 bit)
    size_t v_code;
    size_t k16;       // f16 [B][T][C]  protected rows, compacted by slot
    size_t v16;
    size_t v16t;      // f16 [B][C][96] protected V rows transposed (slot along the last axis)
    size_t image;     // [B][image_bytes] LDS-ready K~/V~ image for the fused block kernel (may be empty)
    size_t image_bytes;
    size_t total;
    int Cb;
};

// LDS-ready image of the integer part of K~/V~ for one batch element (fused block kernel): one
// self-contained block per head, so that the wavefront that owns a head copies and waits for its own
// block only. Offsets are relative to the head block; head_bytes is a multiple of 1 KiB (the unit of
// the direct-to-LDS copy).
struct KvImage {
    int tph;        // 16-channel tiles per head = ceil(d/16)
    int nt16;       // ceil(T/16): score tiles of 16 text tokens
    int ntok;       // 16*nt16: text tokens with padding; length of the per-token arrays below
    int rows_k;     // = ntok: text-token rows of the K part
    int cols_v;     // = ntok: token positions per V^T row (see vt_pos)
    size_t kp;      // i8  [rows_k][tph][4 quarter-lanes][4]  K codes in MFMA operand order (see kp_offset)
    size_t vt;      // u8  [d][cols_v]   V codes (+128) transposed, tokens in accumulator-register order
    size_t s_k;     // f32 [ntok]  per-token K scale of this head, 0 on protected / padding tokens
    size_t s_vp;    // f16 [2][ntok]  s_V * 2^kexp as an fp16 high part [0][t] and the fp16 remainder [1][t]
    size_t bias;    // f32 [ntok]  0 for unprotected tokens, -inf for protected / padding (same in every head)
    size_t oscale;  // f32       2^-kexp / 255
    size_t vpre;    // f32       2^kexp
    size_t head_bytes;  // one head's block, a multiple of 256 bytes
    size_t bytes;   // H * head_bytes
};

// Byte offset, within the K part of a head block, of the 4 codes of text token t, 16-channel tile j, quarter q
// (channels 16*j + 4*q .. +3 of the head). A lane of the score MFMA holds row t, quarter q and needs tiles
// 4*ks .. 4*ks+3 for K step ks. When the head has a multiple of 4 tiles those 16 bytes are laid out contiguously,
// [t][ks][q][tile%4][4], so that the lane reads them with one 16-byte LDS load and the 64 lanes of a wavefront hit
// consecutive 16-byte slots (no bank conflicts; a 64-byte row of [t][tile][q][4] would put 16 rows on 2 bank
// groups). Otherwise [t][tile][q][4].
__host__ __device__ static inline size_t kp_offset(int tph, int t, int j, int q) {
    if ((tph & 3) == 0) return ((((size_t)t * (tph >> 2) + (j >> 2)) * 4 + q) * 4 + (j & 3)) * 4;
    return (((size_t)t * tph + j) * 4 + q) * 4;
}

// Place of text token t in a V^T row of the image. Tokens come in steps of 32 (two score tiles of 16), permuted within
// a step to the accumulator-register order of the score MFMA: token 32*s + 16*a + 4*q + e sits at 32*s + 8*q + 4*a + e,
// so that a lane's 8 probabilities of the step meet 8 consecutive V codes. A last single tile (nt16 odd) keeps its
// natural order 4*q + e: it is contracted with a 16-deep MFMA.
__host__ __device__ static inline int vt_pos(int t, int nt16) {
    if ((nt16 & 1) && (t >> 4) == nt16 - 1) return t;
    return (t & ~31) + 8 * ((t >> 2) & 3) + 4 * ((t >> 4) & 1) + (t & 3);
}

static inline KvImage kv_image(const taq_shape& s) {
    KvImage I;
    const size_t H = s.H, d = s.C / s.H;
    I.tph = (int)((d + 15) / 16);
    I.nt16 = (s.T + 15) / 16;
    I.ntok = 16 * I.nt16;
    I.rows_k = I.ntok;
    I.cols_v = I.ntok;
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes, 16); return o; };
    I.kp = take(I.rows_k * (size_t)I.tph * 16);
    I.vt = take(d * (size_t)I.cols_v);
    I.s_k = take(I.ntok * 4);
    I.s_vp = take(I.ntok * 4);
    I.bias = take(I.ntok * 4);
    I.oscale = take(4);
    I.vpre = take(4);
    I.head_bytes = align_up(off, 256);  // (at least 1 KiB: the kernels copy it in 1 KiB pieces, the last one overlapping)
    I.bytes = H * I.head_bytes;
    return I;
}

// Operand-ordered copy of a [C, C] weight matrix: for head h, 16-row tile j of the head, K step ks (64 codes),
// lane l = r + 16*q: the 16 codes W[min(h*d + 16*j + r, C-1)][64*ks + 16*q ...]; 1 KiB per (h, j, ks).
// It sits behind the row-major codes, 256-byte aligned.
static inline size_t weight_pack_offset(const taq_shape& s) { return align_up((size_t)s.C * s.C, 256); }
static inline size_t weight_pack_bytes(const taq_shape& s) {
    const size_t d = s.C / s.H;
    return weight_pack_offset(s) + (size_t)s.H * ((d + 15) / 16) * (s.C / 64) * 1024;
}

// LDS bytes of the fused block kernel: K~/V~ image, int8 token tile, weight scales, per-token scratch.
static inline size_t fused_lds_bytes(const taq_shape& s, int tok = 32) {
    return kv_image(s).bytes + tok * ((size_t)s.C + 16) + 3 * (size_t)s.C * 4 + tok * 4 + tok * (size_t)s.H * 4;
}

// Shapes the fused block kernel is instantiated for: (d, H) = (40, 8), (80, 8), (64, 10), as long as
// its working set fits the 160 KiB of LDS of a compute unit.
// Any of the full-precision modes (an unquantized projection, Q~ or probabilities): the float32 kernel-per-stage path.
static inline bool fp_mode(const taq_shape& s) { return s.bits_proj == 16 || s.bits_q == 16 || s.bits_prob == 16; }

static inline bool fused_supported(const taq_shape& s) {
    if (fp_mode(s)) return false;
    if (s.bits_kv != 4 && s.bits_kv != 8) return false;
    if (s.C % s.H) return false;
    const int d = s.C / s.H;
    if (!((d == 40 && s.H == 8) || (d == 80 && s.H == 8) || (d == 64 && s.H == 10))) return false;
    if (s.N > 16 * 65535) return false;  // token tiles are a y / z dimension of the grid
    return fused_lds_bytes(s) <= 160 * 1024;
}

// Shapes of the head-group variant (to_q + Q~ + attention per head group; C = 1280 layers):
// (d, H) = (160, 8) with one head per workgroup, (64, 20) with two.
static inline size_t mid_lds_bytes(const taq_shape& s) {
    const int d = s.C / s.H;
    const size_t nh = d == 160 ? 1 : 2;
    // image blocks | 32 token rows of codes | s_wq of the heads | s_h | partial to_q sums [4 K ranges][2 token groups][tiles][1 KiB]
    return nh * kv_image(s).head_bytes + 32 * ((size_t)s.C + 16) + nh * d * 4 + 32 * 4 + 8 * nh * (size_t)((d + 15) / 16) * 1024;
}
static inline bool mid_supported(const taq_shape& s) {
    if (fp_mode(s)) return false;
    if (s.bits_kv != 4 && s.bits_kv != 8) return false;
    if (s.C % s.H) return false;
    const int d = s.C / s.H;
    if (!((d == 160 && s.H == 8) || (d == 64 && s.H == 20))) return false;
    if (s.N > 16 * 65535) return false;  // token tiles are a y dimension of the grid
    return mid_lds_bytes(s) <= 160 * 1024;
}

static inline KvLayout kv_layout(const taq_shape& s) {
    KvLayout L;
    size_t off = 0;
    const size_t B = s.B, T = s.T, C = s.C, H = s.H;
    L.Cb = s.bits_kv == 8 ? s.C : (s.bits_kv == 4 ? s.C / 2 : 0);
    auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes, 256); return o; };
    L.ntrig = take(B * 4);
    L.trig_idx = take(B * T * 4);
    L.slot_of = take(B * T * 4);
    L.s_k = take(B * H * T * 4);
    L.s_v = take(B * H * T * 4);
    L.k_code = take(B * T * (size_t)L.Cb);
    L.v_code = take(B * T * (size_t)L.Cb);
    L.k16 = take(B * T * C * 2);
    L.v16 = take(B * T * C * 2);
    L.v16t = take(B * C * 96 * 2);
    L.image_bytes = (fused_supported(s) || mid_supported(s)) ? align_up(kv_image(s).bytes, 256) : 0;
    L.image = take(B * L.image_bytes);
    L.total = off;
    return L;
}

// Workspace of taq_quantize_kv.
struct KvWorkspace {
    size_t w_code;  // i8  [2C][Cc]   Wk rows then Wv rows
    size_t s_w;     // f32 [2C]
    size_t x_code;  // i8  [B*T][Cc]
    size_t s_x;     // f32 [B*T]
    size_t rows_f;  // f32 [B*T][2C]  dequantised projection rows (K then V channels)
    size_t total;
};

static inline KvWorkspace kv_workspace(const taq_shape& s) {
    KvWorkspace W;
    size_t off = 0;
    const size_t M = (size_t)s.B * s.T, C2 = 2 * (size_t)s.C, Cc = s.Cc;
    auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes, 256); return o; };
    W.w_code = take(C2 * Cc);
    W.s_w = take(C2 * 4);
    W.x_code = take(M * Cc);
    W.s_x = take(M * 4);
    W.rows_f = take(M * C2 * 4);
    W.total = off;
    return W;
}

// Workspace of taq_cross_attn (per request).
struct AttnWorkspace {
    size_t h_code;  // i8  [B*N][C]
    size_t s_h;     // f32 [B*N]
    size_t q_f;     // f32 [B*N][C]
    size_t q_code;  // i8  [B*N][C]
    size_t s_q;     // f32 [B*N][H]
    size_t o_f;     // f32 [B*N][C]
    size_t o_code;  // i8  [B*N][C]
    size_t s_o;     // f32 [B*N]
    size_t total;
};

static inline AttnWorkspace attn_workspace(const taq_shape& s) {
    AttnWorkspace W;
    size_t off = 0;
    const size_t M = (size_t)s.B * s.N, C = s.C, H = s.H;
    auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes, 256); return o; };
    W.h_code = take(M * C);
    W.s_h = take(M * 4);
    W.q_f = take(M * C * 4);
    W.q_code = take(M * C);
    W.s_q = take(M * H * 4);
    W.o_f = take(M * C * 4);
    W.o_code = take(M * C);
    W.s_o = take(M * 4);
    W.total = off;
    return W;
}

// Kernels that use more than 64 KiB of dynamic LDS need that attribute set once per kernel and device. `done` is the
// kernel's bit mask of devices that have it (one static per kernel instantiation, the library's only state); setting
// the attribute twice from two host threads that race here is harmless.
static inline hipError_t ensure_dynamic_lds(const void* kernel, int bytes, std::atomic<unsigned long long>& done) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    const unsigned long long bit = 1ull << (dev & 63);
    if (done.load(std::memory_order_acquire) & bit) return hipSuccess;
    e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    if (e != hipSuccess) return e;
    done.fetch_or(bit, std::memory_order_release);
    return hipSuccess;
}

// ---- kernel launchers (each returns a hipError_t from the launch) ----------------

// Per-row symmetric int8 codes of fp16 rows: x [M][K] -> code [M][K], scale [M].
hipError_t launch_rowquant_f16(const __half* x, int M, int K, int8_t* code, float* scale, hipStream_t st);
// Same for float32 rows.
hipError_t launch_rowquant_f32(const float* x, int M, int K, int8_t* code, float* scale, hipStream_t st);
// Per-(row, head) symmetric codes (8 or 4 bit, one per byte) of float32 rows: x [M][C] -> code [M][C], scale [M][H].
hipError_t launch_headquant_f32(const float* x, int M, int C, int H, int bits, int8_t* code, float* scale, hipStream_t st);

// First launch of taq_quantize_kv: per-row int8 codes of the context rows (context == NULL: skipped) and of the rows of
// Wk / Wv (NULL: codes given by the caller), plus the protected-token bookkeeping, in one kernel.
hipError_t launch_kv_prep(const __half* context, int M, int8_t* x_code, float* s_x, const __half* Wk, const __half* Wv,
                          int C, int8_t* w_code, float* s_w, int K, const uint8_t* mask, int B, int T, int bits,
                          int* ntrig, int* trig_idx, int* slot_of, hipStream_t st);
// Second launch of taq_quantize_kv (bits_kv 4 or 8): per (head, batch element) the integer K/V projection, Eq. (2)
// codes and scales into qkv_packed, and the head's block of the operand-ordered image where the shape has one.
// The same launch computes the protected fp16 rows (K16, V16, V16T) from the unquantized context rows.
hipError_t launch_kv_head(const int8_t* x_code, const float* s_x, const int8_t* w_code, const float* s_w, uint8_t* packed,
                          const __half* context, const taq_shape& s, hipStream_t st);
// Per-(head, token) codes and scales of unprotected K/V rows, written into qkv_packed.
hipError_t launch_kv_pack(const float* rows_f, const int* slot_of, int B, int T, int C, int H, int bits,
                          uint8_t* k_code, uint8_t* v_code, float* s_k, float* s_v, hipStream_t st);
// Protected K/V rows: fp16 context row x int8 weight codes, fp32 accumulate, fp16 store.
hipError_t launch_kv_trigger_rows(const __half* context, const int8_t* w_code, const float* s_w,
                                  const int* ntrig, const int* trig_idx, int B, int T, int C, int Cc,
                                  __half* k16, __half* v16, __half* v16t, hipStream_t st);
// Expansion of qkv_packed for tests.
hipError_t launch_kv_unpack(const uint8_t* packed, const taq_shape& s, int8_t* k_codes, int8_t* v_codes,
                            float* k_scales, float* v_scales, __half* k_trig, __half* v_trig, hipStream_t st);

// int8 GEMM  acc[m][n] = sum_k A[m][k]*W[n][k]  with dequantisation acc*(sa[m]*sw[n]):
//   out_f32 != NULL: float32 result [M][ldo];  out_f16 != NULL: fp16(result + bias[n]).
hipError_t launch_gemm_i8(const int8_t* A, const float* sa, const int8_t* W, const float* sw,
                          const float* bias, int M, int N, int K, float* out_f32, __half* out_f16,
                          int ldo, hipStream_t st);

// Full-precision stages (shape.bits_proj / bits_q / bits_prob = 16), float32 arithmetic:
//   out[m][n] = sum_k A[m][k] * W[n][k] (+ bias[n]); A f16 or f32 [M][K], W f16 [N][K]; float32 and / or fp16 result
hipError_t launch_gemm_fp(const void* A, bool a_is_f32, const __half* W, const float* bias, int M, int N, int K,
                          float* out_f32, __half* out_f16, int ldo, hipStream_t st);
//   protected K / V rows (fp16, compacted by slot, plus the transposed V copy) from float32 projection rows [B*T][2C]
hipError_t launch_kv_rows_from_f32(const float* rows_f, const int* ntrig, const int* trig_idx, int B, int T, int C,
                                   __half* k16, __half* v16, __half* v16t, hipStream_t st);
//   scores, softmax, Eq. (3), A^ V~ with Q unquantized (q_f) or as codes and scales, probabilities at shape.bits_prob
hipError_t launch_attn_fp(const float* q_f, const int8_t* q_code, const float* s_q, const uint8_t* packed, const taq_shape& s,
                          float* o_f, uint8_t* p_code, hipStream_t st);
//   mean squared difference of two fp16 arrays into a device double
hipError_t launch_mse_f16(const __half* x, const __half* y, size_t n, double* out, hipStream_t st);

// K~/V~ image for the fused kernel, from the codes and scales already in qkv_packed.
hipError_t launch_kv_image(uint8_t* packed, const taq_shape& s, hipStream_t st);
// Row-major weight codes -> row-major codes + operand-ordered copy (weight_pack_bytes).
hipError_t launch_pack_weight(const int8_t* codes, const taq_shape& s, int8_t* out, hipStream_t st);

// One request of the fused block kernel.
struct FusedReq {
    const __half* hidden;
    const uint8_t* packed;
    const int8_t* wq;
    const int8_t* wo;
    const float* scales;
    __half* out;
};
// Whole block in one kernel (shapes of fused_supported only). dbg may be NULL. With core_qcode != NULL (R == 1) the
// kernel runs the attention core alone: Q~ codes i8 [B*N][C] and scales f32 [B*N][H] in, float32 A^ V~ [B*N][C] out.
hipError_t launch_fused_block(const FusedReq* reqs, int R, const taq_shape& s, const taq_debug* dbg, hipStream_t st,
                              const int8_t* core_qcode = nullptr, const float* core_sq = nullptr, float* core_of = nullptr);
// Head-group path (shapes of mid_supported), two kernels: (1) per-token codes of `hidden`, to_q, Q~ and the attention
// per head group, writing float32 A^ V~ [B*N][C] and partial row maxima [B*N][<= 40] to the workspace; (2) per-token
// codes of A^ V~ and to_out (with o_code != NULL the codes come from the row quantizer kernel instead). Taps in `dbg`
// are written by the kernel that computes them.
hipError_t launch_fused_mid(const FusedReq& rq, const taq_shape& s, float* o_f, float* o_max, const taq_debug* dbg,
                            hipStream_t st);
hipError_t launch_to_out_tail(const FusedReq& rq, const taq_shape& s, const float* o_f, const float* o_max,
                              const int8_t* o_code, const float* s_o, const taq_debug* dbg, hipStream_t st);

// Attention core: scores, softmax, Eq. (3), A^ V~ for all (batch, head, token).
hipError_t launch_attn_core(const int8_t* q_code, const float* s_q, const uint8_t* packed,
                            const taq_shape& s, float* o_f, hipStream_t st, uint8_t* p_code = nullptr);

}  // namespace taq
