// C ABI of libtaq: argument checks and the launch sequences of the two calls
// (PersonalQ, Section III-B: Eq. 2 for taq_quantize_kv, Eq. 2 third line + Eq. 3 for
// taq_cross_attn). No allocation, no synchronisation, no state.
#include "taq_internal.h"

using namespace taq;

namespace {

inline bool misaligned(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }

int check_shape(const taq_shape* s, bool need_n) {
    if (!s) return TAQ_ERR_INVALID_ARG;
    if (s->B <= 0 || s->C <= 0 || s->H <= 0 || s->T <= 0 || s->Cc <= 0) return TAQ_ERR_INVALID_ARG;
    if (need_n && s->N <= 0) return TAQ_ERR_INVALID_ARG;
    if (s->bits_kv != 4 && s->bits_kv != 8 && s->bits_kv != 16) return TAQ_ERR_UNSUPPORTED_BITS;
    if ((s->bits_prob != 8 && s->bits_prob != 4 && s->bits_prob != 16) || (s->bits_q != 8 && s->bits_q != 4 && s->bits_q != 16) ||
        (s->bits_proj != 8 && s->bits_proj != 16))
        return TAQ_ERR_UNSUPPORTED_BITS;
    if (s->C % s->H != 0) return TAQ_ERR_BAD_SHAPE;
    const int d = s->C / s->H;
    if (d % 8 != 0 || d > TAQ_MAX_D) return TAQ_ERR_BAD_SHAPE;
    if (s->T > TAQ_MAX_T || s->H > TAQ_MAX_H) return TAQ_ERR_BAD_SHAPE;
    if (s->C % 32 != 0 || s->Cc % 32 != 0 || s->Cc > 4096) return TAQ_ERR_BAD_SHAPE;
    if (!(s->softmax_scale >= 0.f)) return TAQ_ERR_INVALID_ARG;
    if (s->w_layout != 0 && s->w_layout != 1) return TAQ_ERR_INVALID_ARG;
    if (s->tok_tile != 0 && s->tok_tile != 16 && s->tok_tile != 32) return TAQ_ERR_INVALID_ARG;
    if (s->prob_grid != TAQ_PROB_LINEAR && s->prob_grid != TAQ_PROB_LOG2 && s->prob_grid != TAQ_PROB_ROWMAX)
        return TAQ_ERR_INVALID_ARG;
    // index arithmetic inside the kernels is 32-bit for token counts
    if ((long long)s->B * (need_n ? s->N : 1) > (1ll << 30)) return TAQ_ERR_BAD_SHAPE;
    return TAQ_OK;
}

#define TAQ_TRY_HIP(expr)                      \
    do {                                       \
        hipError_t e_ = (expr);                \
        if (e_ != hipSuccess) return TAQ_ERR_HIP; \
    } while (0)

}  // namespace

extern "C" {

const char* taq_status_string(int status) {
    switch (status) {
        case TAQ_OK: return "TAQ_OK";
        case TAQ_ERR_INVALID_ARG: return "TAQ_ERR_INVALID_ARG: null pointer, non-positive size or inconsistent arguments";
        case TAQ_ERR_UNSUPPORTED_BITS: return "TAQ_ERR_UNSUPPORTED_BITS: bit width not implemented";
        case TAQ_ERR_BAD_SHAPE: return "TAQ_ERR_BAD_SHAPE: shape outside the supported set";
        case TAQ_ERR_MISALIGNED: return "TAQ_ERR_MISALIGNED: pointer not 16-byte aligned";
        case TAQ_ERR_HIP: return "TAQ_ERR_HIP: HIP runtime error at launch";
        case TAQ_ERR_SCRATCH_TOO_SMALL:
            return "TAQ_ERR_SCRATCH_TOO_SMALL: the shape needs more scratch than the library's static array holds";
        default: return "unknown taq_status";
    }
}

int taq_kv_packed_bytes(const taq_shape* shape, size_t* bytes) {
    if (!bytes) return TAQ_ERR_INVALID_ARG;
    int rc = check_shape(shape, false);
    if (rc != TAQ_OK) return rc;
    *bytes = kv_layout(*shape).total;
    return TAQ_OK;
}

int taq_kv_code_layout(const taq_shape* shape, size_t* k_code_offset, size_t* v_code_offset, size_t* row_bytes) {
    if (!k_code_offset || !v_code_offset || !row_bytes) return TAQ_ERR_INVALID_ARG;
    int rc = check_shape(shape, false);
    if (rc != TAQ_OK) return rc;
    const KvLayout L = kv_layout(*shape);
    *k_code_offset = L.k_code;
    *v_code_offset = L.v_code;
    *row_bytes = (size_t)L.Cb;
    return TAQ_OK;
}

int taq_workspace_bytes(const taq_shape* shape, size_t* bytes) {
    if (!bytes) return TAQ_ERR_INVALID_ARG;
    int rc = check_shape(shape, false);
    if (rc != TAQ_OK) return rc;
    taq_shape s = *shape;
    if (s.N <= 0) s.N = 1;
    const size_t a = attn_workspace(s).total, k = kv_workspace(s).total;
    *bytes = a > k ? a : k;
    return TAQ_OK;
}

int taq_quantize_weight(const void* W_f16, int rows, int cols, int8_t* codes, float* scales, void* hip_stream) {
    if (!W_f16 || !codes || !scales || rows <= 0 || cols <= 0) return TAQ_ERR_INVALID_ARG;
    if (cols % 8 != 0) return TAQ_ERR_BAD_SHAPE;
    if (misaligned(W_f16) || misaligned(codes) || (reinterpret_cast<uintptr_t>(scales) & 3u)) return TAQ_ERR_MISALIGNED;
    TAQ_TRY_HIP(launch_rowquant_f16(static_cast<const __half*>(W_f16), rows, cols, codes, scales,
                                    static_cast<hipStream_t>(hip_stream)));
    return TAQ_OK;
}

int taq_weight_bytes(const taq_shape* shape, size_t* bytes) {
    if (!bytes) return TAQ_ERR_INVALID_ARG;
    int rc = check_shape(shape, false);
    if (rc != TAQ_OK) return rc;
    *bytes = weight_pack_bytes(*shape);
    return TAQ_OK;
}

int taq_pack_weight(const int8_t* codes, const taq_shape* shape, int8_t* out, void* hip_stream) {
    int rc = check_shape(shape, false);
    if (rc != TAQ_OK) return rc;
    if (!codes || !out) return TAQ_ERR_INVALID_ARG;
    if (misaligned(codes) || misaligned(out)) return TAQ_ERR_MISALIGNED;
    if (shape->C % 64 != 0) return TAQ_ERR_BAD_SHAPE;
    TAQ_TRY_HIP(launch_pack_weight(codes, *shape, out, static_cast<hipStream_t>(hip_stream)));
    return TAQ_OK;
}

// Shared body of taq_quantize_kv / taq_quantize_kv_w8: w_code / s_w are the 8-bit codes and scales of Wk (rows 0..C-1)
// and Wv (rows C..2C-1); when Wk / Wv are given they are quantized into those buffers first.
static int quantize_kv_impl(const void* context, const uint8_t* trigger_mask, const void* Wk, const void* Wv,
                            const int8_t* w_code_in, const float* s_w_in, const taq_shape& s, void* qkv_packed,
                            void* workspace, hipStream_t st) {
    const KvLayout L = kv_layout(s);
    const KvWorkspace W = kv_workspace(s);
    uint8_t* pk = static_cast<uint8_t*>(qkv_packed);
    uint8_t* ws = static_cast<uint8_t*>(workspace);
    int8_t* x_code = reinterpret_cast<int8_t*>(ws + W.x_code);
    float* s_x = reinterpret_cast<float*>(ws + W.s_x);
    float* rows_f = reinterpret_cast<float*>(ws + W.rows_f);
    int* ntrig = reinterpret_cast<int*>(pk + L.ntrig);
    int* trig_idx = reinterpret_cast<int*>(pk + L.trig_idx);
    int* slot_of = reinterpret_cast<int*>(pk + L.slot_of);
    const int M = s.B * s.T;
    const int8_t* w_code = w_code_in;
    const float* s_w = s_w_in;

    if (s.bits_proj == 16) {
        // unquantized projections: float32 rows of K and V for every token from the fp16 matrices, Eq. (2) codes of the
        // unprotected rows from those, protected rows by one rounding to fp16
        if (!Wk || !Wv) return TAQ_ERR_INVALID_ARG;
        TAQ_TRY_HIP(launch_kv_prep(nullptr, M, x_code, s_x, nullptr, nullptr, s.C, reinterpret_cast<int8_t*>(ws + W.w_code),
                                   reinterpret_cast<float*>(ws + W.s_w), s.Cc, trigger_mask, s.B, s.T, s.bits_kv, ntrig,
                                   trig_idx, slot_of, st));
        TAQ_TRY_HIP(launch_gemm_fp(context, false, static_cast<const __half*>(Wk), nullptr, M, s.C, s.Cc, rows_f, nullptr, 2 * s.C, st));
        TAQ_TRY_HIP(launch_gemm_fp(context, false, static_cast<const __half*>(Wv), nullptr, M, s.C, s.Cc, rows_f + s.C, nullptr, 2 * s.C, st));
        TAQ_TRY_HIP(launch_kv_pack(rows_f, slot_of, s.B, s.T, s.C, s.H, s.bits_kv, pk + L.k_code, pk + L.v_code,
                                   reinterpret_cast<float*>(pk + L.s_k), reinterpret_cast<float*>(pk + L.s_v), st));
        TAQ_TRY_HIP(launch_kv_image(pk, s, st));
        TAQ_TRY_HIP(launch_kv_rows_from_f32(rows_f, ntrig, trig_idx, s.B, s.T, s.C, reinterpret_cast<__half*>(pk + L.k16),
                                            reinterpret_cast<__half*>(pk + L.v16), reinterpret_cast<__half*>(pk + L.v16t), st));
        return TAQ_OK;
    }

    // one launch: protected-token list, per-token int8 codes of the context (needed for unprotected tokens only) and,
    // unless the caller brings them, the 8-bit weight codes (Wk rows then Wv rows)
    int8_t* wc = reinterpret_cast<int8_t*>(ws + W.w_code);
    float* sw = reinterpret_cast<float*>(ws + W.s_w);
    TAQ_TRY_HIP(launch_kv_prep(s.bits_kv != 16 ? static_cast<const __half*>(context) : nullptr, M, x_code, s_x,
                               w_code ? nullptr : static_cast<const __half*>(Wk),
                               w_code ? nullptr : static_cast<const __half*>(Wv), s.C, wc, sw, s.Cc, trigger_mask, s.B,
                               s.T, s.bits_kv, ntrig, trig_idx, slot_of, st));
    if (!w_code) {
        w_code = wc;
        s_w = sw;
    }
    if (s.bits_kv != 16) {
        // unprotected tokens, one launch per (head, batch element): integer projection, float32 dequantisation, Eq. (2)
        // codes and scales (zero on protected rows), and the operand-ordered image of the single-kernel paths
        // (the same launch carries the workgroups that compute the protected rows in fp16)
        TAQ_TRY_HIP(launch_kv_head(x_code, s_x, w_code, s_w, pk, static_cast<const __half*>(context), s, st));
    } else {
        // every row protected: zero scales, no code section, an image without integer rows, all rows in fp16
        TAQ_TRY_HIP(launch_kv_pack(rows_f, slot_of, s.B, s.T, s.C, s.H, s.bits_kv, pk + L.k_code, pk + L.v_code,
                                   reinterpret_cast<float*>(pk + L.s_k), reinterpret_cast<float*>(pk + L.s_v), st));
        TAQ_TRY_HIP(launch_kv_image(pk, s, st));
        TAQ_TRY_HIP(launch_kv_trigger_rows(static_cast<const __half*>(context), w_code, s_w, ntrig, trig_idx, s.B, s.T,
                                           s.C, s.Cc, reinterpret_cast<__half*>(pk + L.k16),
                                           reinterpret_cast<__half*>(pk + L.v16), reinterpret_cast<__half*>(pk + L.v16t), st));
    }
    return TAQ_OK;
}

int taq_quantize_kv(const void* context, const uint8_t* trigger_mask, const void* Wk, const void* Wv, int bits,
                    const taq_shape* shape, void* qkv_packed, void* workspace, void* hip_stream) {
    int rc = check_shape(shape, false);
    if (rc != TAQ_OK) return rc;
    if (!context || !trigger_mask || !Wk || !Wv || !qkv_packed || !workspace) return TAQ_ERR_INVALID_ARG;
    if (bits != shape->bits_kv) return TAQ_ERR_INVALID_ARG;
    if (misaligned(context) || misaligned(Wk) || misaligned(Wv) || misaligned(qkv_packed) || misaligned(workspace))
        return TAQ_ERR_MISALIGNED;
    return quantize_kv_impl(context, trigger_mask, Wk, Wv, nullptr, nullptr, *shape, qkv_packed, workspace,
                            static_cast<hipStream_t>(hip_stream));
}

int taq_quantize_kv_w8(const void* context, const uint8_t* trigger_mask, const int8_t* Wkv_code, const float* s_wkv,
                       int bits, const taq_shape* shape, void* qkv_packed, void* workspace, void* hip_stream) {
    int rc = check_shape(shape, false);
    if (rc != TAQ_OK) return rc;
    if (!context || !trigger_mask || !Wkv_code || !s_wkv || !qkv_packed || !workspace) return TAQ_ERR_INVALID_ARG;
    if (bits != shape->bits_kv || shape->bits_proj != 8) return TAQ_ERR_INVALID_ARG;  // weight codes: the W8A8 projections only
    if (misaligned(context) || misaligned(Wkv_code) || misaligned(s_wkv) || misaligned(qkv_packed) || misaligned(workspace))
        return TAQ_ERR_MISALIGNED;
    return quantize_kv_impl(context, trigger_mask, nullptr, nullptr, Wkv_code, s_wkv, *shape, qkv_packed, workspace,
                            static_cast<hipStream_t>(hip_stream));
}

int taq_cross_attn_ex(const void* hidden, const void* qkv_packed, const int8_t* Wq, const int8_t* Wo,
                      const float* scales, const uint8_t* trigger_mask, const taq_shape* shape, void* out,
                      void* workspace, void* hip_stream, const taq_debug* dbg) {
    (void)trigger_mask;  // the protected-token list travels inside qkv_packed
    int rc = check_shape(shape, true);
    if (rc != TAQ_OK) return rc;
    if (!hidden || !qkv_packed || !Wq || !Wo || !scales || !out || !workspace) return TAQ_ERR_INVALID_ARG;
    if (misaligned(hidden) || misaligned(qkv_packed) || misaligned(Wq) || misaligned(Wo) || misaligned(scales) ||
        misaligned(out) || misaligned(workspace))
        return TAQ_ERR_MISALIGNED;
    const taq_shape& s = *shape;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    const AttnWorkspace W = attn_workspace(s);
    uint8_t* ws = static_cast<uint8_t*>(workspace);
    int8_t* h_code = reinterpret_cast<int8_t*>(ws + W.h_code);
    float* s_h = reinterpret_cast<float*>(ws + W.s_h);
    float* q_f = reinterpret_cast<float*>(ws + W.q_f);
    int8_t* q_code = reinterpret_cast<int8_t*>(ws + W.q_code);
    float* s_q = reinterpret_cast<float*>(ws + W.s_q);
    float* o_f = reinterpret_cast<float*>(ws + W.o_f);
    int8_t* o_code = reinterpret_cast<int8_t*>(ws + W.o_code);
    float* s_o = reinterpret_cast<float*>(ws + W.s_o);
    const float* s_wq = scales;
    const float* s_wo = scales + s.C;
    const float* bias_o = scales + 2 * s.C;
    const int M = s.B * s.N;
    const unsigned stages = (dbg && dbg->stage_mask) ? dbg->stage_mask : ~0u;

    if (fp_mode(s)) {
        // Full-precision modes, one float32 kernel per stage. With bits_proj = 16 Wq / Wo are the fp16 matrices themselves
        // and only the bias part of `scales` is read.
        if (dbg && dbg->stage_mask) return TAQ_ERR_INVALID_ARG;
        const bool w16 = s.bits_proj == 16;
        if (w16) {
            TAQ_TRY_HIP(launch_gemm_fp(hidden, false, reinterpret_cast<const __half*>(Wq), nullptr, M, s.C, s.C, q_f, nullptr, s.C, st));
        } else {
            TAQ_TRY_HIP(launch_rowquant_f16(static_cast<const __half*>(hidden), M, s.C, h_code, s_h, st));
            TAQ_TRY_HIP(launch_gemm_i8(h_code, s_h, Wq, s_wq, nullptr, M, s.C, s.C, q_f, nullptr, s.C, st));
        }
        if (s.bits_q != 16) TAQ_TRY_HIP(launch_headquant_f32(q_f, M, s.C, s.H, s.bits_q, q_code, s_q, st));
        TAQ_TRY_HIP(launch_attn_fp(q_f, q_code, s_q, static_cast<const uint8_t*>(qkv_packed), s, o_f, dbg ? dbg->p_code : nullptr, st));
        if (w16) {
            TAQ_TRY_HIP(launch_gemm_fp(o_f, true, reinterpret_cast<const __half*>(Wo), bias_o, M, s.C, s.C, nullptr,
                                       static_cast<__half*>(out), s.C, st));
        } else {
            TAQ_TRY_HIP(launch_rowquant_f32(o_f, M, s.C, o_code, s_o, st));
            TAQ_TRY_HIP(launch_gemm_i8(o_code, s_o, Wo, s_wo, bias_o, M, s.C, s.C, nullptr, static_cast<__half*>(out), s.C, st));
        }
        if (dbg) {
            const size_t MC = (size_t)M * s.C;
            if (dbg->h_code && !w16) TAQ_TRY_HIP(hipMemcpyAsync(dbg->h_code, h_code, MC, hipMemcpyDeviceToDevice, st));
            if (dbg->s_h && !w16) TAQ_TRY_HIP(hipMemcpyAsync(dbg->s_h, s_h, (size_t)M * 4, hipMemcpyDeviceToDevice, st));
            if (dbg->q_code && s.bits_q != 16) TAQ_TRY_HIP(hipMemcpyAsync(dbg->q_code, q_code, MC, hipMemcpyDeviceToDevice, st));
            if (dbg->s_Q && s.bits_q != 16) TAQ_TRY_HIP(hipMemcpyAsync(dbg->s_Q, s_q, (size_t)M * s.H * 4, hipMemcpyDeviceToDevice, st));
            if (dbg->O) TAQ_TRY_HIP(hipMemcpyAsync(dbg->O, o_f, MC * 4, hipMemcpyDeviceToDevice, st));
            if (dbg->o_code && !w16) TAQ_TRY_HIP(hipMemcpyAsync(dbg->o_code, o_code, MC, hipMemcpyDeviceToDevice, st));
            if (dbg->s_o && !w16) TAQ_TRY_HIP(hipMemcpyAsync(dbg->s_o, s_o, (size_t)M * 4, hipMemcpyDeviceToDevice, st));
        }
        return TAQ_OK;
    }

    if (fused_supported(s) && !(dbg && dbg->stage_mask)) {
        // the whole block in one kernel; taps are written by the kernel itself
        FusedReq rq = {static_cast<const __half*>(hidden), static_cast<const uint8_t*>(qkv_packed), Wq, Wo, scales,
                       static_cast<__half*>(out)};
        TAQ_TRY_HIP(launch_fused_block(&rq, 1, s, dbg, st));
        return TAQ_OK;
    }

    if (mid_supported(s) && !(dbg && dbg->stage_mask)) {
        // C = 1280 layers, two kernels: hidden codes + to_q + Q~ + attention per head group, then the per-token codes of
        // A^ V~ + to_out; A^ V~ (float32) and its partial row maxima pass through the workspace (the q_f region holds the
        // maxima). Taps are written by the kernels themselves.
        FusedReq rq = {static_cast<const __half*>(hidden), static_cast<const uint8_t*>(qkv_packed), Wq, Wo, scales,
                       static_cast<__half*>(out)};
        TAQ_TRY_HIP(launch_fused_mid(rq, s, o_f, q_f, dbg, st));
        if (M <= 1024) {  // few token tiles: every to_out workgroup quantizes its 16 rows of A^ V~ itself
            TAQ_TRY_HIP(launch_to_out_tail(rq, s, o_f, q_f, nullptr, nullptr, dbg, st));
        } else {          // many: quantize each row once, in a kernel of its own
            TAQ_TRY_HIP(launch_rowquant_f32(o_f, M, s.C, o_code, s_o, st));
            TAQ_TRY_HIP(launch_to_out_tail(rq, s, o_f, q_f, o_code, s_o, dbg, st));
            if (dbg && dbg->o_code) TAQ_TRY_HIP(hipMemcpyAsync(dbg->o_code, o_code, (size_t)M * s.C, hipMemcpyDeviceToDevice, st));
            if (dbg && dbg->s_o) TAQ_TRY_HIP(hipMemcpyAsync(dbg->s_o, s_o, (size_t)M * 4, hipMemcpyDeviceToDevice, st));
        }
        return TAQ_OK;
    }

    if (stages & TAQ_STAGE_HIDDEN_QUANT)
        TAQ_TRY_HIP(launch_rowquant_f16(static_cast<const __half*>(hidden), M, s.C, h_code, s_h, st));
    if (stages & TAQ_STAGE_TO_Q)
        TAQ_TRY_HIP(launch_gemm_i8(h_code, s_h, Wq, s_wq, nullptr, M, s.C, s.C, q_f, nullptr, s.C, st));
    if (stages & TAQ_STAGE_Q_QUANT)
        TAQ_TRY_HIP(launch_headquant_f32(q_f, M, s.C, s.H, s.bits_q, q_code, s_q, st));
    if (stages & TAQ_STAGE_ATTN_CORE) {
        if (fused_supported(s)) {  // (only reached when profiling by stage) the attention phases of the single kernel, alone
            FusedReq rq = {static_cast<const __half*>(hidden), static_cast<const uint8_t*>(qkv_packed), Wq, Wo, scales,
                           static_cast<__half*>(out)};
            TAQ_TRY_HIP(launch_fused_block(&rq, 1, s, nullptr, st, q_code, s_q, o_f));
        } else {
            TAQ_TRY_HIP(launch_attn_core(q_code, s_q, static_cast<const uint8_t*>(qkv_packed), s, o_f, st, dbg ? dbg->p_code : nullptr));
        }
    }
    if (stages & TAQ_STAGE_O_QUANT)
        TAQ_TRY_HIP(launch_rowquant_f32(o_f, M, s.C, o_code, s_o, st));
    if (stages & TAQ_STAGE_TO_OUT)
        TAQ_TRY_HIP(launch_gemm_i8(o_code, s_o, Wo, s_wo, bias_o, M, s.C, s.C, nullptr, static_cast<__half*>(out), s.C, st));

    if (dbg) {
        const size_t MC = (size_t)M * s.C;
        if (dbg->h_code) TAQ_TRY_HIP(hipMemcpyAsync(dbg->h_code, h_code, MC, hipMemcpyDeviceToDevice, st));
        if (dbg->s_h) TAQ_TRY_HIP(hipMemcpyAsync(dbg->s_h, s_h, (size_t)M * 4, hipMemcpyDeviceToDevice, st));
        if (dbg->q_code) TAQ_TRY_HIP(hipMemcpyAsync(dbg->q_code, q_code, MC, hipMemcpyDeviceToDevice, st));
        if (dbg->s_Q) TAQ_TRY_HIP(hipMemcpyAsync(dbg->s_Q, s_q, (size_t)M * s.H * 4, hipMemcpyDeviceToDevice, st));
        if (dbg->O) TAQ_TRY_HIP(hipMemcpyAsync(dbg->O, o_f, MC * 4, hipMemcpyDeviceToDevice, st));
        if (dbg->o_code) TAQ_TRY_HIP(hipMemcpyAsync(dbg->o_code, o_code, MC, hipMemcpyDeviceToDevice, st));
        if (dbg->s_o) TAQ_TRY_HIP(hipMemcpyAsync(dbg->s_o, s_o, (size_t)M * 4, hipMemcpyDeviceToDevice, st));
    }
    return TAQ_OK;
}

int taq_cross_attn(const void* hidden, const void* qkv_packed, const int8_t* Wq, const int8_t* Wo,
                   const float* scales, const uint8_t* trigger_mask, const taq_shape* shape, void* out,
                   void* workspace, void* hip_stream) {
    return taq_cross_attn_ex(hidden, qkv_packed, Wq, Wo, scales, trigger_mask, shape, out, workspace, hip_stream,
                             nullptr);
}

// Scratch of taq_cross_attn_static: a fixed array in device memory, one copy per GPU, each at its own address. In host
// code the array's name is only a stand-in for the symbol; the address kernels can use is looked up once per device
// (with that device current) and kept in scratch_ptr. `used`: no kernel names the array, it must still be emitted.
static __device__ __attribute__((used)) __align__(256) unsigned char scratch[TAQ_STATIC_SCRATCH_BYTES];
static std::atomic<void*> scratch_ptr[64];

static int static_scratch(void** p) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return TAQ_ERR_HIP;
    void* q = scratch_ptr[dev].load(std::memory_order_acquire);
    if (!q) {  // two host threads that race here look up the same address
        if (hipGetSymbolAddress(&q, HIP_SYMBOL(scratch)) != hipSuccess || !q) return TAQ_ERR_HIP;
        scratch_ptr[dev].store(q, std::memory_order_release);
    }
    *p = q;
    return TAQ_OK;
}

int taq_cross_attn_static(const void* hidden, const void* qkv_packed, const int8_t* Wq, const int8_t* Wo,
                          const float* scales, const uint8_t* trigger_mask, const taq_shape* shape, void* out,
                          void* hip_stream) {
    int rc = check_shape(shape, true);
    if (rc != TAQ_OK) return rc;
    // the single-kernel shapes never touch the workspace; every other path uses the layout of attn_workspace
    const size_t need = fused_supported(*shape) ? 0 : attn_workspace(*shape).total;
    if (need > (size_t)TAQ_STATIC_SCRATCH_BYTES) return TAQ_ERR_SCRATCH_TOO_SMALL;
    if (!hidden || !qkv_packed || !Wq || !Wo || !scales || !out) return TAQ_ERR_INVALID_ARG;
    void* ws = nullptr;
    rc = static_scratch(&ws);
    if (rc != TAQ_OK) return rc;
    // nothing in the workspace has to start at zero: every kernel writes what a later one reads
    return taq_cross_attn_ex(hidden, qkv_packed, Wq, Wo, scales, trigger_mask, shape, out, ws, hip_stream, nullptr);
}

int taq_cross_attn_batched(int R, const taq_request* table, const taq_shape* shape, void* workspace,
                           void* hip_stream) {
    if (R <= 0 || !table) return TAQ_ERR_INVALID_ARG;
    int rc = check_shape(shape, true);
    if (rc != TAQ_OK) return rc;
    if (!workspace || misaligned(workspace)) return workspace ? TAQ_ERR_MISALIGNED : TAQ_ERR_INVALID_ARG;
    // validate every request before launching anything
    for (int r = 0; r < R; ++r) {
        const taq_request& q = table[r];
        if (!q.hidden || !q.qkv_packed || !q.Wq || !q.Wo || !q.scales || !q.out) return TAQ_ERR_INVALID_ARG;
        if (misaligned(q.hidden) || misaligned(q.qkv_packed) || misaligned(q.Wq) || misaligned(q.Wo) ||
            misaligned(q.scales) || misaligned(q.out))
            return TAQ_ERR_MISALIGNED;
    }
    size_t per = 0;
    rc = taq_workspace_bytes(shape, &per);
    if (rc != TAQ_OK) return rc;
    {
        taq_shape s = *shape;
        per = attn_workspace(s).total > per ? attn_workspace(s).total : per;
    }
    if (fused_supported(*shape)) {
        // grouped launches: up to 16 requests share one kernel through a pointer table in the arguments
        for (int r0 = 0; r0 < R; r0 += 16) {
            FusedReq rq[16];
            const int n = R - r0 < 16 ? R - r0 : 16;
            for (int i = 0; i < n; ++i) {
                const taq_request& q = table[r0 + i];
                rq[i] = {static_cast<const __half*>(q.hidden), static_cast<const uint8_t*>(q.qkv_packed), q.Wq, q.Wo,
                         q.scales, static_cast<__half*>(q.out)};
            }
            TAQ_TRY_HIP(launch_fused_block(rq, n, *shape, nullptr, static_cast<hipStream_t>(hip_stream)));
        }
        return TAQ_OK;
    }
    for (int r = 0; r < R; ++r) {
        const taq_request& q = table[r];
        rc = taq_cross_attn_ex(q.hidden, q.qkv_packed, q.Wq, q.Wo, q.scales, q.trigger_mask, shape, q.out,
                               static_cast<uint8_t*>(workspace) + (size_t)r * per, hip_stream, nullptr);
        if (rc != TAQ_OK) return rc;
    }
    return TAQ_OK;
}

int taq_mse_f16(const void* x_f16, const void* y_f16, size_t n, double* out, void* hip_stream) {
    if (!x_f16 || !y_f16 || !out || n == 0) return TAQ_ERR_INVALID_ARG;
    if ((reinterpret_cast<uintptr_t>(x_f16) & 1u) || (reinterpret_cast<uintptr_t>(y_f16) & 1u) || (reinterpret_cast<uintptr_t>(out) & 7u))
        return TAQ_ERR_MISALIGNED;
    TAQ_TRY_HIP(launch_mse_f16(static_cast<const __half*>(x_f16), static_cast<const __half*>(y_f16), n, out,
                               static_cast<hipStream_t>(hip_stream)));
    return TAQ_OK;
}

int taq_unpack_kv(const void* qkv_packed, const taq_shape* shape, int8_t* k_codes, int8_t* v_codes,
                  float* k_scales, float* v_scales, void* k_trig_f16, void* v_trig_f16, void* hip_stream) {
    int rc = check_shape(shape, false);
    if (rc != TAQ_OK) return rc;
    if (!qkv_packed) return TAQ_ERR_INVALID_ARG;
    if (misaligned(qkv_packed)) return TAQ_ERR_MISALIGNED;
    TAQ_TRY_HIP(launch_kv_unpack(static_cast<const uint8_t*>(qkv_packed), *shape, k_codes, v_codes, k_scales,
                                 v_scales, static_cast<__half*>(k_trig_f16), static_cast<__half*>(v_trig_f16),
                                 static_cast<hipStream_t>(hip_stream)));
    return TAQ_OK;
}

}  // extern "C"
