// The whole TAQ cross-attention block (PersonalQ, Section III-B) in ONE kernel for gfx950.
//
//   hidden --per-token int8--> to_q (int8 MFMA) --Q_a per (token, head): Eq. 2, line 3-->
//   S^T = K~ Q~^T (int8 MFMA, fp16 MFMA for protected rows) --> softmax --> Eq. 3 -->
//   O^T = V~^T A^^T (fp16 MFMA, split operands) --per-token int8--> to_out (int8 MFMA) --> fp16
//
// Nothing between `hidden` and `out` touches HBM: per image token the kernel reads 2C bytes and
// writes 2C bytes; weights and K~/V~ come from L2.
//
// Work split. A workgroup owns 32 image tokens and all heads: 2 token groups of 16 tokens times
// NW wavefronts that own 2 heads each. Every contraction is computed transposed (output channel
// or text token along the MFMA row axis, image token along the column axis) with 16x16 tiles, so
// an image token stays in lane (token % 16) of its wavefront, in all four quarter-waves, from the
// first GEMM to the last: per-token reductions are register maxima plus two cross-lane steps, and
// every intermediate (Q~ codes, probabilities, O codes) is handed to the next MFMA as its B operand
// straight from registers. The A operands' contraction order is free, so K~ and V~^T are stored
// in LDS in the order in which the accumulator registers of the previous MFMA come out.
//
// Bit-exact steps (same float32 operation order as the definition): per-token codes of hidden,
// the int32 accumulators, Qf = float(acc) * (s_h * s_wq), Q~ codes and scales.
#include "taq_internal.h"

namespace taq {

typedef int int32x4_t __attribute__((ext_vector_type(4)));
typedef float floatx4_t __attribute__((ext_vector_type(4)));
typedef _Float16 half4_t __attribute__((ext_vector_type(4)));
typedef _Float16 half8_t __attribute__((ext_vector_type(8)));

#define TAQ_NEG_INF (-__builtin_inff())
#define TAQ_MAX_REQ 16

__device__ __forceinline__ int symq_code_f(float x, float qmaxf, float amax) {
    float t = x * qmaxf;
    float q = t / amax;  // correctly rounded float32 division
    float r = __builtin_rintf(q);
    r = fminf(fmaxf(r, -qmaxf), qmaxf);
    return (int)r;
}

__device__ __forceinline__ unsigned pack4(int a, int b, int c, int d) {
    return (unsigned)(a & 0xFF) | ((unsigned)(b & 0xFF) << 8) | ((unsigned)(c & 0xFF) << 16) | ((unsigned)(d & 0xFF) << 24);
}

__device__ __forceinline__ float byte_to_float(unsigned w, int e) { return (float)(int)(int8_t)((w >> (8 * e)) & 0xFF); }

// ------------------------------------------------------------------------------------------
// K~/V~ image builder: rearranges the codes of qkv_packed into the order the fused kernel's MFMA
// operands are read in, and precomputes the per-head power-of-two prescale of V.
//   Kp[h][t][tile][q][e]      = k_code[t][h*d + 16*tile + 4*q + e]                (0 outside d / T)
//   Vt[h][j][32*s + 8*q + 4*a + e] = v_code[t = 32*s + 16*a + 4*q + e][h*d + j]   (0 outside T)
// ------------------------------------------------------------------------------------------
__device__ __forceinline__ int code_at(const uint8_t* codes, size_t row, int C, int c, int bits) {
    if (bits == 8) return (int8_t)codes[row * C + c];
    const int nib = (codes[row * (C >> 1) + (c >> 1)] >> (4 * (c & 1))) & 0xF;
    return (nib ^ 8) - 8;
}

__global__ __launch_bounds__(256) void kv_image_kernel(uint8_t* __restrict__ packed, KvLayout L, KvImage I, int T, int C,
                                                       int H, int bits) {
    const int b = blockIdx.x, tid = threadIdx.x;
    const int d = C / H;
    const int* slot_of = reinterpret_cast<const int*>(packed + L.slot_of) + b * T;
    const float* s_k = reinterpret_cast<const float*>(packed + L.s_k) + (size_t)b * H * T;
    const float* s_v = reinterpret_cast<const float*>(packed + L.s_v) + (size_t)b * H * T;
    const uint8_t* k_code = packed + L.k_code;
    const uint8_t* v_code = packed + L.v_code;
    uint8_t* img = packed + L.image + (size_t)b * L.image_bytes;
    __shared__ float vpre_s[TAQ_MAX_H];
    // per-head prescale: largest |s_V * code| goes to [256, 512)
    for (int h = tid; h < H; h += 256) {
        float smax = 0.f;
        for (int t = 0; t < T; ++t)
            if (slot_of[t] < 0) smax = fmaxf(smax, s_v[h * T + t]);
        int kexp = 0;
        const float dmax = smax * (bits == 4 ? 7.f : 127.f);
        if (dmax > 0.f) {
            int e;
            (void)frexpf(dmax, &e);
            kexp = 9 - e;
        }
        vpre_s[h] = ldexpf(1.0f, kexp);
        reinterpret_cast<float*>(img + I.vpre)[h] = ldexpf(1.0f, kexp);
        reinterpret_cast<float*>(img + I.oscale)[h] = ldexpf(1.0f, -kexp) / 255.0f;
    }
    __syncthreads();
    for (int i = tid; i < H * 96; i += 256) {
        const int h = i / 96, t = i % 96;
        const bool isint = t < T && slot_of[t] < 0;
        reinterpret_cast<float*>(img + I.s_k)[i] = isint ? s_k[h * T + t] : 0.f;
        reinterpret_cast<float*>(img + I.s_vp)[i] = isint ? s_v[h * T + t] * vpre_s[h] : 0.f;
        if (h == 0) reinterpret_cast<float*>(img + I.bias)[t] = isint ? 0.f : TAQ_NEG_INF;
    }
    const int rowb = I.tph * 16;  // bytes per (head, token) row of Kp
    for (int i = tid; i < H * I.rows_k * rowb; i += 256) {
        const int e = i & 3, q = (i >> 2) & 3, tile = (i % rowb) >> 4;
        const int t = (i / rowb) % I.rows_k, h = i / (rowb * I.rows_k);
        const int cl = 16 * tile + 4 * q + e;
        int v = 0;
        if (t < T && cl < d && slot_of[t] < 0) v = code_at(k_code, (size_t)b * T + t, C, h * d + cl, bits);
        img[I.kp + i] = (uint8_t)(v & 0xFF);
    }
    for (int i = tid; i < H * d * I.cols_v; i += 256) {
        const int p = i % I.cols_v, j = (i / I.cols_v) % d, h = i / (I.cols_v * d);
        const int s = p >> 5, q = (p >> 3) & 3, a = (p >> 2) & 1, e = p & 3;
        const int t = 32 * s + 16 * a + 4 * q + e;
        int v = 0;
        if (t < T && slot_of[t] < 0) v = code_at(v_code, (size_t)b * T + t, C, h * d + j, bits);
        img[I.vt + i] = (uint8_t)(v & 0xFF);
    }
}

hipError_t launch_kv_image(uint8_t* packed, const taq_shape& s, hipStream_t st) {
    const KvLayout L = kv_layout(s);
    if (L.image_bytes == 0) return hipSuccess;
    const KvImage I = kv_image(s);
    hipLaunchKernelGGL(kv_image_kernel, dim3(s.B), dim3(256), 0, st, packed, L, I, s.T, s.C, s.H, s.bits_kv);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------
// Fused block kernel
// ------------------------------------------------------------------------------------------
struct FusedTable {
    FusedReq req[TAQ_MAX_REQ];
};

struct FusedDims {
    int R, B, N, T;
    int nt16;          // ceil(T/16)
    float sig2;        // softmax scale * log2(e)
    KvLayout L;
    KvImage I;
    taq_debug dbg;     // taps (NULL pointers = off); only used when R == 1
};

template <int D, int NW>
struct FusedCfg {
    static constexpr int H = 2 * NW;
    static constexpr int C = D * H;
    static constexpr int TPH = (D + 15) / 16;     // 16-row tiles per head
    static constexpr int KS = (TPH + 3) / 4;      // K steps of 64 for S^T = K~ Q~^T
    static constexpr int FS = (TPH + 1) / 2;      // K steps of 32 for the protected-row scores
    static constexpr int KC = C / 64;             // K steps of 64 for the projections
    static constexpr int MT = C / (16 * NW);      // 16-row tiles of to_out per wavefront
    static constexpr int NT = 128 * NW;           // threads
    static constexpr int TILE_RS = C + 16;        // bytes per token row of the int8 tile
};

template <int D, int NW>
__global__ __launch_bounds__(128 * NW) void fused_block_kernel(FusedTable tab, FusedDims dm) {
    using F = FusedCfg<D, NW>;
    constexpr int C = F::C, H = F::H, TPH = F::TPH, KS = F::KS, FS = F::FS, KC = F::KC, MT = F::MT, NT = F::NT;
    extern __shared__ __align__(16) unsigned char smem[];

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, r16 = lane & 15, q = lane >> 4;
    const int tg = wave / NW, hp = wave % NW;
    const int RB = dm.R * dm.B;
    const int rb = blockIdx.x % RB, tile = blockIdx.x / RB;
    const int ri = rb / dm.B, b = rb % dm.B;
    const FusedReq rq = tab.req[ri];
    const int N = dm.N, T = dm.T;
    const int n0 = tile * 32;

    // ---- LDS carve-up
    unsigned char* img = smem;                                  // K~/V~ image
    const size_t img_bytes = dm.I.bytes;
    int8_t* tileq = reinterpret_cast<int8_t*>(smem + img_bytes);              // [32][C+16] h codes, later O codes
    float* wsc = reinterpret_cast<float*>(smem + img_bytes + 32 * F::TILE_RS);  // s_wq | s_wo | bias_o  [3C]
    float* s_h = wsc + 3 * C;                                    // [32]
    float* s_o = s_h + 32;                                       // [32]
    unsigned* omax = reinterpret_cast<unsigned*>(s_o + 32);      // [32][NW]

    const uint8_t* packed = rq.packed;
    const int ntrig = reinterpret_cast<const int*>(packed + dm.L.ntrig)[b];
    const int nfp = (ntrig + 15) >> 4;  // tiles of 16 protected tokens

    // ---- phase 0a: copy the K~/V~ image and the weight scales into LDS
    {
        const uint4* src = reinterpret_cast<const uint4*>(packed + dm.L.image + (size_t)b * dm.L.image_bytes);
        uint4* dst = reinterpret_cast<uint4*>(img);
        const int nvec = (int)(img_bytes >> 4);
        for (int i = tid; i < nvec; i += NT) dst[i] = src[i];
        const float4* ssrc = reinterpret_cast<const float4*>(rq.scales);
        float4* sdst = reinterpret_cast<float4*>(wsc);
        for (int i = tid; i < (3 * C) / 4; i += NT) sdst[i] = ssrc[i];
    }
    // ---- phase 0b: per-token int8 codes of the hidden tile (8 threads per token)
    if (tid < 256) {
        const int tok = tid >> 3, part = tid & 7;
        const int n = n0 + tok;
        const size_t row = (size_t)b * N + (n < N ? n : N - 1);
        const uint4* xr = reinterpret_cast<const uint4*>(rq.hidden + row * C);
        uint4 v[KC];
#pragma unroll
        for (int it = 0; it < KC; ++it) v[it] = xr[it * 8 + part];
        float amax = 0.f;
#pragma unroll
        for (int it = 0; it < KC; ++it) {
            const __half2* hh = reinterpret_cast<const __half2*>(&v[it]);
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                float2 p = __half22float2(hh[e]);
                amax = fmaxf(amax, fmaxf(fabsf(p.x), fabsf(p.y)));
            }
        }
        amax = fmaxf(amax, __shfl_xor(amax, 1));
        amax = fmaxf(amax, __shfl_xor(amax, 2));
        amax = fmaxf(amax, __shfl_xor(amax, 4));
        const bool zero = amax == 0.f;
        const float sc = zero ? 1.f : amax / 127.f;
        const float safe = zero ? 1.f : amax;
        if (part == 0) s_h[tok] = sc;
#pragma unroll
        for (int it = 0; it < KC; ++it) {
            const __half2* hh = reinterpret_cast<const __half2*>(&v[it]);
            int c[8];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                float2 p = __half22float2(hh[e]);
                c[2 * e] = symq_code_f(p.x, 127.f, safe);
                c[2 * e + 1] = symq_code_f(p.y, 127.f, safe);
            }
            uint2 o;
            o.x = pack4(c[0], c[1], c[2], c[3]);
            o.y = pack4(c[4], c[5], c[6], c[7]);
            *reinterpret_cast<uint2*>(tileq + tok * F::TILE_RS + (it * 8 + part) * 8) = o;
            if (dm.dbg.h_code && n < N) *reinterpret_cast<uint2*>(dm.dbg.h_code + row * C + (it * 8 + part) * 8) = o;
        }
        if (dm.dbg.s_h && part == 0 && n < N) dm.dbg.s_h[row] = sc;
    }
    __syncthreads();

    // ---- this lane's image token
    const int tl = tg * 16 + r16;           // token within the tile
    const int n = n0 + tl;
    const bool nvalid = n < N;
    const size_t tok = (size_t)b * N + (nvalid ? n : N - 1);
    const float sh = s_h[tl];
    const float* swq = wsc;
    const float* swo = wsc + C;
    const float* bo = wsc + 2 * C;

    // B operand of to_q: this token's hidden codes, 16 bytes per K step
    int32x4_t hb[KC];
#pragma unroll
    for (int ks = 0; ks < KC; ++ks) hb[ks] = *reinterpret_cast<const int32x4_t*>(tileq + tl * F::TILE_RS + 64 * ks + 16 * q);

    const float* img_sk = reinterpret_cast<const float*>(img + dm.I.s_k);
    const float* img_svp = reinterpret_cast<const float*>(img + dm.I.s_vp);
    const float* img_bias = reinterpret_cast<const float*>(img + dm.I.bias);
    const float* img_oscale = reinterpret_cast<const float*>(img + dm.I.oscale);
    const float* img_vpre = reinterpret_cast<const float*>(img + dm.I.vpre);
    const __half* k16 = reinterpret_cast<const __half*>(packed + dm.L.k16) + (size_t)b * T * C;
    const __half* v16t = reinterpret_cast<const __half*>(packed + dm.L.v16t) + (size_t)b * C * 96;

    float oval[2][TPH][4];  // A^ V~ of this wavefront's two heads: channel h*D + 16*jt + 4*q + i
    float omx = 0.f;

#pragma unroll
    for (int hl = 0; hl < 2; ++hl) {
        const int h = 2 * hp + hl;
        // ================= to_q for this head: Qf^T[c][n], c = h*D + 16*j + (row of tile)
        int32x4_t qacc[TPH];
#pragma unroll
        for (int j = 0; j < TPH; ++j) {
            qacc[j] = (int32x4_t){0, 0, 0, 0};
            int c = h * D + 16 * j + r16;
            c = c < C ? c : C - 1;  // rows past the head are discarded; keep the read in bounds
            const int8_t* wr = rq.wq + (size_t)c * C + 16 * q;
#pragma unroll
            for (int ks = 0; ks < KC; ++ks) {
                const int32x4_t wa = *reinterpret_cast<const int32x4_t*>(wr + 64 * ks);
                qacc[j] = __builtin_amdgcn_mfma_i32_16x16x64_i8(wa, hb[ks], qacc[j], 0, 0, 0);
            }
        }
        // ---- Eq. (2), third line: Q~ = Q_a(Q) per (token, head)
        float qf[TPH][4];
        float qmax = 0.f;
#pragma unroll
        for (int j = 0; j < TPH; ++j) {
            const int cl = 16 * j + 4 * q;  // first of this lane's 4 channels in the head
            const bool valid = cl < D;
            const float4 w4 = *reinterpret_cast<const float4*>(swq + h * D + (valid ? cl : 0));
            const float wv[4] = {w4.x, w4.y, w4.z, w4.w};
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const float sc = sh * wv[i];
                const float v = (float)qacc[j][i] * sc;
                qf[j][i] = valid ? v : 0.f;
                qmax = fmaxf(qmax, fabsf(qf[j][i]));
            }
        }
        qmax = fmaxf(qmax, __shfl_xor(qmax, 16));
        qmax = fmaxf(qmax, __shfl_xor(qmax, 32));
        const bool qzero = qmax == 0.f;
        const float sQ = qzero ? 1.f : qmax / 127.f;
        const float qsafe = qzero ? 1.f : qmax;
        unsigned qpk[TPH];
#pragma unroll
        for (int j = 0; j < TPH; ++j)
            qpk[j] = pack4(symq_code_f(qf[j][0], 127.f, qsafe), symq_code_f(qf[j][1], 127.f, qsafe),
                           symq_code_f(qf[j][2], 127.f, qsafe), symq_code_f(qf[j][3], 127.f, qsafe));
        if (dm.dbg.q_code && nvalid) {
#pragma unroll
            for (int j = 0; j < TPH; ++j)
                if (16 * j + 4 * q < D) *reinterpret_cast<unsigned*>(dm.dbg.q_code + tok * C + h * D + 16 * j + 4 * q) = qpk[j];
            if (dm.dbg.s_Q && q == 0) dm.dbg.s_Q[tok * H + h] = sQ;
        }
        // B operand of the score MFMAs: dword jj of step ks = codes of tile 4*ks + jj
        int32x4_t qop[KS];
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
#pragma unroll
            for (int jj = 0; jj < 4; ++jj) qop[ks][jj] = (4 * ks + jj < TPH) ? (int)qpk[4 * ks + jj] : 0;

        // ================= scores in the log2 domain: S^T[t][n]
        const float sq2 = sQ * dm.sig2;
        float S[6][4], Sf[6][4];
        const int8_t* kp = reinterpret_cast<const int8_t*>(img + dm.I.kp) + (size_t)h * dm.I.rows_k * (TPH * 16);
#pragma unroll
        for (int tt = 0; tt < 6; ++tt) {
            if (tt < dm.nt16) {
                int32x4_t acc = (int32x4_t){0, 0, 0, 0};
                const int8_t* krow = kp + (16 * tt + r16) * (TPH * 16) + 4 * q;
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) {
                    int32x4_t ka;
#pragma unroll
                    for (int jj = 0; jj < 4; ++jj)
                        ka[jj] = (4 * ks + jj < TPH) ? *reinterpret_cast<const int*>(krow + 16 * (4 * ks + jj)) : 0;
                    acc = __builtin_amdgcn_mfma_i32_16x16x64_i8(ka, qop[ks], acc, 0, 0, 0);
                }
                const float4 sk = *reinterpret_cast<const float4*>(img_sk + h * 96 + 16 * tt + 4 * q);
                const float4 bi = *reinterpret_cast<const float4*>(img_bias + 16 * tt + 4 * q);
                S[tt][0] = __builtin_fmaf((float)acc[0], sq2 * sk.x, bi.x);
                S[tt][1] = __builtin_fmaf((float)acc[1], sq2 * sk.y, bi.y);
                S[tt][2] = __builtin_fmaf((float)acc[2], sq2 * sk.z, bi.z);
                S[tt][3] = __builtin_fmaf((float)acc[3], sq2 * sk.w, bi.w);
            } else {
#pragma unroll
                for (int i = 0; i < 4; ++i) S[tt][i] = TAQ_NEG_INF;
            }
        }
        // protected rows: fp16 K rows straight from global memory (a handful of rows)
        if (nfp > 0) {
            half8_t qh[FS];  // Q~ codes as fp16: step s covers tiles 2s, 2s+1
#pragma unroll
            for (int s = 0; s < FS; ++s)
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const int j = 2 * s + (e >> 2);
                    qh[s][e] = (j < TPH) ? (_Float16)byte_to_float(qpk[j < TPH ? j : 0], e & 3) : (_Float16)0.f;
                }
#pragma unroll
            for (int ft = 0; ft < 6; ++ft) {
                if (ft < nfp) {
                    floatx4_t acc = (floatx4_t){0.f, 0.f, 0.f, 0.f};
                    const int slot = 16 * ft + r16;
                    const __half* kr = k16 + (size_t)(slot < ntrig ? slot : 0) * C + h * D + 4 * q;
#pragma unroll
                    for (int s = 0; s < FS; ++s) {
                        half8_t ka;
#pragma unroll
                        for (int jj = 0; jj < 2; ++jj) {
                            const int j = 2 * s + jj;
                            uint2 w = make_uint2(0, 0);
                            if (j < TPH && slot < ntrig && 16 * j + 4 * q < D) w = *reinterpret_cast<const uint2*>(kr + 16 * j);
                            const half4_t hv = *reinterpret_cast<const half4_t*>(&w);
                            ka[4 * jj + 0] = hv[0];
                            ka[4 * jj + 1] = hv[1];
                            ka[4 * jj + 2] = hv[2];
                            ka[4 * jj + 3] = hv[3];
                        }
                        acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(ka, qh[s], acc, 0, 0, 0);
                    }
#pragma unroll
                    for (int i = 0; i < 4; ++i) Sf[ft][i] = (16 * ft + 4 * q + i < ntrig) ? acc[i] * sq2 : TAQ_NEG_INF;
                } else {
#pragma unroll
                    for (int i = 0; i < 4; ++i) Sf[ft][i] = TAQ_NEG_INF;
                }
            }
        } else {
#pragma unroll
            for (int ft = 0; ft < 6; ++ft)
#pragma unroll
                for (int i = 0; i < 4; ++i) Sf[ft][i] = TAQ_NEG_INF;
        }

        // ================= softmax over the text tokens of this image token
        float mx = TAQ_NEG_INF;
#pragma unroll
        for (int tt = 0; tt < 6; ++tt)
#pragma unroll
            for (int i = 0; i < 4; ++i) mx = fmaxf(mx, fmaxf(S[tt][i], Sf[tt][i]));
        mx = fmaxf(mx, __shfl_xor(mx, 16));
        mx = fmaxf(mx, __shfl_xor(mx, 32));
        float Z = 0.f;
#pragma unroll
        for (int tt = 0; tt < 6; ++tt)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                S[tt][i] = __builtin_amdgcn_exp2f(S[tt][i] - mx);
                Sf[tt][i] = __builtin_amdgcn_exp2f(Sf[tt][i] - mx);
                Z += S[tt][i] + Sf[tt][i];
            }
        Z += __shfl_xor(Z, 16);
        Z += __shfl_xor(Z, 32);
        const float inv = 1.0f / Z;

        // ================= O^T = V~^T A^^T
        floatx4_t oacc[TPH];
#pragma unroll
        for (int jt = 0; jt < TPH; ++jt) oacc[jt] = (floatx4_t){0.f, 0.f, 0.f, 0.f};
        if (nfp > 0) {
            // protected columns keep A (Eq. 3): 255*A as fp16 high + low parts against the fp16 V row
#pragma unroll
            for (int ft = 0; ft < 6; ++ft) {
                if (ft < nfp) {
                    half4_t phi, plo;
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const float x = (Sf[ft][i] * inv) * 255.0f;
                        const _Float16 xh = (_Float16)x;
                        phi[i] = xh;
                        plo[i] = (_Float16)(x - (float)xh);
                    }
#pragma unroll
                    for (int jt = 0; jt < TPH; ++jt) {
                        int c = h * D + 16 * jt + r16;
                        c = c < C ? c : C - 1;
                        const __half* vr = v16t + (size_t)c * 96 + 16 * ft + 4 * q;
                        uint2 w = *reinterpret_cast<const uint2*>(vr);
                        half4_t va = *reinterpret_cast<const half4_t*>(&w);
#pragma unroll
                        for (int i = 0; i < 4; ++i)
                            if (16 * ft + 4 * q + i >= ntrig) va[i] = (_Float16)0.f;  // unwritten slots
                        oacc[jt] = __builtin_amdgcn_mfma_f32_16x16x16f16(va, phi, oacc[jt], 0, 0, 0);
                        oacc[jt] = __builtin_amdgcn_mfma_f32_16x16x16f16(va, plo, oacc[jt], 0, 0, 0);
                    }
                }
            }
            const float vpre = img_vpre[h];
#pragma unroll
            for (int jt = 0; jt < TPH; ++jt)
#pragma unroll
                for (int i = 0; i < 4; ++i) oacc[jt][i] *= vpre;
        }
        // unprotected columns: weight = code * (s_V * 2^kexp), split into fp16 high + low parts;
        // V codes are exact in fp16
        const int8_t* vt = reinterpret_cast<const int8_t*>(img + dm.I.vt) + (size_t)h * D * dm.I.cols_v;
#pragma unroll
        for (int s = 0; s < 3; ++s) {
            if (2 * s < dm.nt16) {
                half8_t phi, plo;
#pragma unroll
                for (int a = 0; a < 2; ++a) {
                    const float4 sv = *reinterpret_cast<const float4*>(img_svp + h * 96 + 16 * (2 * s + a) + 4 * q);
                    const float svv[4] = {sv.x, sv.y, sv.z, sv.w};
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const float code = __builtin_rintf((S[2 * s + a][i] * inv) * 255.0f);  // Eq. (3)
                        const float w = code * svv[i];
                        const _Float16 wh = (_Float16)w;
                        phi[4 * a + i] = wh;
                        plo[4 * a + i] = (_Float16)(w - (float)wh);
                    }
                }
#pragma unroll
                for (int jt = 0; jt < TPH; ++jt) {
                    int j = 16 * jt + r16;
                    j = j < D ? j : D - 1;
                    const uint2 w = *reinterpret_cast<const uint2*>(vt + (size_t)j * dm.I.cols_v + 32 * s + 8 * q);
                    half8_t va;
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        va[e] = (_Float16)byte_to_float(w.x, e);
                        va[4 + e] = (_Float16)byte_to_float(w.y, e);
                    }
                    oacc[jt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(va, phi, oacc[jt], 0, 0, 0);
                    oacc[jt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(va, plo, oacc[jt], 0, 0, 0);
                }
            }
        }
        const float osc = img_oscale[h];
#pragma unroll
        for (int jt = 0; jt < TPH; ++jt) {
            const bool valid = 16 * jt + 4 * q < D;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const float v = valid ? oacc[jt][i] * osc : 0.f;
                oval[hl][jt][i] = v;
                omx = fmaxf(omx, fabsf(v));
            }
            if (dm.dbg.O && nvalid && valid)
                *reinterpret_cast<float4*>(dm.dbg.O + tok * C + h * D + 16 * jt + 4 * q) =
                    make_float4(oval[hl][jt][0], oval[hl][jt][1], oval[hl][jt][2], oval[hl][jt][3]);
        }
    }

    // ================= per-token int8 codes of O over all heads
    omx = fmaxf(omx, __shfl_xor(omx, 16));
    omx = fmaxf(omx, __shfl_xor(omx, 32));
    if (q == 0) omax[tl * NW + hp] = __float_as_uint(omx);
    __syncthreads();  // every wavefront is past its reads of the hidden codes
    float oamax = 0.f;
#pragma unroll
    for (int w = 0; w < NW; ++w) oamax = fmaxf(oamax, __uint_as_float(omax[tl * NW + w]));
    const bool ozero = oamax == 0.f;
    const float so = ozero ? 1.f : oamax / 127.f;
    const float osafe = ozero ? 1.f : oamax;
#pragma unroll
    for (int hl = 0; hl < 2; ++hl)
#pragma unroll
        for (int jt = 0; jt < TPH; ++jt)
            if (16 * jt + 4 * q < D) {
                const unsigned pk = pack4(symq_code_f(oval[hl][jt][0], 127.f, osafe), symq_code_f(oval[hl][jt][1], 127.f, osafe),
                                          symq_code_f(oval[hl][jt][2], 127.f, osafe), symq_code_f(oval[hl][jt][3], 127.f, osafe));
                const int c = (2 * hp + hl) * D + 16 * jt + 4 * q;
                *reinterpret_cast<unsigned*>(tileq + tl * F::TILE_RS + c) = pk;
                if (dm.dbg.o_code && nvalid) *reinterpret_cast<unsigned*>(dm.dbg.o_code + tok * C + c) = pk;
            }
    if (dm.dbg.s_o && nvalid && q == 0 && hp == 0) dm.dbg.s_o[tok] = so;
    __syncthreads();

    // ================= to_out: Y^T[c][n], c in this wavefront's quarter of the channels
#pragma unroll
    for (int ks = 0; ks < KC; ++ks) hb[ks] = *reinterpret_cast<const int32x4_t*>(tileq + tl * F::TILE_RS + 64 * ks + 16 * q);
    __half* orow = rq.out + tok * C;
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        const int c0 = (C / NW) * hp + 16 * mt;
        const int8_t* wr = rq.wo + (size_t)(c0 + r16) * C + 16 * q;
        int32x4_t acc = (int32x4_t){0, 0, 0, 0};
#pragma unroll
        for (int ks = 0; ks < KC; ++ks) {
            const int32x4_t wa = *reinterpret_cast<const int32x4_t*>(wr + 64 * ks);
            acc = __builtin_amdgcn_mfma_i32_16x16x64_i8(wa, hb[ks], acc, 0, 0, 0);
        }
        const int c = c0 + 4 * q;
        const float4 w4 = *reinterpret_cast<const float4*>(swo + c);
        const float4 b4 = *reinterpret_cast<const float4*>(bo + c);
        const float y0 = (float)acc[0] * (so * w4.x) + b4.x;
        const float y1 = (float)acc[1] * (so * w4.y) + b4.y;
        const float y2 = (float)acc[2] * (so * w4.z) + b4.z;
        const float y3 = (float)acc[3] * (so * w4.w) + b4.w;
        if (nvalid) {
            half4_t y = {(_Float16)y0, (_Float16)y1, (_Float16)y2, (_Float16)y3};
            *reinterpret_cast<half4_t*>(orow + c) = y;
        }
    }
}

template <int D, int NW>
static hipError_t launch_fused_cfg(const FusedTable& tab, const FusedDims& dm, hipStream_t st) {
    using F = FusedCfg<D, NW>;
    static bool attr_set = false;
    const size_t bytes = dm.I.bytes + 32 * F::TILE_RS + 3 * F::C * 4 + 32 * 4 * 2 + 32 * NW * 4;
    if (bytes > 160 * 1024) return hipErrorInvalidValue;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&fused_block_kernel<D, NW>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    const int tiles = (dm.N + 31) / 32;
    hipLaunchKernelGGL((fused_block_kernel<D, NW>), dim3(tiles * dm.R * dm.B), dim3(F::NT), bytes, st, tab, dm);
    return hipGetLastError();
}

hipError_t launch_fused_block(const FusedReq* reqs, int R, const taq_shape& s, const taq_debug* dbg, hipStream_t st) {
    if (R < 1 || R > TAQ_MAX_REQ || !fused_supported(s)) return hipErrorInvalidValue;
    FusedTable tab;
    for (int r = 0; r < TAQ_MAX_REQ; ++r) tab.req[r] = reqs[r < R ? r : 0];
    FusedDims dm;
    dm.R = R;
    dm.B = s.B;
    dm.N = s.N;
    dm.T = s.T;
    dm.nt16 = (s.T + 15) / 16;
    const int d = s.C / s.H;
    const float sigma = s.softmax_scale != 0.f ? s.softmax_scale : 1.0f / sqrtf((float)d);
    dm.sig2 = sigma * 1.4426950408889634f;
    dm.L = kv_layout(s);
    dm.I = kv_image(s);
    taq_debug none = {nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, 0u};
    dm.dbg = (dbg && R == 1) ? *dbg : none;
    if (d == 40 && s.H == 8) return launch_fused_cfg<40, 4>(tab, dm, st);
    if (d == 80 && s.H == 8) return launch_fused_cfg<80, 4>(tab, dm, st);
    if (d == 64 && s.H == 10) return launch_fused_cfg<64, 5>(tab, dm, st);
    return hipErrorInvalidValue;
}

}  // namespace taq
