// Attention core of the TAQ block (PersonalQ, Section III-B) on gfx950 matrix cores:
//   A  = softmax(Q~ K~^T / sqrt(d))            over the T text tokens of one head
//   A^ = M_A*A + (1-M_A)*Q_a(A)                Eq. (3), Q_a(A) = rint(255*A)/255
//   O  = A^ V~
// with K~/V~ mixed precision (Eq. 2): int8/int4 codes with a per-(head, token) scale, or an
// fp16 row for protected (trigger) tokens.
//
// Formulation. Everything is computed transposed, S^T = K~ Q~^T, so that one image token
// lives in one lane (and its partner lane in the other half-wave): the 32x32 accumulator
// layout then gives every lane 16 of the 32 text tokens of a tile for *its* image token, the
// softmax statistics are in-lane reductions plus one exchange between half-waves, and the
// probabilities never leave registers: the accumulator registers, converted to fp16, are
// exactly the B operand of the next contraction O^T = V~^T A^^T once V~^T is stored in LDS
// in the matching token order.
//
// Exactness. Unprotected scores are exact int8 dot products (integer MFMA) scaled in fp32.
// A^ V~ needs float32-grade accuracy because its result is re-quantized to int8 right after:
// the per-token weight s_V[t]*v_code[t][j] is split into an fp16 high part and an fp16 low
// part (two fp16 MFMAs with the exact integer probability code as the other operand), and
// protected columns split the probability itself the same way against the fp16 V row.
#include "taq_internal.h"

namespace taq {

typedef int int32x4_t __attribute__((ext_vector_type(4)));
typedef int int32x16_t __attribute__((ext_vector_type(16)));
typedef float floatx16_t __attribute__((ext_vector_type(16)));
typedef _Float16 half8_t __attribute__((ext_vector_type(8)));

#define TAQ_NEG_INF (-__builtin_inff())

// Position of text token t inside the LDS rows of V~^T: within each block of 16 tokens the
// order follows the accumulator registers of a 32x32 MFMA tile, so that a lane's 8
// consecutive halfs are the 8 tokens its 8 accumulator registers (of that block) hold.
__device__ __forceinline__ int perm_token(int t) {
    const int u = t & 15;
    return (t & ~15) + 8 * ((u >> 2) & 1) + 4 * (u >> 3) + (u & 3);
}

template <int DT>
struct CoreLds {
    static constexpr int RS_K = DT * 32 + 16;    // bytes per row of int8 K codes
    static constexpr int RS_KF = DT * 32 + 8;    // halfs per row of fp16 K rows
    static constexpr int RS_V = TAQ_MAX_T + 8;   // halfs per row of V~^T (token axis)
    static constexpr int OFF_SK = 0;                                   // f32 [96]
    static constexpr int OFF_BIAS = OFF_SK + TAQ_MAX_T * 4;            // f32 [96]
    static constexpr int OFF_BIASF = OFF_BIAS + TAQ_MAX_T * 4;         // f32 [96]
    static constexpr int OFF_SVMAX = OFF_BIASF + TAQ_MAX_T * 4;        // u32 [4] (first: max s_V bits)
    static constexpr int OFF_KC = OFF_SVMAX + 16;                      // i8  [96][RS_K]
    static constexpr int OFF_KF = OFF_KC + TAQ_MAX_T * RS_K;           // f16 [96][RS_KF]
    static constexpr int OFF_M1 = OFF_KF + TAQ_MAX_T * RS_KF * 2;      // f16 [DT*32][RS_V]
    static constexpr int OFF_M2 = OFF_M1 + DT * 32 * RS_V * 2;
    static constexpr int OFF_VF = OFF_M2 + DT * 32 * RS_V * 2;
    static constexpr int BYTES = OFF_VF + DT * 32 * RS_V * 2;
};

struct CoreArgs {
    const int8_t* q_code;   // [B][N][C]
    const float* s_q;       // [B][N][H]
    const int* ntrig;       // [B]
    const int* slot_of;     // [B][T]
    const float* s_k;       // [B][H][T]
    const float* s_v;
    const uint8_t* k_code;  // [B][T][Cb]
    const uint8_t* v_code;
    const __half* k16;      // [B][T][C] by slot
    const __half* v16;
    float* o_f;             // [B][N][C]
    uint8_t* p_code;        // [B][N][H][T] tap of the probability codes, or NULL
    int N, C, H, T, bits;
    float sig2;             // softmax scale * log2(e)
    float pmax;             // linear grid: 255 or 15 (Eq. 3); log2 grid: 2^15, the factor that puts 2^-code into fp16's range
    float plast;            // log2 grid: the last code, 255 or 15
    int plog;               // 1: log2 grid
    int prow;               // 1: linear grid over the row's own range (largest unprotected probability)
};

__device__ __forceinline__ int load_code(const uint8_t* codes, size_t row, int C, int c, int bits) {
    if (bits == 8) return (int8_t)codes[row * C + c];
    const int nib = (codes[row * (C >> 1) + (c >> 1)] >> (4 * (c & 1))) & 0xF;
    return (nib ^ 8) - 8;
}

// grid: (ceil(N/128), H, B); block: 4 wavefronts x 32 image tokens.
template <int DT>
__global__ __launch_bounds__(256) void attn_core_kernel(CoreArgs a) {
    using L = CoreLds<DT>;
    extern __shared__ __align__(16) unsigned char smem[];
    float* sK = reinterpret_cast<float*>(smem + L::OFF_SK);
    float* bias = reinterpret_cast<float*>(smem + L::OFF_BIAS);
    float* biasf = reinterpret_cast<float*>(smem + L::OFF_BIASF);
    int8_t* Kc = reinterpret_cast<int8_t*>(smem + L::OFF_KC);
    _Float16* Kf = reinterpret_cast<_Float16*>(smem + L::OFF_KF);
    _Float16* M1 = reinterpret_cast<_Float16*>(smem + L::OFF_M1);
    _Float16* M2 = reinterpret_cast<_Float16*>(smem + L::OFF_M2);
    _Float16* Vf = reinterpret_cast<_Float16*>(smem + L::OFF_VF);

    const int tid = threadIdx.x;
    const int b = blockIdx.z, h = blockIdx.y;
    const int N = a.N, C = a.C, H = a.H, T = a.T, bits = a.bits;
    const int d = C / H;
    const int ntrig = a.ntrig[b];
    const int nfp = (ntrig + 31) >> 5;   // fp16 tiles of 32 protected tokens
    const int ntt = (T + 31) >> 5;       // tiles of 32 text tokens
    const int* slot_of = a.slot_of + b * T;

    // ---------------- stage K~ / V~ of this (batch, head) in LDS
    unsigned* svmax = reinterpret_cast<unsigned*>(smem + L::OFF_SVMAX);
    if (tid == 0) svmax[0] = 0u;
    __syncthreads();
    for (int t = tid; t < TAQ_MAX_T; t += 256) {
        const bool isint = t < T && slot_of[t] < 0;
        sK[t] = isint ? a.s_k[((size_t)b * H + h) * T + t] * a.sig2 : 0.f;
        bias[t] = isint ? 0.f : TAQ_NEG_INF;
        biasf[t] = t < ntrig ? 0.f : TAQ_NEG_INF;
        if (isint && bits != 16) atomicMax(svmax, __float_as_uint(a.s_v[((size_t)b * H + h) * T + t]));
    }
    __syncthreads();
    // Power-of-two prescale of the dequantised V rows: brings the largest |s_V*code| into
    // [256, 512) so that the fp16 high/low split keeps ~22 bits whatever the data's magnitude.
    int kexp = 0;
    {
        const float dmax = __uint_as_float(svmax[0]) * (bits == 4 ? 7.f : 127.f);
        if (dmax > 0.f) {
            int e;
            (void)frexpf(dmax, &e);
            kexp = 9 - e;
        }
    }
    const float vpre = ldexpf(1.0f, kexp);
    for (int i = tid; i < TAQ_MAX_T * DT * 8; i += 256) {  // K codes, 4 channels per item
        const int t = i / (DT * 8), j = (i % (DT * 8)) * 4;
        unsigned w = 0;
        if (t < T && j < d && bits != 16) {
            const size_t row = (size_t)b * T + t;
            if (bits == 8) {
                w = *reinterpret_cast<const unsigned*>(a.k_code + row * C + h * d + j);
            } else {
                const unsigned short q = *reinterpret_cast<const unsigned short*>(a.k_code + row * (C >> 1) + ((h * d + j) >> 1));
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int nib = (q >> (4 * e)) & 0xF;
                    w |= (unsigned)(((nib ^ 8) - 8) & 0xFF) << (8 * e);
                }
            }
        }
        *reinterpret_cast<unsigned*>(Kc + t * L::RS_K + j) = w;
    }
    for (int i = tid; i < nfp * 32 * DT * 4; i += 256) {  // fp16 K rows, 8 channels per item
        const int slot = i / (DT * 4), j = (i % (DT * 4)) * 8;
        uint4 w = make_uint4(0, 0, 0, 0);
        if (slot < ntrig && j < d)
            w = *reinterpret_cast<const uint4*>(a.k16 + ((size_t)b * T + slot) * C + h * d + j);
        *reinterpret_cast<uint4*>(Kf + slot * L::RS_KF + j) = w;
    }
    for (int i = tid; i < TAQ_MAX_T * DT * 32; i += 256) {  // V~^T high/low parts
        const int t = i / (DT * 32), j = i % (DT * 32);
        float hi = 0.f, lo = 0.f;
        if (t < T && j < d && bits != 16 && slot_of[t] < 0) {
            const float sv = a.s_v[((size_t)b * H + h) * T + t];
            const float D = ((float)load_code(a.v_code, (size_t)b * T + t, C, h * d + j, bits) * sv) * vpre;
            hi = (float)(_Float16)__builtin_amdgcn_cvt_pkrtz(D, 0.f)[0];  // (an intrinsic: one value for both uses, see below)
            lo = D - hi;
        }
        const int p = perm_token(t);
        M1[j * L::RS_V + p] = (_Float16)hi;
        M2[j * L::RS_V + p] = (_Float16)lo;
    }
    for (int i = tid; i < nfp * 32 * DT * 32; i += 256) {  // fp16 V rows, transposed
        const int slot = i / (DT * 32), j = i % (DT * 32);
        _Float16 v = (_Float16)0.f;
        if (slot < ntrig && j < d)
            v = reinterpret_cast<const _Float16*>(a.v16)[((size_t)b * T + slot) * C + h * d + j];
        Vf[j * L::RS_V + perm_token(slot)] = v;
    }
    __syncthreads();

    // ---------------- this lane's image token
    const int wave = tid >> 6, lane = tid & 63, r = lane & 31, half = lane >> 5;
    const int n = blockIdx.x * 128 + wave * 32 + r;
    const bool nvalid = n < N;
    const size_t tok = (size_t)b * N + (nvalid ? n : N - 1);
    const int8_t* qrow = a.q_code + tok * C + h * d;
    int32x4_t qop[DT];
#pragma unroll
    for (int s = 0; s < DT; ++s) {
        const int off = 32 * s + 16 * half;
        uint2 lo = make_uint2(0, 0), hi = make_uint2(0, 0);
        if (off + 8 <= d) lo = *reinterpret_cast<const uint2*>(qrow + off);
        if (off + 16 <= d) hi = *reinterpret_cast<const uint2*>(qrow + off + 8);
        qop[s][0] = (int)lo.x;
        qop[s][1] = (int)lo.y;
        qop[s][2] = (int)hi.x;
        qop[s][3] = (int)hi.y;
    }
    const float sQ = a.s_q[tok * H + h];

    // ---------------- scores (log2 domain): S^T = K~ Q~^T
    float S[3][16], Sf[3][16];
#pragma unroll
    for (int tile = 0; tile < 3; ++tile) {
        if (tile < ntt) {
            int32x16_t acc;
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[i] = 0;
#pragma unroll
            for (int s = 0; s < DT; ++s) {
                const int32x4_t ka = *reinterpret_cast<const int32x4_t*>(Kc + (32 * tile + r) * L::RS_K + 32 * s + 16 * half);
                acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(ka, qop[s], acc, 0, 0, 0);
            }
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int t0 = 32 * tile + 8 * g + 4 * half;
                const float4 sk = *reinterpret_cast<const float4*>(sK + t0);
                const float4 bi = *reinterpret_cast<const float4*>(bias + t0);
                S[tile][4 * g + 0] = __builtin_fmaf((float)acc[4 * g + 0], sQ * sk.x, bi.x);
                S[tile][4 * g + 1] = __builtin_fmaf((float)acc[4 * g + 1], sQ * sk.y, bi.y);
                S[tile][4 * g + 2] = __builtin_fmaf((float)acc[4 * g + 2], sQ * sk.z, bi.z);
                S[tile][4 * g + 3] = __builtin_fmaf((float)acc[4 * g + 3], sQ * sk.w, bi.w);
            }
        } else {
#pragma unroll
            for (int i = 0; i < 16; ++i) S[tile][i] = TAQ_NEG_INF;
        }
    }
    if (nfp > 0) {
        half8_t qh[DT][2];  // Q~ codes as fp16 (exact)
#pragma unroll
        for (int s = 0; s < DT; ++s)
#pragma unroll
            for (int sub = 0; sub < 2; ++sub)
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const int w = qop[s][2 * sub + (e >> 2)];
                    qh[s][sub][e] = (_Float16)(float)(int)(int8_t)((w >> (8 * (e & 3))) & 0xFF);
                }
        const float sq2 = sQ * a.sig2;
#pragma unroll
        for (int ft = 0; ft < 3; ++ft) {
            if (ft < nfp) {
                floatx16_t acc;
#pragma unroll
                for (int i = 0; i < 16; ++i) acc[i] = 0.f;
#pragma unroll
                for (int s = 0; s < DT; ++s)
#pragma unroll
                    for (int sub = 0; sub < 2; ++sub) {
                        const half8_t ka = *reinterpret_cast<const half8_t*>(Kf + (32 * ft + r) * L::RS_KF + 32 * s + 16 * half + 8 * sub);
                        acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(ka, qh[s][sub], acc, 0, 0, 0);
                    }
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const float4 bi = *reinterpret_cast<const float4*>(biasf + 32 * ft + 8 * g + 4 * half);
                    Sf[ft][4 * g + 0] = __builtin_fmaf(acc[4 * g + 0], sq2, bi.x);
                    Sf[ft][4 * g + 1] = __builtin_fmaf(acc[4 * g + 1], sq2, bi.y);
                    Sf[ft][4 * g + 2] = __builtin_fmaf(acc[4 * g + 2], sq2, bi.z);
                    Sf[ft][4 * g + 3] = __builtin_fmaf(acc[4 * g + 3], sq2, bi.w);
                }
            } else {
#pragma unroll
                for (int i = 0; i < 16; ++i) Sf[ft][i] = TAQ_NEG_INF;
            }
        }
    } else {
#pragma unroll
        for (int ft = 0; ft < 3; ++ft)
#pragma unroll
            for (int i = 0; i < 16; ++i) Sf[ft][i] = TAQ_NEG_INF;
    }

    // ---------------- softmax over all text tokens of this image token
    float mx = TAQ_NEG_INF;
#pragma unroll
    for (int tile = 0; tile < 3; ++tile)
#pragma unroll
        for (int i = 0; i < 16; ++i) mx = fmaxf(mx, fmaxf(S[tile][i], Sf[tile][i]));
    mx = fmaxf(mx, __shfl_xor(mx, 32));
    float Z = 0.f, eu = 0.f;
#pragma unroll
    for (int tile = 0; tile < 3; ++tile)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const float arg = S[tile][i] - mx;
            const float ex = __builtin_amdgcn_exp2f(arg);
            Sf[tile][i] = __builtin_amdgcn_exp2f(Sf[tile][i] - mx);
            Z += ex + Sf[tile][i];
            eu = fmaxf(eu, ex);
            S[tile][i] = a.plog ? arg : ex;  // the log2 grid rounds the exponent itself
        }
    Z += __shfl_xor(Z, 32);
    eu = fmaxf(eu, __shfl_xor(eu, 32));
    const float inv = 1.0f / Z;
    const float lz = __builtin_amdgcn_logf(Z);  // log2 Z >= 0 (the largest term is 1)
    // Row-range grid: codes = rint(pmax * E / range) with range = largest unprotected E, A^ = code * (range / Z) / pmax.
    // Unprotected columns that together weigh less than 2^-40 of the row (or none at all) are dropped.
    const bool ranged = a.prow && eu > Z * 9.094947e-13f;
    const float invc = ranged ? 1.0f / eu : inv;    // code = rint((E * invc) * pmax)
    const float rz = ranged ? Z / eu : 1.f;         // protected partial sums into the units of the coded ones
    const float fz = ranged ? eu / Z : 1.f;         // and the result back

    // ---------------- O^T = V~^T A^^T
    floatx16_t oacc[DT];
#pragma unroll
    for (int jt = 0; jt < DT; ++jt)
#pragma unroll
        for (int i = 0; i < 16; ++i) oacc[jt][i] = 0.f;
#pragma unroll
    for (int ft = 0; ft < 3; ++ft) {
        if (ft < nfp) {
#pragma unroll
            for (int blk = 0; blk < 2; ++blk) {
                half8_t phi, plo;  // protected columns keep A: 255*A as fp16 high + low parts
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    // high part by the conversion intrinsic (round toward zero), so that the one value that goes into
                    // the MFMA is also the one subtracted: a plain cast of the product may be merged with the multiply
                    // into a single-rounding instruction in one use and not in the other
                    const float x = (Sf[ft][8 * blk + e] * inv) * a.pmax;
                    const _Float16 xh = (_Float16)__builtin_amdgcn_cvt_pkrtz(x, 0.f)[0];
                    phi[e] = xh;
                    plo[e] = (_Float16)(x - (float)xh);
                }
#pragma unroll
                for (int jt = 0; jt < DT; ++jt) {
                    const half8_t v = *reinterpret_cast<const half8_t*>(Vf + (32 * jt + r) * L::RS_V + 32 * ft + 16 * blk + 8 * half);
                    oacc[jt] = __builtin_amdgcn_mfma_f32_32x32x16_f16(v, phi, oacc[jt], 0, 0, 0);
                    oacc[jt] = __builtin_amdgcn_mfma_f32_32x32x16_f16(v, plo, oacc[jt], 0, 0, 0);
                }
            }
        }
    }

    if (nfp > 0) {  // bring the protected columns' partial sums to the prescaled units
#pragma unroll
        for (int jt = 0; jt < DT; ++jt)
#pragma unroll
            for (int i = 0; i < 16; ++i) oacc[jt][i] *= vpre * rz;
    }
#pragma unroll
    for (int tile = 0; tile < 3; ++tile) {
        if (tile < ntt) {
#pragma unroll
            for (int blk = 0; blk < 2; ++blk) {
                half8_t p;  // Eq. (3): integer probability codes, exact in fp16
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    float code;
                    if (a.plog) {
                        // -code = clip(rint(log2 A)) = clip(rint(arg - log2 Z)); weight 2^(15 - code), a power of
                        // two that fp16 holds exactly down to 2^-24 (smaller ones vanish: below 2^-39 of the row sum)
                        const float c = fminf(fmaxf(__builtin_rintf(S[tile][8 * blk + e] - lz), -a.plast), 0.f);
                        p[e] = (_Float16)ldexpf(1.0f, 15 + (int)c);
                        code = -c;
                    } else {
                        code = __builtin_rintf((S[tile][8 * blk + e] * invc) * a.pmax);
                        p[e] = (_Float16)code;
                    }
                    if (a.p_code && nvalid) {  // tap: register e of this block holds text token t (accumulator order)
                        const int t = 32 * tile + 16 * blk + 8 * (e >> 2) + 4 * half + (e & 3);
                        if (t < T) a.p_code[(tok * H + h) * (size_t)T + t] = (uint8_t)(int)code;
                    }
                }
#pragma unroll
                for (int jt = 0; jt < DT; ++jt) {
                    const int o = (32 * jt + r) * L::RS_V + 32 * tile + 16 * blk + 8 * half;
                    const half8_t v1 = *reinterpret_cast<const half8_t*>(M1 + o);
                    const half8_t v2 = *reinterpret_cast<const half8_t*>(M2 + o);
                    oacc[jt] = __builtin_amdgcn_mfma_f32_32x32x16_f16(v1, p, oacc[jt], 0, 0, 0);
                    oacc[jt] = __builtin_amdgcn_mfma_f32_32x32x16_f16(v2, p, oacc[jt], 0, 0, 0);
                }
            }
        }
    }
    // ---------------- store O (float32): lane holds channels 32*jt + 8*g + 4*half + 0..3
    if (nvalid) {
        float* orow = a.o_f + tok * C + h * d;
        const float k = (ldexpf(1.0f, -kexp) / a.pmax) * fz;
#pragma unroll
        for (int jt = 0; jt < DT; ++jt)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int j = 32 * jt + 8 * g + 4 * half;
                if (j < d) {
                    float4 v = make_float4(oacc[jt][4 * g] * k, oacc[jt][4 * g + 1] * k, oacc[jt][4 * g + 2] * k,
                                           oacc[jt][4 * g + 3] * k);
                    *reinterpret_cast<float4*>(orow + j) = v;
                }
            }
    }
}

template <int DT>
static hipError_t launch_core_dt(const CoreArgs& a, int B, hipStream_t st) {
    static std::atomic<unsigned long long> lds_set{0};
    const int bytes = CoreLds<DT>::BYTES;
    const hipError_t e = ensure_dynamic_lds(reinterpret_cast<const void*>(&attn_core_kernel<DT>), bytes, lds_set);
    if (e != hipSuccess) return e;
    dim3 grid((a.N + 127) / 128, a.H, B);
    hipLaunchKernelGGL(attn_core_kernel<DT>, grid, dim3(256), bytes, st, a);
    return hipGetLastError();
}

hipError_t launch_attn_core(const int8_t* q_code, const float* s_q, const uint8_t* packed, const taq_shape& s,
                            float* o_f, hipStream_t st, uint8_t* p_code) {
    const KvLayout L = kv_layout(s);
    CoreArgs a;
    a.q_code = q_code;
    a.p_code = p_code;
    a.s_q = s_q;
    a.ntrig = reinterpret_cast<const int*>(packed + L.ntrig);
    a.slot_of = reinterpret_cast<const int*>(packed + L.slot_of);
    a.s_k = reinterpret_cast<const float*>(packed + L.s_k);
    a.s_v = reinterpret_cast<const float*>(packed + L.s_v);
    a.k_code = packed + L.k_code;
    a.v_code = packed + L.v_code;
    a.k16 = reinterpret_cast<const __half*>(packed + L.k16);
    a.v16 = reinterpret_cast<const __half*>(packed + L.v16);
    a.o_f = o_f;
    a.N = s.N;
    a.C = s.C;
    a.H = s.H;
    a.T = s.T;
    a.bits = s.bits_kv;
    const int d = s.C / s.H;
    const float sigma = s.softmax_scale != 0.f ? s.softmax_scale : 1.0f / sqrtf((float)d);
    a.sig2 = sigma * 1.4426950408889634f;
    a.pmax = s.prob_grid == TAQ_PROB_LOG2 ? 32768.f : s.bits_prob == 4 ? 15.f : 255.f;
    a.plast = s.bits_prob == 4 ? 15.f : 255.f;
    a.plog = s.prob_grid == TAQ_PROB_LOG2;
    a.prow = s.prob_grid == TAQ_PROB_ROWMAX;
    switch ((d + 31) / 32) {
        case 1: return launch_core_dt<1>(a, s.B, st);
        case 2: return launch_core_dt<2>(a, s.B, st);
        case 3: return launch_core_dt<3>(a, s.B, st);
        case 4: return launch_core_dt<4>(a, s.B, st);
        case 5: return launch_core_dt<5>(a, s.B, st);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace taq
