// Quantizer kernels of libtaq (gfx950): per-row / per-(row, head) symmetric codes,
// K~/V~ packing (Eq. 2 of PersonalQ, Section III-B), protected-row projection.
//
// The symmetric quantizer is a fixed float32 sequence so that codes are reproducible
// bit for bit:  amax = max|x|;  scale = amax/qmax;  code = clamp(rint((x*qmax)/amax)).
// The build disables FMA contraction and keeps IEEE-correct float32 division.
#include "taq_internal.h"

namespace taq {

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
    return v;
}

// One code of the symmetric quantizer; amax > 0.
__device__ __forceinline__ int symq_code(float x, float qmaxf, float amax) {
    float t = x * qmaxf;
    float q = t / amax;  // correctly rounded float32 division
    float r = __builtin_rintf(q);  // half-to-even
    r = fminf(fmaxf(r, -qmaxf), qmaxf);
    return (int)r;
}

__device__ __forceinline__ void unpack_half8(const uint4& u, float f[8]) {
    const __half2* h = reinterpret_cast<const __half2*>(&u);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        float2 p = __half22float2(h[i]);
        f[2 * i] = p.x;
        f[2 * i + 1] = p.y;
    }
}

__device__ __forceinline__ unsigned pack4_i8(int a, int b, int c, int d) {
    return (unsigned)(a & 0xFF) | ((unsigned)(b & 0xFF) << 8) | ((unsigned)(c & 0xFF) << 16) |
           ((unsigned)(d & 0xFF) << 24);
}

// ---------------------------------------------------------------- fp16 rows -> int8
// One wavefront per row. K % 8 == 0.
__global__ __launch_bounds__(256) void rowquant_f16_kernel(const __half* __restrict__ x, int M, int K,
                                                           int8_t* __restrict__ code,
                                                           float* __restrict__ scale) {
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int row = blockIdx.x * 4 + wave;
    if (row >= M) return;
    const uint4* xr = reinterpret_cast<const uint4*>(x + (size_t)row * K);
    const int nv = K >> 3;
    float amax = 0.f;
    for (int v = lane; v < nv; v += 64) {
        float f[8];
        unpack_half8(xr[v], f);
#pragma unroll
        for (int i = 0; i < 8; ++i) amax = fmaxf(amax, fabsf(f[i]));
    }
    amax = wave_max(amax);
    const bool zero = amax == 0.f;
    const float sc = zero ? 1.f : amax / 127.f;
    const float safe = zero ? 1.f : amax;
    if (lane == 0) scale[row] = sc;
    uint2* cr = reinterpret_cast<uint2*>(code + (size_t)row * K);
    for (int v = lane; v < nv; v += 64) {
        float f[8];
        unpack_half8(xr[v], f);
        int c[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) c[i] = symq_code(f[i], 127.f, safe);
        uint2 o;
        o.x = pack4_i8(c[0], c[1], c[2], c[3]);
        o.y = pack4_i8(c[4], c[5], c[6], c[7]);
        cr[v] = o;
    }
}

// First launch of taq_quantize_kv: the per-row codes of up to three fp16 matrices that share the row length K (the
// context rows and, unless cached, the rows of Wk and Wv), and the protected-token list, each part on workgroups of
// its own: one launch instead of four.
struct KvPrepJob {
    const __half* x;   // rows to quantize (NULL: none)
    int M;             // number of rows
    int8_t* code;
    float* scale;
};

__device__ __forceinline__ void rowquant_f16_row(const __half* __restrict__ x, int row, int K, int8_t* __restrict__ code,
                                                  float* __restrict__ scale, int lane) {
    const uint4* xr = reinterpret_cast<const uint4*>(x + (size_t)row * K);
    const int nv = K >> 3;
    float amax = 0.f;
    for (int v = lane; v < nv; v += 64) {
        float f[8];
        unpack_half8(xr[v], f);
#pragma unroll
        for (int i = 0; i < 8; ++i) amax = fmaxf(amax, fabsf(f[i]));
    }
    amax = wave_max(amax);
    const bool zero = amax == 0.f;
    const float sc = zero ? 1.f : amax / 127.f;
    const float safe = zero ? 1.f : amax;
    if (lane == 0) scale[row] = sc;
    uint2* cr = reinterpret_cast<uint2*>(code + (size_t)row * K);
    for (int v = lane; v < nv; v += 64) {
        float f[8];
        unpack_half8(xr[v], f);
        int c[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) c[i] = symq_code(f[i], 127.f, safe);
        uint2 o;
        o.x = pack4_i8(c[0], c[1], c[2], c[3]);
        o.y = pack4_i8(c[4], c[5], c[6], c[7]);
        cr[v] = o;
    }
}

__global__ __launch_bounds__(256) void kv_prep_kernel(KvPrepJob j0, KvPrepJob j1, KvPrepJob j2, int K,
                                                      const uint8_t* __restrict__ mask, int B, int T, int bits,
                                                      int* __restrict__ ntrig, int* __restrict__ trig_idx,
                                                      int* __restrict__ slot_of) {
    __shared__ int flag[128];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    int blk = blockIdx.x;
    if (blk < B) {  // protected-token list of batch element blk (T <= 96: a direct count is cheaper than a scan)
        const int t = threadIdx.x;
        const bool prot = t < T && (bits == 16 || mask[blk * T + t] != 0);
        if (t < 128) flag[t] = prot ? 1 : 0;
        __syncthreads();
        if (t >= 128) return;
        int before = 0, total = 0;
        for (int u = 0; u < T; ++u) {
            before += (u < t) ? flag[u] : 0;
            total += flag[u];
        }
        if (t < T) {
            slot_of[blk * T + t] = prot ? before : -1;
            if (prot) trig_idx[blk * T + before] = t;
            if (t >= total) trig_idx[blk * T + t] = -1;
        }
        if (t == 0) ntrig[blk] = total;
        return;
    }
    blk -= B;
    const KvPrepJob jobs[3] = {j0, j1, j2};
#pragma unroll
    for (int k = 0; k < 3; ++k) {
        const int nb = (jobs[k].M + 3) / 4;
        if (blk < nb) {
            const int row = blk * 4 + wave;
            if (jobs[k].x && row < jobs[k].M) rowquant_f16_row(jobs[k].x, row, K, jobs[k].code, jobs[k].scale, lane);
            return;
        }
        blk -= nb;
    }
}

hipError_t launch_kv_prep(const __half* context, int M, int8_t* x_code, float* s_x, const __half* Wk, const __half* Wv,
                          int C, int8_t* w_code, float* s_w, int K, const uint8_t* mask, int B, int T, int bits,
                          int* ntrig, int* trig_idx, int* slot_of, hipStream_t st) {
    KvPrepJob j0 = {context, context ? M : 0, x_code, s_x};
    KvPrepJob j1 = {Wk, Wk ? C : 0, w_code, s_w};
    KvPrepJob j2 = {Wv, Wv ? C : 0, w_code + (size_t)C * K, s_w + C};
    const int blocks = B + (j0.M + 3) / 4 + (j1.M + 3) / 4 + (j2.M + 3) / 4;
    hipLaunchKernelGGL(kv_prep_kernel, dim3(blocks), dim3(256), 0, st, j0, j1, j2, K, mask, B, T, bits, ntrig, trig_idx,
                       slot_of);
    return hipGetLastError();
}

hipError_t launch_rowquant_f16(const __half* x, int M, int K, int8_t* code, float* scale, hipStream_t st) {
    if (M <= 0) return hipSuccess;
    hipLaunchKernelGGL(rowquant_f16_kernel, dim3((M + 3) / 4), dim3(256), 0, st, x, M, K, code, scale);
    return hipGetLastError();
}

// ---------------------------------------------------------------- f32 rows -> int8
// One wavefront per row. K % 4 == 0.
__global__ __launch_bounds__(256) void rowquant_f32_kernel(const float* __restrict__ x, int M, int K,
                                                           int8_t* __restrict__ code,
                                                           float* __restrict__ scale) {
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int row = blockIdx.x * 4 + wave;
    if (row >= M) return;
    const float4* xr = reinterpret_cast<const float4*>(x + (size_t)row * K);
    const int nv = K >> 2;
    float amax = 0.f;
    for (int v = lane; v < nv; v += 64) {
        float4 f = xr[v];
        amax = fmaxf(amax, fmaxf(fmaxf(fabsf(f.x), fabsf(f.y)), fmaxf(fabsf(f.z), fabsf(f.w))));
    }
    amax = wave_max(amax);
    const bool zero = amax == 0.f;
    const float sc = zero ? 1.f : amax / 127.f;
    const float safe = zero ? 1.f : amax;
    if (lane == 0) scale[row] = sc;
    unsigned* cr = reinterpret_cast<unsigned*>(code + (size_t)row * K);
    for (int v = lane; v < nv; v += 64) {
        float4 f = xr[v];
        cr[v] = pack4_i8(symq_code(f.x, 127.f, safe), symq_code(f.y, 127.f, safe),
                         symq_code(f.z, 127.f, safe), symq_code(f.w, 127.f, safe));
    }
}

hipError_t launch_rowquant_f32(const float* x, int M, int K, int8_t* code, float* scale, hipStream_t st) {
    if (M <= 0) return hipSuccess;
    hipLaunchKernelGGL(rowquant_f32_kernel, dim3((M + 3) / 4), dim3(256), 0, st, x, M, K, code, scale);
    return hipGetLastError();
}

// ---------------------------------------------------------------- f32 rows -> int8 per head
// One wavefront per row; per-head maxima through LDS atomics on the bit pattern of |x|
// (non-negative floats order like unsigned integers). d % 4 == 0, H <= TAQ_MAX_H.
__global__ __launch_bounds__(256) void headquant_f32_kernel(const float* __restrict__ x, int M, int C, int H,
                                                            float qmaxf, int8_t* __restrict__ code,
                                                            float* __restrict__ scale) {
    __shared__ unsigned smax[4][TAQ_MAX_H];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int row = blockIdx.x * 4 + wave;
    const bool live = row < M;
    const int d = C / H;
    for (int h = lane; h < H; h += 64) smax[wave][h] = 0u;
    __syncthreads();
    const float4* xr = reinterpret_cast<const float4*>(x + (size_t)(live ? row : 0) * C);
    const int nv = C >> 2;
    if (live) {
        for (int v = lane; v < nv; v += 64) {
            float4 f = xr[v];
            float a = fmaxf(fmaxf(fabsf(f.x), fabsf(f.y)), fmaxf(fabsf(f.z), fabsf(f.w)));
            atomicMax(&smax[wave][(v * 4) / d], __float_as_uint(a));
        }
    }
    __syncthreads();
    if (!live) return;
    for (int h = lane; h < H; h += 64) {
        float amax = __uint_as_float(smax[wave][h]);
        scale[(size_t)row * H + h] = amax == 0.f ? 1.f : amax / qmaxf;
    }
    unsigned* cr = reinterpret_cast<unsigned*>(code + (size_t)row * C);
    for (int v = lane; v < nv; v += 64) {
        float4 f = xr[v];
        float amax = __uint_as_float(smax[wave][(v * 4) / d]);
        float safe = amax == 0.f ? 1.f : amax;
        cr[v] = pack4_i8(symq_code(f.x, qmaxf, safe), symq_code(f.y, qmaxf, safe),
                         symq_code(f.z, qmaxf, safe), symq_code(f.w, qmaxf, safe));
    }
}

hipError_t launch_headquant_f32(const float* x, int M, int C, int H, int bits, int8_t* code, float* scale,
                                hipStream_t st) {
    if (M <= 0) return hipSuccess;
    hipLaunchKernelGGL(headquant_f32_kernel, dim3((M + 3) / 4), dim3(256), 0, st, x, M, C, H, bits == 4 ? 7.f : 127.f,
                       code, scale);
    return hipGetLastError();
}

// ---------------------------------------------------------------- K~/V~ codes, Eq. (2)
// One wavefront per (batch, token). rows_f holds that token's K channels then V channels;
// each head's d channels are one quantization row. Protected tokens get zero codes/scales.
__global__ __launch_bounds__(64) void kv_pack_kernel(const float* __restrict__ rows_f,
                                                     const int* __restrict__ slot_of, int T, int C, int H,
                                                     int bits, uint8_t* __restrict__ k_code,
                                                     uint8_t* __restrict__ v_code, float* __restrict__ s_k,
                                                     float* __restrict__ s_v) {
    __shared__ unsigned smax[2 * TAQ_MAX_H];
    const int bt = blockIdx.x, b = bt / T, t = bt % T, lane = threadIdx.x;
    const int d = C / H;
    const bool prot = slot_of[bt] >= 0;
    const float qmaxf = bits == 4 ? 7.f : 127.f;
    for (int g = lane; g < 2 * H; g += 64) smax[g] = 0u;
    __syncthreads();
    const float4* xr = reinterpret_cast<const float4*>(rows_f + (size_t)bt * 2 * C);
    const int nv = (2 * C) >> 2;
    if (!prot) {
        for (int v = lane; v < nv; v += 64) {
            float4 f = xr[v];
            float a = fmaxf(fmaxf(fabsf(f.x), fabsf(f.y)), fmaxf(fabsf(f.z), fabsf(f.w)));
            atomicMax(&smax[(v * 4) / d], __float_as_uint(a));
        }
    }
    __syncthreads();
    for (int g = lane; g < 2 * H; g += 64) {
        float amax = __uint_as_float(smax[g]);
        float sc = prot ? 0.f : (amax == 0.f ? 1.f : amax / qmaxf);
        float* dst = g < H ? s_k : s_v;
        dst[((size_t)b * H + (g % H)) * T + t] = sc;
    }
    if (bits == 16) return;  // every row protected: there is no code section
    for (int v = lane; v < nv; v += 64) {
        const int ch = v * 4;  // channel within the 2C-wide row
        int c0 = 0, c1 = 0, c2 = 0, c3 = 0;
        if (!prot) {
            float4 f = xr[v];
            float amax = __uint_as_float(smax[ch / d]);
            float safe = amax == 0.f ? 1.f : amax;
            c0 = symq_code(f.x, qmaxf, safe);
            c1 = symq_code(f.y, qmaxf, safe);
            c2 = symq_code(f.z, qmaxf, safe);
            c3 = symq_code(f.w, qmaxf, safe);
        }
        uint8_t* base = ch < C ? k_code : v_code;
        const int c = ch < C ? ch : ch - C;
        if (bits == 8) {
            *reinterpret_cast<unsigned*>(base + (size_t)bt * C + c) = pack4_i8(c0, c1, c2, c3);
        } else {
            unsigned short w = (unsigned short)((c0 & 0xF) | ((c1 & 0xF) << 4) | ((c2 & 0xF) << 8) |
                                                ((c3 & 0xF) << 12));
            *reinterpret_cast<unsigned short*>(base + (size_t)bt * (C / 2) + c / 2) = w;
        }
    }
}

hipError_t launch_kv_pack(const float* rows_f, const int* slot_of, int B, int T, int C, int H, int bits,
                          uint8_t* k_code, uint8_t* v_code, float* s_k, float* s_v, hipStream_t st) {
    hipLaunchKernelGGL(kv_pack_kernel, dim3(B * T), dim3(64), 0, st, rows_f, slot_of, T, C, H, bits, k_code,
                       v_code, s_k, s_v);
    return hipGetLastError();
}

// ---------------------------------------------------------------- protected K/V rows
// One workgroup (512 threads) per (slot, batch, 128 output channels): y[c] = s_w[c] * sum_k ctx[t][k] * w_code[c][k].
// Four threads share an output channel, each summing every fourth 16-code piece of the row in float32 (four
// partial sums per thread), combined by two shuffles; one rounding to fp16. Cc % 16 == 0, Cc <= 4096.
__device__ __forceinline__ void kv_trigger_rows_block(float* xs, int slot, int b, int cblk, const __half* __restrict__ context,
                                                      const int8_t* __restrict__ w_code, const float* __restrict__ s_w,
                                                      const int* __restrict__ ntrig, const int* __restrict__ trig_idx,
                                                      int T, int C, int Cc, __half* __restrict__ k16,
                                                      __half* __restrict__ v16, __half* __restrict__ v16t) {
    const int c = cblk * 128 + (threadIdx.x >> 2), part = threadIdx.x & 3;  // output channel in [0, 2C)
    // unused slots of all three copies read as zeros: the padding slots T..95 of the transposed copy ...
    if (slot == T - 1 && c >= C && c < 2 * C && part == 0)
        for (int sp = T; sp < 96; ++sp) v16t[((size_t)b * C + (c - C)) * 96 + sp] = __float2half(0.f);
    if (slot >= ntrig[b]) {  // ... and every slot past the protected tokens
        if (c < 2 * C && part == 0) {
            if (c < C) {
                k16[((size_t)b * T + slot) * C + c] = __float2half(0.f);
            } else {
                v16[((size_t)b * T + slot) * C + (c - C)] = __float2half(0.f);
                v16t[((size_t)b * C + (c - C)) * 96 + slot] = __float2half(0.f);
            }
        }
        return;
    }
    const int t = trig_idx[b * T + slot];
    const __half* xr = context + ((size_t)b * T + t) * Cc;
    for (int k = threadIdx.x; k < Cc; k += 512) xs[k] = __half2float(xr[k]);
    __syncthreads();
    float sum = 0.f;
    if (c < 2 * C) {
        const int4* wr = reinterpret_cast<const int4*>(w_code + (size_t)c * Cc);
        float acc[4] = {0.f, 0.f, 0.f, 0.f};
        for (int kv = part; kv < (Cc >> 4); kv += 4) {
            const int4 w = wr[kv];
            const int wd[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
            for (int qd = 0; qd < 4; ++qd) {
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const float wf = (float)(int)(int8_t)((wd[qd] >> (8 * e)) & 0xFF);
                    acc[e] = __builtin_fmaf(xs[kv * 16 + qd * 4 + e], wf, acc[e]);
                }
            }
        }
        sum = (acc[0] + acc[1]) + (acc[2] + acc[3]);
    }
    sum += __shfl_xor(sum, 1);
    sum += __shfl_xor(sum, 2);
    if (c < 2 * C && part == 0) {
        const __half yh = __float2half_rn(sum * s_w[c]);
        if (c < C) {
            k16[((size_t)b * T + slot) * C + c] = yh;
        } else {
            v16[((size_t)b * T + slot) * C + (c - C)] = yh;
            v16t[((size_t)b * C + (c - C)) * 96 + slot] = yh;  // transposed copy, slot along the row
        }
    }
}

__global__ __launch_bounds__(512) void kv_trigger_rows_kernel(const __half* __restrict__ context,
                                                              const int8_t* __restrict__ w_code,
                                                              const float* __restrict__ s_w,
                                                              const int* __restrict__ ntrig,
                                                              const int* __restrict__ trig_idx, int T, int C,
                                                              int Cc, __half* __restrict__ k16,
                                                              __half* __restrict__ v16,
                                                              __half* __restrict__ v16t) {
    __shared__ float xs[4096];
    kv_trigger_rows_block(xs, blockIdx.x, blockIdx.y, blockIdx.z, context, w_code, s_w, ntrig, trig_idx, T, C, Cc, k16, v16, v16t);
}

hipError_t launch_kv_trigger_rows(const __half* context, const int8_t* w_code, const float* s_w,
                                  const int* ntrig, const int* trig_idx, int B, int T, int C, int Cc,
                                  __half* k16, __half* v16, __half* v16t, hipStream_t st) {
    hipLaunchKernelGGL(kv_trigger_rows_kernel, dim3(T, B, (2 * C + 127) / 128), dim3(512), 0, st, context, w_code, s_w,
                       ntrig, trig_idx, T, C, Cc, k16, v16, v16t);
    return hipGetLastError();
}

// ---------------------------------------------------------------- K/V projection + Eq. (2) codes + image, per head
// Second launch of taq_quantize_kv for 4/8-bit rows: a workgroup does, for one head and every text
// token, the integer projection of the head's K (or V) channels (acc = x_code . w_code over Cc, 16x16x64 int8 MFMA,
// channels as rows and tokens as columns), the float32 dequantisation float(acc) * (s_x * s_w), the per-(head, token)
// symmetric quantizer of Eq. (2) (zero codes and scales on protected tokens), and writes the plain code / scale
// sections of qkv_packed and, where the shape has one, this head's block of the operand-ordered image.
// One workgroup per (head, batch element, K or V), one wavefront per 16-token column tile. d % 8 == 0, Cc % 16 == 0.
// The same launch carries the workgroups of the protected fp16 rows (they need only the first launch's results too).
// WLDS: the head's weight slice (16*TPH rows x Cc codes, Cc % 64 == 0) is fetched once per workgroup, straight into LDS
// in MFMA operand order (one KiB per 16 rows x 64 codes, LDS address = base + lane * 16), and every wavefront reads its
// A operands from there; otherwise each of the up to six wavefronts fetches the slice itself.
typedef int kvh_int32x4_t __attribute__((ext_vector_type(4)));
#ifndef TAQ_NEG_INF
#define TAQ_NEG_INF (-__builtin_inff())
#endif

__device__ __forceinline__ float kvh_quad_allmax(float x) {  // over the lanes l, l^16, l^32, l^48
    const auto a = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    const float y = fmaxf(__uint_as_float(a[0]), __uint_as_float(a[1]));
    const auto b = __builtin_amdgcn_permlane32_swap(__float_as_uint(y), __float_as_uint(y), false, false);
    return fmaxf(__uint_as_float(b[0]), __uint_as_float(b[1]));
}

// Epilogue of one wavefront's 16-token column tile: float32 dequantisation of the integer sums, Eq. (2) quantizer per
// (head, token), plain code / scale sections and the head's image block. This lane: token 16*st + r16, channels
// 16*j + 4*q .. +3 of the head.
template <int TPH>
__device__ __forceinline__ void kvh_finish(const kvh_int32x4_t (&acc)[TPH], int st, int h, int b, int side, int d, int r16, int q,
                                           int T, int C, int H, int bits, float qmaxf, const float* __restrict__ s_x,
                                           const float* __restrict__ s_w, const int* __restrict__ slot_of, uint8_t* codes,
                                           float* scales, uint8_t* img, const KvImage& I, bool has_image, float* sc_l,
                                           unsigned* scmax) {
    const int t = 16 * st + r16, tc = t < T ? t : T - 1;
    const bool tv = t < T;
    const bool prot = !tv || slot_of[tc] >= 0;
    const float sx = s_x[(size_t)b * T + tc];
    float v[TPH][4];
    float amax = 0.f;
#pragma unroll
    for (int j = 0; j < TPH; ++j) {
        const int cl = 16 * j + 4 * q;
        const bool valid = cl < d;
        float4 sw4 = make_float4(0.f, 0.f, 0.f, 0.f);
        if (valid) sw4 = *reinterpret_cast<const float4*>(s_w + side * C + h * d + cl);
        const float swv[4] = {sw4.x, sw4.y, sw4.z, sw4.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const float sc = sx * swv[i];
            v[j][i] = valid ? (float)acc[j][i] * sc : 0.f;
            amax = fmaxf(amax, fabsf(v[j][i]));
        }
    }
    amax = kvh_quad_allmax(amax);
    const float sc = prot ? 0.f : (amax == 0.f ? 1.f : amax / qmaxf);
    const float safe = amax == 0.f ? 1.f : amax;
    if (tv && q == 0) scales[t] = sc;
    if (!prot && q == 0) {
        sc_l[t] = sc;
        atomicMax(scmax, __float_as_uint(sc));
    }
    const int pos = vt_pos(t, I.nt16);  // place of token t in a V^T row
#pragma unroll
    for (int j = 0; j < TPH; ++j) {
        const int cl = 16 * j + 4 * q;
        int c[4] = {0, 0, 0, 0};
        if (!prot && cl < d) {
#pragma unroll
            for (int i = 0; i < 4; ++i) c[i] = symq_code(v[j][i], qmaxf, safe);
        }
        if (tv && cl < d) {
            if (bits == 8) {
                *reinterpret_cast<unsigned*>(codes + ((size_t)b * T + t) * C + h * d + cl) = pack4_i8(c[0], c[1], c[2], c[3]);
            } else {
                const unsigned short w = (unsigned short)((c[0] & 0xF) | ((c[1] & 0xF) << 4) | ((c[2] & 0xF) << 8) |
                                                          ((c[3] & 0xF) << 12));
                *reinterpret_cast<unsigned short*>(codes + ((size_t)b * T + t) * (C / 2) + (h * d + cl) / 2) = w;
            }
        }
        if (has_image) {
            if (!side) {  // Kp[t][tile][quarter][4]; zeros past the head and past the last token
                if (t < I.rows_k)
                    *reinterpret_cast<unsigned*>(img + I.kp + kp_offset(I.tph, t, j, q)) = pack4_i8(c[0], c[1], c[2], c[3]);
            } else if (cl < d) {  // Vt[channel][pos], stored with the sign bit flipped
#pragma unroll
                for (int i = 0; i < 4; ++i) img[I.vt + (size_t)(cl + i) * I.cols_v + pos] = (uint8_t)((c[i] & 0xFF) ^ 0x80);
            }
        }
    }
}

template <int TPH, bool WLDS>
__global__ __launch_bounds__(512) void kv_head_kernel(const int8_t* __restrict__ x_code, const float* __restrict__ s_x,
                                                      const int8_t* __restrict__ w_code, const float* __restrict__ s_w,
                                                      uint8_t* __restrict__ packed, KvLayout L, KvImage I, int T, int C,
                                                      int H, int Cc, int bits, int B, const __half* __restrict__ context) {
    __shared__ float xs[4096];  // protected-row workgroups: the context row in float32
    __shared__ float sc_l[96];  // scales of the unprotected tokens of this head and side (0: protected / padding)
    __shared__ unsigned scmax;
    extern __shared__ __align__(16) unsigned char kvh_w[];  // WLDS: [TPH][Cc/64][64 lanes][16 bytes]
    // workgroups [0, 2*H*B): (head, batch element, K or V); the rest: protected fp16 rows, (slot, batch, 128 channels)
    const int nhead = 2 * H * B;
    if ((int)blockIdx.x >= nhead) {
        const int r = (int)blockIdx.x - nhead, nc = (2 * C + 127) / 128;
        kv_trigger_rows_block(xs, r % T, (r / T) % B, r / (T * B), context, w_code, s_w,
                              reinterpret_cast<const int*>(packed + L.ntrig), reinterpret_cast<const int*>(packed + L.trig_idx), T,
                              C, Cc, reinterpret_cast<__half*>(packed + L.k16), reinterpret_cast<__half*>(packed + L.v16),
                              reinterpret_cast<__half*>(packed + L.v16t));
        (void)nc;
        return;
    }
    const int h = (int)blockIdx.x % H, b = ((int)blockIdx.x / H) % B, side = (int)blockIdx.x / (H * B);  // side 0: K, 1: V
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, r16 = lane & 15, q = lane >> 4;
    const int d = C / H;
    const bool has_image = L.image_bytes != 0;
    const int nsub = has_image ? I.cols_v / 16 : (T + 15) / 16;  // 16-token column tiles to produce (image: padded)
    if (tid < 96) sc_l[tid] = 0.f;
    if (tid == 0) scmax = 0u;
    const int ksteps = Cc / 64;  // used by WLDS only (there Cc % 64 == 0)
    if constexpr (WLDS) {
        // all eight wavefronts: piece f = j * ksteps + ks of the slice (rows 16*j .. 16*j+15, codes 64*ks .. 64*ks+63)
        for (int f = wave; f < TPH * ksteps; f += 8) {
            const int j = f / ksteps, ks = f - j * ksteps;
            int c = side * C + h * d + 16 * j + r16;  // rows past the head are computed and dropped; stay inside [0, 2C)
            c = c < 2 * C ? c : 2 * C - 1;
            __builtin_amdgcn_global_load_lds(
                (const __attribute__((address_space(1))) void*)(w_code + (size_t)c * Cc + 64 * ks + 16 * q),
                (__attribute__((address_space(3))) void*)(kvh_w + (size_t)f * 1024), 16, 0, 0);
        }
    }
    const float qmaxf = bits == 4 ? 7.f : 127.f;
    const int* slot_of = reinterpret_cast<const int*>(packed + L.slot_of) + b * T;
    uint8_t* codes = packed + (side ? L.v_code : L.k_code);
    float* scales = reinterpret_cast<float*>(packed + (side ? L.s_v : L.s_k)) + ((size_t)b * H + h) * T;
    uint8_t* img = packed + L.image + (size_t)b * L.image_bytes + (size_t)h * I.head_bytes;
    const int st = wave;  // one 16-token column tile per wavefront (at most 6)
    if constexpr (WLDS) {
        // the token codes of the first K steps travel with the weight slice; then everybody waits for the slice
        const int t = 16 * st + r16, tc = t < T ? t : T - 1;
        const int8_t* xrow = x_code + ((size_t)b * T + tc) * Cc + 16 * q;
        constexpr int XB = 16;  // K steps of token codes in flight per wavefront
        kvh_int32x4_t xb[XB];
        kvh_int32x4_t acc[TPH];
#pragma unroll
        for (int j = 0; j < TPH; ++j) acc[j] = (kvh_int32x4_t){0, 0, 0, 0};
        if (st < nsub) {
#pragma unroll
            for (int u = 0; u < XB; ++u) {
                xb[u] = (kvh_int32x4_t){0, 0, 0, 0};
                if (u < ksteps) xb[u] = *reinterpret_cast<const kvh_int32x4_t*>(xrow + 64 * u);
            }
        }
        __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): this wavefront's pieces of the slice are in LDS
        __syncthreads();                     // ... and so are everybody else's; sc_l and scmax are cleared
        if (st < nsub) {
            for (int k0 = 0; k0 < ksteps; k0 += XB) {
                if (k0 > 0) {
#pragma unroll
                    for (int u = 0; u < XB; ++u) {
                        xb[u] = (kvh_int32x4_t){0, 0, 0, 0};
                        if (k0 + u < ksteps) xb[u] = *reinterpret_cast<const kvh_int32x4_t*>(xrow + 64 * (k0 + u));
                    }
                }
#pragma unroll
                for (int u = 0; u < XB; ++u) {
                    if (k0 + u < ksteps) {
#pragma unroll
                        for (int j = 0; j < TPH; ++j) {
                            const kvh_int32x4_t wa =
                                *reinterpret_cast<const kvh_int32x4_t*>(kvh_w + (size_t)(j * ksteps + k0 + u) * 1024 + lane * 16);
                            acc[j] = __builtin_amdgcn_mfma_i32_16x16x64_i8(wa, xb[u], acc[j], 0, 0, 0);
                        }
                    }
                }
            }
            kvh_finish<TPH>(acc, st, h, b, side, d, r16, q, T, C, H, bits, qmaxf, s_x, s_w, slot_of, codes, scales, img, I, has_image,
                            sc_l, &scmax);
        }
    } else {
    __syncthreads();
    if (st < nsub) {
        const int8_t* wrow[TPH];
#pragma unroll
        for (int j = 0; j < TPH; ++j) {
            int c = side * C + h * d + 16 * j + r16;  // rows past the head are computed and dropped; stay inside [0, 2C)
            c = c < 2 * C ? c : 2 * C - 1;
            wrow[j] = w_code + (size_t)c * Cc + 16 * q;
        }
        const int t = 16 * st + r16, tc = t < T ? t : T - 1;
        const int8_t* xrow = x_code + ((size_t)b * T + tc) * Cc + 16 * q;
        kvh_int32x4_t acc[TPH];
#pragma unroll
        for (int j = 0; j < TPH; ++j) acc[j] = (kvh_int32x4_t){0, 0, 0, 0};
        // K steps of 64 codes, KB at a time: all their loads are issued before the first MFMA consumes one
        constexpr int KB = TPH <= 3 ? 12 : TPH <= 5 ? 6 : 2;  // (TPH + 1) * KB * 4 operand registers in flight
        for (int k0 = 0; k0 < Cc; k0 += 64 * KB) {
            kvh_int32x4_t xb[KB], wa[KB][TPH];
#pragma unroll
            for (int u = 0; u < KB; ++u) {
                const bool in = k0 + 64 * u + 16 * q < Cc;  // past the end of the row (its length need not divide)
                xb[u] = (kvh_int32x4_t){0, 0, 0, 0};
                if (in) xb[u] = *reinterpret_cast<const kvh_int32x4_t*>(xrow + k0 + 64 * u);
#pragma unroll
                for (int j = 0; j < TPH; ++j) {
                    wa[u][j] = (kvh_int32x4_t){0, 0, 0, 0};
                    if (in) wa[u][j] = *reinterpret_cast<const kvh_int32x4_t*>(wrow[j] + k0 + 64 * u);
                }
            }
#pragma unroll
            for (int u = 0; u < KB; ++u)
#pragma unroll
                for (int j = 0; j < TPH; ++j) acc[j] = __builtin_amdgcn_mfma_i32_16x16x64_i8(wa[u][j], xb[u], acc[j], 0, 0, 0);
        }
        kvh_finish<TPH>(acc, st, h, b, side, d, r16, q, T, C, H, bits, qmaxf, s_x, s_w, slot_of, codes, scales, img, I, has_image,
                        sc_l, &scmax);
    }
    }
    if (!has_image) return;
    __syncthreads();
    if (!side) {  // token scales of K and the 0 / -inf token bias
        if (tid < I.ntok) {
            reinterpret_cast<float*>(img + I.s_k)[tid] = sc_l[tid];
            reinterpret_cast<float*>(img + I.bias)[tid] = sc_l[tid] != 0.f ? 0.f : TAQ_NEG_INF;  // an unprotected token's scale is never 0
        }
        return;
    }
    // per-head power-of-two prescale of V: the largest |s_V * code| goes to [256, 512)
    int kexp = 0;
    {
        const float dmax = __uint_as_float(scmax) * qmaxf;
        if (dmax > 0.f) {
            int e;
            (void)frexpf(dmax, &e);
            kexp = 9 - e;
        }
    }
    const float vpre = ldexpf(1.0f, kexp);
    if (tid < I.ntok) {  // s' = s_V * 2^kexp as two fp16 numbers, high part and remainder
        const float sp = sc_l[tid] * vpre;
        const __half hi = __float2half_rn(sp);
        reinterpret_cast<__half*>(img + I.s_vp)[tid] = hi;
        reinterpret_cast<__half*>(img + I.s_vp)[I.ntok + tid] = __float2half_rn(sp - __half2float(hi));
    }
    if (tid == 0) {
        reinterpret_cast<float*>(img + I.vpre)[0] = vpre;
        reinterpret_cast<float*>(img + I.oscale)[0] = ldexpf(1.0f, -kexp);
    }
}

template <int TPH, bool WLDS>
static hipError_t launch_kv_head_cfg(const int8_t* x_code, const float* s_x, const int8_t* w_code, const float* s_w,
                                     uint8_t* packed, const __half* context, const taq_shape& s, size_t lds, hipStream_t st) {
    const KvLayout L = kv_layout(s);
    const KvImage I = kv_image(s);
    if (WLDS) {
        static std::atomic<unsigned long long> lds_set{0};
        const hipError_t e = ensure_dynamic_lds(reinterpret_cast<const void*>(&kv_head_kernel<TPH, WLDS>), 140 * 1024, lds_set);
        if (e != hipSuccess) return e;
    }
    const dim3 grid(2 * s.H * s.B + s.T * s.B * ((2 * s.C + 127) / 128)), block(512);
    hipLaunchKernelGGL((kv_head_kernel<TPH, WLDS>), grid, block, lds, st, x_code, s_x, w_code, s_w, packed, L, I, s.T, s.C, s.H,
                       s.Cc, s.bits_kv, s.B, context);
    return hipGetLastError();
}

hipError_t launch_kv_head(const int8_t* x_code, const float* s_x, const int8_t* w_code, const float* s_w, uint8_t* packed,
                          const __half* context, const taq_shape& s, hipStream_t st) {
    const int tph = (s.C / s.H + 15) / 16;
    // weight slice of a head in LDS (one KiB per 16 rows x 64 codes) when the row length allows whole K steps and the
    // slice fits beside the 17 KiB of static LDS
    const size_t slice = (size_t)tph * (s.Cc / 64) * 1024;
    const bool wlds = s.Cc % 64 == 0 && slice <= 140 * 1024;
#define TAQ_KVH(N)                                                                                                       \
    case N:                                                                                                              \
        return wlds ? launch_kv_head_cfg<N, true>(x_code, s_x, w_code, s_w, packed, context, s, slice, st)               \
                    : launch_kv_head_cfg<N, false>(x_code, s_x, w_code, s_w, packed, context, s, 0, st);
    switch (tph) {
        TAQ_KVH(1) TAQ_KVH(2) TAQ_KVH(3) TAQ_KVH(4) TAQ_KVH(5) TAQ_KVH(6) TAQ_KVH(7) TAQ_KVH(8) TAQ_KVH(9) TAQ_KVH(10)
        default: return hipErrorInvalidValue;
    }
#undef TAQ_KVH
}

// ---------------------------------------------------------------- expansion for tests
__global__ __launch_bounds__(256) void kv_unpack_kernel(const uint8_t* __restrict__ packed, KvLayout L, int T,
                                                        int C, int H, int bits, int8_t* k_codes,
                                                        int8_t* v_codes, float* k_scales, float* v_scales,
                                                        __half* k_trig, __half* v_trig) {
    const int bt = blockIdx.x, b = bt / T, t = bt % T;
    const int slot = reinterpret_cast<const int*>(packed + L.slot_of)[bt];
    const float* s_k = reinterpret_cast<const float*>(packed + L.s_k);
    const float* s_v = reinterpret_cast<const float*>(packed + L.s_v);
    for (int h = threadIdx.x; h < H; h += 256) {
        size_t i = ((size_t)b * H + h) * T + t;
        if (k_scales) k_scales[i] = s_k[i];
        if (v_scales) v_scales[i] = s_v[i];
    }
    for (int side = 0; side < 2; ++side) {
        const uint8_t* codes = packed + (side ? L.v_code : L.k_code);
        const __half* full = reinterpret_cast<const __half*>(packed + (side ? L.v16 : L.k16));
        int8_t* oc = side ? v_codes : k_codes;
        __half* ot = side ? v_trig : k_trig;
        for (int c = threadIdx.x; c < C; c += 256) {
            int code = 0;
            if (slot < 0 && bits == 8) code = (int8_t)codes[(size_t)bt * C + c];
            if (slot < 0 && bits == 4) {
                int nib = (codes[(size_t)bt * (C / 2) + c / 2] >> (4 * (c & 1))) & 0xF;
                code = (nib ^ 8) - 8;  // sign-extend the two's-complement nibble
            }
            if (oc) oc[(size_t)bt * C + c] = (int8_t)code;
            if (ot) ot[(size_t)bt * C + c] = slot >= 0 ? full[((size_t)b * T + slot) * C + c] : __float2half(0.f);
        }
    }
}

hipError_t launch_kv_unpack(const uint8_t* packed, const taq_shape& s, int8_t* k_codes, int8_t* v_codes,
                            float* k_scales, float* v_scales, __half* k_trig, __half* v_trig, hipStream_t st) {
    KvLayout L = kv_layout(s);
    hipLaunchKernelGGL(kv_unpack_kernel, dim3(s.B * s.T), dim3(256), 0, st, packed, L, s.T, s.C, s.H, s.bits_kv,
                       k_codes, v_codes, k_scales, v_scales, k_trig, v_trig);
    return hipGetLastError();
}

}  // namespace taq
