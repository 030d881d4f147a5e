// Full-precision stages of libtaq (gfx950): what runs when shape.bits_proj, bits_q or bits_prob is 16, i.e. when a
// projection, Q~ or the probabilities of PersonalQ's Eq. (2) / Eq. (3) are to stay unquantized. These modes exist for
// reference runs (Eq. (1): "all other parameters and activations in full precision"; the identity "every row protected,
// nothing quantized = plain softmax attention"), not for speed: plain float32 arithmetic, one simple kernel per stage.
#include "taq_internal.h"

namespace taq {

// ---------------------------------------------------------------- out[m][n] = sum_k A[m][k] * W[n][k]  (+ bias[n])
// A: f16 or f32 [M][K]; W: f16 [N][K] (out x in, as the projections are stored); float32 accumulation in K order.
// 64 x 64 outputs per workgroup of 256 threads (4 x 4 each), K in chunks of 16 through LDS.
template <typename AT>
__global__ __launch_bounds__(256) void gemm_nt_fp_kernel(const AT* __restrict__ A, const __half* __restrict__ W,
                                                         const float* __restrict__ bias, int M, int N, int K,
                                                         float* __restrict__ out_f32, __half* __restrict__ out_f16, int ldo) {
    __shared__ float As[16][65], Ws[16][65];
    const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
    const int m0 = blockIdx.x * 64, n0 = blockIdx.y * 64;
    float acc[4][4] = {};
    for (int k0 = 0; k0 < K; k0 += 16) {
        for (int i = threadIdx.x; i < 64 * 16; i += 256) {
            const int r = i >> 4, k = i & 15;
            const int m = m0 + r, n = n0 + r;
            As[k][r] = (m < M && k0 + k < K) ? (float)A[(size_t)m * K + k0 + k] : 0.f;
            Ws[k][r] = (n < N && k0 + k < K) ? __half2float(W[(size_t)n * K + k0 + k]) : 0.f;
        }
        __syncthreads();
#pragma unroll
        for (int k = 0; k < 16; ++k) {
            float a[4], w[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                a[i] = As[k][ty * 4 + i];
                w[i] = Ws[k][tx * 4 + i];
            }
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = __builtin_fmaf(a[i], w[j], acc[i][j]);
        }
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int m = m0 + ty * 4 + i;
        if (m >= M) continue;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int n = n0 + tx * 4 + j;
            if (n >= N) continue;
            const float y = acc[i][j] + (bias ? bias[n] : 0.f);
            if (out_f32) out_f32[(size_t)m * ldo + n] = y;
            if (out_f16) out_f16[(size_t)m * ldo + n] = __float2half_rn(y);
        }
    }
}

hipError_t launch_gemm_fp(const void* A, bool a_is_f32, const __half* W, const float* bias, int M, int N, int K,
                          float* out_f32, __half* out_f16, int ldo, hipStream_t st) {
    const dim3 grid((M + 63) / 64, (N + 63) / 64), block(256);
    if (a_is_f32)
        hipLaunchKernelGGL(gemm_nt_fp_kernel<float>, grid, block, 0, st, static_cast<const float*>(A), W, bias, M, N, K, out_f32, out_f16, ldo);
    else
        hipLaunchKernelGGL(gemm_nt_fp_kernel<__half>, grid, block, 0, st, static_cast<const __half*>(A), W, bias, M, N, K, out_f32, out_f16, ldo);
    return hipGetLastError();
}

// ---------------------------------------------------------------- protected rows from float32 projection rows
// rows_f [B*T][2C] (K channels then V channels of every text token) -> K16, V16 (compacted by slot) and the transposed
// V16T [B][C][96], one rounding to fp16; unused slots and the padding of V16T read as zeros. One workgroup per
// (slot, batch element).
__global__ __launch_bounds__(256) void kv_rows_from_f32_kernel(const float* __restrict__ rows_f, const int* __restrict__ ntrig,
                                                               const int* __restrict__ trig_idx, int T, int C,
                                                               __half* __restrict__ k16, __half* __restrict__ v16,
                                                               __half* __restrict__ v16t) {
    const int slot = blockIdx.x, b = blockIdx.y;
    const bool live = slot < ntrig[b];
    const int t = live ? trig_idx[b * T + slot] : 0;
    for (int c = threadIdx.x; c < 2 * C; c += 256) {
        const __half y = live ? __float2half_rn(rows_f[((size_t)b * T + t) * 2 * C + c]) : __float2half(0.f);
        if (c < C) {
            k16[((size_t)b * T + slot) * C + c] = y;
        } else {
            v16[((size_t)b * T + slot) * C + (c - C)] = y;
            v16t[((size_t)b * C + (c - C)) * 96 + slot] = y;
            if (slot == T - 1)
                for (int sp = T; sp < 96; ++sp) v16t[((size_t)b * C + (c - C)) * 96 + sp] = __float2half(0.f);
        }
    }
}

hipError_t launch_kv_rows_from_f32(const float* rows_f, const int* ntrig, const int* trig_idx, int B, int T, int C,
                                   __half* k16, __half* v16, __half* v16t, hipStream_t st) {
    hipLaunchKernelGGL(kv_rows_from_f32_kernel, dim3(T, B), dim3(256), 0, st, rows_f, ntrig, trig_idx, T, C, k16, v16, v16t);
    return hipGetLastError();
}

// ---------------------------------------------------------------- attention with unquantized Q and / or probabilities
// A = softmax(Q~ K~^T * sigma), Eq. (3), O = A^ V~ in float32, for any mix of bits_q in {4, 8, 16} and bits_prob in
// {4, 8, 16} and the three probability grids. K~ and V~ (Eq. 2) are expanded to float32 in LDS: s * code for unprotected
// rows, the fp16 row for protected ones. One workgroup per (16 image tokens, head, batch element); a wavefront takes four
// tokens in turn, lanes over text tokens for the scores and the softmax, lanes over channels for A^ V~.
struct FpAttnArgs {
    const float* q_f;       // [B*N][C]  unquantized Q (bits_q = 16)
    const int8_t* q_code;   // [B*N][C]  Q~ codes and scales otherwise
    const float* s_q;       // [B*N][H]
    const uint8_t* packed;
    KvLayout L;
    float* o_f;             // [B*N][C]
    uint8_t* p_code;        // [B*N][H][T] tap or NULL
    int N, C, H, T, bits_kv, bits_q, bits_prob, grid;
    float sigma;
};

__device__ __forceinline__ float fp_wave_max(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
    return v;
}
__device__ __forceinline__ float fp_wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
    return v;
}

__global__ __launch_bounds__(256) void attn_fp_kernel(FpAttnArgs a) {
    extern __shared__ __align__(16) unsigned char smem[];
    const int b = blockIdx.z, h = blockIdx.y, n0 = blockIdx.x * 16;
    const int N = a.N, C = a.C, H = a.H, T = a.T, d = C / H;
    float* Kd = reinterpret_cast<float*>(smem);   // [T][d]
    float* Vd = Kd + (size_t)T * d;               // [T][d]
    float* qs = Vd + (size_t)T * d;               // [4 wavefronts][d]
    float* ah = qs + 4 * d;                       // [4 wavefronts][96]
    int* prot = reinterpret_cast<int*>(ah + 4 * 96);  // [96]
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const uint8_t* pk = a.packed;
    const int* slot_of = reinterpret_cast<const int*>(pk + a.L.slot_of) + b * T;
    const float* s_k = reinterpret_cast<const float*>(pk + a.L.s_k) + ((size_t)b * H + h) * T;
    const float* s_v = reinterpret_cast<const float*>(pk + a.L.s_v) + ((size_t)b * H + h) * T;
    const __half* k16 = reinterpret_cast<const __half*>(pk + a.L.k16);
    const __half* v16 = reinterpret_cast<const __half*>(pk + a.L.v16);
    auto code_at = [&](const uint8_t* codes, int t, int c) -> float {
        if (a.bits_kv == 8) return (float)(int8_t)codes[((size_t)b * T + t) * C + c];
        const int nib = (codes[((size_t)b * T + t) * (C >> 1) + (c >> 1)] >> (4 * (c & 1))) & 0xF;
        return (float)((nib ^ 8) - 8);
    };
    for (int i = tid; i < T * d; i += 256) {
        const int t = i / d, j = i % d, slot = slot_of[t];
        if (slot >= 0) {
            Kd[i] = __half2float(k16[((size_t)b * T + slot) * C + h * d + j]);
            Vd[i] = __half2float(v16[((size_t)b * T + slot) * C + h * d + j]);
        } else {
            Kd[i] = code_at(pk + a.L.k_code, t, h * d + j) * s_k[t];
            Vd[i] = code_at(pk + a.L.v_code, t, h * d + j) * s_v[t];
        }
    }
    for (int t = tid; t < 96; t += 256) prot[t] = (t < T && slot_of[t] >= 0) ? 1 : 0;
    __syncthreads();
    const float pmax = a.bits_prob == 4 ? 15.f : 255.f;
    for (int it = 0; it < 4; ++it) {
        const int n = n0 + wave * 4 + it;
        const bool nvalid = n < N;
        const size_t tok = (size_t)b * N + (nvalid ? n : N - 1);
        for (int j = lane; j < d; j += 64)
            qs[wave * d + j] = a.bits_q == 16 ? a.q_f[tok * C + h * d + j]
                                              : (float)a.q_code[tok * C + h * d + j] * a.s_q[tok * H + h];
        __syncthreads();
        float sc[2], A[2];
        float mx = -__builtin_inff();
#pragma unroll
        for (int r = 0; r < 2; ++r) {
            const int t = lane + 64 * r;
            sc[r] = -__builtin_inff();
            if (t < T) {
                float s = 0.f;
                for (int j = 0; j < d; ++j) s = __builtin_fmaf(qs[wave * d + j], Kd[t * d + j], s);
                sc[r] = s * a.sigma;
            }
            mx = fmaxf(mx, sc[r]);
        }
        mx = fp_wave_max(mx);
        float Z = 0.f;
#pragma unroll
        for (int r = 0; r < 2; ++r) {
            A[r] = (lane + 64 * r < T) ? __expf(sc[r] - mx) : 0.f;
            Z += A[r];
        }
        Z = fp_wave_sum(Z);
        float amax = 0.f;  // row-range grid: largest unprotected probability
#pragma unroll
        for (int r = 0; r < 2; ++r) {
            const int t = lane + 64 * r;
            A[r] = A[r] / Z;
            if (t < T && !prot[t]) amax = fmaxf(amax, A[r]);
        }
        amax = fp_wave_max(amax);
#pragma unroll
        for (int r = 0; r < 2; ++r) {
            const int t = lane + 64 * r;
            if (t >= T) continue;
            float ahat = A[r], code = 0.f;
            if (a.bits_prob != 16 && !prot[t]) {  // Eq. (3): Q_a on unprotected columns
                if (a.grid == TAQ_PROB_LOG2) {
                    code = A[r] > 0.f ? fminf(fmaxf(__builtin_rintf(-__log2f(A[r])), 0.f), pmax) : pmax;
                    ahat = exp2f(-code);
                } else if (a.grid == TAQ_PROB_ROWMAX) {
                    const float safe = amax == 0.f ? 1.f : amax;
                    const float scale = amax == 0.f ? 1.f : amax / pmax;
                    code = fminf(fmaxf(__builtin_rintf((A[r] * pmax) / safe), 0.f), pmax);
                    ahat = code * scale;
                } else {
                    code = __builtin_rintf(A[r] * pmax);
                    ahat = code / pmax;
                }
            }
            ah[wave * 96 + t] = ahat;
            if (a.p_code && nvalid) a.p_code[(tok * H + h) * (size_t)T + t] = (uint8_t)(int)code;
        }
        __syncthreads();
        for (int j = lane; j < d; j += 64) {
            float o = 0.f;
            for (int t = 0; t < T; ++t) o = __builtin_fmaf(ah[wave * 96 + t], Vd[t * d + j], o);
            if (nvalid) a.o_f[tok * C + h * d + j] = o;
        }
        __syncthreads();
    }
}

hipError_t launch_attn_fp(const float* q_f, const int8_t* q_code, const float* s_q, const uint8_t* packed, const taq_shape& s,
                          float* o_f, uint8_t* p_code, hipStream_t st) {
    FpAttnArgs a;
    a.q_f = q_f;
    a.q_code = q_code;
    a.s_q = s_q;
    a.packed = packed;
    a.L = kv_layout(s);
    a.o_f = o_f;
    a.p_code = p_code;
    a.N = s.N;
    a.C = s.C;
    a.H = s.H;
    a.T = s.T;
    a.bits_kv = s.bits_kv;
    a.bits_q = s.bits_q;
    a.bits_prob = s.bits_prob;
    a.grid = s.prob_grid;
    const int d = s.C / s.H;
    a.sigma = s.softmax_scale != 0.f ? s.softmax_scale : 1.0f / sqrtf((float)d);
    const size_t bytes = ((size_t)2 * s.T * d + 4 * d + 4 * 96) * 4 + 96 * 4;
    static std::atomic<unsigned long long> lds_set{0};
    const hipError_t e = ensure_dynamic_lds(reinterpret_cast<const void*>(&attn_fp_kernel), 160 * 1024, lds_set);
    if (e != hipSuccess) return e;
    if (bytes > 160 * 1024) return hipErrorInvalidValue;
    hipLaunchKernelGGL(attn_fp_kernel, dim3((s.N + 15) / 16, s.H, s.B), dim3(256), bytes, st, a);
    return hipGetLastError();
}

// ---------------------------------------------------------------- mean squared difference of two fp16 arrays
// The loss of the token-sensitivity experiment (Section III-B, Eq. 1) on block outputs. One workgroup; float64 sum.
__global__ __launch_bounds__(1024) void mse_f16_kernel(const __half* __restrict__ x, const __half* __restrict__ y, size_t n,
                                                       double* __restrict__ out) {
    __shared__ double part[1024];
    double s = 0.0;
    for (size_t i = threadIdx.x; i < n; i += 1024) {
        const double dlt = (double)__half2float(x[i]) - (double)__half2float(y[i]);
        s += dlt * dlt;
    }
    part[threadIdx.x] = s;
    __syncthreads();
    for (int w = 512; w > 0; w >>= 1) {
        if ((int)threadIdx.x < w) part[threadIdx.x] += part[threadIdx.x + w];
        __syncthreads();
    }
    if (threadIdx.x == 0) out[0] = part[0] / (double)n;
}

hipError_t launch_mse_f16(const __half* x, const __half* y, size_t n, double* out, hipStream_t st) {
    hipLaunchKernelGGL(mse_f16_kernel, dim3(1), dim3(1024), 0, st, x, y, n, out);
    return hipGetLastError();
}

}  // namespace taq
