// int8 x int8 -> int32 GEMM on the gfx950 matrix cores with fused dequantisation.
//
// Serves the W8A8 contractions of the TAQ block (to_q, to_out, and the K/V projections of
// unprotected text tokens): acc[m][n] = sum_k A[m][k] * W[n][k], both operands K-contiguous,
// result = float(acc) * (sa[m] * sw[n]) (+ bias[n]), in that order of float32 operations.
#include "taq_internal.h"

namespace taq {

typedef int int32x4_t __attribute__((ext_vector_type(4)));
typedef int int32x16_t __attribute__((ext_vector_type(16)));

// Workgroup = 4 wavefronts in a 2x2 arrangement, each owning one 32x32 accumulator tile
// (V_MFMA_I32_32X32X32_I8: a lane supplies 16 consecutive k of row/column lane%32, the
// upper half-wave the next 16). Operands are read straight from global memory: a lane's
// 16 bytes are contiguous and both operands stay resident in L2 at these sizes.
// K % 32 == 0. Rows beyond M / N are clamped on load and masked on store.
__global__ __launch_bounds__(256) void gemm_i8_kernel(const int8_t* __restrict__ A, const float* __restrict__ sa,
                                                      const int8_t* __restrict__ W, const float* __restrict__ sw,
                                                      const float* __restrict__ bias, int M, int N, int K,
                                                      float* __restrict__ out_f32, __half* __restrict__ out_f16,
                                                      int ldo) {
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int r = lane & 31, half = lane >> 5;
    const int m0 = blockIdx.y * 64 + (wave & 1) * 32;
    const int n0 = blockIdx.x * 64 + (wave >> 1) * 32;
    if (m0 >= M || n0 >= N) return;
    const int am = min(m0 + r, M - 1);
    const int wn = min(n0 + r, N - 1);
    const int8_t* ap = A + (size_t)am * K + 16 * half;
    const int8_t* wp = W + (size_t)wn * K + 16 * half;
    int32x16_t acc;
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[i] = 0;
#pragma unroll 4
    for (int k = 0; k < K; k += 32) {
        int32x4_t a = *reinterpret_cast<const int32x4_t*>(ap + k);
        int32x4_t b = *reinterpret_cast<const int32x4_t*>(wp + k);
        acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, acc, 0, 0, 0);
    }
    const int col = n0 + r;
    if (col >= N) return;
    const float swc = sw[col];
    const float bc = bias ? bias[col] : 0.f;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const int row = m0 + 8 * (i >> 2) + 4 * half + (i & 3);
        if (row < M) {
            const float sc = sa[row] * swc;
            const float v = (float)acc[i] * sc;
            if (out_f32) out_f32[(size_t)row * ldo + col] = v;
            if (out_f16) out_f16[(size_t)row * ldo + col] = __float2half_rn(v + bc);
        }
    }
}

hipError_t launch_gemm_i8(const int8_t* A, const float* sa, const int8_t* W, const float* sw, const float* bias,
                          int M, int N, int K, float* out_f32, __half* out_f16, int ldo, hipStream_t st) {
    if (M <= 0 || N <= 0) return hipSuccess;
    dim3 grid((N + 63) / 64, (M + 63) / 64);
    hipLaunchKernelGGL(gemm_i8_kernel, grid, dim3(256), 0, st, A, sa, W, sw, bias, M, N, K, out_f32, out_f16, ldo);
    return hipGetLastError();
}

}  // namespace taq
