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
    const int m0 = blockIdx.x * 64 + (wave & 1) * 32;
    const int n0 = blockIdx.y * 64 + (wave >> 1) * 32;
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

// ------------------------------------------------------------------------------------------
// LDS-staged kernel for K % 64 == 0 (every configured channel count): a workgroup of four wavefronts owns 128 rows of A
// (image tokens) x 80 rows of W (output channels: 320, 640 and 1280 are multiples of 80, and 2048 x 1280 outputs are then
// exactly 256 workgroups, one per compute unit). Per K step of 64 the 13 operand blocks (16 rows x 64 codes = 1 KiB
// each) go through LDS, row-major with the 16-byte segments of a row swizzled (below). Software pipeline, one barrier
// per K step, three LDS stages, four register sets for loads in flight: while the ten MFMAs of step k run on one operand
// register set, step k + 1 is read from LDS into the other, steps k + 2 and k + 3 move from registers to LDS and the
// global loads of up to four later steps are outstanding.
// (Direct global->LDS loads are not used here: the compiler waits for every outstanding one before any LDS read, which
// would serialise the stages.)
// The product is formed transposed (W rows as the A operand, tokens as the B operand), so that a lane ends up with four
// consecutive output channels of one token: 16-byte float32 / 8-byte fp16 stores.
// ------------------------------------------------------------------------------------------
template <int MB, int NB, int RD>
__global__ __launch_bounds__(256) void gemm_i8_lds_kernel(const int8_t* __restrict__ A, const float* __restrict__ sa,
                                                          const int8_t* __restrict__ W, const float* __restrict__ sw,
                                                          const float* __restrict__ bias, int M, int N, int K,
                                                          float* __restrict__ out_f32, __half* __restrict__ out_f16, int ldo) {
    constexpr int BLK = MB + NB, STAGES = 3, MW = MB / 4;  // blocks per stage; token tiles per wavefront
    constexpr int NLD = (BLK + 3) / 4;                     // loads per wavefront and stage (the last may be idle)
    static_assert(MB % 4 == 0, "four wavefronts share the token tiles");
    __shared__ __align__(16) unsigned char lds[STAGES * BLK * 1024];
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63, r16 = lane & 15, q = lane >> 4;
    const int m0 = blockIdx.x * (16 * MB), n0 = blockIdx.y * (16 * NB);
    const int KC = K >> 6;
    // global loads: four consecutive lanes fetch the 64 contiguous bytes of one row; MFMA operands: lane (r16, q) holds
    // codes 16q .. 16q+15 of row r16. Segment g of row r sits at r * 64 + (g ^ f(r)) * 16 inside its block, with
    // f(r) = (r >> 1 ^ r >> 2) & 3: the wave-wide 16-byte stores stay contiguous, and the 16-byte operand reads of any
    // eight consecutive lanes fall into eight different 16-byte columns of a 128-byte bank row (of any sixteen lanes:
    // sixteen columns of a 256-byte row).
    const int lrow = lane >> 2, lseg = lane & 3;
    const int st_off = lrow * 64 + ((lseg ^ ((lrow >> 1 ^ lrow >> 2) & 3)) << 4);
    const int ld_off = r16 * 64 + ((q ^ ((r16 >> 1 ^ r16 >> 2) & 3)) << 4);
    // this wavefront's loads of a stage: blocks wave, wave + 4, ... (token blocks first, then weight blocks)
    const int8_t* src[NLD];
#pragma unroll
    for (int u = 0; u < NLD; ++u) {
        const int blk = wave + 4 * u < BLK ? wave + 4 * u : BLK - 1;  // (an idle slot re-reads the last block and drops it)
        const int8_t* base = A;
        int row = 0;
        if (blk < MB) {
            row = m0 + 16 * blk + lrow;
            row = row < M ? row : M - 1;
        } else {
            base = W;
            row = n0 + 16 * (blk - MB) + lrow;
            row = row < N ? row : N - 1;
        }
        src[u] = base + (size_t)row * K + 16 * lseg;
    }
    int32x4_t g[RD][NLD];  // stages on their way from global memory to LDS
    // (No step of the pipeline is conditional: a load past the last stage re-reads the last stage, and what the steps
    // past the end store to and read from LDS is never multiplied. With loads under a condition the compiler's wait
    // counts assume the fewest outstanding loads, which makes every wait a wait for the newest load.)
    auto load_stage = [&](int kc, int slot) {
        const int off = 64 * (kc < KC ? kc : KC - 1);
#pragma unroll
        for (int u = 0; u < NLD; ++u) g[slot][u] = *reinterpret_cast<const int32x4_t*>(src[u] + off);
    };
    auto store_stage = [&](int kc, int slot) {
        unsigned char* dst = lds + (kc % STAGES) * (BLK * 1024) + st_off;
#pragma unroll
        for (int u = 0; u < NLD; ++u)
            if (4 * u + 3 < BLK || wave + 4 * u < BLK) *reinterpret_cast<int32x4_t*>(dst + (wave + 4 * u) * 1024) = g[slot][u];
    };
    int32x4_t acc[NB][MW];
#pragma unroll
    for (int j = 0; j < NB; ++j)
#pragma unroll
        for (int i = 0; i < MW; ++i) acc[j][i] = (int32x4_t){0, 0, 0, 0};
    int32x4_t wa[2][NB], xb[2][MW];
    auto read_ops = [&](int kc, int set) {
        const unsigned char* st = lds + (kc % STAGES) * (BLK * 1024) + ld_off;
#pragma unroll
        for (int i = 0; i < MW; ++i) xb[set][i] = *reinterpret_cast<const int32x4_t*>(st + (MW * wave + i) * 1024);
#pragma unroll
        for (int j = 0; j < NB; ++j) wa[set][j] = *reinterpret_cast<const int32x4_t*>(st + (MB + j) * 1024);
    };
    // prologue: stages 0 and 1 in LDS, stages 2 .. 5 in flight, operands of step 0 in registers
    static_assert(RD == 4, "four register sets: the main loop is unrolled four times");
    load_stage(0, 0);
    load_stage(1, 1);
    store_stage(0, 0);
    store_stage(1, 1);
    load_stage(2, 2);
    load_stage(3, 3);
    load_stage(4, 0);
    load_stage(5, 1);
    __syncthreads();
    read_ops(0, 0);
    auto mfmas = [&](int set) {
#pragma unroll
        for (int j = 0; j < NB; ++j)
#pragma unroll
            for (int i = 0; i < MW; ++i) acc[j][i] = __builtin_amdgcn_mfma_i32_16x16x64_i8(wa[set][j], xb[set][i], acc[j][i], 0, 0, 0);
    };
    // Steps come in pairs. The even step kc moves stages kc + 2 and kc + 3 from registers to LDS and issues the loads of
    // stages kc + 6 and kc + 7 back to back: the two are the halves of the same 128-byte lines, so the second is served
    // by the line the first brought in. At the barrier of step kc every wavefront is through with reading stage kc
    // (buffer kc % 3, which stage kc + 3 overwrites) and stage kc - 1 (which stage kc + 2 overwrites).
    auto even_step = [&](int kc, int slot) {  // slot = (kc + 2) % 4
        __syncthreads();
        read_ops(kc + 1, 1);
        store_stage(kc + 2, slot);
        store_stage(kc + 3, slot + 1);
        load_stage(kc + 6, slot);
        load_stage(kc + 7, slot + 1);
        mfmas(0);
    };
    auto odd_step = [&](int kc) {
        __syncthreads();
        read_ops(kc + 1, 0);
        mfmas(1);
    };
    int kc = 0;
    for (; kc + 4 <= KC; kc += 4) {
        even_step(kc, 2);
        odd_step(kc + 1);
        even_step(kc + 2, 0);
        odd_step(kc + 3);
    }
    if (kc < KC) even_step(kc, 2);
    if (kc + 1 < KC) odd_step(kc + 1);
    if (kc + 2 < KC) even_step(kc + 2, 0);
    // epilogue: result = float(acc) * (sa[m] * sw[n]) (+ bias[n]). The MFMA leaves lane (r16, q) with channels
    // 16j + 4q .. + 3 of token r16 of its tile; a lane exchange hands lane l the four channels 16j + 4 (l & 3) .. of
    // token l >> 2, so that four consecutive lanes store 64 (fp16: 32) contiguous bytes.
    const int from = ((lane >> 2) + 16 * (lane & 3)) << 2;
#pragma unroll
    for (int i = 0; i < MW; ++i) {
        const int m = m0 + 16 * (MW * wave + i) + lrow;
        const float sam = sa[m < M ? m : M - 1];
#pragma unroll
        for (int j = 0; j < NB; ++j) {
            int c[4];
#pragma unroll
            for (int e2 = 0; e2 < 4; ++e2) c[e2] = __builtin_amdgcn_ds_bpermute(from, acc[j][i][e2]);
            const int n = n0 + 16 * j + 4 * lseg;
            if (m >= M || n >= N) continue;  // (N % 4 == 0: a lane's four channels are inside or outside together)
            const float4 w4 = *reinterpret_cast<const float4*>(sw + n);
            const float v0 = (float)c[0] * (sam * w4.x), v1 = (float)c[1] * (sam * w4.y);
            const float v2 = (float)c[2] * (sam * w4.z), v3 = (float)c[3] * (sam * w4.w);
            if (out_f32) *reinterpret_cast<float4*>(out_f32 + (size_t)m * ldo + n) = make_float4(v0, v1, v2, v3);
            if (out_f16) {
                float4 b4 = make_float4(0.f, 0.f, 0.f, 0.f);
                if (bias) b4 = *reinterpret_cast<const float4*>(bias + n);
                __half2 h01 = __floats2half2_rn(v0 + b4.x, v1 + b4.y), h23 = __floats2half2_rn(v2 + b4.z, v3 + b4.w);
                uint2 o;
                o.x = *reinterpret_cast<unsigned*>(&h01);
                o.y = *reinterpret_cast<unsigned*>(&h23);
                *reinterpret_cast<uint2*>(out_f16 + (size_t)m * ldo + n) = o;
            }
        }
    }
}

hipError_t launch_gemm_i8(const int8_t* A, const float* sa, const int8_t* W, const float* sw, const float* bias,
                          int M, int N, int K, float* out_f32, __half* out_f16, int ldo, hipStream_t st) {
    if (M <= 0 || N <= 0) return hipSuccess;
    if (K % 64 == 0 && N % 4 == 0 && ldo % 4 == 0) {
        // While 128-token tiles would give every compute unit at most one workgroup, 64-token tiles (two workgroups per
        // unit, each hiding the other's waits) are faster: 7.8 -> 7.0 us at (8192, 320), 11.7 -> 11.2 us at (2048, 1280);
        // with more tiles than that the larger tile's fewer weight reads win (12.1 vs 12.9 us at (8192, 640)).
        const long tiles128 = (long)((M + 127) / 128) * ((N + 79) / 80);
        if (tiles128 <= 256) {
            dim3 grid((M + 63) / 64, (N + 79) / 80);
            hipLaunchKernelGGL((gemm_i8_lds_kernel<4, 5, 4>), grid, dim3(256), 0, st, A, sa, W, sw, bias, M, N, K, out_f32, out_f16, ldo);
        } else {
            dim3 grid((M + 127) / 128, (N + 79) / 80);
            hipLaunchKernelGGL((gemm_i8_lds_kernel<8, 5, 4>), grid, dim3(256), 0, st, A, sa, W, sw, bias, M, N, K, out_f32, out_f16, ldo);
        }
        return hipGetLastError();
    }
    dim3 grid((M + 63) / 64, (N + 63) / 64);  // (M, which may be large, along x)
    hipLaunchKernelGGL(gemm_i8_kernel, grid, dim3(256), 0, st, A, sa, W, sw, bias, M, N, K, out_f32, out_f16, ldo);
    return hipGetLastError();
}

}  // namespace taq
