// The fused TAQ cross-attention block kernel (PersonalQ, Section III-B) for gfx950: template, configuration
// constants and per-instantiation launchers. Included by one translation unit per (head dimension, heads) family
// (taq_fused_d40.hip, ...), so that the families compile in parallel; taq_fused.hip holds the dispatch.
//
//   hidden --per-token int8--> to_q (int8 MFMA) --Q_a per (token, head): Eq. 2, line 3-->
//   S^T = K~ Q~^T (int8 MFMA, fp16 MFMA for protected rows) --> softmax --> Eq. 3 -->
//   O^T = V~^T A^^T (fp16 MFMA, split operands) --per-token int8--> to_out (int8 MFMA) --> fp16
//
// Nothing between `hidden` and `out` touches HBM: per image token the kernel reads 2C bytes and
// writes 2C bytes; weights and K~/V~ come from L2.
//
// Work split. A workgroup owns 32 image tokens and all heads, one wavefront per head; each wavefront
// carries two column tiles of 16 tokens. Every contraction is computed transposed (output channel or
// text token along the MFMA row axis, image token along the column axis) with 16x16 tiles, so an image
// token stays in lane (token % 16) of its wavefront, in all four quarter-waves, from the first GEMM to
// the last: per-token reductions are register maxima plus two cross-lane swaps, and every intermediate
// (Q~ codes, probabilities, O codes) is handed to the next MFMA as its B operand straight from registers.
// The A operands' contraction order is free, so K~ and V~^T are stored in LDS in the order in which the
// accumulator registers of the previous MFMA come out.
//
// Bit-exact steps (same float32 operation order as the definition): per-token codes of hidden,
// the int32 accumulators, Qf = float(acc) * (s_h * s_wq), Q~ codes and scales.
#pragma once
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

// Buffer descriptor of a weight matrix: base address, no stride (raw byte offsets), `bytes` addressable, 32-bit data
// format; out-of-range reads return zero.
__device__ __forceinline__ __amdgpu_buffer_rsrc_t weight_rsrc(const int8_t* p, unsigned bytes) {
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<int8_t*>(p), 0, (int)bytes, 0x00020000);
}

__device__ __forceinline__ float byte_to_float(unsigned w, int e) { return (float)(int)(int8_t)((w >> (8 * e)) & 0xFF); }

// ------------------------------------------------------------------------------------------
// Fused block kernel
// ------------------------------------------------------------------------------------------
struct FusedTable {
    FusedReq req[TAQ_MAX_REQ];
};

struct FusedDims {
    int R, B, N, T;
    int nt16;          // ceil(T/16)
    int w_layout;      // 1: Wq / Wo carry an operand-ordered copy at w_pack_off
    unsigned w_pack_off;
    unsigned w_bytes;  // bytes of each weight buffer (row-major codes, plus the operand-ordered copy if present)
    float sig2;        // softmax scale * log2(e)
    float qmaxq;       // 127 or 7: grid of Q~ (Eq. 2, third line)
    float pmax;        // linear grid: 255 or 15 (Eq. 3); log2 grid: 256, which brings 2^-code * s_V to the linear grid's magnitudes
    float plast;       // log2 grid: the last code, 255 or 15
    KvLayout L;
    KvImage I;
    taq_debug dbg;     // taps (NULL pointers = off); only used when R == 1
    // head-group variant (NG > 1): A^ V~ and the partial row maxima pass through the workspace
    float* ws_of;            // f32 [B*N][C]
    float* ws_omax;          // f32 [B*N][omax_n]  max |A^ V~| over each wavefront's share of a token's row
    int omax_n;              // partial maxima per token (heads x wavefronts per head and token group)
    const int8_t* core_qcode;  // i8  [B*N][C]  Q~ codes (attention-core-only variant)
    const float* core_sq;      // f32 [B*N][H]  ... and their scales
    const int8_t* ws_ocode;  // i8  [B*N][C]  per-token codes of A^ V~ when a separate kernel formed them (else NULL)
    const float* ws_so;      // f32 [B*N]     ... and their scales
};

template <int D, int NH, int NTT, int NG, int TOK = 32, bool DENSE = false>
struct FusedCfg {
    static constexpr int G = TOK / (16 * NTT);    // wavefronts per head (token groups of 16*NTT tokens)
    static constexpr int H = NH * NG;             // heads of the layer; a workgroup owns NH of them
    static constexpr int C = D * H;
    static constexpr int TPH = (D + 15) / 16;     // 16-row tiles per head
    static constexpr int KS = (TPH + 3) / 4;      // K steps of 64 for S^T = K~ Q~^T
    static constexpr int FS = (TPH + 1) / 2;      // K steps of 32 for the protected-row scores
    static constexpr int KC = C / 64;             // K steps of 64 for the projections
    // Head-group variant (NG > 1): SUB wavefronts share one (head, token group); each owns every SUB-th channel tile
    // of A^ V~, and all eight wavefronts of the workgroup split to_q by weight tile and K range.
    static constexpr int SUB = NG > 1 ? 4 / NH : 1;
    static constexpr int TPS = (TPH + SUB - 1) / SUB;  // channel tiles of A^ V~ per wavefront
    static constexpr int ROLES = NH * G * SUB;    // wavefronts with a (head, token group, channel share) of the attention
    static constexpr int NT = NG > 1 ? 512 : 64 * ROLES;  // threads (head-group variant: always eight wavefronts for the
                                                          // hidden codes and to_q; those without a role stop after to_q)
    static constexpr int TILE_RS = C + 16;        // bytes per token row of the int8 tile
    // bytes of one head's image block at T = 96, in 1 KiB pieces (one direct-to-LDS load each)
    static constexpr int IMG_HEAD_MAX = 96 * TPH * 16 + D * 96 + 3 * 96 * 4 + 32;
    static constexpr int IMGC = (IMG_HEAD_MAX + 1023) / 1024;
    // DENSE: the instantiation meant to run two workgroups per compute unit (layers with more token tiles than compute
    // units): at most 128 registers per lane, so the weights pass through a short ring instead of sitting in registers.
    static constexpr bool PREFETCH_W = TPH * KC <= 16 && NTT == 2 && NG == 1 && !DENSE;  // a head's whole weight slice in registers
    // Otherwise a ring of RING weight loads stays in flight ahead of the projection MFMAs (K step outermost, so that
    // only one step's B operands are live); left to itself the compiler keeps one to ten loads ahead and the loop
    // waits on latency.
    static constexpr int NF = TPH * KC;  // weight loads (16 rows x 64 bytes) of one projection per wavefront
    // two wavefronts per SIMD (256 registers each), or three at ten heads (168)
    static constexpr int RING_MAX = DENSE ? 6 : NH <= 8 ? (NTT == 1 ? 32 : 24) : (NTT == 1 ? 12 : 8);
    static constexpr int RING = (!PREFETCH_W && NG == 1) ? (NF < RING_MAX ? NF : RING_MAX) : 0;
};

// Symmetric 8-bit codes of four values of one row, packed into a dword (low byte first).
//   exact definition: code = rint((x * qmax) / amax) with IEEE float32 multiply and divide (qmax = 127, or 7 for
//   4-bit Q~; the bounds below are stated for 127 and only shrink for 7).
//   fast path: with c = qmax * rcp(amax) (rcp within 1 ulp, the product rounded once: c is within 1.5 * 2^-23 of
//   qmax / amax, relatively), m = fma(x, c, 1.5 * 2^23) is the EXACT product x * c rounded half-to-even to an integer
//   (plus the magic constant, whose low mantissa byte is then the code's byte), and e = fma(x, c, -(m - magic)) is the
//   distance of that exact product from the integer. x * c lies within 1.5 * 2^-23 * 127 = 2.3e-5 of the exact ratio
//   and the defined quotient within 2 * 2^-24 * 127 = 1.5e-5, so both round to the same integer unless x * c is
//   within 3.8e-5 of a half-integer; lanes with |e| > 0.49995 redo their four values by the definition.
__device__ __forceinline__ unsigned quant4_i8(float x0, float x1, float x2, float x3, float c, float amax,
                                              float qmaxf = 127.f) {
    const float magic = 12582912.0f;
    const float m0 = __builtin_fmaf(x0, c, magic), m1 = __builtin_fmaf(x1, c, magic);
    const float m2 = __builtin_fmaf(x2, c, magic), m3 = __builtin_fmaf(x3, c, magic);
    const float e0 = __builtin_fmaf(x0, c, magic - m0), e1 = __builtin_fmaf(x1, c, magic - m1);
    const float e2 = __builtin_fmaf(x2, c, magic - m2), e3 = __builtin_fmaf(x3, c, magic - m3);
    const unsigned lo = __builtin_amdgcn_perm(__float_as_uint(m1), __float_as_uint(m0), 0x0c0c0400u);
    const unsigned hi = __builtin_amdgcn_perm(__float_as_uint(m3), __float_as_uint(m2), 0x0c0c0400u);
    unsigned pk = __builtin_amdgcn_perm(hi, lo, 0x05040100u);
    if (fmaxf(fmaxf(fabsf(e0), fabsf(e1)), fmaxf(fabsf(e2), fabsf(e3))) > 0.49995f)
        pk = pack4(symq_code_f(x0, qmaxf, amax), symq_code_f(x1, qmaxf, amax), symq_code_f(x2, qmaxf, amax),
                   symq_code_f(x3, qmaxf, amax));
    return pk;
}

// The same for values x_i * f whose products have not been formed yet (f > 0 common to the four): the fast path
// rounds the exact product x * (f * c), f * c rounded once, which lies within 2.5 * 2^-23 * 127 = 3.8e-5 of the exact
// ratio of y = fl(x * f) to amax (one more rounding in f * c, one in y itself); with the defined quotient's 1.5e-5 the
// two agree unless the product is within 5.3e-5 of a half-integer. Flagged lanes form y and follow the definition.
__device__ __forceinline__ unsigned quant4_i8_scaled(float x0, float x1, float x2, float x3, float f, float c, float amax) {
    const float magic = 12582912.0f;
    const float fc = f * c;
    const float m0 = __builtin_fmaf(x0, fc, magic), m1 = __builtin_fmaf(x1, fc, magic);
    const float m2 = __builtin_fmaf(x2, fc, magic), m3 = __builtin_fmaf(x3, fc, magic);
    const float e0 = __builtin_fmaf(x0, fc, magic - m0), e1 = __builtin_fmaf(x1, fc, magic - m1);
    const float e2 = __builtin_fmaf(x2, fc, magic - m2), e3 = __builtin_fmaf(x3, fc, magic - m3);
    const unsigned lo = __builtin_amdgcn_perm(__float_as_uint(m1), __float_as_uint(m0), 0x0c0c0400u);
    const unsigned hi = __builtin_amdgcn_perm(__float_as_uint(m3), __float_as_uint(m2), 0x0c0c0400u);
    unsigned pk = __builtin_amdgcn_perm(hi, lo, 0x05040100u);
    if (fmaxf(fmaxf(fabsf(e0), fabsf(e1)), fmaxf(fabsf(e2), fabsf(e3))) > 0.49994f)
        pk = pack4(symq_code_f(x0 * f, 127.f, amax), symq_code_f(x1 * f, 127.f, amax), symq_code_f(x2 * f, 127.f, amax),
                   symq_code_f(x3 * f, 127.f, amax));
    return pk;
}

typedef _Float16 half2_t __attribute__((ext_vector_type(2)));

// All-reduce over the four quarter-wave lanes that hold one image token (l, l^16, l^32, l^48) with the
// gfx950 row / half-wave swaps: no LDS round trip.
__device__ __forceinline__ float quad_allmax(float x) {
    const auto a = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    const float y = fmaxf(__uint_as_float(a[0]), __uint_as_float(a[1]));
    const auto b = __builtin_amdgcn_permlane32_swap(__float_as_uint(y), __float_as_uint(y), false, false);
    return fmaxf(__uint_as_float(b[0]), __uint_as_float(b[1]));
}
__device__ __forceinline__ float quad_allsum(float x) {
    const auto a = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    const float y = __uint_as_float(a[0]) + __uint_as_float(a[1]);
    const auto b = __builtin_amdgcn_permlane32_swap(__float_as_uint(y), __float_as_uint(y), false, false);
    return __uint_as_float(b[0]) + __uint_as_float(b[1]);
}
// Maximum over the 16 lanes of a row (DPP: xor 1, xor 2, mirror within 8, mirror within 16).
__device__ __forceinline__ float row16_allmax(float x) {
    x = fmaxf(x, __uint_as_float(__builtin_amdgcn_update_dpp(0u, __float_as_uint(x), 0xB1, 0xF, 0xF, true)));
    x = fmaxf(x, __uint_as_float(__builtin_amdgcn_update_dpp(0u, __float_as_uint(x), 0x4E, 0xF, 0xF, true)));
    x = fmaxf(x, __uint_as_float(__builtin_amdgcn_update_dpp(0u, __float_as_uint(x), 0x141, 0xF, 0xF, true)));
    x = fmaxf(x, __uint_as_float(__builtin_amdgcn_update_dpp(0u, __float_as_uint(x), 0x140, 0xF, 0xF, true)));
    return x;
}

// Four biased bytes (code + 128) -> four fp16 codes: 0x6400 | byte is the fp16 number 1152 + code.
__device__ __forceinline__ void biased4_to_half(unsigned w, half2_t& a, half2_t& b) {
    const unsigned lo = __builtin_amdgcn_perm(0x64646464u, w, 0x04010400u);
    const unsigned hi = __builtin_amdgcn_perm(0x64646464u, w, 0x04030402u);
    const half2_t off = {(_Float16)1152.0f, (_Float16)1152.0f};
    a = *reinterpret_cast<const half2_t*>(&lo) - off;
    b = *reinterpret_cast<const half2_t*>(&hi) - off;
}

// TOK = 32 image tokens per workgroup. NTT = 2: one wavefront per head carrying two column tiles of 16 tokens
// (A operands shared by both tiles). NTT = 1: two wavefronts per head, one tile each (16 wavefronts per CU
// instead of 8: more latency hiding for twice the A-operand traffic). TOK = 16 (with NTT = 1): one wavefront per
// head and half the tokens, for layers whose 32-token tiles would leave most compute units without a workgroup.
// CORE: only the attention core (profiling by stage): Q~ codes and scales come from the workspace instead of the
// hidden tile and to_q, and the kernel stops after writing A^ V~ as float32.
// NG > 1 (layers too wide for one workgroup's LDS): the workgroup owns one head group (NH of the NH*NG
// heads), takes the per-token codes of `hidden` from the workspace, and stops after A^ V~, which it writes to
// the workspace as float32; the per-token quantization of that result and to_out run as separate kernels.
// NT16 > 0: the number of 16-token score tiles, ceil(T / 16), is this compile-time constant (5 for the 77 text tokens
// of every configured workload: no run-time guards around the tiles) and the taps on intermediate results are
// compiled out; NT16 = 0: any T up to 96, guards at run time, taps where the caller asks for them.
template <int D, int NH, int NTT, int NG, int PG, int TOK = 32, bool CORE = false, int NT16 = 0, bool DENSE = false>
__global__ __launch_bounds__(NG > 1 ? 512 : 64 * NH * (TOK / (16 * NTT)))
__attribute__((amdgpu_waves_per_eu(DENSE ? 4 : 1, DENSE ? 4 : NG > 1 ? 2 : (NH * (TOK / (16 * NTT)) + 3) / 4)))
void fused_block_kernel(FusedTable tab, FusedDims dm) {
    using F = FusedCfg<D, NH, NTT, NG, TOK, DENSE>;
    static_assert(!DENSE || (NG == 1 && !CORE && NH * (TOK / (16 * NTT)) == 8), "two 8-wavefront workgroups per compute unit");
    static_assert(TOK == 32 || (TOK == 16 && NTT == 1), "a workgroup owns 32 image tokens, or 16 with one tile per wavefront");
    static_assert(!CORE || NG == 1, "the attention-core-only variant exists for the single-kernel shapes");
    constexpr int C = F::C, H = F::H, TPH = F::TPH, KS = F::KS, FS = F::FS, KC = F::KC, NT = F::NT;
    constexpr int SUB = F::SUB, TPS = F::TPS;
    constexpr bool LOGP = PG == TAQ_PROB_LOG2, ROWMAX = PG == TAQ_PROB_ROWMAX;  // grid of the probabilities, Eq. (3)
    constexpr int MT16 = NT16 ? NT16 : 6;  // score tiles the code is unrolled for
    constexpr bool TAPS = NT16 == 0;       // taps of intermediate codes and scales (tests, profiling)
    extern __shared__ __align__(16) unsigned char smem[];

    const int tid = threadIdx.x, hl = (tid >> 6) % NH, lane = tid & 63, r16 = lane & 15, q = lane >> 4;
    // Grid: x = batch element, y = request, z = token tile; head-group variant (one request): x = batch element,
    // y = token tile, z = head group. Workgroups are dispatched x fastest, so consecutive ones (which round-robin over
    // the 8 XCDs) share a token tile index and differ in the batch element / request: one XCD, few K~/V~ images. The
    // indices come straight from the grid: no integer divisions in front of the first loads.
    const int b = (int)blockIdx.x;
    const int ri = NG > 1 ? 0 : (int)blockIdx.y;
    const int tile = NG > 1 ? (int)blockIdx.y : (int)blockIdx.z;
    const int by = NG > 1 ? (int)blockIdx.z : 0;  // head group
    const int h = by * NH + hl;  // head of the layer; hl = head within the workgroup
    const int tbase = (((tid >> 6) / NH) % F::G) * 16 * NTT;  // first tile row of this wavefront's tokens
    const int sub = SUB == 1 ? 0 : (tid >> 6) / (NH * F::G);  // which share of the channel tiles of A^ V~
    const FusedReq rq = tab.req[ri];
    const int N = dm.N, T = dm.T;
    const int nt16 = NT16 ? NT16 : dm.nt16;
    const int n0 = tile * TOK;

    // ---- The hidden tile's loads are issued before anything else: they are the head of the kernel's one unavoidable
    // latency chain (HBM), and everything below (scalar loads of layout fields, of the protected-token count from
    // global memory, address arithmetic for the weights) would otherwise sit in front of them.
    constexpr bool HQ1 = NG == 1 && !CORE;         // single-kernel variant: 16 threads per token, 8-byte loads
    constexpr int TPT = NG > 1 ? NT / TOK : 16;    // threads per token
    constexpr int CH = NG > 1 ? C / (8 * TPT) : 1; // head-group variant: 16-byte pieces of a hidden row per thread
    const int tok0 = tid / TPT, part0 = tid % TPT;
    const int nq0 = n0 + tok0;
    const size_t row0 = (size_t)b * N + (nq0 < N ? nq0 : N - 1);
    const bool HOLDS = NT == 16 * TOK || tid < 16 * TOK;  // this thread holds a piece of the tile (all do, at 8 heads)
    uint2 xin[HQ1 ? KC : 1];
    uint4 xin4[NG > 1 ? CH : 1];
    if constexpr (HQ1) {
        if (HOLDS) {
            const uint2* xr = reinterpret_cast<const uint2*>(rq.hidden + row0 * C);
#pragma unroll
            for (int it = 0; it < KC; ++it) xin[it] = xr[it * 16 + part0];
        }
    }
    if constexpr (NG > 1) {
        const uint4* xr = reinterpret_cast<const uint4*>(rq.hidden + row0 * C);
#pragma unroll
        for (int it = 0; it < CH; ++it) xin4[it] = xr[it * TPT + part0];
    }
    __builtin_amdgcn_sched_barrier(0);

    // ---- LDS carve-up
    unsigned char* img = smem;                                  // K~/V~ image blocks of this workgroup's heads
    const size_t img_bytes = (size_t)NH * dm.I.head_bytes;
    int8_t* tileq = reinterpret_cast<int8_t*>(smem + img_bytes);                 // [TOK][C+16] hidden codes, later O codes
    float* wsc = reinterpret_cast<float*>(smem + img_bytes + TOK * F::TILE_RS);  // s_wq | s_wo | bias_o  [3C]
    float* s_h = wsc + (NG == 1 ? 3 * C : NH * D);               // [TOK]  (NG > 1: only s_wq of the workgroup's heads)
    unsigned* omax = reinterpret_cast<unsigned*>(s_h + TOK);     // [TOK][NH]  (NG == 1)
    int* qacc = reinterpret_cast<int*>(s_h + TOK);               // [K ranges][TOK/16][NH*TPH][64][4] partial to_q sums (NG > 1)

    const uint8_t* packed = rq.packed;
    const int ntrig = reinterpret_cast<const int*>(packed + dm.L.ntrig)[b];
    const int nfp = (ntrig + 15) >> 4;  // tiles of 16 protected tokens

    // weight rows of this head: row c = h*D + 16*j + r16 (rows past the head are discarded; clamp keeps reads in bounds)
    // (byte offset of K step ks = wrow[j] + ks * wstep; with the operand-ordered copy a wavefront-wide load is
    // one contiguous KiB, otherwise 16 rows x 64 bytes)
    int wrow[TPH];
    const int wstep = dm.w_layout ? 1024 : 64;
#pragma unroll
    for (int j = 0; j < TPH; ++j) {
        const int c = h * D + 16 * j + r16;
        wrow[j] = dm.w_layout ? (int)dm.w_pack_off + ((h * TPH + j) * KC) * 1024 + lane * 16 : (c < C ? c : C - 1) * C + 16 * q;
        // Weight rows past the head (the upper lanes of a partly filled last tile) are not fetched: their products are
        // dropped anyway, and at d = 40 they are a sixth of the bytes every CU pulls through its L2. Their lanes carry
        // an offset past the end of the buffer, for which a buffer load returns zero without a memory access.
        if (!((D % 16 == 0) || 16 * j + 16 <= D || r16 < D - 16 * j)) wrow[j] = 0x7fffffff;
    }
    // Buffer loads: the descriptor (base, size) and the step sit in scalar registers and the lane's part is a 32-bit
    // offset, so a load costs no vector address arithmetic (a 64-bit vector add per load otherwise) and the lanes
    // without a row need neither a branch nor registers cleared by hand.
    const __amdgpu_buffer_rsrc_t rs_wq = weight_rsrc(rq.wq, dm.w_bytes), rs_wo = weight_rsrc(rq.wo, dm.w_bytes);
    auto load_w = [&](const __amdgpu_buffer_rsrc_t rs, int j, int off) -> int32x4_t {
        return (int32x4_t)__builtin_amdgcn_raw_buffer_load_b128(rs, wrow[j], off, 0);
    };
    int32x4_t wreg[F::PREFETCH_W ? TPH : 1][F::PREFETCH_W ? KC : 1];
    constexpr int RING = CORE ? 0 : F::RING, NF = F::NF;
    constexpr int RPS = RING ? (RING + KC - 1) / KC : 0;  // ring loads issued per step of the hidden quantizer
    int32x4_t wring[RING ? RING : 1];
    const float* swq = wsc;
    const float* swo = wsc + C;
    const float* bo = wsc + 2 * C;
    unsigned char* imgh = img + (size_t)hl * dm.I.head_bytes;  // this head's block of the K~/V~ image
    const float* img_sk = reinterpret_cast<const float*>(imgh + dm.I.s_k);
    const float* img_bias = reinterpret_cast<const float*>(imgh + dm.I.bias);
    const __half* k16 = reinterpret_cast<const __half*>(packed + dm.L.k16) + (size_t)b * T * C;
    const __half* v16t = reinterpret_cast<const __half*>(packed + dm.L.v16t) + (size_t)b * C * 96;

    // protected (trigger) rows of this head, first tile of 16: fp16 K rows and transposed V rows straight from
    // global memory into MFMA operand registers (slots past the protected tokens hold zeros; K channels past the
    // head are not read: they would belong to the next head, or lie past the last row of the last head, and a
    // non-finite bit pattern there would survive the multiplication with a zero Q~ code)
    uint2 k16r[FS][2], v16r[TPS];
    auto load_protected = [&]() {
        if (nfp > 0) {
            const int slot = r16 < T ? r16 : T - 1;
            const __half* kr = k16 + (size_t)slot * C + h * D + 4 * q;
#pragma unroll
            for (int s = 0; s < FS; ++s)
#pragma unroll
                for (int jj = 0; jj < 2; ++jj)
                    k16r[s][jj] = (2 * s + jj < TPH && 16 * (2 * s + jj) + 4 * q < D)
                                      ? *reinterpret_cast<const uint2*>(kr + 16 * (2 * s + jj)) : make_uint2(0, 0);
#pragma unroll
            for (int k = 0; k < TPS; ++k) {
                const int jt = sub + SUB * k;  // this wavefront's k-th channel tile of A^ V~ (may lie past the head: clamped)
                int c = h * D + 16 * jt + r16;
                c = c < C ? c : C - 1;
                v16r[k] = *reinterpret_cast<const uint2*>(v16t + (size_t)c * 96 + 4 * q);
            }
        }
    };

    if constexpr (NG == 1 && !CORE) {
        // ---- phase 0: issue every global read up front, oldest first in the order of use (loads return in
        // order): hidden tile, weight scales, this head's to_q weight slice, the K~/V~ image
        // (16 threads per token, 4 channels per load: the first 16*TOK threads hold the tile, requested above)
        constexpr int SCV = (3 * C / 4 + NT - 1) / NT;
        float4 scv[SCV];
    #pragma unroll
        for (int k = 0; k < SCV; ++k) {
            const int i = tid + k * NT;
            scv[k] = i < 3 * C / 4 ? reinterpret_cast<const float4*>(rq.scales)[i] : make_float4(0.f, 0.f, 0.f, 0.f);
        }
        // ---- per-token int8 codes of the hidden tile. The row maximum is taken on the fp16 values themselves, two per
        // instruction (a maximum is exact in any precision); the quantizer's FMAs read the fp16 operands directly.
        float amax = 0.f;
        if (HOLDS) {
            half2_t am2 = {(_Float16)0.f, (_Float16)0.f};
    #pragma unroll
            for (int it = 0; it < KC; ++it) {
                const unsigned a0 = xin[it].x & 0x7fff7fffu, a1 = xin[it].y & 0x7fff7fffu;
                am2 = __builtin_elementwise_max(am2, __builtin_elementwise_max(*reinterpret_cast<const half2_t*>(&a0),
                                                                                 *reinterpret_cast<const half2_t*>(&a1)));
            }
            amax = fmaxf((float)am2[0], (float)am2[1]);
        }
        // The hidden tile has arrived (the unpacking above waited for it). Only now are the 10x larger weight reads
        // issued: the texture path serves requests in arrival order, and the first barrier waits for nothing else.
        __builtin_amdgcn_sched_barrier(0);
        // The weight slice is fetched a few loads at a time between pieces of arithmetic: a wavefront stalls at a
        // vector-memory instruction while the texture unit's queue is full (it coalesces 64 B per clock, and every
        // CU pulls ~300 KB of weights and image per launch), so the requests are spread under the ALU work.
        amax = row16_allmax(amax);
        const bool zero0 = amax == 0.f;
        const float sc0 = zero0 ? 1.f : amax / 127.f;
        const float safe0 = zero0 ? 1.f : amax;
        const float cq0 = 127.f * __builtin_amdgcn_rcpf(safe0);
        if (HOLDS && part0 == 0) s_h[tok0] = sc0;
    #pragma unroll
        for (int it = 0; it < KC; ++it) {
            if (F::PREFETCH_W) {
    #pragma unroll
                for (int j = 0; j < TPH; ++j) wreg[j][it] = load_w(rs_wq, j, wstep * it);
            }
            if constexpr (RING > 0) {  // the first RING loads of to_q, in the order the MFMAs use them
    #pragma unroll
                for (int f = it * RPS; f < (it + 1) * RPS && f < RING; ++f) wring[f] = load_w(rs_wq, f % TPH, wstep * (f / TPH));
            }
            if (HOLDS) {
                const half2_t x01 = *reinterpret_cast<const half2_t*>(&xin[it].x), x23 = *reinterpret_cast<const half2_t*>(&xin[it].y);
                const unsigned pk = quant4_i8((float)x01[0], (float)x01[1], (float)x23[0], (float)x23[1], cq0, safe0);
                *reinterpret_cast<unsigned*>(tileq + tok0 * F::TILE_RS + (it * 16 + part0) * 4) = pk;
                if (TAPS && dm.dbg.h_code && nq0 < N) *reinterpret_cast<unsigned*>(dm.dbg.h_code + row0 * C + (it * 16 + part0) * 4) = pk;
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        if (TAPS && HOLDS && dm.dbg.s_h && part0 == 0 && nq0 < N) dm.dbg.s_h[row0] = sc0;
        // ---- weight scales into LDS
    #pragma unroll
        for (int k = 0; k < SCV; ++k) {
            const int i = tid + k * NT;
            if (i < 3 * C / 4) reinterpret_cast<float4*>(wsc)[i] = scv[k];
        }
    }
    // ---- head-group variant, phase 0: every global read of the first two phases is issued up front, oldest first in
    // the order of use: the hidden tile, this wavefront's share of the to_q weights, the K~/V~ image blocks
    constexpr int TW = NH * TPH;                       // weight tiles (16 output channels) of this workgroup
    constexpr int KP = NG > 1 ? NT / 128 : 1;          // the wavefronts split to_q into two tile groups x KP K ranges
    constexpr int N2 = TOK / 16;                       // token groups of 16, all covered by every wavefront's share
    constexpr int TJ = NG > 1 ? TW / 2 : 1;            // weight tiles per tile group
    constexpr int KW = NG > 1 ? KC / KP : 1;           // K steps per K range
    constexpr int IMV = NG > 1 ? (NH * F::IMGC * 64 + NT - 1) / NT : 1;
    int32x4_t wpre[TJ][KW];
    int32x4_t imv[IMV];
    if constexpr (NG > 1) {
        static_assert(NG == 1 || (TW % 2 == 0 && KC % KP == 0 && C % (8 * TPT) == 0 && (TPT == 16 || TPT == 32)), "head-group split");
        const int wv = tid >> 6, js = wv & 1, kp = wv >> 1;
        float4 swv = make_float4(0.f, 0.f, 0.f, 0.f);  // s_wq of this workgroup's heads: NH*D floats
        if (tid < NH * D / 4) swv = reinterpret_cast<const float4*>(rq.scales + (size_t)by * NH * D)[tid];
        // ---- per-token int8 codes of the hidden tile (every head group of a token tile computes the same codes)
        float amax = 0.f;
#pragma unroll
        for (int it = 0; it < CH; ++it) {
            const __half2* hh2 = reinterpret_cast<const __half2*>(&xin4[it]);
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float2 p = __half22float2(hh2[e]);
                amax = fmaxf(amax, fmaxf(fabsf(p.x), fabsf(p.y)));
            }
        }
        // The hidden tile has arrived. The 3x larger weight and image reads are issued a few at a time between
        // pieces of the quantizer arithmetic: a wavefront stalls at a vector-memory instruction while the texture
        // unit's queue is full, so the requests are spread under the ALU work.
        __builtin_amdgcn_sched_barrier(0);
        amax = row16_allmax(amax);
        if constexpr (TPT == 32) {  // the other 16 lanes of this token
            const auto sw = __builtin_amdgcn_permlane16_swap(__float_as_uint(amax), __float_as_uint(amax), false, false);
            amax = fmaxf(__uint_as_float(sw[0]), __uint_as_float(sw[1]));
        }
        const bool zero0 = amax == 0.f;
        const float sc0 = zero0 ? 1.f : amax / 127.f;
        const float safe0 = zero0 ? 1.f : amax;
        const float cq0 = 127.f * __builtin_amdgcn_rcpf(safe0);
        if (tid < NH * D / 4) reinterpret_cast<float4*>(wsc)[tid] = swv;
        const bool tap = by == 0 && nq0 < N;
        if (part0 == 0) s_h[tok0] = sc0;
        if (TAPS && tap && dm.dbg.s_h && part0 == 0) dm.dbg.s_h[row0] = sc0;
        const int img16 = (int)((NH * dm.I.head_bytes) >> 4);  // the workgroup's head blocks are contiguous
        const int32x4_t* gimg = reinterpret_cast<const int32x4_t*>(packed + dm.L.image + (size_t)b * dm.L.image_bytes +
                                                                   (size_t)by * NH * dm.I.head_bytes);
        constexpr int NLD = TJ * KW + IMV, LPI = (NLD + CH - 1) / CH;  // loads to spread, loads per quantizer step
#pragma unroll
        for (int it = 0; it < CH; ++it) {
#pragma unroll
            for (int f = it * LPI; f < (it + 1) * LPI && f < NLD; ++f) {
                if (f < TJ * KW) {  // this wavefront's share of the to_q weights: tile group js, K range kp
                    const int jj = f / KW, kk = f % KW;
                    const int tw = js * TJ + jj;                       // weight tile within the workgroup
                    const int hh = by * NH + tw / TPH;    // its head and tile within the head
                    const int c = hh * D + 16 * (tw % TPH) + r16;
                    const int off = dm.w_layout ? (int)dm.w_pack_off + ((hh * TPH + tw % TPH) * KC) * 1024 + lane * 16
                                                : (c < C ? c : C - 1) * C + 16 * q;
                    wpre[jj][kk] = *reinterpret_cast<const int32x4_t*>(rq.wq + off + wstep * (kp * KW + kk));
                } else {            // the K~/V~ image blocks of this workgroup's heads
                    const int i = tid + (f - TJ * KW) * NT;
                    imv[f - TJ * KW] = gimg[i < img16 ? i : img16 - 1];
                }
            }
            const __half2* hh2 = reinterpret_cast<const __half2*>(&xin4[it]);
            const float2 p0 = __half22float2(hh2[0]), p1 = __half22float2(hh2[1]);
            const float2 p2 = __half22float2(hh2[2]), p3 = __half22float2(hh2[3]);
            uint2 pk;
            pk.x = quant4_i8(p0.x, p0.y, p1.x, p1.y, cq0, safe0);
            pk.y = quant4_i8(p2.x, p2.y, p3.x, p3.y, cq0, safe0);
            *reinterpret_cast<uint2*>(tileq + tok0 * F::TILE_RS + (it * TPT + part0) * 8) = pk;
            if (TAPS && tap && dm.dbg.h_code) *reinterpret_cast<uint2*>(dm.dbg.h_code + row0 * C + (it * TPT + part0) * 8) = pk;
            __builtin_amdgcn_sched_barrier(0);
        }
    }
    __syncthreads();

    // this lane's two image tokens: tile rows r16 and 16 + r16
    bool nvalid[NTT];
    size_t tok[NTT];
#pragma unroll
    for (int nt = 0; nt < NTT; ++nt) {
        const int n = n0 + tbase + 16 * nt + r16;
        nvalid[nt] = n < N;
        tok[nt] = (size_t)b * N + (n < N ? n : N - 1);
    }

    // ================= to_q for this head: Qf^T[c][n]
    int32x4_t hb[NTT][NG == 1 && RING == 0 ? KC : 1];
    if constexpr (NG == 1 && !CORE && RING == 0) {
#pragma unroll
        for (int nt = 0; nt < NTT; ++nt)
#pragma unroll
            for (int ks = 0; ks < KC; ++ks)
                hb[nt][ks] = *reinterpret_cast<const int32x4_t*>(tileq + (tbase + 16 * nt + r16) * F::TILE_RS + 64 * ks + 16 * q);
    }
    int32x4_t pacc[NTT][TPH];
    if constexpr (CORE) {
        // no projection: Q~ comes from the workspace
    } else if constexpr (F::PREFETCH_W) {
        // K step outermost: the order in which the weight loads were issued, so that the MFMAs follow the weights as they
        // arrive and only one step's worth is left to do after the last load
#pragma unroll
        for (int j = 0; j < TPH; ++j)
#pragma unroll
            for (int nt = 0; nt < NTT; ++nt) pacc[nt][j] = (int32x4_t){0, 0, 0, 0};
#pragma unroll
        for (int ks = 0; ks < KC; ++ks)
#pragma unroll
            for (int j = 0; j < TPH; ++j)
#pragma unroll
                for (int nt = 0; nt < NTT; ++nt)
                    pacc[nt][j] = __builtin_amdgcn_mfma_i32_16x16x64_i8(wreg[j][ks], hb[nt][ks], pacc[nt][j], 0, 0, 0);
    } else if constexpr (NG == 1 && RING > 0) {
#pragma unroll
        for (int j = 0; j < TPH; ++j)
#pragma unroll
            for (int nt = 0; nt < NTT; ++nt) pacc[nt][j] = (int32x4_t){0, 0, 0, 0};
#pragma unroll
        for (int ks = 0; ks < KC; ++ks) {
            int32x4_t hbk[NTT];
#pragma unroll
            for (int nt = 0; nt < NTT; ++nt)
                hbk[nt] = *reinterpret_cast<const int32x4_t*>(tileq + (tbase + 16 * nt + r16) * F::TILE_RS + 64 * ks + 16 * q);
#pragma unroll
            for (int j = 0; j < TPH; ++j) {
                const int f = ks * TPH + j;
                const int32x4_t wa = wring[f % RING];
#pragma unroll
                for (int nt = 0; nt < NTT; ++nt) pacc[nt][j] = __builtin_amdgcn_mfma_i32_16x16x64_i8(wa, hbk[nt], pacc[nt][j], 0, 0, 0);
                // the slot is free again: the load RING places ahead takes it
                if (f + RING < NF) wring[f % RING] = load_w(rs_wq, (f + RING) % TPH, wstep * ((f + RING) / TPH));
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    } else if constexpr (NG == 1) {
#pragma unroll
        for (int j = 0; j < TPH; ++j) {
#pragma unroll
            for (int nt = 0; nt < NTT; ++nt) pacc[nt][j] = (int32x4_t){0, 0, 0, 0};
#pragma unroll
            for (int ks = 0; ks < KC; ++ks) {
                const int32x4_t wa = load_w(rs_wq, j, wstep * ks);
#pragma unroll
                for (int nt = 0; nt < NTT; ++nt) pacc[nt][j] = __builtin_amdgcn_mfma_i32_16x16x64_i8(wa, hb[nt][ks], pacc[nt][j], 0, 0, 0);
            }
        }
    } else {
        // Head-group variant: the wavefronts split the workgroup's to_q by weight tile group (js) and K range (kp),
        // each for all of the workgroup's tokens; every wavefront leaves its int32 partial sums in a slot of its own
        // in LDS, and then adds up the KP partial sums of its own (head, token group): integer adds, exact in any order.
        const int wv = tid >> 6, js = wv & 1, kp = wv >> 1;
        if (sub < SUB) load_protected();  // needed only after the second barrier: they travel during the MFMAs
        int32x4_t hb2[N2][KW];
#pragma unroll
        for (int n2 = 0; n2 < N2; ++n2)
#pragma unroll
            for (int kk = 0; kk < KW; ++kk)
                hb2[n2][kk] = *reinterpret_cast<const int32x4_t*>(tileq + (16 * n2 + r16) * F::TILE_RS + 64 * (kp * KW + kk) + 16 * q);
#pragma unroll
        for (int jj = 0; jj < TJ; ++jj) {
            int32x4_t a2[N2];
#pragma unroll
            for (int n2 = 0; n2 < N2; ++n2) a2[n2] = (int32x4_t){0, 0, 0, 0};
#pragma unroll
            for (int kk = 0; kk < KW; ++kk)
#pragma unroll
                for (int n2 = 0; n2 < N2; ++n2) a2[n2] = __builtin_amdgcn_mfma_i32_16x16x64_i8(wpre[jj][kk], hb2[n2][kk], a2[n2], 0, 0, 0);
#pragma unroll
            for (int n2 = 0; n2 < N2; ++n2)
                *reinterpret_cast<int32x4_t*>(qacc + (((kp * N2 + n2) * TW + js * TJ + jj) * 64 + lane) * 4) = a2[n2];
        }
        {   // the K~/V~ image blocks (read into registers in phase 0) go to LDS
            const int img16 = (int)((NH * dm.I.head_bytes) >> 4);
#pragma unroll
            for (int k = 0; k < IMV; ++k) {
                const int i = tid + k * NT;
                if (i < img16) reinterpret_cast<int32x4_t*>(img)[i] = imv[k];
            }
        }
        __syncthreads();
        if (sub >= SUB) return;  // 16-token variant: only ROLES of the eight wavefronts carry on (no barrier follows)
#pragma unroll
        for (int j = 0; j < TPH; ++j) {
            pacc[0][j] = *reinterpret_cast<const int32x4_t*>(qacc + (((tbase >> 4) * TW + hl * TPH + j) * 64 + lane) * 4);
#pragma unroll
            for (int p = 1; p < KP; ++p)
                pacc[0][j] += *reinterpret_cast<const int32x4_t*>(qacc + (((p * N2 + (tbase >> 4)) * TW + hl * TPH + j) * 64 + lane) * 4);
        }
    }
    // Everything the Q~ step reads from LDS is fetched now, so that no LDS access sits between the issue of the
    // image copy below and the wait for it (the compiler orders LDS accesses after outstanding direct-to-LDS loads).
    float4 wq4[TPH];
    float shv[NTT];
    if constexpr (!CORE) {
#pragma unroll
        for (int j = 0; j < TPH; ++j) {
            const int cl = 16 * j + 4 * q;
            wq4[j] = *reinterpret_cast<const float4*>((NG == 1 ? swq + h * D : wsc + hl * D) + (((16 * j + 16 <= D) || cl < D) ? cl : 0));
        }
#pragma unroll
        for (int nt = 0; nt < NTT; ++nt) shv[nt] = s_h[tbase + 16 * nt + r16];
    }
    // This head's block of the K~/V~ image: straight into LDS, 1 KiB per wavefront-wide load (LDS address =
    // base + lane * 16), no registers in between; it travels while to_q and Q~ are computed, and only this
    // wavefront reads it, so only this wavefront waits for it. The last piece may be fetched more than once.
    if constexpr (NG == 1) {
        const unsigned char* gsrc = packed + dm.L.image + (size_t)b * dm.L.image_bytes + (size_t)h * dm.I.head_bytes;
        const int last = (int)dm.I.head_bytes - 1024;  // the block is a multiple of 256 bytes: the last piece overlaps
#pragma unroll
        for (int k = 0; k < F::IMGC; ++k) {
            if (k == 0 || k * 1024 < last + 1024) {  // (pieces past the block's end at this T are not fetched)
                const int c = k * 1024 < last ? k * 1024 : last;
                __builtin_amdgcn_global_load_lds(
                    (const __attribute__((address_space(1))) void*)(gsrc + c + lane * 16),
                    (__attribute__((address_space(3))) void*)(imgh + c), 16, 0, 0);
            }
        }
    }
    if constexpr (NG == 1) load_protected();

    // ---- Eq. (2), third line: Q~ = Q_a(Q) per (token, head)
    unsigned qpk[NTT][TPH];
    float sq2[NTT];
#pragma unroll
    for (int nt = 0; nt < NTT; ++nt) {
        if constexpr (CORE) {  // Q~ codes (one per byte) and per-(token, head) scales as a separate kernel formed them
#pragma unroll
            for (int j = 0; j < TPH; ++j) {
                const int cl = 16 * j + 4 * q;
                qpk[nt][j] = cl < D ? *reinterpret_cast<const unsigned*>(dm.core_qcode + tok[nt] * C + h * D + cl) : 0u;
            }
            sq2[nt] = fmaxf(dm.core_sq[tok[nt] * H + h] * dm.sig2, 1e-37f);
            continue;
        }
        const float sh = shv[nt];
        float qf[TPH][4];
        float qmax = 0.f;
#pragma unroll
        for (int j = 0; j < TPH; ++j) {
            const int cl = 16 * j + 4 * q;  // first of this lane's 4 channels in the head
            const bool valid = (16 * j + 16 <= D) || cl < D;
            const float wv[4] = {wq4[j].x, wq4[j].y, wq4[j].z, wq4[j].w};
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const float sc = sh * wv[i];
                const float v = (float)pacc[nt][j][i] * sc;
                qf[j][i] = valid ? v : 0.f;
                qmax = fmaxf(qmax, fabsf(qf[j][i]));
            }
        }
        qmax = quad_allmax(qmax);
        const bool qzero = qmax == 0.f;
        const float sQ = qzero ? 1.f : qmax / dm.qmaxq;
        const float qsafe = qzero ? 1.f : qmax;
        const float cq = dm.qmaxq * __builtin_amdgcn_rcpf(qsafe);
#pragma unroll
        for (int j = 0; j < TPH; ++j) qpk[nt][j] = quant4_i8(qf[j][0], qf[j][1], qf[j][2], qf[j][3], cq, qsafe, dm.qmaxq);
        if (TAPS && dm.dbg.q_code && nvalid[nt]) {
#pragma unroll
            for (int j = 0; j < TPH; ++j)
                if (16 * j + 4 * q < D) *reinterpret_cast<unsigned*>(dm.dbg.q_code + tok[nt] * C + h * D + 16 * j + 4 * q) = qpk[nt][j];
            if (dm.dbg.s_Q && q == 0) dm.dbg.s_Q[tok[nt] * H + h] = sQ;
        }
        sq2[nt] = fmaxf(sQ * dm.sig2, 1e-37f);
    }

    // the head's image block travelled meanwhile; it is private to this wavefront: wait (vmcnt(0)), no barrier
    __builtin_amdgcn_s_waitcnt(0x0F70);
    if constexpr (RING > 0 && NTT == 1) {  // ... or its first RING loads
#pragma unroll
        for (int f = 0; f < RING; ++f) wring[f] = load_w(rs_wo, f % TPH, wstep * (f / TPH));
    }

    // ================= scores: x[t][n] = (K~ Q~^T)[t][n] * s_K[t]   (times sQ * sigma * log2 e later)
    float S[NTT][MT16][4];
    {
        int32x4_t qop[NTT][KS];  // B operand: dword jj of step ks = codes of tile 4*ks + jj
#pragma unroll
        for (int nt = 0; nt < NTT; ++nt)
#pragma unroll
            for (int ks = 0; ks < KS; ++ks)
#pragma unroll
                for (int jj = 0; jj < 4; ++jj) qop[nt][ks][jj] = (4 * ks + jj < TPH) ? (int)qpk[nt][4 * ks + jj] : 0;
        const int8_t* kp = reinterpret_cast<const int8_t*>(imgh + dm.I.kp);
#pragma unroll
        for (int tt = 0; tt < MT16; ++tt) {
            if (tt < nt16) {
                int32x4_t acc[NTT];
#pragma unroll
                for (int nt = 0; nt < NTT; ++nt) acc[nt] = (int32x4_t){0, 0, 0, 0};
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) {
                    int32x4_t ka;
                    if constexpr (TPH % 4 == 0) {  // the lane's 16 bytes of this K step are contiguous
                        ka = *reinterpret_cast<const int32x4_t*>(kp + kp_offset(TPH, 16 * tt + r16, 4 * ks, q));
                    } else {
#pragma unroll
                        for (int jj = 0; jj < 4; ++jj)
                            ka[jj] = (4 * ks + jj < TPH) ? *reinterpret_cast<const int*>(kp + kp_offset(TPH, 16 * tt + r16, 4 * ks + jj, q)) : 0;
                    }
#pragma unroll
                    for (int nt = 0; nt < NTT; ++nt) acc[nt] = __builtin_amdgcn_mfma_i32_16x16x64_i8(ka, qop[nt][ks], acc[nt], 0, 0, 0);
                }
                const float4 sk = *reinterpret_cast<const float4*>(img_sk + 16 * tt + 4 * q);
                const float4 bi = *reinterpret_cast<const float4*>(img_bias + 16 * tt + 4 * q);
#pragma unroll
                for (int nt = 0; nt < NTT; ++nt) {
                    S[nt][tt][0] = __builtin_fmaf((float)acc[nt][0], sk.x, bi.x);
                    S[nt][tt][1] = __builtin_fmaf((float)acc[nt][1], sk.y, bi.y);
                    S[nt][tt][2] = __builtin_fmaf((float)acc[nt][2], sk.z, bi.z);
                    S[nt][tt][3] = __builtin_fmaf((float)acc[nt][3], sk.w, bi.w);
                }
            }
        }
    }
    // protected rows: fp16 K rows (the first 16 from registers, further ones straight from global memory: a handful of
    // rows). Their scores are formed twice by a run-time loop over tiles of 16 protected tokens, once for the row
    // maximum and once more for the exponentials, which go straight into the MFMAs against the fp16 V rows: only
    // one tile of protected scores is ever held in registers.
    half8_t qh[NTT][FS];  // Q~ codes as fp16: step s covers tiles 2s, 2s+1
    if (nfp > 0) {
#pragma unroll
        for (int nt = 0; nt < NTT; ++nt)
#pragma unroll
            for (int s = 0; s < FS; ++s) {
                half2_t c0 = {(_Float16)0.f, (_Float16)0.f}, c1 = c0, c2 = c0, c3 = c0;
                biased4_to_half(qpk[nt][2 * s] ^ 0x80808080u, c0, c1);
                if (2 * s + 1 < TPH) biased4_to_half(qpk[nt][2 * s + 1 < TPH ? 2 * s + 1 : 0] ^ 0x80808080u, c2, c3);
                qh[nt][s] = (half8_t){c0[0], c0[1], c1[0], c1[1], c2[0], c2[1], c3[0], c3[1]};
            }
    }
    // scores of protected tile ft (tokens of slots 16*ft .. 16*ft+15) for this lane's image tokens; -inf past ntrig
    auto protected_scores = [&](int ft, floatx4_t (&facc)[NTT]) {
#pragma unroll
        for (int nt = 0; nt < NTT; ++nt) facc[nt] = (floatx4_t){0.f, 0.f, 0.f, 0.f};
        int slot = 16 * ft + r16;
        slot = slot < T ? slot : T - 1;
        const __half* kr = k16 + (size_t)slot * C + h * D + 4 * q;
#pragma unroll
        for (int s = 0; s < FS; ++s) {
            half8_t ka;
#pragma unroll
            for (int jj = 0; jj < 2; ++jj) {
                const int j = 2 * s + jj;
                uint2 w = k16r[s][jj];
                if (ft > 0) w = (j < TPH && 16 * j + 4 * q < D) ? *reinterpret_cast<const uint2*>(kr + 16 * j) : make_uint2(0, 0);
                const half4_t hv = *reinterpret_cast<const half4_t*>(&w);
                ka[4 * jj + 0] = hv[0];
                ka[4 * jj + 1] = hv[1];
                ka[4 * jj + 2] = hv[2];
                ka[4 * jj + 3] = hv[3];
            }
#pragma unroll
            for (int nt = 0; nt < NTT; ++nt) facc[nt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(ka, qh[nt][s], facc[nt], 0, 0, 0);
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const bool live = 16 * ft + 4 * q + i < ntrig;
#pragma unroll
            for (int nt = 0; nt < NTT; ++nt) facc[nt][i] = live ? facc[nt][i] : TAQ_NEG_INF;
        }
    };

    // The LDS operands of O^T = V~^T A^^T (this wavefront's V~ codes and the split V scales) are read now, into
    // registers: issued next to their use, each read's round trip would stand between the softmax and its MFMAs.
    // (Only where registers are plentiful: the instantiation that also holds its weight slices in registers.)
    constexpr bool PRE_V = F::PREFETCH_W && NG == 1;
    uint2 vw2[PRE_V ? 3 : 1][PRE_V ? TPS : 1];  // V~^T codes of 32-token step s (s = 0, 1, 2; a single last tile uses .x only)
    uint2 svh[PRE_V ? MT16 : 1], svl[PRE_V ? MT16 : 1];  // fp16 high parts and remainders of s_V * 2^kexp, four text tokens of each tile
    const uint8_t* vt = imgh + dm.I.vt;
    const _Float16* img_sv = reinterpret_cast<const _Float16*>(imgh + dm.I.s_vp);  // [ntok] high parts | [ntok] low parts
    if constexpr (PRE_V) {
#pragma unroll
        for (int tt = 0; tt < MT16; ++tt) {
            svh[tt] = svl[tt] = make_uint2(0u, 0u);
            if (tt < nt16) {
                svh[tt] = *reinterpret_cast<const uint2*>(img_sv + 16 * tt + 4 * q);
                svl[tt] = *reinterpret_cast<const uint2*>(img_sv + dm.I.ntok + 16 * tt + 4 * q);
            }
        }
#pragma unroll
        for (int s = 0; s < 3; ++s)
#pragma unroll
            for (int k = 0; k < TPS; ++k) {
                vw2[s][k] = make_uint2(0u, 0u);
                const int jt = sub + SUB * k;
                if (2 * s >= nt16 || (SUB > 1 && jt >= TPH)) continue;
                int j = 16 * jt + r16;
                j = j < D ? j : D - 1;
                if (2 * s + 1 < nt16) vw2[s][k] = *reinterpret_cast<const uint2*>(vt + (size_t)j * dm.I.cols_v + 32 * s + 8 * q);
                else vw2[s][k].x = *reinterpret_cast<const unsigned*>(vt + (size_t)j * dm.I.cols_v + 32 * s + 4 * q);
            }
    }
    __builtin_amdgcn_sched_barrier(0);

    // ================= softmax over the text tokens; Eq. (3); weights of O^T = V~^T A^^T
    float kq[NTT];   // code = rint(E * kq): pmax / Z per image token (row-range grid: pmax / largest unprotected E)
    float kqp[NTT];  // protected columns: weight = E * kqp = pmax * A
    float lz[NTT];   // log2 Z (log2 grid only)
    float rz[NTT], fz[NTT];  // row-range grid only: Z / range and range / Z, which move between the two units
    float mxs[NTT];  // row maximum of the raw scores
#pragma unroll
    for (int nt = 0; nt < NTT; ++nt) {
        float mx = TAQ_NEG_INF;
#pragma unroll
        for (int tt = 0; tt < MT16; ++tt)
            if (tt < nt16) mx = fmaxf(mx, fmaxf(fmaxf(S[nt][tt][0], S[nt][tt][1]), fmaxf(S[nt][tt][2], S[nt][tt][3])));
        mxs[nt] = mx;
    }
    for (int ft = 0; ft < nfp; ++ft) {  // first pass over the protected tiles: their share of the row maximum
        floatx4_t facc[NTT];
        protected_scores(ft, facc);
#pragma unroll
        for (int nt = 0; nt < NTT; ++nt)
            mxs[nt] = fmaxf(mxs[nt], fmaxf(fmaxf(facc[nt][0], facc[nt][1]), fmaxf(facc[nt][2], facc[nt][3])));
    }
    float Zs[NTT], eus[NTT], offs[NTT];
#pragma unroll
    for (int nt = 0; nt < NTT; ++nt) {
        const float mx = quad_allmax(mxs[nt]);
        const float sc = sq2[nt], off = -mx * sc;
        offs[nt] = off;
        float Z = 0.f, eu = 0.f;
#pragma unroll
        for (int tt = 0; tt < MT16; ++tt)
            if (tt < nt16) {
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const float arg = __builtin_fmaf(S[nt][tt][i], sc, off);
                    const float ex = __builtin_amdgcn_exp2f(arg);
                    Z += ex;
                    if (ROWMAX) eu = fmaxf(eu, ex);  // the row's range: its largest unprotected probability (times Z)
                    S[nt][tt][i] = LOGP ? arg : ex;  // the log2 grid rounds the exponent itself
                }
            }
        Zs[nt] = Z;
        eus[nt] = eu;
    }

    // oacc[nt][k]: channel tile jt = sub + SUB*k of this head (NG == 1: SUB = 1, every tile; head-group variant: every
    // SUB-th tile, the other wavefronts of the (head, token group) take the rest; tiles past the head are skipped)
    floatx4_t oacc[NTT][TPS];
#pragma unroll
    for (int nt = 0; nt < NTT; ++nt)
#pragma unroll
        for (int k = 0; k < TPS; ++k) oacc[nt][k] = (floatx4_t){0.f, 0.f, 0.f, 0.f};
    // protected columns keep A (Eq. 3). Second pass over the protected tiles: E = exp2(score - max), not yet divided
    // by Z, as fp16 high + low parts against the fp16 V rows; the accumulators are brought to the unit of the
    // unprotected columns' weights (pmax * A * 2^kexp) once Z is known.
    for (int ft = 0; ft < nfp; ++ft) {
        floatx4_t facc[NTT];
        protected_scores(ft, facc);
        half4_t phi[NTT], plo[NTT];
#pragma unroll
        for (int nt = 0; nt < NTT; ++nt)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const float ex = __builtin_amdgcn_exp2f(__builtin_fmaf(facc[nt][i], sq2[nt], offs[nt]));
                Zs[nt] += ex;
                // (high part by the conversion intrinsic: the value that enters the MFMA is the one subtracted, whatever
                // instruction the compiler would pick for a plain cast in either place)
                const _Float16 xh = (_Float16)__builtin_amdgcn_cvt_pkrtz(ex, 0.f)[0];
                phi[nt][i] = xh;
                plo[nt][i] = (_Float16)(ex - (float)xh);
            }
#pragma unroll
        for (int k = 0; k < TPS; ++k) {
            const int jt = sub + SUB * k;
            if (SUB > 1 && jt >= TPH) continue;
            int c = h * D + 16 * jt + r16;
            c = c < C ? c : C - 1;
            uint2 w = v16r[k];
            if (ft > 0) w = *reinterpret_cast<const uint2*>(v16t + (size_t)c * 96 + 16 * ft + 4 * q);
            const half4_t va = *reinterpret_cast<const half4_t*>(&w);  // slots past ntrig hold zeros
#pragma unroll
            for (int nt = 0; nt < NTT; ++nt) {
                oacc[nt][k] = __builtin_amdgcn_mfma_f32_16x16x16f16(va, phi[nt], oacc[nt][k], 0, 0, 0);
                oacc[nt][k] = __builtin_amdgcn_mfma_f32_16x16x16f16(va, plo[nt], oacc[nt][k], 0, 0, 0);
            }
        }
    }
#pragma unroll
    for (int nt = 0; nt < NTT; ++nt) {
        const float Z = quad_allsum(Zs[nt]);
        kqp[nt] = dm.pmax * __builtin_amdgcn_rcpf(Z);
        kq[nt] = kqp[nt];
        lz[nt] = LOGP ? __builtin_amdgcn_logf(Z) : 0.f;  // log2 Z >= 0: the largest term of Z is 1
        rz[nt] = 1.f;
        fz[nt] = 1.f;
        if constexpr (ROWMAX) {
            // codes = rint(pmax * E / range), A^ = code * (range / Z) / pmax. Unprotected columns that together weigh
            // less than 2^-40 of the row (or none at all) are dropped: their codes would scale a vanishing range.
            const float eu = quad_allmax(eus[nt]);
            if (eu > Z * 9.094947e-13f) {
                const float re = __builtin_amdgcn_rcpf(eu);
                kq[nt] = dm.pmax * re;
                rz[nt] = Z * re;
                fz[nt] = eu * __builtin_amdgcn_rcpf(Z);
            }
        }
    }
    if (nfp > 0) {
        const float vpre = reinterpret_cast<const float*>(imgh + dm.I.vpre)[0];
#pragma unroll
        for (int nt = 0; nt < NTT; ++nt) {
            const float f = kqp[nt] * (ROWMAX ? vpre * rz[nt] : vpre);
#pragma unroll
            for (int k = 0; k < TPS; ++k)
#pragma unroll
                for (int i = 0; i < 4; ++i) oacc[nt][k][i] *= f;
        }
    }
    // unprotected columns: weight = code * s', s' = s_V * 2^kexp, as fp16 high + low parts (V codes are exact in fp16).
    // s' comes from the image already split, s' = sh + sl (two fp16 numbers, |sl| <= 2^-11 |sh|). The code c (an integer
    // below 256) is exact in fp16; in packed fp16 arithmetic, two columns per instruction:
    //   wh = fl(c * sh),  r = fma(c, sh, -wh)  (the rounding error of wh: exact, it needs at most 8 bits),
    //   wl = fma(c, sl, r)                      => wh + wl = c * s' to about 2^-22, relatively.
    // The code itself is formed with one FMA: P * kq + (1.5 * 2^23 + 0x6400) rounds P * kq half-to-even to an integer
    // and leaves 0x6400 + code in the low half of the result: the bit pattern of the fp16 number 1024 + code.
    {
        const half2_t k1024 = {(_Float16)1024.0f, (_Float16)1024.0f};
        // tap: the codes of text tokens t, t + 1 for this lane's image token of tile nt (one wavefront per (head, token group))
        auto tap_pcode = [&](int nt, int t, unsigned c0, unsigned c1) {
            if (sub == 0 && nvalid[nt]) {
                uint8_t* row = dm.dbg.p_code + (tok[nt] * H + h) * (size_t)T;
                if (t < T) row[t] = (uint8_t)c0;
                if (t + 1 < T) row[t + 1] = (uint8_t)c1;
            }
        };
#pragma unroll
        for (int s = 0; s < 3; ++s) {
            if (2 * s < nt16) {
                const bool second = 2 * s + 1 < nt16;
                half8_t phi[NTT], plo[NTT];
#pragma unroll
                for (int a = 0; a < 2; ++a) {
                    if (a == 0 || second) {
                        uint2 h4, l4;
                        if constexpr (PRE_V) {
                            h4 = svh[2 * s + a < MT16 ? 2 * s + a : 0];
                            l4 = svl[2 * s + a < MT16 ? 2 * s + a : 0];
                        } else {
                            h4 = *reinterpret_cast<const uint2*>(img_sv + 16 * (2 * s + a) + 4 * q);
                            l4 = *reinterpret_cast<const uint2*>(img_sv + dm.I.ntok + 16 * (2 * s + a) + 4 * q);
                        }
                        const half2_t sh[2] = {*reinterpret_cast<const half2_t*>(&h4.x), *reinterpret_cast<const half2_t*>(&h4.y)};
                        const half2_t sl[2] = {*reinterpret_cast<const half2_t*>(&l4.x), *reinterpret_cast<const half2_t*>(&l4.y)};
#pragma unroll
                        for (int nt = 0; nt < NTT; ++nt)
#pragma unroll
                            for (int i2 = 0; i2 < 2; ++i2) {
                                half2_t c;
                                if constexpr (LOGP) {
                                    // -code = clip(rint(log2 A)) = clip(rint(arg - log2 Z)); weight 2^(8 - code) * s': exact
                                    // scalings of sh and sl (a weight below fp16's range is below 2^-30 of the largest)
                                    const float c0 = __builtin_amdgcn_fmed3f(__builtin_rintf(S[nt][2 * s + a][2 * i2] - lz[nt]), -dm.plast, 0.f);
                                    const float c1 = __builtin_amdgcn_fmed3f(__builtin_rintf(S[nt][2 * s + a][2 * i2 + 1] - lz[nt]), -dm.plast, 0.f);
                                    const auto pw = __builtin_amdgcn_cvt_pkrtz(ldexpf(256.0f, (int)c0), ldexpf(256.0f, (int)c1));
                                    c = (half2_t){(_Float16)pw[0], (_Float16)pw[1]};
                                    if (TAPS && dm.dbg.p_code) tap_pcode(nt, 16 * (2 * s + a) + 4 * q + 2 * i2, (unsigned)(int)(-c0), (unsigned)(int)(-c1));
                                } else {
                                    const float m0 = __builtin_fmaf(S[nt][2 * s + a][2 * i2], kq[nt], 12608512.0f);
                                    const float m1 = __builtin_fmaf(S[nt][2 * s + a][2 * i2 + 1], kq[nt], 12608512.0f);
                                    const unsigned u = __builtin_amdgcn_perm(__float_as_uint(m1), __float_as_uint(m0), 0x05040100u);
                                    c = *reinterpret_cast<const half2_t*>(&u) - k1024;
                                    if (TAPS && dm.dbg.p_code) tap_pcode(nt, 16 * (2 * s + a) + 4 * q + 2 * i2, u & 0xFFu, (u >> 16) & 0xFFu);
                                }
                                const half2_t wh = c * sh[i2];
                                const half2_t wl = __builtin_elementwise_fma(c, sl[i2], __builtin_elementwise_fma(c, sh[i2], -wh));
                                phi[nt][4 * a + 2 * i2] = wh[0];
                                phi[nt][4 * a + 2 * i2 + 1] = wh[1];
                                plo[nt][4 * a + 2 * i2] = wl[0];
                                plo[nt][4 * a + 2 * i2 + 1] = wl[1];
                            }
                    } else {
#pragma unroll
                        for (int nt = 0; nt < NTT; ++nt)
#pragma unroll
                            for (int i = 0; i < 4; ++i) {
                                phi[nt][4 * a + i] = (_Float16)0.f;
                                plo[nt][4 * a + i] = (_Float16)0.f;
                            }
                    }
                }
#pragma unroll
                for (int k = 0; k < TPS; ++k) {
                    const int jt = sub + SUB * k;
                    if (SUB > 1 && jt >= TPH) continue;
                    int j = 16 * jt + r16;
                    j = j < D ? j : D - 1;
                    if (second) {  // two score tiles: 32 tokens deep, a lane's 8 codes are consecutive (vt_pos)
                        const uint2 w = PRE_V ? vw2[PRE_V ? s : 0][PRE_V ? k : 0]
                                              : *reinterpret_cast<const uint2*>(vt + (size_t)j * dm.I.cols_v + 32 * s + 8 * q);
                        half2_t v0, v1, v2, v3;
                        biased4_to_half(w.x, v0, v1);
                        biased4_to_half(w.y, v2, v3);
                        const half8_t va = {v0[0], v0[1], v1[0], v1[1], v2[0], v2[1], v3[0], v3[1]};
#pragma unroll
                        for (int nt = 0; nt < NTT; ++nt) {
                            oacc[nt][k] = __builtin_amdgcn_mfma_f32_16x16x32_f16(va, phi[nt], oacc[nt][k], 0, 0, 0);
                            oacc[nt][k] = __builtin_amdgcn_mfma_f32_16x16x32_f16(va, plo[nt], oacc[nt][k], 0, 0, 0);
                        }
                    } else {       // a last single tile: 16 tokens deep, in their natural order
                        const unsigned w = PRE_V ? vw2[PRE_V ? s : 0][PRE_V ? k : 0].x
                                                 : *reinterpret_cast<const unsigned*>(vt + (size_t)j * dm.I.cols_v + 32 * s + 4 * q);
                        half2_t v0, v1;
                        biased4_to_half(w, v0, v1);
                        const half4_t va = {v0[0], v0[1], v1[0], v1[1]};
#pragma unroll
                        for (int nt = 0; nt < NTT; ++nt) {
                            const half4_t ph = {phi[nt][0], phi[nt][1], phi[nt][2], phi[nt][3]};
                            const half4_t pl = {plo[nt][0], plo[nt][1], plo[nt][2], plo[nt][3]};
                            oacc[nt][k] = __builtin_amdgcn_mfma_f32_16x16x16f16(va, ph, oacc[nt][k], 0, 0, 0);
                            oacc[nt][k] = __builtin_amdgcn_mfma_f32_16x16x16f16(va, pl, oacc[nt][k], 0, 0, 0);
                        }
                    }
                }
            }
        }
    }

    if (F::PREFETCH_W && !CORE) {  // to_out's weight slice travels while A^ V~ is quantized (two barriers away from its use)
#pragma unroll
        for (int j = 0; j < TPH; ++j)
#pragma unroll
            for (int ks = 0; ks < KC; ++ks) wreg[j][ks] = load_w(rs_wo, j, wstep * ks);
    }
    if constexpr (RING > 0 && NTT == 2) {  // two token tiles per wavefront: the attention needs the registers; the first
#pragma unroll                         // RING loads of to_out travel while A^ V~ is quantized
        for (int f = 0; f < RING; ++f) wring[f] = load_w(rs_wo, f % TPH, wstep * (f / TPH));
    }
    // ================= per-token int8 codes of O over all heads
    // O = oacc * of, of = 2^-kexp / pmax (times range / Z on the row-range grid). Where nobody needs O itself (no tap, no
    // workspace copy) the products are not formed: the row maximum is max|oacc| * of (a product with a positive
    // constant is monotone, so this IS the maximum of the products), and the quantizer takes oacc and of apart.
    constexpr bool KEEP_O = NG > 1 || CORE || TAPS;
    const float osc = reinterpret_cast<const float*>(imgh + dm.I.oscale)[0] * (1.0f / dm.pmax);
    float of[NTT];
#pragma unroll
    for (int nt = 0; nt < NTT; ++nt) {
        of[nt] = ROWMAX ? osc * fz[nt] : osc;
        float omx = 0.f;
#pragma unroll
        for (int k = 0; k < TPS; ++k) {
            const int jt = sub + SUB * k;
            const bool valid = jt < TPH && ((16 * jt + 16 <= D) || 16 * jt + 4 * q < D);
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                if constexpr (KEEP_O) oacc[nt][k][i] = valid ? oacc[nt][k][i] * of[nt] : 0.f;
                omx = fmaxf(omx, valid ? fabsf(oacc[nt][k][i]) : 0.f);
            }
            if (KEEP_O && nvalid[nt] && valid) {
                const float4 o4 = make_float4(oacc[nt][k][0], oacc[nt][k][1], oacc[nt][k][2], oacc[nt][k][3]);
                if (TAPS && dm.dbg.O) *reinterpret_cast<float4*>(dm.dbg.O + tok[nt] * C + h * D + 16 * jt + 4 * q) = o4;
                if constexpr (NG > 1 || CORE) *reinterpret_cast<float4*>(dm.ws_of + tok[nt] * C + h * D + 16 * jt + 4 * q) = o4;
            }
        }
        if constexpr (!KEEP_O) omx *= of[nt];
        omx = quad_allmax(omx);
        if (NG == 1 && !CORE && q == 0) omax[(tbase + 16 * nt + r16) * NH + hl] = __float_as_uint(omx);
        // head-group variant: this wavefront's share of the token's row maximum, for the kernel that quantizes the row
        if (NG > 1 && q == 0 && nvalid[nt]) dm.ws_omax[tok[nt] * (H * SUB) + h * SUB + sub] = omx;
    }
    if constexpr (NG > 1 || CORE) return;  // the per-token quantization of A^ V~ and to_out are separate kernels
    __syncthreads();  // every wavefront is past its reads of the hidden codes
    float so[NTT];
#pragma unroll
    for (int nt = 0; nt < NTT; ++nt) {
        float oamax = 0.f;
#pragma unroll
        for (int w = 0; w < NH; ++w) oamax = fmaxf(oamax, __uint_as_float(omax[(tbase + 16 * nt + r16) * NH + w]));
        const bool ozero = oamax == 0.f;
        so[nt] = ozero ? 1.f : oamax / 127.f;
        const float osafe = ozero ? 1.f : oamax;
        const float cq = 127.f * __builtin_amdgcn_rcpf(osafe);
#pragma unroll
        for (int jt = 0; jt < TPH; ++jt)
            if (16 * jt + 4 * q < D) {
                const unsigned pk = KEEP_O ? quant4_i8(oacc[nt][jt][0], oacc[nt][jt][1], oacc[nt][jt][2], oacc[nt][jt][3], cq, osafe)
                                           : quant4_i8_scaled(oacc[nt][jt][0], oacc[nt][jt][1], oacc[nt][jt][2], oacc[nt][jt][3], of[nt], cq, osafe);
                const int c = h * D + 16 * jt + 4 * q;
                *reinterpret_cast<unsigned*>(tileq + (tbase + 16 * nt + r16) * F::TILE_RS + c) = pk;
                if (TAPS && dm.dbg.o_code && nvalid[nt]) *reinterpret_cast<unsigned*>(dm.dbg.o_code + tok[nt] * C + c) = pk;
            }
        if (TAPS && dm.dbg.s_o && nvalid[nt] && q == 0 && h == 0) dm.dbg.s_o[tok[nt]] = so[nt];
    }
    __syncthreads();

    // ================= to_out: Y^T[c][n] for this head's D output channels
    if constexpr (RING > 0) {
#pragma unroll
        for (int j = 0; j < TPH; ++j)
#pragma unroll
            for (int nt = 0; nt < NTT; ++nt) pacc[nt][j] = (int32x4_t){0, 0, 0, 0};
#pragma unroll
        for (int ks = 0; ks < KC; ++ks) {
            int32x4_t hbk[NTT];
#pragma unroll
            for (int nt = 0; nt < NTT; ++nt)
                hbk[nt] = *reinterpret_cast<const int32x4_t*>(tileq + (tbase + 16 * nt + r16) * F::TILE_RS + 64 * ks + 16 * q);
#pragma unroll
            for (int j = 0; j < TPH; ++j) {
                const int f = ks * TPH + j;
                const int32x4_t wa = wring[f % RING];
#pragma unroll
                for (int nt = 0; nt < NTT; ++nt) pacc[nt][j] = __builtin_amdgcn_mfma_i32_16x16x64_i8(wa, hbk[nt], pacc[nt][j], 0, 0, 0);
                if (f + RING < NF) wring[f % RING] = load_w(rs_wo, (f + RING) % TPH, wstep * ((f + RING) / TPH));
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    } else {
#pragma unroll
        for (int nt = 0; nt < NTT; ++nt)
#pragma unroll
            for (int ks = 0; ks < KC; ++ks)
                hb[nt][ks] = *reinterpret_cast<const int32x4_t*>(tileq + (tbase + 16 * nt + r16) * F::TILE_RS + 64 * ks + 16 * q);
#pragma unroll
        for (int j = 0; j < TPH; ++j) {
#pragma unroll
            for (int nt = 0; nt < NTT; ++nt) pacc[nt][j] = (int32x4_t){0, 0, 0, 0};
#pragma unroll
            for (int ks = 0; ks < KC; ++ks) {
                const int32x4_t wa = F::PREFETCH_W ? wreg[j][ks] : load_w(rs_wo, j, wstep * ks);
#pragma unroll
                for (int nt = 0; nt < NTT; ++nt) pacc[nt][j] = __builtin_amdgcn_mfma_i32_16x16x64_i8(wa, hb[nt][ks], pacc[nt][j], 0, 0, 0);
            }
        }
    }
#pragma unroll
    for (int j = 0; j < TPH; ++j) {
        const int cl = 16 * j + 4 * q;
        if (cl < D) {
            const int c = h * D + cl;
            const float4 w4 = *reinterpret_cast<const float4*>(swo + c);
            const float4 b4 = *reinterpret_cast<const float4*>(bo + c);
#pragma unroll
            for (int nt = 0; nt < NTT; ++nt) {
                const float y0 = (float)pacc[nt][j][0] * (so[nt] * w4.x) + b4.x;
                const float y1 = (float)pacc[nt][j][1] * (so[nt] * w4.y) + b4.y;
                const float y2 = (float)pacc[nt][j][2] * (so[nt] * w4.z) + b4.z;
                const float y3 = (float)pacc[nt][j][3] * (so[nt] * w4.w) + b4.w;
                if (nvalid[nt]) {
                    const half4_t y = {(_Float16)y0, (_Float16)y1, (_Float16)y2, (_Float16)y3};
                    *reinterpret_cast<half4_t*>(rq.out + tok[nt] * C + c) = y;
                }
            }
        }
    }
}

// Compute units of the current device (asked once per device).
static inline int device_cu_count() {
    static std::atomic<int> cus[64];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 256;
    int n = cus[dev].load(std::memory_order_acquire);
    if (n <= 0) {
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) n = 256;
        cus[dev].store(n, std::memory_order_release);
    }
    return n;
}

template <int D, int NH, int NTT, int NG, int PG, int TOK, bool CORE, int NT16 = 0, bool DENSE = false>
static hipError_t launch_fused_grid(const FusedTable& tab, const FusedDims& dm, hipStream_t st) {
    if constexpr (NT16 == 0) {  // 65 to 80 text tokens: the instantiation without run-time guards around the score tiles
        const bool taps = dm.dbg.h_code || dm.dbg.s_h || dm.dbg.q_code || dm.dbg.s_Q || dm.dbg.O || dm.dbg.o_code || dm.dbg.s_o || dm.dbg.p_code;
        if (dm.nt16 == 5 && !taps) return launch_fused_grid<D, NH, NTT, NG, PG, TOK, CORE, 5>(tab, dm, st);
    }
    using F = FusedCfg<D, NH, NTT, NG, TOK, DENSE>;
    static std::atomic<unsigned long long> lds_set{0};
    const size_t bytes = NG == 1 ? dm.I.bytes + TOK * F::TILE_RS + 3 * F::C * 4 + TOK * 4 + TOK * NH * 4  // = fused_lds_bytes
                                 : (size_t)NH * dm.I.head_bytes + TOK * F::TILE_RS + NH * D * 4 + TOK * 4 +
                                       (F::NT / 128) * (TOK / 16) * NH * F::TPH * 1024;  // = mid_lds_bytes at TOK = 32
    if (bytes > 160 * 1024 || dm.I.head_bytes > (size_t)F::IMGC * 1024) return hipErrorInvalidValue;
    if constexpr (!DENSE && NT16 == 5 && D == 40 && NH == 8 && NTT == 2 && NG == 1 && !CORE) {
        // More token tiles than compute units and a working set of at most half a compute unit's LDS: the instantiation
        // of which two workgroups share a compute unit (one is in its arithmetic while the other waits for memory).
        if ((dm.N + TOK - 1) / TOK * dm.R * dm.B > device_cu_count() && bytes <= 80 * 1024)
            return launch_fused_grid<D, NH, NTT, NG, PG, TOK, CORE, NT16, true>(tab, dm, st);
    }
    const hipError_t e = ensure_dynamic_lds(reinterpret_cast<const void*>(&fused_block_kernel<D, NH, NTT, NG, PG, TOK, CORE, NT16, DENSE>), 160 * 1024, lds_set);
    if (e != hipSuccess) return e;
    const int tiles = (dm.N + TOK - 1) / TOK;
    if (tiles > 65535 || dm.R > 65535 || (NG > 1 && dm.R != 1)) return hipErrorInvalidValue;
    const dim3 grid = NG > 1 ? dim3(dm.B, tiles, NG) : dim3(dm.B, dm.R, tiles);
    hipLaunchKernelGGL((fused_block_kernel<D, NH, NTT, NG, PG, TOK, CORE, NT16, DENSE>), grid, dim3(F::NT), bytes, st, tab, dm);
    return hipGetLastError();
}

template <int D, int NH, int NTT, int NG, int TOK = 32, bool CORE = false>
static hipError_t launch_fused_cfg(const FusedTable& tab, const FusedDims& dm, int grid, hipStream_t st) {
    if (grid == TAQ_PROB_LOG2) return launch_fused_grid<D, NH, NTT, NG, TAQ_PROB_LOG2, TOK, CORE>(tab, dm, st);
    if (grid == TAQ_PROB_ROWMAX) return launch_fused_grid<D, NH, NTT, NG, TAQ_PROB_ROWMAX, TOK, CORE>(tab, dm, st);
    return launch_fused_grid<D, NH, NTT, NG, TAQ_PROB_LINEAR, TOK, CORE>(tab, dm, st);
}

// Family launchers, one translation unit each. tok = 32 or 16 image tokens per workgroup; core: the attention core
// alone (single-kernel families only).
hipError_t launch_fused_d40(const FusedTable& tab, const FusedDims& dm, int grid, int tok, bool core, hipStream_t st);   // (d, H) = (40, 8)
hipError_t launch_fused_d80(const FusedTable& tab, const FusedDims& dm, int grid, int tok, bool core, hipStream_t st);   // (80, 8)
hipError_t launch_fused_d64(const FusedTable& tab, const FusedDims& dm, int grid, int tok, bool core, hipStream_t st);   // (64, 10)
hipError_t launch_fused_mid160(const FusedTable& tab, const FusedDims& dm, int grid, int tok, hipStream_t st);           // (160, 8): 8 groups of 1 head
hipError_t launch_fused_mid64(const FusedTable& tab, const FusedDims& dm, int grid, int tok, hipStream_t st);            // (64, 20): 10 groups of 2 heads

}  // namespace taq
