// Dispatch of the fused TAQ cross-attention block (PersonalQ, Section III-B), the K~/V~ image and weight re-layout
// kernels, and the to_out tail kernel of the head-group path. The block kernel itself is in taq_fused_kernel.h.
#include "taq_fused_kernel.h"

namespace taq {

// ------------------------------------------------------------------------------------------
// K~/V~ image builder: rearranges the codes of qkv_packed into the order the fused kernel's MFMA
// operands are read in, and precomputes the per-head power-of-two prescale of V.
//   per head h:  Kp[t][tile][q][e] = k_code[t][h*d + 16*tile + 4*q + e]         (0 outside d / T; heads with a
//                multiple of 4 tiles use the order [t][tile/4][q][tile%4][e])
//                Vt[j][vt_pos(t)] = v_code[t][h*d + j] ^ 0x80   (vt_pos: 32*s + 8*q + 4*a + e for t = 32*s + 16*a + 4*q + e)
// ------------------------------------------------------------------------------------------
__device__ __forceinline__ int code_at(const uint8_t* codes, size_t row, int C, int c, int bits) {
    if (bits == 8) return (int8_t)codes[row * C + c];
    const int nib = (codes[row * (C >> 1) + (c >> 1)] >> (4 * (c & 1))) & 0xF;
    return (nib ^ 8) - 8;
}

__global__ __launch_bounds__(256) void kv_image_kernel(uint8_t* __restrict__ packed, KvLayout L, KvImage I, int T, int C,
                                                       int H, int bits) {
    const int h = blockIdx.x, b = blockIdx.y, tid = threadIdx.x + 256 * blockIdx.z, nth = 256 * gridDim.z;
    const int d = C / H;
    const int* slot_of = reinterpret_cast<const int*>(packed + L.slot_of) + b * T;
    const float* s_k = reinterpret_cast<const float*>(packed + L.s_k) + ((size_t)b * H + h) * T;
    const float* s_v = reinterpret_cast<const float*>(packed + L.s_v) + ((size_t)b * H + h) * T;
    const uint8_t* k_code = packed + L.k_code;
    const uint8_t* v_code = packed + L.v_code;
    uint8_t* img = packed + L.image + (size_t)b * L.image_bytes + (size_t)h * I.head_bytes;  // this head's block
    __shared__ float vpre_s;
    if (threadIdx.x == 0) {  // (every z-slice recomputes it; only slice 0 stores it)  // per-head prescale: the largest |s_V * code| goes to [256, 512)
        float smax = 0.f;
        for (int t = 0; t < T; ++t)
            if (slot_of[t] < 0) smax = fmaxf(smax, s_v[t]);
        int kexp = 0;
        const float dmax = smax * (bits == 4 ? 7.f : 127.f);
        if (dmax > 0.f) {
            int e;
            (void)frexpf(dmax, &e);
            kexp = 9 - e;
        }
        vpre_s = ldexpf(1.0f, kexp);
        if (blockIdx.z == 0) {
            reinterpret_cast<float*>(img + I.vpre)[0] = ldexpf(1.0f, kexp);
            reinterpret_cast<float*>(img + I.oscale)[0] = ldexpf(1.0f, -kexp);
        }
    }
    __syncthreads();
    for (int t = tid; t < I.ntok; t += nth) {
        const bool isint = t < T && slot_of[t] < 0;
        reinterpret_cast<float*>(img + I.s_k)[t] = isint ? s_k[t] : 0.f;
        const float sp = isint ? s_v[t] * vpre_s : 0.f;  // s' = s_V * 2^kexp as two fp16 numbers, high part and remainder
        const __half sph = __float2half_rn(sp);
        reinterpret_cast<__half*>(img + I.s_vp)[t] = sph;
        reinterpret_cast<__half*>(img + I.s_vp)[I.ntok + t] = __float2half_rn(sp - __half2float(sph));
        reinterpret_cast<float*>(img + I.bias)[t] = isint ? 0.f : TAQ_NEG_INF;
    }
    const int rowb = I.tph * 16;  // bytes per (head, token) row of Kp
    for (int i = tid; i < I.rows_k * rowb; i += nth) {
        const int e = i & 3, q = (i >> 2) & 3, tile = (i % rowb) >> 4, t = i / rowb;
        const int cl = 16 * tile + 4 * q + e;
        int v = 0;
        if (t < T && cl < d && slot_of[t] < 0) v = code_at(k_code, (size_t)b * T + t, C, h * d + cl, bits);
        img[I.kp + kp_offset(I.tph, t, tile, q) + e] = (uint8_t)(v & 0xFF);
    }
    for (int i = tid; i < d * I.cols_v; i += nth) {
        const int t = i % I.cols_v, j = i / I.cols_v;  // token t of channel j goes to position vt_pos(t)
        int v = 0;
        if (t < T && slot_of[t] < 0) v = code_at(v_code, (size_t)b * T + t, C, h * d + j, bits);
        // stored with the sign bit flipped (code + 128 as an unsigned byte): 0x6400 | byte is then the
        // fp16 number 1024 + 128 + code, one packed subtraction away from the code itself
        img[I.vt + (size_t)j * I.cols_v + vt_pos(t, I.nt16)] = (uint8_t)((v & 0xFF) ^ 0x80);
    }
}

hipError_t launch_kv_image(uint8_t* packed, const taq_shape& s, hipStream_t st) {
    const KvLayout L = kv_layout(s);
    if (L.image_bytes == 0) return hipSuccess;
    const KvImage I = kv_image(s);
    hipLaunchKernelGGL(kv_image_kernel, dim3(s.H, s.B, 8), dim3(256), 0, st, packed, L, I, s.T, s.C, s.H, s.bits_kv);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------
// Weight re-layout for the fused kernel (optional, shape.w_layout = 1)
// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void pack_weight_kernel(const int8_t* __restrict__ codes, int C, int d, int tph, int kc,
                                                          size_t pack_off, int8_t* __restrict__ out) {
    // one 16-byte vector per thread: first the row-major copy, then the operand-ordered copy
    const size_t nrow = (size_t)C * C / 16;
    const size_t npack = (size_t)(C / d) * tph * kc * 64;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < nrow + npack; i += (size_t)gridDim.x * 256) {
        if (i < nrow) {
            if (codes != out) reinterpret_cast<uint4*>(out)[i] = reinterpret_cast<const uint4*>(codes)[i];
        } else {
            const size_t v = i - nrow;
            const int lane = (int)(v & 63), r = lane & 15, q = lane >> 4;
            const size_t blk = v >> 6;  // (h * tph + j) * kc + ks
            const int ks = (int)(blk % kc), j = (int)((blk / kc) % tph), h = (int)(blk / ((size_t)kc * tph));
            int row = h * d + 16 * j + r;
            row = row < C ? row : C - 1;
            reinterpret_cast<uint4*>(out + pack_off)[v] =
                *reinterpret_cast<const uint4*>(codes + (size_t)row * C + 64 * ks + 16 * q);
        }
    }
}

hipError_t launch_pack_weight(const int8_t* codes, const taq_shape& s, int8_t* out, hipStream_t st) {
    const int d = s.C / s.H;
    hipLaunchKernelGGL(pack_weight_kernel, dim3(256), dim3(256), 0, st, codes, s.C, d, (d + 15) / 16, s.C / 64,
                       weight_pack_offset(s), out);
    return hipGetLastError();
}

// Per-token quantization of A^ V~ and to_out for the head-group shapes (C = 1280):
// Y^T[c][n] = Wo[c][:] . o_code[n][:]. A workgroup owns 16 TG image tokens and OT output tiles of 16 channels; one
// wavefront per (output tile, token group of 16), so that each wavefront has only C/64 weight loads in front of its
// MFMAs. (TG = 1: what a workgroup pulls through its compute unit's vector memory path, its rows plus one 20 KiB weight
// slice per wavefront, is half of TG = 2's 480 KiB, and that transfer is most of the kernel's time.) FUSEQ: the float32 rows of A^ V~ and the partial row maxima come from the workspace and every workgroup of
// a token tile forms the same int8 codes of its rows (32 threads per row) in LDS: one kernel less, worth it while
// the layer has few token tiles. Otherwise the codes and scales were formed once by the row quantizer kernel.
// Same operand layout and epilogue as the last phase of the fused kernel.
// (At most 128 registers per lane, so that two 8-wavefront workgroups share a compute unit: the 256-token layers have
// 320 workgroups, and with one per compute unit the last 64 of them ran as a second round after the first had finished.)
template <int C, int OT, bool FUSEQ, int TT = 1, int TG = 2>
__global__ __launch_bounds__(64 * OT * TG) __attribute__((amdgpu_waves_per_eu(4, 4)))
void to_out_tail_kernel(FusedTable tab, FusedDims dm) {
    constexpr int KC = C / 64, NT = 64 * OT * TG, TILE_RS = C + 16;
    constexpr int TOKS = 16 * TG * TT;  // image tokens per workgroup: every weight load serves TT token groups of 16
    static_assert(C % 128 == 0, "32 threads per token row");
    static_assert(!FUSEQ || NT == 32 * TOKS, "the in-kernel quantizer maps 32 threads to each row");
    constexpr int CH = C / 128;  // float4 pieces of a row per thread
    extern __shared__ __align__(16) unsigned char smem[];
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, r16 = lane & 15, q = lane >> 4;
    const int gt = (int)blockIdx.z * OT + (wave % OT);  // output tile of the layer: channels 16*gt .. 16*gt+15
    const int tl = (wave / OT) * 16 + r16;              // this lane's token within the 32-token tile
    const int b = blockIdx.x, tile = blockIdx.y;  // (grid: batch element, token tile, group of OT output tiles)
    const FusedReq rq = tab.req[0];
    const int N = dm.N, n0 = tile * TOKS;
    int8_t* tileq = reinterpret_cast<int8_t*>(smem);               // [TOKS][C+16]
    float* s_o = reinterpret_cast<float*>(smem + TOKS * TILE_RS);  // [TOKS]
    // The rows of the tile are requested first: they are needed first (quantizer), and loads return in order; the
    // weights, needed only after the barrier, travel while the rows are quantized.
    const int cr = 16 * gt + r16;
    const int wrow = dm.w_layout ? (int)dm.w_pack_off + (gt * KC) * 1024 + lane * 16 : cr * C + 16 * q;
    const int wstep = dm.w_layout ? 1024 : 64;
    int32x4_t wa[KC];
    if constexpr (!FUSEQ) {
        for (int v = tid; v < TOKS * (C / 16); v += NT) {
            const int tk = v / (C / 16), col = (v % (C / 16)) * 16;
            const int nq = n0 + tk;
            const size_t row = (size_t)b * N + (nq < N ? nq : N - 1);
            *reinterpret_cast<uint4*>(tileq + tk * TILE_RS + col) = *reinterpret_cast<const uint4*>(dm.ws_ocode + row * C + col);
        }
        if (tid < TOKS) {
            const int nq = n0 + tid;
            s_o[tid] = dm.ws_so[(size_t)b * N + (nq < N ? nq : N - 1)];
        }
#pragma unroll
        for (int ks = 0; ks < KC; ++ks) wa[ks] = *reinterpret_cast<const int32x4_t*>(rq.wo + wrow + wstep * ks);
    } else {
        const int tk = tid >> 5, part = tid & 31;  // token of the tile, piece of its row
        const int nq = n0 + tk;
        const size_t row = (size_t)b * N + (nq < N ? nq : N - 1);
        float4 xv[CH];
        const float4* xr = reinterpret_cast<const float4*>(dm.ws_of + row * C);
#pragma unroll
        for (int it = 0; it < CH; ++it) xv[it] = xr[it * 32 + part];
        float amax = 0.f;
        for (int i = part; i < dm.omax_n; i += 32) amax = fmaxf(amax, dm.ws_omax[row * dm.omax_n + i]);
        __builtin_amdgcn_sched_barrier(0);
        // (the first KPRE weight loads now, the rest once the rows' registers are free: 128 registers per lane in all)
        constexpr int KPRE = KC < 12 ? KC : 12;
#pragma unroll
        for (int ks = 0; ks < KPRE; ++ks) wa[ks] = *reinterpret_cast<const int32x4_t*>(rq.wo + wrow + wstep * ks);
        __builtin_amdgcn_sched_barrier(0);
        amax = row16_allmax(amax);
        {   // the other 16 lanes of this token
            const auto sw = __builtin_amdgcn_permlane16_swap(__float_as_uint(amax), __float_as_uint(amax), false, false);
            amax = fmaxf(__uint_as_float(sw[0]), __uint_as_float(sw[1]));
        }
        const bool zero = amax == 0.f;
        const float sc = zero ? 1.f : amax / 127.f;
        const float safe = zero ? 1.f : amax;
        const float cq = 127.f * __builtin_amdgcn_rcpf(safe);
        const bool tap = blockIdx.z == 0 && nq < N;
        if (part == 0) s_o[tk] = sc;
        if (tap && dm.dbg.s_o && part == 0) dm.dbg.s_o[row] = sc;
#pragma unroll
        for (int it = 0; it < CH; ++it) {
            const unsigned pk = quant4_i8(xv[it].x, xv[it].y, xv[it].z, xv[it].w, cq, safe);
            *reinterpret_cast<unsigned*>(tileq + tk * TILE_RS + (it * 32 + part) * 4) = pk;
            if (tap && dm.dbg.o_code) *reinterpret_cast<unsigned*>(dm.dbg.o_code + row * C + (it * 32 + part) * 4) = pk;
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int ks = KPRE; ks < KC; ++ks) wa[ks] = *reinterpret_cast<const int32x4_t*>(rq.wo + wrow + wstep * ks);
    }
    __syncthreads();
    int32x4_t acc[TT];
#pragma unroll
    for (int g = 0; g < TT; ++g) acc[g] = (int32x4_t){0, 0, 0, 0};
#pragma unroll
    for (int ks = 0; ks < KC; ++ks) {
#pragma unroll
        for (int g = 0; g < TT; ++g) {
            const int32x4_t hb = *reinterpret_cast<const int32x4_t*>(tileq + (16 * TG * g + tl) * TILE_RS + 64 * ks + 16 * q);
            acc[g] = __builtin_amdgcn_mfma_i32_16x16x64_i8(wa[ks], hb, acc[g], 0, 0, 0);
        }
    }
    const int c = 16 * gt + 4 * q;
    const float4 w4 = *reinterpret_cast<const float4*>(rq.scales + C + c);
    const float4 b4 = *reinterpret_cast<const float4*>(rq.scales + 2 * C + c);
#pragma unroll
    for (int g = 0; g < TT; ++g) {
        const int n = n0 + 16 * TG * g + tl;
        const size_t tok = (size_t)b * N + (n < N ? n : N - 1);
        const float so = s_o[16 * TG * g + tl];
        const float y0 = (float)acc[g][0] * (so * w4.x) + b4.x;
        const float y1 = (float)acc[g][1] * (so * w4.y) + b4.y;
        const float y2 = (float)acc[g][2] * (so * w4.z) + b4.z;
        const float y3 = (float)acc[g][3] * (so * w4.w) + b4.w;
        if (n < N) {
            const half4_t y = {(_Float16)y0, (_Float16)y1, (_Float16)y2, (_Float16)y3};
            *reinterpret_cast<half4_t*>(rq.out + tok * C + c) = y;
        }
    }
}

template <int C, int OT, bool FUSEQ, int TT, int TG>
static hipError_t launch_tail_cfg(const FusedTable& tab, const FusedDims& dm, hipStream_t st) {
    constexpr int TOKS = 16 * TG * TT;
    const size_t bytes = TOKS * (C + 16) + TOKS * 4;
    static std::atomic<unsigned long long> lds_set{0};
    const hipError_t e = ensure_dynamic_lds(reinterpret_cast<const void*>(&to_out_tail_kernel<C, OT, FUSEQ, TT, TG>), 160 * 1024, lds_set);
    if (e != hipSuccess) return e;
    const int tiles = (dm.N + TOKS - 1) / TOKS;
    if (tiles > 65535) return hipErrorInvalidValue;
    hipLaunchKernelGGL((to_out_tail_kernel<C, OT, FUSEQ, TT, TG>), dim3(dm.B, tiles, C / 16 / OT), dim3(64 * OT * TG), bytes, st, tab, dm);
    return hipGetLastError();
}

hipError_t launch_fused_block(const FusedReq* reqs, int R, const taq_shape& s, const taq_debug* dbg, hipStream_t st,
                              const int8_t* core_qcode, const float* core_sq, float* core_of) {
    if (R < 1 || R > TAQ_MAX_REQ || !fused_supported(s)) return hipErrorInvalidValue;
    if (core_qcode && (R != 1 || !core_sq || !core_of)) return hipErrorInvalidValue;
    FusedTable tab;
    for (int r = 0; r < TAQ_MAX_REQ; ++r) tab.req[r] = reqs[r < R ? r : 0];
    FusedDims dm;
    dm.R = R;
    dm.B = s.B;
    dm.N = s.N;
    dm.T = s.T;
    dm.nt16 = (s.T + 15) / 16;
    dm.w_layout = s.w_layout;
    dm.w_pack_off = (unsigned)weight_pack_offset(s);
    dm.w_bytes = (unsigned)(s.w_layout ? weight_pack_bytes(s) : (size_t)s.C * s.C);
    const int d = s.C / s.H;
    const float sigma = s.softmax_scale != 0.f ? s.softmax_scale : 1.0f / sqrtf((float)d);
    dm.sig2 = sigma * 1.4426950408889634f;
    dm.qmaxq = s.bits_q == 4 ? 7.f : 127.f;
    const bool logp = s.prob_grid == TAQ_PROB_LOG2;
    dm.plast = s.bits_prob == 4 ? 15.f : 255.f;
    dm.pmax = logp ? 256.f : dm.plast;
    dm.L = kv_layout(s);
    dm.I = kv_image(s);
    taq_debug none = {nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, 0u};
    dm.dbg = (dbg && R == 1) ? *dbg : none;
    dm.ws_of = core_of;
    dm.ws_omax = nullptr;
    dm.omax_n = 0;
    dm.core_qcode = core_qcode;
    dm.core_sq = core_sq;
    dm.ws_ocode = nullptr;
    dm.ws_so = nullptr;
    const int grid = s.prob_grid;
    if (core_qcode) {  // the attention core alone, from Q~ codes and scales in the workspace to float32 A^ V~
        if (d == 40 && s.H == 8) return launch_fused_d40(tab, dm, grid, 32, true, st);
        if (d == 80 && s.H == 8) return launch_fused_d80(tab, dm, grid, 32, true, st);
        if (d == 64 && s.H == 10) return launch_fused_d64(tab, dm, grid, 32, true, st);
        return hipErrorInvalidValue;
    }
    // 32-token tiles that would occupy under half of the 256 compute units: 16-token workgroups instead
    // (shape.tok_tile = 32 or 16 forces one variant: for tests and tuning)
    const bool few = s.tok_tile == 16 ? true : s.tok_tile == 32 ? false : ((s.N + 31) / 32) * R * s.B <= 128;
    const int tok = few ? 16 : 32;
    if (d == 40 && s.H == 8) return launch_fused_d40(tab, dm, grid, tok, false, st);
    if (d == 80 && s.H == 8) return launch_fused_d80(tab, dm, grid, tok, false, st);
    if (d == 64 && s.H == 10) return launch_fused_d64(tab, dm, grid, tok, false, st);
    return hipErrorInvalidValue;
}

// Head-group variant for layers too wide for one workgroup (C = 1280): per-token codes of `hidden`, to_q, Q~ and the
// attention per head group; A^ V~ (float32) and the partial row maxima go to the workspace.
static int mid_omax_n(const taq_shape& s) { return s.H * (s.C / s.H == 160 ? 4 : 2); }

hipError_t launch_fused_mid(const FusedReq& rq, const taq_shape& s, float* o_f, float* o_max, const taq_debug* dbg,
                            hipStream_t st) {
    if (!mid_supported(s)) return hipErrorInvalidValue;
    FusedTable tab;
    for (int r = 0; r < TAQ_MAX_REQ; ++r) tab.req[r] = rq;
    FusedDims dm;
    dm.R = 1;
    dm.B = s.B;
    dm.N = s.N;
    dm.T = s.T;
    dm.nt16 = (s.T + 15) / 16;
    dm.w_layout = s.w_layout;
    dm.w_pack_off = (unsigned)weight_pack_offset(s);
    dm.w_bytes = (unsigned)(s.w_layout ? weight_pack_bytes(s) : (size_t)s.C * s.C);
    const int d = s.C / s.H;
    const float sigma = s.softmax_scale != 0.f ? s.softmax_scale : 1.0f / sqrtf((float)d);
    dm.sig2 = sigma * 1.4426950408889634f;
    dm.qmaxq = s.bits_q == 4 ? 7.f : 127.f;
    const bool logp = s.prob_grid == TAQ_PROB_LOG2;
    dm.plast = s.bits_prob == 4 ? 15.f : 255.f;
    dm.pmax = logp ? 256.f : dm.plast;
    dm.L = kv_layout(s);
    dm.I = kv_image(s);
    taq_debug none = {nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, 0u};
    dm.dbg = dbg ? *dbg : none;
    dm.dbg.o_code = nullptr;  // taps of the stages this kernel does not run are written by the kernel that runs them
    dm.dbg.s_o = nullptr;
    dm.ws_of = o_f;
    dm.ws_omax = o_max;
    dm.omax_n = mid_omax_n(s);
    dm.core_qcode = nullptr;
    dm.core_sq = nullptr;
    dm.ws_ocode = nullptr;
    dm.ws_so = nullptr;
    // 16-token workgroups (all eight wavefronts load, four carry on with the attention) unless the layer is large:
    // measured faster up to 640 workgroups of 32 tokens (SDXL 1024-token layer, batch 2: 36.4 -> 33.6 us), not
    // measured beyond (shape.tok_tile = 32 or 16 forces one variant: for tests and tuning)
    const bool few = s.tok_tile == 16 ? true : s.tok_tile == 32 ? false : ((s.N + 31) / 32) * s.B * (d == 160 ? 8 : 10) <= 1024;
    if (d == 160 && s.H == 8) return launch_fused_mid160(tab, dm, s.prob_grid, few ? 16 : 32, st);
    if (d == 64 && s.H == 20) return launch_fused_mid64(tab, dm, s.prob_grid, few ? 16 : 32, st);
    return hipErrorInvalidValue;
}

// to_out for the head-group shapes: from the float32 rows of A^ V~ and their partial maxima in the workspace (o_code ==
// NULL: the kernel forms the per-token codes itself), or from codes and scales a separate kernel formed.
hipError_t launch_to_out_tail(const FusedReq& rq, const taq_shape& s, const float* o_f, const float* o_max,
                              const int8_t* o_code, const float* s_o, const taq_debug* dbg, hipStream_t st) {
    if (!mid_supported(s)) return hipErrorInvalidValue;
    FusedTable tab;
    for (int r = 0; r < TAQ_MAX_REQ; ++r) tab.req[r] = rq;
    FusedDims dm = {};
    dm.R = 1;
    dm.B = s.B;
    dm.N = s.N;
    dm.T = s.T;
    dm.w_layout = s.w_layout;
    dm.w_pack_off = (unsigned)weight_pack_offset(s);
    dm.w_bytes = (unsigned)(s.w_layout ? weight_pack_bytes(s) : (size_t)s.C * s.C);
    taq_debug none = {nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, 0u};
    dm.dbg = dbg ? *dbg : none;
    dm.ws_of = const_cast<float*>(o_f);
    dm.ws_omax = const_cast<float*>(o_max);
    dm.omax_n = mid_omax_n(s);
    dm.ws_ocode = o_code;
    dm.ws_so = s_o;
    // codes from the row quantizer (large layers): 64 tokens per workgroup, so that a weight load serves four token groups
    if (s.C == 1280) return o_code ? launch_tail_cfg<1280, 8, false, 3, 1>(tab, dm, st) : launch_tail_cfg<1280, 8, true, 1, 1>(tab, dm, st);
    return hipErrorInvalidValue;
}

}  // namespace taq