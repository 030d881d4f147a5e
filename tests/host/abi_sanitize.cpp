// Host-side exercise of the C ABI for AddressSanitizer / UBSan builds of the library's host code: argument checks,
// size and layout queries over many shapes, the batched table validation, the static-scratch size limit. Nothing here
// reaches a kernel launch (every call either is host-only or is rejected first), so it runs without a GPU.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "taq.h"

#define CHECK(cond)                                                        \
    do {                                                                   \
        if (!(cond)) {                                                     \
            std::fprintf(stderr, "%s:%d: check failed: %s\n", __FILE__, __LINE__, #cond); \
            std::exit(1);                                                  \
        }                                                                  \
    } while (0)

static taq_shape shape(int B, int N, int C, int H, int T, int Cc, int bkv = 8) {
    taq_shape s = {};
    s.B = B; s.N = N; s.C = C; s.H = H; s.T = T; s.Cc = Cc;
    s.bits_kv = bkv; s.bits_prob = 8; s.bits_q = 8; s.bits_proj = 8;
    return s;
}

int main() {
    void* fake = reinterpret_cast<void*>(0x7F0000001000ull);  // aligned, never dereferenced on error paths
    void* odd = reinterpret_cast<void*>(0x7F0000001004ull);
    const uint8_t* fm = static_cast<const uint8_t*>(fake);   // typed views of the same fake address
    const int8_t* fi = static_cast<const int8_t*>(fake);
    const float* ff = static_cast<const float*>(fake);
    // ---- size and layout queries over a grid of shapes (valid and invalid)
    unsigned long long seen = 0;
    const int Cs[] = {64, 96, 320, 640, 1280, 324, 2048}, Hs[] = {1, 2, 4, 8, 10, 20, 64, 65}, Ts[] = {1, 13, 77, 96, 97};
    for (int C : Cs) for (int H : Hs) for (int T : Ts) for (int bkv : {4, 8, 16, 5}) for (int bp : {8, 16}) {
        taq_shape s = shape(2, 100, C, H, T, 768, bkv);
        s.bits_proj = bp;
        size_t kvb = 0, wsb = 0, wb = 0, ko = 0, vo = 0, rb = 0;
        const int rc = taq_kv_packed_bytes(&s, &kvb);
        CHECK(rc <= 0);
        CHECK(taq_workspace_bytes(&s, &wsb) == rc);
        CHECK(taq_weight_bytes(&s, &wb) == rc);
        CHECK(taq_kv_code_layout(&s, &ko, &vo, &rb) == rc);
        if (rc == TAQ_OK) {
            ++seen;
            CHECK(kvb % 256 == 0 && wsb % 256 == 0 && wb >= (size_t)C * C);
            CHECK(rb == (bkv == 8 ? (size_t)C : bkv == 4 ? (size_t)C / 2 : 0u));
            CHECK(ko <= vo && vo + 2 * (size_t)T * rb <= kvb);
        }
        CHECK(taq_status_string(rc) != nullptr);
    }
    CHECK(seen > 50);
    // ---- argument checks of the entry points (no launch)
    taq_shape s = shape(1, 64, 320, 8, 77, 768);
    CHECK(taq_kv_packed_bytes(nullptr, nullptr) == TAQ_ERR_INVALID_ARG);
    CHECK(taq_quantize_kv(nullptr, fm, fake, fake, 8, &s, fake, fake, nullptr) == TAQ_ERR_INVALID_ARG);
    CHECK(taq_quantize_kv(fake, fm, fake, fake, 4, &s, fake, fake, nullptr) == TAQ_ERR_INVALID_ARG);
    CHECK(taq_quantize_kv(odd, fm, fake, fake, 8, &s, fake, fake, nullptr) == TAQ_ERR_MISALIGNED);
    CHECK(taq_quantize_kv_w8(fake, fm, nullptr, nullptr, 8, &s, fake, fake, nullptr) == TAQ_ERR_INVALID_ARG);
    CHECK(taq_cross_attn(fake, fake, fi, fi, ff, nullptr, &s, nullptr, fake, nullptr) == TAQ_ERR_INVALID_ARG);
    CHECK(taq_cross_attn(fake, fake, fi, static_cast<const int8_t*>(odd), ff, nullptr, &s, fake, fake, nullptr) == TAQ_ERR_MISALIGNED);
    CHECK(taq_cross_attn_ex(fake, fake, fi, fi, ff, nullptr, nullptr, fake, fake, nullptr, nullptr) == TAQ_ERR_INVALID_ARG);
    taq_shape big = shape(2, 4096, 1280, 8, 77, 768);
    CHECK(taq_cross_attn_static(fake, fake, fi, fi, ff, nullptr, &big, fake, nullptr) == TAQ_ERR_SCRATCH_TOO_SMALL);
    CHECK(taq_cross_attn_static(fake, fake, fi, fi, ff, nullptr, &s, nullptr, nullptr) == TAQ_ERR_INVALID_ARG);
    CHECK(taq_quantize_weight(fake, 8, 60, const_cast<int8_t*>(fi), const_cast<float*>(ff), nullptr) == TAQ_ERR_BAD_SHAPE);
    CHECK(taq_pack_weight(fi, &s, static_cast<int8_t*>(odd), nullptr) == TAQ_ERR_MISALIGNED);
    CHECK(taq_unpack_kv(nullptr, &s, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr) == TAQ_ERR_INVALID_ARG);
    CHECK(taq_mse_f16(fake, fake, 0, static_cast<double*>(fake), nullptr) == TAQ_ERR_INVALID_ARG);
    // ---- batched call: every request is validated before anything is launched
    std::vector<taq_request> tab(33);
    for (auto& q : tab) q = taq_request{fake, fake, fi, fi, ff, nullptr, fake};
    tab[32].out = nullptr;
    CHECK(taq_cross_attn_batched(33, tab.data(), &s, fake, nullptr) == TAQ_ERR_INVALID_ARG);
    tab[32].out = odd;
    CHECK(taq_cross_attn_batched(33, tab.data(), &s, fake, nullptr) == TAQ_ERR_MISALIGNED);
    CHECK(taq_cross_attn_batched(0, tab.data(), &s, fake, nullptr) == TAQ_ERR_INVALID_ARG);
    std::puts("abi_sanitize: ok");
    return 0;
}
