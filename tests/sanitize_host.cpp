// Host-side sanitizer check of libdbf: the sign packer / tile layout (dbf_layout.cpp) and the
// argument-validation paths of the C ABI (dbf_api.hip and the entry points beside it), compiled with
// -fsanitize=address,undefined for the host and run on the CPU.  Every buffer is heap allocated at exactly
// the size the header documents, so a read or write past an end, a shift by too much or a misaligned
// access in the host code ends the program with a sanitizer report.  No kernel is launched: every call
// here either is host-only or must return its error code before touching the GPU.
//
// Built and run by tests/test_boundary_cpu.py (paper_2505_11076_amd/build.py: build_sanitize_check).
#include <climits>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "../include/dbf.h"

static int failures = 0;
#define EXPECT(cond)                                                        \
    do {                                                                    \
        if (!(cond)) {                                                      \
            std::fprintf(stderr, "line %d: %s\n", __LINE__, #cond);         \
            ++failures;                                                     \
        }                                                                   \
    } while (0)

static uint32_t rng_state = 12345u;
static uint32_t rnd() {  // xorshift32
    rng_state ^= rng_state << 13;
    rng_state ^= rng_state >> 17;
    rng_state ^= rng_state << 5;
    return rng_state;
}

// signs -> words -> tiles -> words, on exact-size heap buffers
static void layout_round_trip(int rows, int cols) {
    const size_t wpr = ((size_t)cols + 31) / 32;
    std::vector<int8_t> pm1((size_t)rows * cols);
    for (auto& v : pm1) v = (rnd() & 1) ? 1 : -1;
    uint32_t* bits = static_cast<uint32_t*>(std::malloc(sizeof(uint32_t) * rows * wpr));
    uint32_t* back = static_cast<uint32_t*>(std::malloc(sizeof(uint32_t) * rows * wpr));
    const size_t tb = dbf_tiled_bytes(rows, cols);
    EXPECT(tb == (size_t)((rows + 127) / 128) * ((cols + 63) / 64) * 1024);
    uint8_t* tiled = static_cast<uint8_t*>(std::malloc(tb));
    EXPECT(dbf_signs_to_bits_host(rows, cols, pm1.data(), bits) == DBF_OK);
    for (int r = 0; r < rows; ++r)
        for (int c = 0; c < cols; ++c)
            EXPECT((((bits[r * wpr + c / 32] >> (c % 32)) & 1u) == 1u) == (pm1[(size_t)r * cols + c] == 1));
    if (cols % 32) EXPECT((bits[wpr - 1] >> (cols % 32)) == 0u);
    EXPECT(dbf_tile_host(rows, cols, bits, tiled) == DBF_OK);
    // the documented position of every sign: byte 256 g + 16 r + j of its tile, bit s
    const int n_ct = (cols + 63) / 64;
    for (int r = 0; r < rows; r += (rows > 64 ? 7 : 1))
        for (int c = 0; c < cols; c += (cols > 64 ? 5 : 1)) {
            const uint8_t* tile = tiled + ((size_t)(r / 128) * n_ct + c / 64) * 1024;
            const int rr = r % 128, cc = c % 64;
            const int byte = 256 * (cc / 16) + 16 * (rr % 16) + cc % 16, s = rr / 16;
            EXPECT((((tile[byte] >> s) & 1) == 1) == (pm1[(size_t)r * cols + c] == 1));
        }
    std::memset(back, 0xEE, sizeof(uint32_t) * rows * wpr);
    EXPECT(dbf_untile_host(rows, cols, tiled, back) == DBF_OK);
    EXPECT(std::memcmp(bits, back, sizeof(uint32_t) * rows * wpr) == 0);
    if (cols % 32) {  // dirty tail bits are refused
        bits[wpr - 1] |= 0x80000000u;
        EXPECT(dbf_tile_host(rows, cols, bits, tiled) == DBF_ENOTSIGN);
    }
    pm1[pm1.size() - 1] = 0;  // not a sign
    EXPECT(dbf_signs_to_bits_host(rows, cols, pm1.data(), bits) == DBF_ENOTSIGN);
    std::free(bits);
    std::free(back);
    std::free(tiled);
}

int main() {
    const int shapes[][2] = {{1, 1}, {3, 5}, {16, 64}, {17, 65}, {128, 64}, {129, 63}, {130, 2985}, {300, 97}, {257, 640}};
    for (const auto& sh : shapes) layout_round_trip(sh[0], sh[1]);
    EXPECT(dbf_tiled_bytes(0, 4) == 0 && dbf_tiled_bytes(4, (1 << 20) + 1) == 0 && dbf_tiled_bytes(-3, 4) == 0);
    uint32_t w = 0;
    uint8_t t8 = 0;
    int8_t s8 = 1;
    EXPECT(dbf_signs_to_bits_host(1, 1, nullptr, &w) == DBF_EINVAL);
    EXPECT(dbf_signs_to_bits_host(0, 1, &s8, &w) == DBF_ESHAPE);
    EXPECT(dbf_tile_host(1, 1, nullptr, &t8) == DBF_EINVAL && dbf_untile_host(1, 0, &t8, &w) == DBF_ESHAPE);

    // ---- argument validation of the device entry points: all of these return before any GPU call
    const int n_in = 40, n_out = 24, k = 33;
    std::vector<int8_t> A((size_t)n_out * k, 1), Bm((size_t)k * n_in, -1);
    std::vector<uint16_t> a(n_out, 0x3C00), m(k, 0x3C00), b(n_in, 0x3C00);
    dbf_layer* L = reinterpret_cast<dbf_layer*>(0x1);
    EXPECT(dbf_pack(n_in, n_out, k, nullptr, Bm.data(), a.data(), m.data(), b.data(), &L) == DBF_EINVAL && L == nullptr);
    EXPECT(dbf_pack(n_in, n_out, k, A.data(), Bm.data(), a.data(), m.data(), b.data(), nullptr) == DBF_EINVAL);
    EXPECT(dbf_pack(0, n_out, k, A.data(), Bm.data(), a.data(), m.data(), b.data(), &L) == DBF_ESHAPE);
    EXPECT(dbf_pack(n_in, n_out, (1 << 20) + 1, A.data(), Bm.data(), a.data(), m.data(), b.data(), &L) == DBF_ESHAPE);
    Bm[Bm.size() - 1] = 3;
    EXPECT(dbf_pack(n_in, n_out, k, A.data(), Bm.data(), a.data(), m.data(), b.data(), &L) == DBF_ENOTSIGN);
    Bm[Bm.size() - 1] = -1;
    std::vector<uint32_t> Ab((size_t)n_out * 2, 0xFFFFFFFFu), Bb((size_t)k * 2, 0u);
    EXPECT(dbf_pack_bits(n_in, n_out, k, Ab.data(), Bb.data(), a.data(), m.data(), b.data(), &L) == DBF_ENOTSIGN);
    for (int r = 0; r < n_out; ++r) Ab[2 * r + 1] = 1u;  // k = 33: one valid bit in the second word
    // valid operands: packs on a machine with a GPU, DBF_EHIP without one -- never anything else
    int rc = dbf_pack_bits(n_in, n_out, k, Ab.data(), Bb.data(), a.data(), m.data(), b.data(), &L);
    EXPECT(rc == DBF_OK || rc == DBF_EHIP);
    if (rc == DBF_OK) {
        int d[3] = {0, 0, 0};
        size_t bytes = 0;
        EXPECT(dbf_dims(L, &d[0], &d[1], &d[2], &bytes) == DBF_OK && d[0] == n_in && d[1] == n_out && d[2] == k);
        EXPECT(dbf_gemv(L, nullptr, &t8, 1, nullptr) == DBF_EINVAL);
        EXPECT(dbf_gemv(L, &t8, &t8, 0, nullptr) == DBF_EINVAL && dbf_gemv(L, &t8, &t8, DBF_MAX_BATCH + 1, nullptr) == DBF_EINVAL);
        EXPECT(dbf_gemv_kind(L, &t8, &t8, 1, 9, nullptr) == DBF_EINVAL);
        EXPECT(dbf_gemm(L, &t8, &t8, 4, nullptr, 1 << 20, nullptr) == DBF_EWORKSPACE);
        const dbf_layer* twice[2] = {L, L};
        dbf_stack* S = nullptr;
        EXPECT(dbf_stack_create(twice, 2, &S) == DBF_EINVAL && S == nullptr);
        int32_t keep_bad[2] = {5, 5};
        dbf_layer* P = nullptr;
        EXPECT(dbf_prune_middle(L, keep_bad, 2, &P) == DBF_EINVAL && P == nullptr);
        dbf_free(L);
    } else {
        EXPECT(L == nullptr);
    }
    EXPECT(dbf_gemv(nullptr, &t8, &t8, 1, nullptr) == DBF_EINVAL);
    EXPECT(dbf_gemm(nullptr, &t8, &t8, 1, &t8, 1, nullptr) == DBF_EINVAL);
    EXPECT(dbf_gemm_workspace_bytes(nullptr, 4) == 0);
    EXPECT(dbf_unpack_bits(nullptr, nullptr, nullptr, nullptr, nullptr, nullptr) == DBF_EINVAL);
    dbf_stack* S = reinterpret_cast<dbf_stack*>(0x1);
    EXPECT(dbf_stack_create(nullptr, 1, &S) == DBF_EINVAL && S == nullptr);
    const dbf_layer* none[1] = {nullptr};
    EXPECT(dbf_stack_create(none, 1, &S) == DBF_EINVAL);
    int groups[1] = {1};
    EXPECT(dbf_stack_create_grouped(none, 1, groups, 1, &S) == DBF_EINVAL);
    EXPECT(dbf_stack_gemv(nullptr, &t8, &t8, 1, 0, nullptr) == DBF_EINVAL);
    EXPECT(dbf_stack_offsets(nullptr, 0, 1, nullptr, nullptr) == DBF_EINVAL);
    EXPECT(dbf_prune_middle(nullptr, nullptr, 1, &L) == DBF_EINVAL);
    EXPECT(dbf_svid(nullptr, 4, 4, 1, nullptr, nullptr, nullptr, nullptr, 0, nullptr) == DBF_EINVAL);
    EXPECT(dbf_svid_workspace_bytes(0, 4) == 0 && dbf_svid_workspace_bytes(64, 64) > 0);
    EXPECT(dbf_admm_step(nullptr, nullptr, 4, 4, 1.f, 1, nullptr, nullptr, nullptr, nullptr, nullptr, 0, nullptr) == DBF_EINVAL);
    EXPECT(dbf_admm_workspace_bytes(4, 0) == 0);
    EXPECT(dbf_probe_read(nullptr, 1 << 20, nullptr, nullptr) == DBF_EINVAL);
    dbf_free(nullptr);
    dbf_stack_free(nullptr);

    // ---- tuning hooks
    dbf_tuning_reset();
    EXPECT(dbf_tuning_get(DBF_TUNE_WAIT_LIMIT_US) == 250000 && dbf_tuning_get(DBF_TUNE_COUNT_) == INT_MIN);
    EXPECT(dbf_tuning_set(DBF_TUNE_COUNT_, 0) == DBF_EINVAL && dbf_tuning_set(-1, 0) == DBF_EINVAL);
    EXPECT(dbf_tuning_set(DBF_TUNE_COL_PIECES, 65) == DBF_EINVAL && dbf_tuning_set(DBF_TUNE_COL_PIECES, 4) == DBF_OK);
    EXPECT(dbf_tuning_get(DBF_TUNE_COL_PIECES) == 4);
    dbf_tuning_reset();
    EXPECT(dbf_tuning_get(DBF_TUNE_COL_PIECES) == -1);
    for (int code = 1; code >= -8; --code) EXPECT(dbf_strerror(code) != nullptr && dbf_strerror(code)[0] != 0);

    if (failures) {
        std::fprintf(stderr, "sanitize_host: %d expectation(s) failed\n", failures);
        return 1;
    }
    std::puts("sanitize_host: ok");
    return 0;
}
