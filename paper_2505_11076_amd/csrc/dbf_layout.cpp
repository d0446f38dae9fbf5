// Host-side sign packing and the gfx950 tile layout (no GPU calls in this file).
//
// A rows x cols sign matrix (reduction over cols) is stored on the device as tiles of
// 128 rows x 64 cols, 1024 bytes each, row-tile major.  Byte (256*g + 16*r + j) of a tile
// holds in bit s the sign of tile element (row 16*s + r, col 16*g + j).  One wavefront
// reads a tile with a single 16-byte load per lane (lane = 16*g + r): every lane then owns
// sixteen consecutive columns, one per byte, and the eight bits of each byte belong to the
// eight 16-row groups of the tile.  Masking all bytes with (1 << s) therefore yields, with
// one AND per register, the operand of an int8 matrix-core instruction for row group s.
#include "dbf_internal.h"

#include <cstring>

namespace {

// Transpose an 8x8 bit matrix held in a uint64: bit (8*i + j) <-> bit (8*j + i).
inline uint64_t transpose8x8(uint64_t x) {
    uint64_t t;
    t = (x ^ (x >> 7)) & 0x00AA00AA00AA00AAull;
    x = x ^ t ^ (t << 7);
    t = (x ^ (x >> 14)) & 0x0000CCCC0000CCCCull;
    x = x ^ t ^ (t << 14);
    t = (x ^ (x >> 28)) & 0x00000000F0F0F0F0ull;
    x = x ^ t ^ (t << 28);
    return x;
}

inline bool dims_ok(int rows, int cols) {
    return rows >= 1 && cols >= 1 && rows <= DBF_MAX_DIM && cols <= DBF_MAX_DIM;
}

}  // namespace

extern "C" size_t dbf_tiled_bytes(int rows, int cols) {
    if (!dims_ok(rows, cols)) return 0;
    return (size_t)dbf_row_tiles(rows) * (size_t)dbf_col_tiles(cols) * DBF_TILE_BYTES;
}

extern "C" int dbf_signs_to_bits_host(int rows, int cols, const int8_t* pm1, uint32_t* bits) {
    if (!pm1 || !bits) return DBF_EINVAL;
    if (!dims_ok(rows, cols)) return DBF_ESHAPE;
    const int wpr = (cols + 31) / 32;
    for (int r = 0; r < rows; ++r) {
        const int8_t* src = pm1 + (size_t)r * cols;
        uint32_t* dst = bits + (size_t)r * wpr;
        for (int w = 0; w < wpr; ++w) {
            const int c0 = w * 32;
            const int n = (cols - c0 < 32) ? (cols - c0) : 32;
            uint32_t word = 0;
            for (int i = 0; i < n; ++i) {
                const int8_t v = src[c0 + i];
                if (v == 1)
                    word |= (1u << i);
                else if (v != -1)
                    return DBF_ENOTSIGN;
            }
            dst[w] = word;
        }
    }
    return DBF_OK;
}

extern "C" int dbf_tile_host(int rows, int cols, const uint32_t* bits, uint8_t* tiled) {
    if (!bits || !tiled) return DBF_EINVAL;
    if (!dims_ok(rows, cols)) return DBF_ESHAPE;
    const int wpr = (cols + 31) / 32;
    const int n_rt = dbf_row_tiles(rows), n_ct = dbf_col_tiles(cols);
    if (cols & 31) {  // unused tail bits must be clean
        const uint32_t keep = (1u << (cols & 31)) - 1u;
        for (int r = 0; r < rows; ++r)
            if (bits[(size_t)r * wpr + wpr - 1] & ~keep) return DBF_ENOTSIGN;
    }
    for (int rt = 0; rt < n_rt; ++rt) {
        for (int ct = 0; ct < n_ct; ++ct) {
            uint8_t* tile = tiled + ((size_t)rt * n_ct + ct) * DBF_TILE_BYTES;
            for (int r = 0; r < 16; ++r) {
                uint64_t v[8];  // the 64 columns of this tile for rows 16*s + r
                for (int s = 0; s < 8; ++s) {
                    const int row = rt * 128 + 16 * s + r;
                    uint64_t lo = 0, hi = 0;
                    if (row < rows) {
                        const uint32_t* src = bits + (size_t)row * wpr;
                        if (2 * ct < wpr) lo = src[2 * ct];
                        if (2 * ct + 1 < wpr) hi = src[2 * ct + 1];
                    }
                    v[s] = lo | (hi << 32);
                }
                for (int byte = 0; byte < 8; ++byte) {  // columns 8*byte .. 8*byte+7
                    uint64_t x = 0;
                    for (int s = 0; s < 8; ++s) x |= ((v[s] >> (8 * byte)) & 0xFFull) << (8 * s);
                    x = transpose8x8(x);  // byte i of x: column 8*byte+i, bit s: row group s
                    const int g = byte >> 1, j0 = (byte & 1) * 8;
                    std::memcpy(tile + 256 * g + 16 * r + j0, &x, 8);
                }
            }
        }
    }
    return DBF_OK;
}

extern "C" int dbf_untile_host(int rows, int cols, const uint8_t* tiled, uint32_t* bits) {
    if (!bits || !tiled) return DBF_EINVAL;
    if (!dims_ok(rows, cols)) return DBF_ESHAPE;
    const int wpr = (cols + 31) / 32;
    const int n_rt = dbf_row_tiles(rows), n_ct = dbf_col_tiles(cols);
    for (int rt = 0; rt < n_rt; ++rt) {
        for (int ct = 0; ct < n_ct; ++ct) {
            const uint8_t* tile = tiled + ((size_t)rt * n_ct + ct) * DBF_TILE_BYTES;
            for (int r = 0; r < 16; ++r) {
                uint64_t v[8] = {0, 0, 0, 0, 0, 0, 0, 0};
                for (int byte = 0; byte < 8; ++byte) {
                    const int g = byte >> 1, j0 = (byte & 1) * 8;
                    uint64_t x;
                    std::memcpy(&x, tile + 256 * g + 16 * r + j0, 8);
                    x = transpose8x8(x);  // byte s of x: row group s, bit i: column 8*byte+i
                    for (int s = 0; s < 8; ++s) v[s] |= ((x >> (8 * s)) & 0xFFull) << (8 * byte);
                }
                for (int s = 0; s < 8; ++s) {
                    const int row = rt * 128 + 16 * s + r;
                    if (row >= rows) continue;
                    uint32_t* dst = bits + (size_t)row * wpr;
                    if (2 * ct < wpr) dst[2 * ct] = (uint32_t)v[s];
                    if (2 * ct + 1 < wpr) dst[2 * ct + 1] = (uint32_t)(v[s] >> 32);
                }
            }
        }
    }
    return DBF_OK;
}
