// Host-side packers: logical row-major arrays -> the tile-major stored formats of eora.h.
// Each output word is produced by gathering the codes it holds (word-walk direction).
#include "eora.h"

#include <cstring>

namespace {

bool shape_ok(int rows, int K, int KT) { return rows > 0 && K > 0 && rows % 16 == 0 && K % KT == 0; }

// 4-bit tiles with k-tile KT (128 or 64).
int pack_q4_tiles(const uint8_t* codes, int rows, int K, int KT, uint32_t* out)
{
    const int wpl = KT / 32, ntk = K / KT, cpl = KT / 4;
    const size_t nwords = (size_t)rows * K / 8;
    for (size_t w = 0; w < nwords; ++w) {
        const size_t tile = w / (64 * wpl);
        const int rem = (int)(w % (64 * wpl));
        const int lane = rem / wpl, t = rem % wpl;
        const int R = (int)(tile / ntk), g = (int)(tile % ntk);
        const int j = lane / 16, n = lane % 16;
        const uint8_t* src = codes + (size_t)(16 * R + n) * K + (size_t)g * KT + j * cpl + 8 * t;
        uint32_t word = 0;
        for (int kk = 0; kk < 8; ++kk) {
            if (src[kk] > 15) return EORA_ERR_VALUE;
            const int e = 4 * (kk % 2) + kk / 2;
            word |= (uint32_t)src[kk] << (4 * e);
        }
        out[w] = word;
    }
    return EORA_OK;
}

int pack_q3_tiles(const uint8_t* codes, int rows, int K, uint32_t* out)
{
    const int ntk = K / 128;
    const size_t nlanes = (size_t)rows * K / 32;
    for (size_t L = 0; L < nlanes; ++L) {
        const size_t tile = L / 64;
        const int lane = (int)(L % 64);
        const int R = (int)(tile / ntk), g = (int)(tile % ntk);
        const int j = lane / 16, n = lane % 16;
        const uint8_t* src = codes + (size_t)(16 * R + n) * K + (size_t)g * 128 + 32 * j;
        uint32_t d[3] = {0, 0, 0};
        for (int cc = 0; cc < 32; ++cc) {
            const uint32_t q = src[cc];
            if (q > 7) return EORA_ERR_VALUE;
            if (cc < 30) {
                const int p = cc / 2, h = cc % 2;
                d[p / 5] |= q << (16 * h + 3 * (p % 5));
            } else {
                const int h = cc - 30;
                for (int b = 0; b < 3; ++b) d[b] |= ((q >> b) & 1u) << (16 * h + 15);
            }
        }
        out[3 * L + 0] = d[0];
        out[3 * L + 1] = d[1];
        out[3 * L + 2] = d[2];
    }
    return EORA_OK;
}

int pack_q2_tiles(const uint8_t* codes, int rows, int K, uint32_t* out)
{
    const int ntk = K / 128;
    const size_t nlanes = (size_t)rows * K / 32;
    for (size_t L = 0; L < nlanes; ++L) {
        const size_t tile = L / 64;
        const int lane = (int)(L % 64);
        const int R = (int)(tile / ntk), g = (int)(tile % ntk);
        const int j = lane / 16, n = lane % 16;
        const uint8_t* src = codes + (size_t)(16 * R + n) * K + (size_t)g * 128 + 32 * j;
        for (int u = 0; u < 2; ++u) {
            uint32_t word = 0;
            for (int c = 0; c < 16; ++c) {
                const uint32_t q = src[16 * u + c];
                if (q > 3) return EORA_ERR_VALUE;
                word |= q << (16 * (c % 2) + 2 * (c / 2));      // pair c/2: even column low half, odd column high half
            }
            out[2 * L + u] = word;
        }
    }
    return EORA_OK;
}

// scales are stored as they come: row-major rows x NG
void pack_scale_tiles(const uint16_t* scales, int rows, int NG, uint16_t* out)
{
    std::memcpy(out, scales, (size_t)rows * NG * sizeof(uint16_t));
}

}  // namespace

extern "C" {

size_t eora_qweight_bytes(int d_in, int d_out, int w_bits)
{
    if (!shape_ok(d_out, d_in, 128) || w_bits < 2 || w_bits > 4) return 0;
    return (size_t)d_out * d_in * w_bits / 8;
}

size_t eora_qzeros_bytes(int d_in, int d_out, int group)
{
    if (!shape_ok(d_out, d_in, 128) || group <= 0 || group % 128 || d_in % group) return 0;
    return (size_t)d_out * ((d_in / group + 7) / 8) * 4;
}

size_t eora_scales_bytes(int d_in, int d_out, int group)
{
    if (!shape_ok(d_out, d_in, 128) || group <= 0 || group % 128 || d_in % group) return 0;
    return (size_t)d_out * (d_in / group) * 2;
}

size_t eora_sp24_values_bytes(int d_in, int d_out)
{
    return shape_ok(d_out, d_in, 128) ? (size_t)d_out * d_in : 0;
}

size_t eora_sp24_indices_bytes(int d_in, int d_out)
{
    return shape_ok(d_out, d_in, 128) ? (size_t)d_out * d_in / 8 : 0;
}

int eora_pack_q(const uint8_t* codes, const uint8_t* zeros, const uint16_t* scales,
                int d_in, int d_out, int w_bits, int group,
                void* qweight_out, void* qzeros_out, void* scales_out)
{
    if (!codes || !zeros || !scales || !qweight_out || !qzeros_out || !scales_out) return EORA_ERR_NULL;
    if (w_bits < 2 || w_bits > 4) return EORA_ERR_UNSUPPORTED;
    if (!shape_ok(d_out, d_in, 128) || group <= 0 || group % 128 || d_in % group) return EORA_ERR_SHAPE;
    const int NG = d_in / group;
    const int zmax = (1 << w_bits) - 1;
    for (size_t i = 0; i < (size_t)d_out * NG; ++i)
        if (zeros[i] > zmax) return EORA_ERR_VALUE;
    int rc = (w_bits == 4)   ? pack_q4_tiles(codes, d_out, d_in, 128, (uint32_t*)qweight_out)
             : (w_bits == 3) ? pack_q3_tiles(codes, d_out, d_in, (uint32_t*)qweight_out)
                             : pack_q2_tiles(codes, d_out, d_in, (uint32_t*)qweight_out);
    if (rc != EORA_OK) return rc;
    uint32_t* zw = (uint32_t*)qzeros_out;
    const int NGW = (NG + 7) / 8;
    for (int row = 0; row < d_out; ++row)
        for (int wq = 0; wq < NGW; ++wq) {
            uint32_t word = 0;
            for (int e = 0; e < 8 && 8 * wq + e < NG; ++e)
                word |= (uint32_t)zeros[(size_t)row * NG + 8 * wq + e] << (4 * e);
            zw[(size_t)row * NGW + wq] = word;
        }
    pack_scale_tiles(scales, d_out, NG, (uint16_t*)scales_out);
    return EORA_OK;
}

int eora_pack_factor_f16(const uint16_t* mat, int rows, int cols, void* out)
{
    if (!mat || !out) return EORA_ERR_NULL;
    if (!shape_ok(rows, cols, 32)) return EORA_ERR_SHAPE;
    uint16_t* o = (uint16_t*)out;
    const int ntk = cols / 32;
    const size_t nchunks = (size_t)rows * cols / 8;          // one 16-byte chunk per (tile, lane)
    for (size_t c = 0; c < nchunks; ++c) {
        const size_t tile = c / 64;
        const int lane = (int)(c % 64);
        const int R = (int)(tile / ntk), g = (int)(tile % ntk);
        const int j = lane / 16, n = lane % 16;
        std::memcpy(o + 8 * c, mat + (size_t)(16 * R + n) * cols + 32 * g + 8 * j, 16);
    }
    return EORA_OK;
}

int eora_pack_factor_q4(const uint8_t* codes, const uint16_t* scales, int rows, int cols,
                        void* q_out, void* scales_out)
{
    if (!codes || !scales || !q_out || !scales_out) return EORA_ERR_NULL;
    if (rows <= 0 || rows % 16 || !(cols == 64 || (cols > 0 && cols % 128 == 0))) return EORA_ERR_SHAPE;
    const int KT = cols < 128 ? cols : 128;
    int rc = pack_q4_tiles(codes, rows, cols, KT, (uint32_t*)q_out);
    if (rc != EORA_OK) return rc;
    pack_scale_tiles(scales, rows, cols / KT, (uint16_t*)scales_out);
    return EORA_OK;
}

int eora_pack_factor_q3(const uint8_t* codes, const uint16_t* scales, int rows, int cols,
                        void* q_out, void* scales_out)
{
    if (!codes || !scales || !q_out || !scales_out) return EORA_ERR_NULL;
    if (rows <= 0 || rows % 16 || cols <= 0 || cols % 128) return EORA_ERR_SHAPE;
    int rc = pack_q3_tiles(codes, rows, cols, (uint32_t*)q_out);
    if (rc != EORA_OK) return rc;
    pack_scale_tiles(scales, rows, cols / 128, (uint16_t*)scales_out);
    return EORA_OK;
}

int eora_pack_sp24(const uint16_t* vals, const uint8_t* pos, int d_in, int d_out,
                   void* values_out, void* indices_out)
{
    if (!vals || !pos || !values_out || !indices_out) return EORA_ERR_NULL;
    if (!shape_ok(d_out, d_in, 128)) return EORA_ERR_SHAPE;
    uint16_t* vo = (uint16_t*)values_out;
    uint32_t* io = (uint32_t*)indices_out;
    const int ntk = d_in / 128, half = d_in / 2;
    const size_t nlanes = (size_t)d_out * d_in / 32;         // one index word per (tile, lane)
    for (size_t L = 0; L < nlanes; ++L) {
        const size_t tile = L / 64;
        const int lane = (int)(L % 64);
        const int R = (int)(tile / ntk), g = (int)(tile % ntk);
        const int j = lane / 16, n = lane % 16;
        uint32_t word = 0;
        for (int s = 0; s < 2; ++s)
            for (int q = 0; q < 4; ++q) {
                const int dense0 = 128 * g + 64 * s + 16 * j + 4 * q;
                const size_t u = (size_t)(16 * R + n) * half + dense0 / 2;
                if (pos[u] > 3 || pos[u + 1] > 3 || pos[u] >= pos[u + 1]) return EORA_ERR_VALUE;
                for (int v = 0; v < 2; ++v) {
                    word |= (uint32_t)pos[u + v] << (16 * s + 4 * q + 2 * v);
                    vo[tile * 1024 + s * 512 + lane * 8 + 2 * q + v] = vals[u + v];
                }
            }
        io[L] = word;
    }
    return EORA_OK;
}

size_t eora_sp24q4_tiles_bytes(int d_in, int d_out)
{
    return shape_ok(d_out, d_in, 128) ? (size_t)d_out * d_in * 3 / 8 : 0;
}

size_t eora_sp24q4_meta_bytes(int d_in, int d_out)
{
    return shape_ok(d_out, d_in, 128) ? (size_t)d_out * (d_in / 128) * 4 : 0;
}

int eora_pack_sp24q4(const uint8_t* codes, const uint8_t* pos, const uint8_t* zeros, const uint16_t* scales,
                     int d_in, int d_out, int group, void* qtiles_out, void* qmeta_out)
{
    if (!codes || !pos || !zeros || !scales || !qtiles_out || !qmeta_out) return EORA_ERR_NULL;
    if (!shape_ok(d_out, d_in, 128) || group <= 0 || group % 128 || d_in % group) return EORA_ERR_SHAPE;
    const int NG = d_in / group;
    for (size_t i = 0; i < (size_t)d_out * NG; ++i)
        if (zeros[i] > 15) return EORA_ERR_VALUE;
    uint32_t* to = (uint32_t*)qtiles_out;
    uint32_t* mo = (uint32_t*)qmeta_out;
    const int ntk = d_in / 128, half = d_in / 2;
    const size_t nlanes = (size_t)d_out * d_in / 32;         // three words per (tile, lane)
    for (size_t L = 0; L < nlanes; ++L) {
        const size_t tile = L / 64;
        const int lane = (int)(L % 64);
        const int R = (int)(tile / ntk), g = (int)(tile % ntk);
        const int j = lane / 16, n = lane % 16;
        uint32_t word = 0;
        for (int s = 0; s < 2; ++s) {
            uint32_t cw = 0;
            for (int q = 0; q < 4; ++q) {
                const int dense0 = 128 * g + 64 * s + 16 * j + 4 * q;
                const size_t u = (size_t)(16 * R + n) * half + dense0 / 2;
                if (pos[u] > 3 || pos[u + 1] > 3 || pos[u] >= pos[u + 1]) return EORA_ERR_VALUE;
                for (int v = 0; v < 2; ++v) {
                    if (codes[u + v] > 15) return EORA_ERR_VALUE;
                    const int e = 2 * q + v;
                    word |= (uint32_t)pos[u + v] << (16 * s + 4 * q + 2 * v);
                    cw |= (uint32_t)codes[u + v] << (4 * (4 * (e % 2) + e / 2));
                }
            }
            to[3 * L + s] = cw;
        }
        to[3 * L + 2] = word;
        if (j == 0) {                                        // the tile's meta word of row n
            const size_t q = (size_t)(16 * R + n) * NG + (128 * g) / group;
            mo[tile * 16 + n] = (uint32_t)scales[q] | ((uint32_t)zeros[q] << 16);
        }
    }
    return EORA_OK;
}

const char* eora_status_string(int status)
{
    switch (status) {
        case EORA_OK: return "ok";
        case EORA_ERR_NULL: return "null pointer";
        case EORA_ERR_SHAPE: return "invalid shape";
        case EORA_ERR_UNSUPPORTED: return "unsupported format";
        case EORA_ERR_ALIGN: return "misaligned pointer";
        case EORA_ERR_WORKSPACE: return "workspace missing or too small";
        case EORA_ERR_LAUNCH: return "kernel launch failed";
        case EORA_ERR_VALUE: return "value out of range";
        case EORA_ERR_TIMEOUT: return "in-kernel wait timed out";
        case EORA_ERR_NOT_CONVERGED: return "Jacobi sweeps did not converge";
        default: return "unknown status";
    }
}

}  // extern "C"
