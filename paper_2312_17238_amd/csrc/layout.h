// Private layout of one expert's contiguous blob (Sec. 3.3: all of an expert's parameters live in
// one buffer that moves in a single host-to-device copy) and the host-side repacking into it.
//
// A matrix [out][in] is stored row by row; a row is its packed codes followed by its (scale, zero)
// fp16 pairs, padded to 16 bytes, so one output row is one contiguous stream.  w1 and w3 are
// interleaved row-wise (w1 row r, w3 row r, w1 row r+1, ...) because the SwiGLU product needs the
// same row of both; w2 follows.
//
// 4-bit codes: 8 per 32-bit word.  Element i of the 8 (consecutive along `in`) sits at bit
// 4*(i/2) of the low (i even) or high (i odd) half-word, so that masking the word with
// 0x000F000F (after shifting by 0 or 8) or 0x00F000F0 yields two fp16 bit patterns holding
// elements (2n, 2n+1) -- the pair order of the activation vector.
//
// 2-bit codes (group 16): a group is one 32-bit word of 16 codes followed directly by its
// (scale, zero) pair, 8 bytes per group; element i sits at bit 2*(i/2) of the low (i even) or
// high (i odd) half-word.
//
// 3-bit codes (group 64): stored as a 2-bit plane (low two bits, packed like the 2-bit format,
// 16 per word) and a 1-bit plane (the high bit, 32 per word: element i at bit i/2 of the low or
// high half-word); per row: all 2-bit-plane words, then all 1-bit-plane words, then the pairs.
// 3.0 bits per weight, the same as dense packing.
#pragma once
#include <cstdint>
#include <cstring>

namespace moe {

struct MatLayout {
    uint32_t rows = 0, cols = 0;
    uint32_t code_bytes = 0;   // packed codes per row
    uint32_t meta_off = 0;     // byte offset of the (scale, zero) pairs inside a row (4/3-bit)
    uint32_t row_stride = 0;   // bytes from one row of this matrix to the next row of the same matrix's stream
};

struct BlobLayout {
    int32_t hidden = 0, ffn = 0, bits = 0, group = 0;
    MatLayout m13;             // w1 and w3 rows: [F][H]; interleaved, so consecutive rows of w1 are 2*row_stride apart
    MatLayout m2;              // w2 rows: [H][F]
    uint64_t off_w13 = 0, off_w2 = 0, total = 0;
    bool ok = false;
};

inline uint32_t align_up(uint32_t v, uint32_t a) { return (v + a - 1) / a * a; }

inline MatLayout mat_layout(uint32_t rows, uint32_t cols, int bits, int group)
{
    MatLayout m;
    m.rows = rows;
    m.cols = cols;
    uint32_t groups = cols / group;
    if (bits == 2) {                       // interleaved: 8 bytes per group of 16
        m.code_bytes = groups * 8;
        m.meta_off = 0;
        m.row_stride = align_up(m.code_bytes, 16);
    } else {
        m.code_bytes = cols * bits / 8;
        m.meta_off = m.code_bytes;
        m.row_stride = align_up(m.code_bytes + groups * 4, 16);
    }
    return m;
}

inline bool format_supported(int bits, int group)
{
    if (bits == 4) return group == 32 || group == 64 || group == 128;
    if (bits == 3) return group == 64;
    if (bits == 2) return group == 16;
    return false;
}

inline BlobLayout blob_layout(int32_t hidden, int32_t ffn, int32_t bits, int32_t group)
{
    BlobLayout b;
    b.hidden = hidden; b.ffn = ffn; b.bits = bits; b.group = group;
    if (hidden <= 0 || ffn <= 0 || hidden % 64 || ffn % 64 || !format_supported(bits, group)) return b;
    if (hidden % group || ffn % group) return b;
    b.m13 = mat_layout(ffn, hidden, bits, group);
    b.m2 = mat_layout(hidden, ffn, bits, group);
    b.off_w13 = 0;
    b.off_w2 = (uint64_t)2 * ffn * b.m13.row_stride;
    b.total = b.off_w2 + (uint64_t)hidden * b.m2.row_stride;
    b.total = (b.total + 255) / 256 * 256;
    b.ok = true;
    return b;
}

// byte offset of row r of matrix m (0 = w1, 1 = w3, 2 = w2) inside the blob
inline uint64_t row_offset(const BlobLayout &b, int matrix, uint32_t r)
{
    if (matrix == 2) return b.off_w2 + (uint64_t)r * b.m2.row_stride;
    return b.off_w13 + ((uint64_t)2 * r + matrix) * b.m13.row_stride;
}

inline const MatLayout &mat_of(const BlobLayout &b, int matrix) { return matrix == 2 ? b.m2 : b.m13; }

// ---- packing one row ------------------------------------------------------------------------

inline void pack_row(const BlobLayout &b, const MatLayout &m, const uint8_t *codes, const uint16_t *scale,
                     const uint16_t *zero, uint8_t *dst)
{
    const uint32_t cols = m.cols, groups = cols / b.group;
    uint32_t *w = reinterpret_cast<uint32_t *>(dst);
    if (b.bits == 4) {
        for (uint32_t i = 0; i < cols / 8; ++i) {
            const uint8_t *c = codes + 8 * i;
            uint32_t v = 0;
            for (int n = 0; n < 4; ++n)
                v |= (uint32_t)(c[2 * n] & 15) << (4 * n) | (uint32_t)(c[2 * n + 1] & 15) << (16 + 4 * n);
            w[i] = v;
        }
    } else if (b.bits == 2) {
        for (uint32_t g = 0; g < groups; ++g) {
            const uint8_t *c = codes + 16 * g;
            uint32_t v = 0;
            for (int n = 0; n < 8; ++n)
                v |= (uint32_t)(c[2 * n] & 3) << (2 * n) | (uint32_t)(c[2 * n + 1] & 3) << (16 + 2 * n);
            w[2 * g] = v;
            w[2 * g + 1] = (uint32_t)scale[g] | (uint32_t)zero[g] << 16;
        }
        return;
    } else {  // 3-bit: 2-bit plane then 1-bit plane
        uint32_t *lo = w, *hi = w + cols / 16;
        for (uint32_t i = 0; i < cols / 16; ++i) {
            const uint8_t *c = codes + 16 * i;
            uint32_t v = 0;
            for (int n = 0; n < 8; ++n)
                v |= (uint32_t)(c[2 * n] & 3) << (2 * n) | (uint32_t)(c[2 * n + 1] & 3) << (16 + 2 * n);
            lo[i] = v;
        }
        for (uint32_t i = 0; i < cols / 32; ++i) {
            const uint8_t *c = codes + 32 * i;
            uint32_t v = 0;
            for (int n = 0; n < 16; ++n)
                v |= (uint32_t)((c[2 * n] >> 2) & 1) << n | (uint32_t)((c[2 * n + 1] >> 2) & 1) << (16 + n);
            hi[i] = v;
        }
    }
    uint32_t *meta = reinterpret_cast<uint32_t *>(dst + m.meta_off);
    for (uint32_t g = 0; g < groups; ++g) meta[g] = (uint32_t)scale[g] | (uint32_t)zero[g] << 16;
}

inline void peek_row(const BlobLayout &b, const MatLayout &m, const uint8_t *src, uint32_t col, uint8_t *code,
                     uint16_t *scale, uint16_t *zero)
{
    const uint32_t *w = reinterpret_cast<const uint32_t *>(src);
    uint32_t g = col / b.group, meta;
    if (b.bits == 4) {
        uint32_t v = w[col / 8], i = col % 8;
        *code = (v >> (4 * (i / 2) + 16 * (i & 1))) & 15;
        meta = reinterpret_cast<const uint32_t *>(src + m.meta_off)[g];
    } else if (b.bits == 2) {
        uint32_t v = w[2 * g], i = col % 16;
        *code = (v >> (2 * (i / 2) + 16 * (i & 1))) & 3;
        meta = w[2 * g + 1];
    } else {
        uint32_t v = w[col / 16], i = col % 16;
        uint32_t low = (v >> (2 * (i / 2) + 16 * (i & 1))) & 3;
        uint32_t u = w[m.cols / 16 + col / 32], j = col % 32;
        uint32_t high = (u >> ((j / 2) + 16 * (j & 1))) & 1;
        *code = (uint8_t)(low | high << 2);
        meta = reinterpret_cast<const uint32_t *>(src + m.meta_off)[g];
    }
    *scale = (uint16_t)(meta & 0xffff);
    *zero = (uint16_t)(meta >> 16);
}

}  // namespace moe
