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
// 3-bit codes (group 64): a row is three regions, each indexed by the group (64 consecutive codes):
// region A, 16 bytes per group; region B, 8 bytes per group; then the (scale, zero) pairs, 4 bytes per
// group.  With T_j (j = 0..7) the eight 32-bit words the 64 codes would occupy in the 4-bit layout above
// (3-bit value in each nibble), A_i = (T_2i & 0x33333333) | (T_2i+1 & 0x33333333) << 2 holds the low two
// bits of two such words and B_i = sum_j ((T_4i+j >> 2) & 0x11111111) << j the third bits of four, so a
// decoder rebuilds T_j with three bit operations and reuses the 4-bit arithmetic.  3.0 bits per weight.
//
// Two-level metadata (Sec. 4.2 "scale group size"): the row's codes are followed by one (scale code, zero code)
// byte pair per group, then, 8-byte aligned, one fp16 quad per run of scale_group consecutive groups (the whole
// row if it has fewer; the last run of a row may be shorter): (step of the scale codes, zero of the scale codes,
// step of the zero codes, zero of the zero codes).  4.25 / 3.25 / 3.0 bits per weight for the 4-bit g64, 3-bit g64
// and 2-bit g16 codes, plus 8 bytes per run.  The codes are laid out as above, except that the 2-bit words are
// no longer interleaved with metadata: word g holds group g.
#pragma once
#include <cstdint>
#include <cstring>

namespace moe {

struct MatLayout {
    uint32_t rows = 0, cols = 0;
    uint32_t code_bytes = 0;   // packed codes per row
    uint32_t meta_off = 0;     // byte offset of the (scale, zero) pairs inside a row (4/3-bit)
    uint32_t row_stride = 0;   // bytes from one row of this matrix to the next row of the same matrix's stream
    uint32_t meta2_off = 0;    // two-level metadata: byte offset of the per-run fp16 quads
    uint32_t run_len = 0;      // ... groups per run (0: one-level metadata)
};

struct BlobLayout {
    int32_t hidden = 0, ffn = 0, bits = 0, group = 0, scale_group = 0;
    MatLayout m13;             // w1 and w3 rows: [F][H]; interleaved, so consecutive rows of w1 are 2*row_stride apart
    MatLayout m2;              // w2 rows: [H][F]
    uint64_t off_w13 = 0, off_w2 = 0, total = 0;
    bool ok = false;
};

inline uint32_t align_up(uint32_t v, uint32_t a) { return (v + a - 1) / a * a; }

inline MatLayout mat_layout(uint32_t rows, uint32_t cols, int bits, int group, int scale_group = 0)
{
    MatLayout m;
    m.rows = rows;
    m.cols = cols;
    uint32_t groups = cols / group;
    if (scale_group > 0) {                 // codes, byte pairs, per-run quads
        m.code_bytes = bits == 4 ? cols / 2 : (bits == 3 ? groups * 24 : groups * 4);
        m.meta_off = m.code_bytes;
        m.run_len = groups < (uint32_t)scale_group ? groups : (uint32_t)scale_group;
        m.meta2_off = align_up(m.meta_off + groups * 2, 8);
        m.row_stride = align_up(m.meta2_off + (groups + m.run_len - 1) / m.run_len * 8, 16);
    } else if (bits == 2) {                       // interleaved: 8 bytes per group of 16
        m.code_bytes = groups * 8;
        m.meta_off = 0;
        m.row_stride = align_up(m.code_bytes, 16);
    } else if (bits == 3) {                // per group of 64: 16 B (region A) + 8 B (region B) + 4 B pair
        m.code_bytes = groups * 24;
        m.meta_off = m.code_bytes;
        m.row_stride = align_up(groups * 28, 16);
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

// scale_group: 0, or a power of two.  The 2-bit kernels read four groups (64 codes) per lane, which must not
// straddle runs: there a run is at least four groups, or the whole row.
inline bool scale_group_supported(int bits, int group, int scale_group, int cols)
{
    if (scale_group == 0) return true;
    if (scale_group < 1 || (scale_group & (scale_group - 1))) return false;
    const int groups = cols / group;
    return bits != 2 || groups <= scale_group || scale_group >= 4;
}

inline BlobLayout blob_layout(int32_t hidden, int32_t ffn, int32_t bits, int32_t group, int32_t scale_group = 0)
{
    BlobLayout b;
    b.hidden = hidden; b.ffn = ffn; b.bits = bits; b.group = group; b.scale_group = scale_group;
    if (hidden <= 0 || ffn <= 0 || hidden % 64 || ffn % 64 || !format_supported(bits, group)) return b;
    if (hidden % group || ffn % group) return b;
    if (!scale_group_supported(bits, group, scale_group, hidden) || !scale_group_supported(bits, group, scale_group, ffn)) return b;
    b.m13 = mat_layout(ffn, hidden, bits, group, scale_group);
    b.m2 = mat_layout(hidden, ffn, bits, group, scale_group);
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

// 8 consecutive 4-bit (or 3-bit, `mask` 7) codes as one word of the 4-bit layout
inline uint32_t word_of_8(const uint8_t *c, uint32_t mask)
{
    uint32_t v = 0;
    for (int n = 0; n < 4; ++n)
        v |= (uint32_t)(c[2 * n] & mask) << (4 * n) | (uint32_t)(c[2 * n + 1] & mask) << (16 + 4 * n);
    return v;
}

// 16 consecutive 2-bit codes as one word
inline uint32_t word_of_16(const uint8_t *c)
{
    uint32_t v = 0;
    for (int n = 0; n < 8; ++n)
        v |= (uint32_t)(c[2 * n] & 3) << (2 * n) | (uint32_t)(c[2 * n + 1] & 3) << (16 + 2 * n);
    return v;
}

// the 4-bit code words of a row, or the regions A and B of a 3-bit row
inline void pack_codes_43(int bits, uint32_t cols, const uint8_t *codes, uint32_t *w)
{
    if (bits == 4) {
        for (uint32_t i = 0; i < cols / 8; ++i) w[i] = word_of_8(codes + 8 * i, 15);
        return;
    }
    const uint32_t groups = cols / 64;
    uint32_t *ra = w, *rb = w + groups * 4;
    for (uint32_t g = 0; g < groups; ++g) {
        uint32_t t[8];
        for (int j = 0; j < 8; ++j) t[j] = word_of_8(codes + 64 * g + 8 * j, 7);
        for (int i = 0; i < 4; ++i) ra[4 * g + i] = (t[2 * i] & 0x33333333u) | (t[2 * i + 1] & 0x33333333u) << 2;
        for (int i = 0; i < 2; ++i) {
            uint32_t v = 0;
            for (int j = 0; j < 4; ++j) v |= ((t[4 * i + j] >> 2) & 0x11111111u) << j;
            rb[2 * g + i] = v;
        }
    }
}

inline void pack_row(const BlobLayout &b, const MatLayout &m, const uint8_t *codes, const uint16_t *scale,
                     const uint16_t *zero, uint8_t *dst)
{
    const uint32_t cols = m.cols, groups = cols / b.group;
    uint32_t *w = reinterpret_cast<uint32_t *>(dst);
    if (b.bits == 2) {
        for (uint32_t g = 0; g < groups; ++g) {
            w[2 * g] = word_of_16(codes + 16 * g);
            w[2 * g + 1] = (uint32_t)scale[g] | (uint32_t)zero[g] << 16;
        }
        return;
    }
    pack_codes_43(b.bits, cols, codes, w);
    uint32_t *meta = reinterpret_cast<uint32_t *>(dst + m.meta_off);
    for (uint32_t g = 0; g < groups; ++g) meta[g] = (uint32_t)scale[g] | (uint32_t)zero[g] << 16;
}

// two-level metadata: the codes, then the byte pairs, then the per-run quads
inline void pack_row_meta8(const BlobLayout &b, const MatLayout &m, const uint8_t *codes, const uint8_t *scale_code,
                           const uint8_t *zero_code, const uint16_t *run_meta, uint8_t *dst)
{
    const uint32_t cols = m.cols, groups = cols / b.group;
    uint32_t *w = reinterpret_cast<uint32_t *>(dst);
    if (b.bits == 2)
        for (uint32_t g = 0; g < groups; ++g) w[g] = word_of_16(codes + 16 * g);
    else
        pack_codes_43(b.bits, cols, codes, w);
    uint8_t *pairs = dst + m.meta_off;
    for (uint32_t g = 0; g < groups; ++g) { pairs[2 * g] = scale_code[g]; pairs[2 * g + 1] = zero_code[g]; }
    memset(pairs + 2 * groups, 0, m.meta2_off - (m.meta_off + 2 * groups));
    memcpy(dst + m.meta2_off, run_meta, (size_t)((groups + m.run_len - 1) / m.run_len) * 8);
}

// code at column col of a 4-bit or 3-bit row
inline uint8_t peek_code_43(int bits, uint32_t cols, const uint32_t *w, uint32_t col)
{
    if (bits == 4) {
        const uint32_t v = w[col / 8], i = col % 8;
        return (v >> (4 * (i / 2) + 16 * (i & 1))) & 15;
    }
    const uint32_t groups = cols / 64, g = col / 64, e = col % 64, j = e / 8, pos = e % 8;
    const uint32_t p = 4 * (pos / 2) + 16 * (pos & 1);
    const uint32_t low = (w[4 * g + j / 2] >> (p + 2 * (j & 1))) & 3;
    const uint32_t high = (w[groups * 4 + 2 * g + j / 4] >> (p + (j % 4))) & 1;
    return (uint8_t)(low | high << 2);
}

inline uint8_t peek_code_2(uint32_t word, uint32_t col)
{
    const uint32_t i = col % 16;
    return (word >> (2 * (i / 2) + 16 * (i & 1))) & 3;
}

inline void peek_row_meta8(const BlobLayout &b, const MatLayout &m, const uint8_t *src, uint32_t col, uint8_t *code,
                           uint8_t *scale_code, uint8_t *zero_code, uint16_t run_meta[4])
{
    const uint32_t *w = reinterpret_cast<const uint32_t *>(src);
    const uint32_t g = col / b.group;
    *code = b.bits == 2 ? peek_code_2(w[g], col) : peek_code_43(b.bits, m.cols, w, col);
    *scale_code = src[m.meta_off + 2 * g];
    *zero_code = src[m.meta_off + 2 * g + 1];
    memcpy(run_meta, src + m.meta2_off + (size_t)(g / m.run_len) * 8, 8);
}

inline void peek_row(const BlobLayout &b, const MatLayout &m, const uint8_t *src, uint32_t col, uint8_t *code,
                     uint16_t *scale, uint16_t *zero)
{
    const uint32_t *w = reinterpret_cast<const uint32_t *>(src);
    uint32_t g = col / b.group, meta;
    if (b.bits == 2) {
        *code = peek_code_2(w[2 * g], col);
        meta = w[2 * g + 1];
    } else {
        *code = peek_code_43(b.bits, m.cols, w, col);
        meta = reinterpret_cast<const uint32_t *>(src + m.meta_off)[g];
    }
    *scale = (uint16_t)(meta & 0xffff);
    *zero = (uint16_t)(meta >> 16);
}

}  // namespace moe
