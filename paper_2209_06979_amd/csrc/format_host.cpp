// Host-side format builder: interchange BCRS (V x 1 blocks) <-> device panel format.
//
// The device format follows the idea of SR-BCRS (paper, Section 4.1): inside a row
// panel the stored vectors are grouped into strides whose length equals the reduction
// depth of the matrix instruction, the last stride is zero-padded, values are stored
// row-major inside a stride, and each panel carries two pointers (aligned start, real
// end).  Here a stride ("chunk") is 64 vectors = one v_mfma_i32_16x16x64_i8, and it is
// cut into 4 sub-strides of 16 vectors because one MFMA lane group consumes 16
// consecutive reduction bytes of one row.
#include "internal.h"

#include <algorithm>
#include <climits>
#include <cstring>
#include <vector>

namespace {

inline int64_t pad_to_chunk(int64_t n) { return (n + MC_CHUNK - 1) / MC_CHUNK * MC_CHUNK; }

// bytes of one chunk of packed values
// (a 12-bit operand is an int16 array restricted to [-2048, 2047] and is stored like a 16-bit one)
inline int storage_bits(int bits) { return bits == 12 ? 16 : bits; }
inline int64_t chunk_value_bytes(int V, int bits) { return (int64_t)MC_CHUNK * V * storage_bits(bits) / 8; }
inline bool valid_lhs_bits(int b) { return b == 0 || b == 4 || b == 8 || b == 12 || b == 16; }

// signed int8 planes of a 16-bit value: a = 256 * hi + lo, lo in [-128, 127]
inline bool split_balanced(int a, int8_t *hi, int8_t *lo)
{
    int h = (a + 128) >> 8; // arithmetic shift, floor
    int l = a - h * 256;
    if (h < -128 || h > 127) return false;
    *hi = (int8_t)h;
    *lo = (int8_t)l;
    return true;
}

inline int nibble_at(const uint8_t *bytes, int64_t elem)
{
    uint8_t b = bytes[elem >> 1];
    return (elem & 1) ? (b >> 4) : (b & 15);
}

// Writes the V elements of interchange vector `vec` into slot `slot` (0..63) of a chunk of packed
// values (layout: see mc_pack_host).  The chunk must have been zeroed.
inline int put_vector(uint8_t *chunk, int V, int lhs_bits, int slot, const void *values, int64_t vec)
{
    const int g = slot / 16, b = slot % 16;
    for (int v = 0; v < V; ++v) {
        const int64_t e = vec * V + v; // element in interchange order
        if (lhs_bits == 8) {
            chunk[g * (16 * V) + v * 16 + b] = static_cast<const uint8_t *>(values)[e];
        } else if (lhs_bits == 16 || lhs_bits == 12) {
            int8_t hi, l8;
            const int x = static_cast<const int16_t *>(values)[e];
            if (lhs_bits == 12 && (x < -2048 || x > 2047)) return MC_ERANGE;
            if (!split_balanced(x, &hi, &l8)) return MC_ERANGE;
            chunk[g * (32 * V) + v * 16 + b] = (uint8_t)hi;
            chunk[g * (32 * V) + 16 * V + v * 16 + b] = (uint8_t)l8;
        } else { // 4 bits
            const int nib = nibble_at(static_cast<const uint8_t *>(values), e);
            uint8_t *byte = &chunk[g * (8 * V) + v * 8 + (b & 7)];
            *byte |= (uint8_t)((b < 8) ? nib : (nib << 4));
        }
    }
    return MC_OK;
}

// Position of slot s (0..63) of a chunk in the K-blocked format's row array: the two slots one lane of the
// kernel addresses (s and s + 8 inside a sub-stride of 16) are neighbours, so that they travel as one 32-bit word.
inline int64_t chunk_base(int64_t slot) { return slot / MC_CHUNK * MC_CHUNK; }
inline int row_position(int s) { return (s / 16) * 16 + (s % 8) * 2 + (s % 16) / 8; }

} // namespace

// The builders below exist in two forms: the exported ones take the vector lengths of the interchange format
// (2, 4, 8); the *_wide ones also take 16 for 4- and 8-bit values, which only the library's own merged copy of
// an operand uses (see mc_merge_host): sixteen rows fill the MFMA's row operand completely.
static bool valid_V_wide(int V, int lhs_bits)
{
    return V == 2 || V == 4 || V == 8 || (V == 16 && (lhs_bits == 4 || lhs_bits == 8));
}

extern "C" int mc_layout_query(int M, int K, int V, int lhs_bits, const int32_t *row_ptr, mc_layout *out)
{
    return V == 16 ? MC_EINVAL : mc_layout_query_wide(M, K, V, lhs_bits, row_ptr, out);
}

int mc_layout_query_wide(int M, int K, int V, int lhs_bits, const int32_t *row_ptr, mc_layout *out)
{
    if (!row_ptr || !out) return MC_EINVAL;
    if (M <= 0 || K <= 0) return MC_EINVAL;
    if (!valid_V_wide(V, lhs_bits)) return MC_EINVAL;
    if (M % V != 0) return MC_EINVAL;
    if (!valid_lhs_bits(lhs_bits)) return MC_EINVAL;
    const int P = M / V;
    if (row_ptr[0] != 0) return MC_EINVAL;
    int64_t nslots = 0;
    for (int p = 0; p < P; ++p) {
        const int64_t n = (int64_t)row_ptr[p + 1] - row_ptr[p];
        if (n < 0 || n > K) return MC_EINVAL;
        nslots += pad_to_chunk(n);
    }
    if (nslots > (int64_t)INT32_MAX - MC_CHUNK) return MC_EINVAL;
    out->P = P;
    out->nvec = row_ptr[P];
    out->nslots = nslots;
    out->vals_bytes = lhs_bits ? (nslots / MC_CHUNK) * chunk_value_bytes(V, lhs_bits) : 0;
    return MC_OK;
}

extern "C" int mc_pack_host(int M, int K, int V, int lhs_bits, const int32_t *row_ptr, const int32_t *col_idx,
                            const void *values, int32_t *panel_ptr, int32_t *slot_idx, void *slot_vals)
{
    return V == 16 ? MC_EINVAL : mc_pack_host_wide(M, K, V, lhs_bits, row_ptr, col_idx, values, panel_ptr, slot_idx, slot_vals);
}

int mc_pack_host_wide(int M, int K, int V, int lhs_bits, const int32_t *row_ptr, const int32_t *col_idx,
                      const void *values, int32_t *panel_ptr, int32_t *slot_idx, void *slot_vals)
{
    mc_layout lay;
    int rc = mc_layout_query_wide(M, K, V, lhs_bits, row_ptr, &lay);
    if (rc != MC_OK) return rc;
    if (!panel_ptr || (lay.nslots && !slot_idx) || (lay.nvec && !col_idx)) return MC_EINVAL;
    const bool with_vals = lhs_bits != 0 && values != nullptr;
    if (with_vals && lay.vals_bytes && !slot_vals) return MC_EINVAL;

    // pattern
    int64_t slot0 = 0;
    for (int p = 0; p < lay.P; ++p) {
        const int64_t lo = row_ptr[p], n = (int64_t)row_ptr[p + 1] - lo;
        panel_ptr[2 * p] = (int32_t)slot0;
        panel_ptr[2 * p + 1] = (int32_t)(slot0 + n);
        int32_t prev = -1;
        for (int64_t i = 0; i < n; ++i) {
            const int32_t c = col_idx[lo + i];
            if (c <= prev || c >= K) return MC_EINVAL;
            slot_idx[slot0 + i] = c;
            prev = c;
        }
        for (int64_t i = n; i < pad_to_chunk(n); ++i) slot_idx[slot0 + i] = prev; // n > 0 here
        slot0 += pad_to_chunk(n);
    }
    if (!with_vals) return MC_OK;

    std::memset(slot_vals, 0, (size_t)lay.vals_bytes);
    uint8_t *dst = static_cast<uint8_t *>(slot_vals);
    const int64_t cbytes = chunk_value_bytes(V, lhs_bits);
    for (int p = 0; p < lay.P; ++p) {
        const int64_t lo = row_ptr[p], n = (int64_t)row_ptr[p + 1] - lo;
        const int64_t s0 = panel_ptr[2 * p];
        for (int64_t i = 0; i < n; ++i) {
            const int64_t s = s0 + i;
            rc = put_vector(dst + (s / MC_CHUNK) * cbytes, V, lhs_bits, (int)(s % MC_CHUNK), values, lo + i);
            if (rc != MC_OK) return rc;
        }
    }
    return MC_OK;
}

extern "C" int mc_unpack_host(int M, int K, int V, int lhs_bits, const int32_t *panel_ptr,
                              const int32_t *slot_idx, const void *slot_vals, int32_t *row_ptr,
                              int32_t *col_idx, void *values)
{
    if (M <= 0 || K <= 0 || (V != 2 && V != 4 && V != 8) || M % V) return MC_EINVAL;
    if (!valid_lhs_bits(lhs_bits)) return MC_EINVAL;
    if (!panel_ptr || !row_ptr) return MC_EINVAL;
    const int P = M / V;
    const uint8_t *src = static_cast<const uint8_t *>(slot_vals);
    const int64_t cbytes = lhs_bits ? chunk_value_bytes(V, lhs_bits) : 0;
    const bool with_vals = lhs_bits != 0 && slot_vals != nullptr && values != nullptr;
    int64_t out = 0;
    row_ptr[0] = 0;
    for (int p = 0; p < P; ++p) {
        const int64_t s0 = panel_ptr[2 * p], n = (int64_t)panel_ptr[2 * p + 1] - s0;
        if (n < 0 || s0 % MC_CHUNK) return MC_EINVAL;
        for (int64_t i = 0; i < n; ++i, ++out) {
            const int64_t s = s0 + i;
            col_idx[out] = slot_idx[s];
            if (!with_vals) continue;
            const uint8_t *chunk = src + (s / MC_CHUNK) * cbytes;
            const int g = (int)(s % MC_CHUNK) / 16, b = (int)(s % 16);
            for (int v = 0; v < V; ++v) {
                const int64_t e = out * V + v;
                if (lhs_bits == 8) {
                    static_cast<uint8_t *>(values)[e] = chunk[g * (16 * V) + v * 16 + b];
                } else if (lhs_bits == 16 || lhs_bits == 12) {
                    const int hi = (int8_t)chunk[g * (32 * V) + v * 16 + b];
                    const int l8 = (int8_t)chunk[g * (32 * V) + 16 * V + v * 16 + b];
                    static_cast<int16_t *>(values)[e] = (int16_t)(hi * 256 + l8);
                } else {
                    const uint8_t byte = chunk[g * (8 * V) + v * 8 + (b & 7)];
                    const int nib = (b < 8) ? (byte & 15) : (byte >> 4);
                    uint8_t *o = &static_cast<uint8_t *>(values)[e >> 1];
                    if (e & 1) *o = (uint8_t)((*o & 0x0F) | (nib << 4));
                    else *o = (uint8_t)((*o & 0xF0) | nib);
                }
            }
        }
        row_ptr[p + 1] = (int32_t)out;
    }
    return MC_OK;
}

// ---- K-blocked variant of the format -------------------------------------------------------
// For kernels that keep a block of MC_KBLOCK consecutive rows of the dense operand resident in
// on-chip memory: the vectors of a panel are additionally grouped by the K-block their column
// falls in, and each (panel, block) list is padded to whole chunks on its own, so that every
// chunk only names rows of one block (as 16-bit row numbers inside that block).
extern "C" int mc_blocked_query(int M, int K, int V, int lhs_bits, const int32_t *row_ptr, const int32_t *col_idx,
                                mc_blocked_layout *out)
{
    return V == 16 ? MC_EINVAL : mc_blocked_query_wide(M, K, V, lhs_bits, row_ptr, col_idx, out);
}

int mc_blocked_query_wide(int M, int K, int V, int lhs_bits, const int32_t *row_ptr, const int32_t *col_idx,
                          mc_blocked_layout *out)
{
    mc_layout lay;
    int rc = mc_layout_query_wide(M, K, V, lhs_bits, row_ptr, &lay);
    if (rc != MC_OK) return rc;
    if (!out || (lay.nvec && !col_idx)) return MC_EINVAL;
    const int nblk = (K + MC_KBLOCK - 1) / MC_KBLOCK;
    int64_t nchunks = 0;
    for (int p = 0; p < lay.P; ++p) {
        int64_t i = row_ptr[p];
        const int64_t end = row_ptr[p + 1];
        int32_t prev = -1;
        for (int b = 0; b < nblk; ++b) {
            int64_t n = 0;
            while (i < end && col_idx[i] < (int64_t)(b + 1) * MC_KBLOCK) {
                if (col_idx[i] <= prev || col_idx[i] >= K) return MC_EINVAL;
                prev = col_idx[i];
                ++i; ++n;
            }
            nchunks += (n + MC_CHUNK - 1) / MC_CHUNK;
        }
        if (i != end) return MC_EINVAL; // a column at or beyond K
    }
    if (nchunks * MC_CHUNK > (int64_t)INT32_MAX - MC_CHUNK) return MC_EINVAL;
    out->nblk = nblk;
    out->nchunks = nchunks;
    out->vals_bytes = lhs_bits ? nchunks * chunk_value_bytes(V, lhs_bits) : 0;
    return MC_OK;
}

extern "C" int mc_pack_blocked_host(int M, int K, int V, int lhs_bits, const int32_t *row_ptr, const int32_t *col_idx,
                                    const void *values, int32_t *blk_ptr, uint16_t *blk_rows, void *blk_vals,
                                    int32_t *blk_src)
{
    return V == 16 ? MC_EINVAL : mc_pack_blocked_host_wide(M, K, V, lhs_bits, row_ptr, col_idx, values, blk_ptr, blk_rows, blk_vals, blk_src);
}

int mc_pack_blocked_host_wide(int M, int K, int V, int lhs_bits, const int32_t *row_ptr, const int32_t *col_idx,
                              const void *values, int32_t *blk_ptr, uint16_t *blk_rows, void *blk_vals, int32_t *blk_src)
{
    mc_blocked_layout bl;
    int rc = mc_blocked_query_wide(M, K, V, lhs_bits, row_ptr, col_idx, &bl);
    if (rc != MC_OK) return rc;
    if (!blk_ptr || (bl.nchunks && (!blk_rows || !blk_src))) return MC_EINVAL;
    const bool with_vals = lhs_bits != 0 && values != nullptr;
    if (with_vals && bl.vals_bytes && !blk_vals) return MC_EINVAL;
    if (with_vals) std::memset(blk_vals, 0, (size_t)bl.vals_bytes);
    uint8_t *dst = static_cast<uint8_t *>(blk_vals);
    const int64_t cbytes = lhs_bits ? chunk_value_bytes(V, lhs_bits) : 0;
    const int P = M / V;
    int64_t chunk = 0;
    for (int p = 0; p < P; ++p) {
        int64_t i = row_ptr[p];
        const int64_t end = row_ptr[p + 1];
        for (int b = 0; b < bl.nblk; ++b) {
            blk_ptr[(int64_t)p * bl.nblk + b] = (int32_t)chunk;
            int64_t n = 0;
            int last_row = 0;
            while (i < end && col_idx[i] < (int64_t)(b + 1) * MC_KBLOCK) {
                const int64_t slot = chunk * MC_CHUNK + n;
                last_row = col_idx[i] - b * MC_KBLOCK;
                blk_rows[chunk_base(slot) + row_position((int)(slot % MC_CHUNK))] = (uint16_t)last_row;
                blk_src[slot] = (int32_t)i;
                if (with_vals) {
                    rc = put_vector(dst + (slot / MC_CHUNK) * cbytes, V, lhs_bits, (int)(slot % MC_CHUNK), values, i);
                    if (rc != MC_OK) return rc;
                }
                ++i; ++n;
            }
            const int64_t npad = (n + MC_CHUNK - 1) / MC_CHUNK * MC_CHUNK;
            for (int64_t k = n; k < npad; ++k) { // padded slots: a row of this block, zero values, no source vector
                blk_rows[chunk_base(chunk * MC_CHUNK + k) + row_position((int)(k % MC_CHUNK))] = (uint16_t)last_row;
                blk_src[chunk * MC_CHUNK + k] = -1;
            }
            chunk += npad / MC_CHUNK;
        }
    }
    blk_ptr[(int64_t)P * bl.nblk] = (int32_t)chunk;
    return MC_OK;
}

// ---- merged panels ----------------------------------------------------------------------------
// `group` consecutive panels of V rows become one panel of V * group rows whose stored vectors sit at the
// union of the panels' columns; a panel that has no vector at a column of the union contributes zeros there
// (explicit zeros are legal inside stored vectors).  The product with a dense matrix is unchanged, the rows
// of the dense operand named by a column are fetched once for all the panels of a group instead of once per
// panel that holds it, and the MFMA's 16-row operand fills up.
extern "C" int mc_merged_query(int M, int K, int V, int lhs_bits, const int32_t *row_ptr, const int32_t *col_idx, int group,
                               mc_merged_layout *out)
{
    mc_layout lay;
    int rc = mc_layout_query(M, K, V, lhs_bits, row_ptr, &lay);
    if (rc != MC_OK) return rc;
    if (!out || (lay.nvec && !col_idx)) return MC_EINVAL;
    if (group < 2 || (V * group != 8 && V * group != 16)) return MC_EINVAL;
    if (V * group == 16 && lhs_bits != 4 && lhs_bits != 8) return MC_EINVAL;
    const int Pm = (lay.P + group - 1) / group;
    int64_t nvec = 0;
    std::vector<int64_t> at((size_t)group);
    for (int sp = 0; sp < Pm; ++sp) {
        const int p0 = sp * group, np = std::min(group, lay.P - p0);
        for (int g = 0; g < np; ++g) {
            at[(size_t)g] = row_ptr[p0 + g];
            int32_t prev = -1;
            for (int64_t i = row_ptr[p0 + g]; i < row_ptr[p0 + g + 1]; ++i) { // ascending, inside [0, K)
                if (col_idx[i] <= prev || col_idx[i] >= K) return MC_EINVAL;
                prev = col_idx[i];
            }
        }
        for (;;) { // one column of the union per round: the smallest column any panel still has
            int32_t c = INT32_MAX;
            for (int g = 0; g < np; ++g)
                if (at[(size_t)g] < row_ptr[p0 + g + 1]) c = std::min(c, col_idx[at[(size_t)g]]);
            if (c == INT32_MAX) break;
            for (int g = 0; g < np; ++g)
                if (at[(size_t)g] < row_ptr[p0 + g + 1] && col_idx[at[(size_t)g]] == c) ++at[(size_t)g];
            ++nvec;
        }
    }
    if (nvec > (int64_t)INT32_MAX - MC_CHUNK) return MC_EINVAL;
    out->group = group;
    out->P = Pm;
    out->nvec = nvec;
    return MC_OK;
}

extern "C" int mc_merge_host(int M, int K, int V, int lhs_bits, const int32_t *row_ptr, const int32_t *col_idx, const void *values,
                             int group, int32_t *m_row_ptr, int32_t *m_col_idx, void *m_values, int32_t *m_src)
{
    mc_merged_layout ml;
    int rc = mc_merged_query(M, K, V, lhs_bits, row_ptr, col_idx, group, &ml);
    if (rc != MC_OK) return rc;
    if (!m_row_ptr || (ml.nvec && (!m_col_idx || !m_src))) return MC_EINVAL;
    const bool with_vals = lhs_bits != 0 && values != nullptr && m_values != nullptr;
    const int P = M / V;
    const int64_t vb = (int64_t)V * storage_bits(lhs_bits) / 8; // bytes of one panel's share of a merged vector
    const uint8_t *src = static_cast<const uint8_t *>(values);
    uint8_t *dst = static_cast<uint8_t *>(m_values);
    if (with_vals) std::memset(dst, 0, (size_t)(ml.nvec * group * vb));
    std::vector<int64_t> at((size_t)group);
    int64_t out = 0;
    m_row_ptr[0] = 0;
    for (int sp = 0; sp < ml.P; ++sp) {
        const int p0 = sp * group, np = std::min(group, P - p0);
        for (int g = 0; g < np; ++g) at[(size_t)g] = row_ptr[p0 + g];
        for (;;) {
            int32_t c = INT32_MAX;
            for (int g = 0; g < np; ++g)
                if (at[(size_t)g] < row_ptr[p0 + g + 1]) c = std::min(c, col_idx[at[(size_t)g]]);
            if (c == INT32_MAX) break;
            m_col_idx[out] = c;
            for (int g = 0; g < group; ++g) {
                int64_t from = -1;
                if (g < np && at[(size_t)g] < row_ptr[p0 + g + 1] && col_idx[at[(size_t)g]] == c) from = at[(size_t)g]++;
                m_src[out * group + g] = (int32_t)from;
                if (with_vals && from >= 0) std::memcpy(dst + (out * group + g) * vb, src + from * vb, (size_t)vb);
            }
            ++out;
        }
        m_row_ptr[sp + 1] = (int32_t)out;
    }
    return MC_OK;
}
