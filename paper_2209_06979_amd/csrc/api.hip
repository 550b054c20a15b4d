// C-ABI entry points: argument checks on the host, then kernel launches on the caller's
// stream.  See include/magicube.h for the contract of every function.
#include "internal.h"

#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <mutex>
#include <new>
#include <vector>

namespace {

// The calling thread's default choices (all zero = automatic).  A compute call copies either the
// options it was handed or these once, at entry, and never looks at shared state afterwards.
thread_local mc_options t_options = {};

bool valid_options(const mc_options &o)
{
    const int b = o.spmm_row_tile_bytes, w = o.spmm_waves, d = o.sddmm_waves;
    if (b != 0 && b != 64 && b != 128 && b != 256) return false;
    if (w != 0 && w != 1 && w != 2 && w != 4 && w != 8) return false;
    if (o.spmm_stages < 0 || o.spmm_stages > 2) return false;
    if (o.spmm_splitting < -1 || o.spmm_splitting > 1) return false;
    if (o.spmm_slab < -1 || o.spmm_slab > 1) return false;
    if (o.spmm_slab_waves < 0 || o.spmm_slab_waves > 15) return false;
    if (o.spmm_slab_panels != 0 && o.spmm_slab_panels != 1 && o.spmm_slab_panels != 2 && o.spmm_slab_panels != 4) return false;
    if (d != 0 && d != -1 && d != 1 && d != 2 && d != 4 && d != 8) return false;
    if (o.softmax_variant < 0 || o.softmax_variant > 2) return false;
    if (o.attention_mode < 0 || o.attention_mode > 6) return false;
    if (o.spmm_merge < -1 || o.spmm_merge > 1) return false;
    return true;
}

// The options of one call: the caller's (validated), or the thread's defaults.
int resolve_options(const mc_options *given, mc_options *out)
{
    if (given) {
        if (!valid_options(*given)) return MC_EINVAL;
        *out = *given;
    } else {
        *out = t_options;
    }
    return MC_OK;
}

inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline int lhs_bits_of(mc_prec p)
{
    switch (p) {
    case MC_L4R4: return 4;
    case MC_L16R8: case MC_L16R16: case MC_L16R4: return 16;
    case MC_L12R4: return 12;
    default: return 8;
    }
}
inline int rhs_bits_of(mc_prec p)
{
    switch (p) {
    case MC_L8R4: case MC_L4R4: case MC_L16R4: case MC_L12R4: return 4;
    case MC_L16R16: return 16;
    default: return 8;
    }
}
inline bool valid_prec(int p) { return p >= MC_L8R8 && p <= MC_L12R4; }

thread_local char g_detail[256] = "";

// Remembers which HIP call failed and why (read back with mc_last_error_detail).
bool hip_ok(hipError_t e, const char *what)
{
    if (e == hipSuccess) return true;
    snprintf(g_detail, sizeof g_detail, "%s: %s", what, hipGetErrorString(e));
    (void)hipGetLastError();
    return false;
}

#define MC_HIP(call)                               \
    do {                                           \
        if (!hip_ok((call), #call)) return MC_EHIP; \
    } while (0)

// Every compute call works on the device the operand was created on: its buffers are not
// addressable from another one.
bool on_device_of(const mc_mat *A)
{
    int cur = -1;
    if (!hip_ok(hipGetDevice(&cur), "hipGetDevice")) return false;
    if (cur != A->device) {
        snprintf(g_detail, sizeof g_detail, "sparse operand lives on device %d, the current device is %d", A->device, cur);
        return false;
    }
    return true;
}

void free_device(mc_mat *A)
{
    if (A->d_panel_ptr) (void)hipFree(A->d_panel_ptr);
    if (A->d_row_ptr) (void)hipFree(A->d_row_ptr);
    if (A->d_slot_idx) (void)hipFree(A->d_slot_idx);
    if (A->d_vals) (void)hipFree(A->d_vals);
    if (A->d_items) (void)hipFree(A->d_items);
    if (A->d_split_panels) (void)hipFree(A->d_split_panels);
    if (A->d_blk_ptr) (void)hipFree(A->d_blk_ptr);
    if (A->d_blk_rows) (void)hipFree(A->d_blk_rows);
    if (A->d_blk_vals) (void)hipFree(A->d_blk_vals);
    if (A->d_blk_src) (void)hipFree(A->d_blk_src);
    if (A->d_class_panels) (void)hipFree(A->d_class_panels);
    if (A->d_merge_src) (void)hipFree(A->d_merge_src);
    if (A->d_merge_vals) (void)hipFree(A->d_merge_vals);
    if (A->merged) {
        free_device(A->merged);
        delete A->merged;
        A->merged = nullptr;
    }
}

// Waves per panel for SDDMM: enough to put about 2048 waves on the chip (4096 of the light ones
// that stage rows of 32 bytes, or 64 bytes of nibbles), fewer than twice the chunks of an average panel.
int choose_sddmm_waves(const mc_mat *mask, int batch, int row_bytes, int bits, const mc_options &o)
{
    if (o.sddmm_waves != 0) return o.sddmm_waves < 0 ? 0 : o.sddmm_waves; // 0 selects the direct-load kernel in launch_sddmm
    const double avg = mask->P ? (double)(mask->nslots / MC_CHUNK) / mask->P : 0.0;
    const double groups = (double)mask->P * (batch > 0 ? batch : 1);
    const double target = (row_bytes <= 32 || (bits == 4 && row_bytes <= 64)) ? 4096.0 : 2048.0;
    int w = 1;
    // (down to one chunk per wave, e.g. 32 panels of 7 chunks: 2.8 us with 4 waves, 2.4 us with 8)
    while (w < 8 && groups * w * 2 <= target && w < avg) w *= 2;
    return w;
}

// SpMM tile variant for a problem (from sweeps on MI355X).  Rows are cut into 128-byte tiles, into
// 256-byte tiles when panels are long, into 64-byte tiles when rows or panels are short; the chunks
// of a panel are shared by as many waves as it takes to put about 2048 waves on the chip, but
// never more waves than a panel has chunks.
// max_unit: chunks of the longest unit of work (panel or work item) of this launch.
// lhs_bits: width of the sparse operand's values in this launch (a mask carries none of its own).
void choose_variant(const mc_mat *A, int lhs_bits, int row_bytes, bool r4, int batch, int max_unit, const mc_options &o, int *bnb,
                    int *waves)
{
    int b = o.spmm_row_tile_bytes, w = o.spmm_waves;
    const double avg = A->P ? (double)(A->nslots / MC_CHUNK) / A->P : 0.0;
    if (b == 0) {
        if (r4) {
            // a 64-byte tile of nibbles already yields 128 output columns
            // (rows of 128 bytes: the wider tile only for long panels, and not with a two-plane A and V = 8,
            // i.e. 16 output rows per tile: L16-R4, N=256, 70 % sparse 13.4 us on 128-byte, 11.2 us on 64-byte tiles)
            const bool two_planes = (lhs_bits != 8 && lhs_bits != 4 && A->V == 8) || A->V == 16; // 16 output rows per tile
            b = ((row_bytes >= 256 && avg >= 2.0) || (row_bytes >= 128 && avg >= 16.0 && !two_planes)) ? 128 : 64;
        } else {
            b = 128;
            if (row_bytes < 128 || (row_bytes == 128 && avg < 4.0) || (row_bytes < 512 && avg < 2.0) || avg < 3.0) b = 64;
            // wide tiles for panels of 8 chunks and more; with a two-plane A and V = 8 (16 output rows per
            // tile) only for long rows
            if (row_bytes >= 256 && avg >= 8.0 && ((lhs_bits == 8 && A->V <= 8) || A->V < 8 || row_bytes >= 512)) b = 256;
            if (row_bytes >= 1024 && avg >= 6.0) b = 256; // eight and more 128-byte tiles would each re-read A
        }
    }
    if (b == 256 && r4) b = 128;
    // few panels: narrower tiles until there is a workgroup for every compute unit (a 256 x 2304 matrix
    // with rows of 512 bytes: 5.7 us on 256-byte tiles, 3.3 us on 64-byte ones)
    // (rows of nibbles, fewer than 512 panels: until the panels' chunks can occupy 4096 of the light waves)
    if (o.spmm_row_tile_bytes == 0) {
        const double nb = (batch > 0 ? batch : 1), per_group = std::min(8.0, std::max(1.0, avg));
        while (b > 64 && (double)A->P * ((row_bytes + b - 1) / b) * nb < 256.0) b /= 2;
        if (r4 && A->P < 512)
            while (b > 64 && (double)A->P * ((row_bytes + b - 1) / b) * nb * per_group < 4096.0) b /= 2;
    }
    if (w == 0) {
        const double groups = (double)A->P * ((row_bytes + b - 1) / b) * (batch > 0 ? batch : 1);
        // about 2048 waves on the chip; 4096 of the lighter ones that gather 64-byte pieces of nibbles
        const double target = (r4 && b == 64) ? 4096.0 : 2048.0;
        w = 1;
        while (w < 8 && groups * w * 2 <= target && w * 2 <= avg) w *= 2;
        // long panels on the narrower tiles: at most 16 chunks per wave (8 with a two-plane A and V = 8)
        if (!r4 && b != 256) {
            const double per_wave = ((lhs_bits != 8 && A->V == 8) || A->V == 16) ? 8.0 : 16.0;
            while (w < 8 && avg > per_wave * w) w *= 2;
        }
        // unequal panels (longest unit above twice the average): the longest unit sets the time of the
        // launch; no wave gets more than 8 chunks of it
        while (w < 8 && max_unit > 2.0 * avg && max_unit > 8 * w) w *= 2;
    }
    *bnb = b;
    *waves = w;
}

} // namespace

extern "C" const char *mc_strerror(int status)
{
    switch (status) {
    case MC_OK: return "ok";
    case MC_EINVAL: return "invalid argument";
    case MC_EUNSUPPORTED: return "unsupported precision or operation";
    case MC_EALIGN: return "pointer or leading dimension not 16-byte aligned";
    case MC_EHIP: return "HIP runtime error";
    case MC_ENOMEM: return "out of memory or workspace too small";
    case MC_ERANGE: return "value out of representable range";
    default: return "unknown status";
    }
}

#ifndef MC_SOURCE_ID
#define MC_SOURCE_ID "unidentified"
#endif
extern "C" const char *mc_version(void) { return "0.2+" MC_SOURCE_ID " gfx950"; }

extern "C" const char *mc_last_error_detail(void) { return g_detail; }

extern "C" void mc_options_init(mc_options *o)
{
    if (o) *o = mc_options{};
}

extern "C" int mc_set_thread_options(const mc_options *o)
{
    if (!o) {
        t_options = mc_options{};
        return MC_OK;
    }
    if (!valid_options(*o)) return MC_EINVAL;
    t_options = *o;
    return MC_OK;
}

extern "C" int mc_get_thread_options(mc_options *o)
{
    if (!o) return MC_EINVAL;
    *o = t_options;
    return MC_OK;
}

// The older one-knob setters: each changes one field of the calling thread's defaults.
namespace {
template <class F> int set_field(F &&f)
{
    mc_options o = t_options;
    f(o);
    if (!valid_options(o)) return MC_EINVAL;
    t_options = o;
    return MC_OK;
}
} // namespace

extern "C" int mc_set_spmm_variant(int bytes_per_row_tile, int waves)
{
    return set_field([&](mc_options &o) { o.spmm_row_tile_bytes = bytes_per_row_tile; o.spmm_waves = waves; });
}

extern "C" int mc_set_spmm_stages(int stages)
{
    if (stages != 1 && stages != 2) return MC_EINVAL;
    return set_field([&](mc_options &o) { o.spmm_stages = stages; });
}

extern "C" int mc_set_spmm_splitting(int enable)
{
    return set_field([&](mc_options &o) { o.spmm_splitting = enable ? 0 : -1; });
}

extern "C" int mc_set_sddmm_variant(int waves)
{
    // this setter's own convention: -1 automatic, 0 the direct-load kernel
    if (waves < -1) return MC_EINVAL;
    return set_field([&](mc_options &o) { o.sddmm_waves = (waves == -1) ? 0 : (waves == 0 ? -1 : waves); });
}

extern "C" int mc_set_softmax_variant(int variant)
{
    return set_field([&](mc_options &o) { o.softmax_variant = variant; });
}

extern "C" int mc_set_attention_mode(int mode)
{
    return set_field([&](mc_options &o) { o.attention_mode = mode; });
}

namespace {
// Whether mc_mat_create builds the merged copy (lay: the operand, ml: its merged form).  The copy holds
// ml.nvec * rows values; which of the two a call uses is decided per call (merged_pays).
bool merged_worth_building(const mc_layout &lay, const mc_merged_layout &ml, int V)
{
    (void)V;
    return ml.nvec <= lay.nvec;
}

// child: the merged copy of another operand (V up to 16, never merged again)
int mat_create_impl(int M, int K, int V, int lhs_bits, const int32_t *row_ptr, const int32_t *col_idx, const void *values,
                    void *stream, bool child, mc_mat **out)
{
    if (!out) return MC_EINVAL;
    *out = nullptr;
    if (!values) lhs_bits = 0;
    if (!child && V == 16) return MC_EINVAL;
    mc_layout lay;
    int rc = mc_layout_query_wide(M, K, V, lhs_bits, row_ptr, &lay);
    if (rc != MC_OK) return rc;

    std::vector<int32_t> panel_ptr, slot_idx;
    std::vector<uint8_t> vals;
    try {
        panel_ptr.resize((size_t)2 * lay.P);
        slot_idx.resize((size_t)lay.nslots);
        vals.resize((size_t)lay.vals_bytes);
    } catch (const std::bad_alloc &) {
        return MC_ENOMEM;
    }
    rc = mc_pack_host_wide(M, K, V, lhs_bits, row_ptr, col_idx, values, panel_ptr.data(), slot_idx.data(),
                           vals.empty() ? nullptr : vals.data());
    if (rc != MC_OK) return rc;

    mc_mat *A = new (std::nothrow) mc_mat();
    if (!A) return MC_ENOMEM;
    A->M = M; A->K = K; A->V = V; A->lhs_bits = lhs_bits; A->P = lay.P;
    A->nvec = lay.nvec; A->nslots = lay.nslots; A->vals_bytes = lay.vals_bytes;
    A->max_panel_chunks = 0;
    int min_panel_chunks = INT32_MAX;
    for (int p = 0; p < lay.P; ++p) {
        const int c = (row_ptr[p + 1] - row_ptr[p] + MC_CHUNK - 1) / MC_CHUNK;
        if (c > A->max_panel_chunks) A->max_panel_chunks = c;
        if (c < min_panel_chunks) min_panel_chunks = c;
    }
    A->uniform_chunks = (lay.P > 0 && min_panel_chunks == A->max_panel_chunks && min_panel_chunks > 0) ? min_panel_chunks : 0;
    A->d_panel_ptr = A->d_row_ptr = A->d_slot_idx = nullptr;
    A->d_vals = nullptr;
    A->d_items = A->d_split_panels = nullptr;
    A->n_items = A->n_split = 0;
    A->max_item_chunks = 0;
    A->nblk = 0; A->blk_chunks = 0; A->blk_valid = false;
    A->d_blk_ptr = nullptr; A->d_blk_rows = nullptr; A->d_blk_vals = nullptr; A->d_blk_src = nullptr;
    A->d_class_panels = nullptr;
    A->merged = nullptr; A->merge_group = 0; A->d_merge_src = nullptr; A->d_merge_vals = nullptr; A->merged_valid = false;
    // Length classes of the panels (V = 8: the attention kernel gives a panel 1, 2, 4 or 8 waves)
    std::vector<int32_t> class_panels;
    for (int b = 0; b <= 4; ++b) A->class_start[b] = 0;
    if (V == 8 && lay.P > 0) {
        auto class_of = [&](int p) {
            const int c = (row_ptr[p + 1] - row_ptr[p] + MC_CHUNK - 1) / MC_CHUNK;
            return c <= 8 ? 0 : (c <= 16 ? 1 : (c <= 32 ? 2 : 3));
        };
        int count[4] = {0, 0, 0, 0};
        for (int p = 0; p < lay.P; ++p) ++count[class_of(p)];
        if ((count[0] > 0) + (count[1] > 0) + (count[2] > 0) + (count[3] > 0) > 1) {
            try {
                class_panels.resize((size_t)lay.P);
            } catch (const std::bad_alloc &) {
                delete A;
                return MC_ENOMEM;
            }
            int next[4];
            for (int b = 0, at = 0; b < 4; ++b) { A->class_start[b] = next[b] = at; at += count[b]; }
            A->class_start[4] = lay.P;
            for (int p = 0; p < lay.P; ++p) class_panels[(size_t)next[class_of(p)]++] = p;
        }
    }
    // Work items: only when the longest panel is far above the average; a panel is then cut into
    // pieces of at most `cap` chunks (cap = three times the average, at least 8: smaller pieces
    // balance better but cost the SpMM more in atomics than they gain; measured).
    std::vector<int32_t> items, split_panels;
    {
        const double avg = lay.P ? (double)(lay.nslots / MC_CHUNK) / lay.P : 0.0;
        // A pattern-only mask (SDDMM: every item writes its own outputs, nothing to add up) is cut
        // as soon as a panel exceeds the average rounded up to 8 chunks.
        // With fewer than 256 panels the pieces also get short enough to make 256 of them.
        const bool mask_only = (lhs_bits == 0);
        double piece = (mask_only ? 1.0 : 3.0) * avg;
        if (mask_only && lay.P < 256) piece = std::min(piece, (double)(lay.nslots / MC_CHUNK) / 256.0);
        const int cap = std::max(8, (int)std::ceil(piece));
        if (A->max_panel_chunks > (mask_only ? cap : 2 * cap)) {
            try {
                for (int p = 0; p < lay.P; ++p) {
                    const int c = (row_ptr[p + 1] - row_ptr[p] + MC_CHUNK - 1) / MC_CHUNK;
                    const int pieces = (c + cap - 1) / cap;
                    if (pieces > 1) split_panels.push_back(p);
                    if (pieces <= 1) {
                        items.insert(items.end(), {p, 0, c, 0});
                    } else {
                        const int per = (c + pieces - 1) / pieces;
                        // (fourth field: 1 + the panel's position in split_panels)
                        for (int b = 0; b < c; b += per) items.insert(items.end(), {p, b, std::min(c, b + per), (int)split_panels.size()});
                    }
                }
            } catch (const std::bad_alloc &) {
                delete A;
                return MC_ENOMEM;
            }
            // longest first: workgroups start in this order, so the long items do not form the tail
            {
                const size_t ni = items.size() / 4;
                std::vector<size_t> order(ni);
                for (size_t i = 0; i < ni; ++i) order[i] = i;
                std::stable_sort(order.begin(), order.end(), [&](size_t x, size_t y) {
                    return items[4 * x + 2] - items[4 * x + 1] > items[4 * y + 2] - items[4 * y + 1];
                });
                std::vector<int32_t> sorted(items.size());
                for (size_t i = 0; i < ni; ++i) std::copy(items.begin() + 4 * order[i], items.begin() + 4 * order[i] + 4, sorted.begin() + 4 * i);
                items.swap(sorted);
            }
            A->n_items = (int)(items.size() / 4);
            A->n_split = (int)split_panels.size();
            A->max_item_chunks = 0;
            for (size_t i = 0; i < items.size(); i += 4) A->max_item_chunks = std::max(A->max_item_chunks, items[i + 2] - items[i + 1]);
        }
    }
    // K-blocked copy for the SpMM that keeps blocks of B resident in LDS: for operands with values whose
    // panels are about equally long and dense enough that the per-(panel, block) padding stays moderate
    // (at most half as many slots again as there are vectors), unless the thread's options rule that kernel out.
    std::vector<int32_t> blk_ptr, blk_src;
    std::vector<uint16_t> blk_rows;
    std::vector<uint8_t> blk_vals;
    if (lhs_bits != 0 && lay.nvec > 0 && (A->n_items == 0 || t_options.spmm_slab == 1) && t_options.spmm_slab != -1) {
        mc_blocked_layout bl;
        // (spmm_slab == 1 on the creating thread: built whatever the shape, so that the form can be forced)
        const bool forced = t_options.spmm_slab == 1;
        if (mc_blocked_query_wide(M, K, V, lhs_bits, row_ptr, col_idx, &bl) == MC_OK && bl.nblk <= 63 && bl.nchunks > 0 &&
            (forced || ((double)lay.nvec >= 160.0 * lay.P * bl.nblk && // (below about 160 vectors per list the form never won)
                        bl.nchunks * MC_CHUNK <= lay.nvec + lay.nvec / 2 &&
                        A->max_panel_chunks <= 2.0 * (double)(lay.nslots / MC_CHUNK) / lay.P + 1.0))) {
            try {
                blk_ptr.resize((size_t)lay.P * bl.nblk + 1);
                blk_rows.resize((size_t)bl.nchunks * MC_CHUNK);
                blk_src.resize((size_t)bl.nchunks * MC_CHUNK);
                blk_vals.resize((size_t)bl.vals_bytes);
            } catch (const std::bad_alloc &) {
                delete A;
                return MC_ENOMEM;
            }
            rc = mc_pack_blocked_host_wide(M, K, V, lhs_bits, row_ptr, col_idx, values, blk_ptr.data(), blk_rows.data(),
                                           blk_vals.data(), blk_src.data());
            if (rc != MC_OK) {
                delete A;
                return rc;
            }
            A->nblk = bl.nblk;
            A->blk_chunks = bl.nchunks;
        }
    }
    hipStream_t s = static_cast<hipStream_t>(stream);
#define MC_TRY(call) (ok = ok && hip_ok((call), #call))
    bool ok = true;
    MC_TRY(hipGetDevice(&A->device));
    // the index array gets one spare chunk so that 16-byte index reads never leave it
    MC_TRY(hipMalloc(&A->d_panel_ptr, sizeof(int32_t) * 2 * (size_t)(lay.P + 1)));
    MC_TRY(hipMalloc(&A->d_row_ptr, sizeof(int32_t) * (size_t)(lay.P + 1)));
    MC_TRY(hipMalloc(&A->d_slot_idx, sizeof(int32_t) * (size_t)(lay.nslots + MC_CHUNK)));
    if (lay.vals_bytes) MC_TRY(hipMalloc(&A->d_vals, (size_t)lay.vals_bytes));
    MC_TRY(hipMemcpyAsync(A->d_panel_ptr, panel_ptr.data(), sizeof(int32_t) * 2 * (size_t)lay.P, hipMemcpyHostToDevice, s));
    MC_TRY(hipMemcpyAsync(A->d_row_ptr, row_ptr, sizeof(int32_t) * (size_t)(lay.P + 1), hipMemcpyHostToDevice, s));
    if (lay.nslots)
        MC_TRY(hipMemcpyAsync(A->d_slot_idx, slot_idx.data(), sizeof(int32_t) * (size_t)lay.nslots, hipMemcpyHostToDevice, s));
    if (lay.vals_bytes)
        MC_TRY(hipMemcpyAsync(A->d_vals, vals.data(), (size_t)lay.vals_bytes, hipMemcpyHostToDevice, s));
    if (A->n_items) {
        MC_TRY(hipMalloc(&A->d_items, sizeof(int32_t) * items.size()));
        MC_TRY(hipMalloc(&A->d_split_panels, sizeof(int32_t) * split_panels.size()));
        MC_TRY(hipMemcpyAsync(A->d_items, items.data(), sizeof(int32_t) * items.size(), hipMemcpyHostToDevice, s));
        MC_TRY(hipMemcpyAsync(A->d_split_panels, split_panels.data(), sizeof(int32_t) * split_panels.size(),
                              hipMemcpyHostToDevice, s));
    }
    if (A->blk_chunks) {
        MC_TRY(hipMalloc(&A->d_blk_ptr, sizeof(int32_t) * blk_ptr.size()));
        MC_TRY(hipMalloc(&A->d_blk_rows, sizeof(uint16_t) * blk_rows.size()));
        MC_TRY(hipMalloc(&A->d_blk_src, sizeof(int32_t) * blk_src.size()));
        MC_TRY(hipMalloc(&A->d_blk_vals, blk_vals.size()));
        MC_TRY(hipMemcpyAsync(A->d_blk_ptr, blk_ptr.data(), sizeof(int32_t) * blk_ptr.size(), hipMemcpyHostToDevice, s));
        MC_TRY(hipMemcpyAsync(A->d_blk_rows, blk_rows.data(), sizeof(uint16_t) * blk_rows.size(), hipMemcpyHostToDevice, s));
        MC_TRY(hipMemcpyAsync(A->d_blk_src, blk_src.data(), sizeof(int32_t) * blk_src.size(), hipMemcpyHostToDevice, s));
        MC_TRY(hipMemcpyAsync(A->d_blk_vals, blk_vals.data(), blk_vals.size(), hipMemcpyHostToDevice, s));
        A->blk_valid = true;
    }
    if (!class_panels.empty()) {
        MC_TRY(hipMalloc(&A->d_class_panels, sizeof(int32_t) * class_panels.size()));
        MC_TRY(hipMemcpyAsync(A->d_class_panels, class_panels.data(), sizeof(int32_t) * class_panels.size(), hipMemcpyHostToDevice, s));
    }
    // Merged copy for the SpMM: panels of fewer rows than the matrix unit takes share one panel of 16 rows (4- and
    // 8-bit values) or 8 rows (two byte planes), see mc_merge_host.  Not for operands without vectors, and not
    // when the thread's options rule it out.
    std::vector<int32_t> m_src;
    int64_t m_vals_bytes = 0;
    if (!child && lhs_bits != 0 && lay.nvec > 0 && t_options.spmm_merge != -1) {
        const int rows = (lhs_bits == 4 || lhs_bits == 8) ? 16 : 8, group = rows / V;
        mc_merged_layout ml;
        if (group >= 2 && mc_merged_query(M, K, V, lhs_bits, row_ptr, col_idx, group, &ml) == MC_OK && ml.nvec > 0 &&
            (t_options.spmm_merge == 1 || merged_worth_building(lay, ml, V))) {
            std::vector<int32_t> m_row_ptr, m_col_idx;
            std::vector<uint8_t> m_values;
            const int64_t vb = (int64_t)V * (lhs_bits == 12 ? 16 : lhs_bits) / 8;
            try {
                m_row_ptr.resize((size_t)ml.P + 1);
                m_col_idx.resize((size_t)ml.nvec);
                m_values.resize((size_t)(ml.nvec * group * vb));
                m_src.resize((size_t)(ml.nvec * group));
            } catch (const std::bad_alloc &) {
                free_device(A);
                delete A;
                return MC_ENOMEM;
            }
            rc = mc_merge_host(M, K, V, lhs_bits, row_ptr, col_idx, values, group, m_row_ptr.data(), m_col_idx.data(), m_values.data(),
                               m_src.data());
            if (rc == MC_OK)
                rc = mat_create_impl(ml.P * rows, K, rows, lhs_bits, m_row_ptr.data(), m_col_idx.data(), m_values.data(), stream, true,
                                     &A->merged);
            if (rc != MC_OK) {
                free_device(A);
                delete A;
                return rc;
            }
            A->merge_group = group;
            m_vals_bytes = (int64_t)m_values.size();
        }
    }
    if (A->merged) {
        MC_TRY(hipMalloc(&A->d_merge_src, sizeof(int32_t) * m_src.size()));
        MC_TRY(hipMalloc(&A->d_merge_vals, (size_t)m_vals_bytes));
        MC_TRY(hipMemcpyAsync(A->d_merge_src, m_src.data(), sizeof(int32_t) * m_src.size(), hipMemcpyHostToDevice, s));
        A->merged_valid = true;
    }
    MC_TRY(hipStreamSynchronize(s)); // host staging buffers die at return
#undef MC_TRY
    if (!ok) {
        free_device(A);
        delete A;
        return MC_EHIP;
    }
    *out = A;
    return MC_OK;
}
} // namespace

extern "C" int mc_mat_create(int M, int K, int V, int lhs_bits, const int32_t *row_ptr, const int32_t *col_idx,
                             const void *values, void *stream, mc_mat **out)
{
    return mat_create_impl(M, K, V, lhs_bits, row_ptr, col_idx, values, stream, false, out);
}

extern "C" int mc_mat_merged_info(const mc_mat *A, int *group, int64_t *nvec)
{
    if (!A) return MC_EINVAL;
    if (group) *group = A->merged ? A->merge_group : 0;
    if (nvec) *nvec = A->merged ? A->merged->nvec : 0;
    return MC_OK;
}

extern "C" void mc_mat_destroy(mc_mat *A)
{
    if (!A) return;
    free_device(A);
    delete A;
}

extern "C" int mc_mat_info(const mc_mat *A, int *M, int *K, int *V, int *lhs_bits, int64_t *nvec, int64_t *nslots)
{
    if (!A) return MC_EINVAL;
    if (M) *M = A->M;
    if (K) *K = A->K;
    if (V) *V = A->V;
    if (lhs_bits) *lhs_bits = A->lhs_bits;
    if (nvec) *nvec = A->nvec;
    if (nslots) *nslots = A->nslots;
    return MC_OK;
}

extern "C" int mc_mat_set_values_device(mc_mat *A, const void *values_dev, void *stream)
{
    if (!A) return MC_EINVAL;
    if (A->lhs_bits == 0) return MC_EINVAL;        // a pattern-only mask holds no values
    if (A->nslots == 0) return MC_OK;              // no stored vector: nothing to replace
    if (!values_dev) return MC_EINVAL;
    if (!on_device_of(A)) return MC_EINVAL;
    RepackArgs r;
    r.panel_ptr = A->d_panel_ptr; r.row_ptr = A->d_row_ptr;
    r.src = static_cast<const uint8_t *>(values_dev); r.src_batch_stride = 0;
    r.dst = A->d_vals; r.dst_batch_stride = 0;
    r.P = A->P; r.V = A->V; r.bits = (A->lhs_bits == 12) ? 16 : A->lhs_bits; r.batch = 1;
    MC_HIP(launch_repack(r, static_cast<hipStream_t>(stream)));
    if (A->d_blk_vals) { // the K-blocked copy follows
        MC_HIP(launch_repack_blocked(A->d_blk_src, r.src, A->d_blk_vals, A->blk_chunks, A->V, r.bits, static_cast<hipStream_t>(stream)));
        A->blk_valid = true;
    }
    if (A->merged) { // and the merged copy: its values in interchange order first, then its own formats
        const int vb = A->V * r.bits / 8;
        MC_HIP(launch_merge_values(A->d_merge_src, r.src, A->d_merge_vals, A->merged->nvec * A->merge_group, vb,
                                   static_cast<hipStream_t>(stream)));
        const int rc = mc_mat_set_values_device(A->merged, A->d_merge_vals, stream);
        if (rc != MC_OK) return rc;
        A->merged_valid = true;
    }
    return MC_OK;
}

namespace {
inline int spmm_stages_for(const mc_options &o, int K, int64_t ldb_bytes, int row_bytes)
{
    // (the two-chunk form works out a lane's offset into B with one 24-bit multiply-add)
    return (o.spmm_stages != 1 && (int64_t)(K - 1) * ldb_bytes + row_bytes < ((int64_t)1 << 32) && K <= (1 << 24) &&
            ldb_bytes < (1 << 24)) ? 2 : 1;
}

// Work split of the SpMM that keeps K-blocks of B resident in LDS: one workgroup per (64-byte column
// tile, group of ppg consecutive panels); about one workgroup per compute unit (each takes 128 KB of
// LDS), more groups when a wave would otherwise own more panels than its registers hold.
struct SlabPlan { int groups, ppg, wpp, nc, ppw, passes; int64_t workgroups; };
bool plan_slab(const mc_mat *A, int row_bytes, bool r4, int batch, const mc_options &o, SlabPlan *pl)
{
    const int T = (row_bytes + 63) / 64, max_ppw = r4 ? 2 : 4;
    int64_t G = (256 + (int64_t)T * batch - 1) / ((int64_t)T * batch);
    if (G > A->P) G = A->P;
    if (G < 1) G = 1;
    const int ppg = (int)((A->P + G - 1) / G);
    G = (A->P + ppg - 1) / ppg;
    pl->groups = (int)G;
    pl->ppg = ppg;
    pl->workgroups = G * T * batch;
    // Twelve computing waves and four filling ones (one filling wave alone is bound by the latency of its own
    // copies: 3.3 against 1.6 us per 64 KB block).  More panels than waves: two panels per wave and as many
    // passes over K as it takes (measured against 8 x 2, 8 x 4, 12 x 1 and 15 x 1/2/4: 12 x 2 is the fastest or
    // within 5 % of it from 13 panels per workgroup on).  Fewer panels than waves: several waves share a panel's
    // chunks, at most four and no more than a (panel, block) list has chunks on average.
    if (ppg > 12) {
        pl->nc = 12; pl->wpp = 1; pl->ppw = 2; pl->passes = (ppg + 23) / 24;
    } else {
        const double per_list = (double)A->blk_chunks / ((double)A->P * A->nblk);
        int wpp = 12 / ppg;
        if (wpp > 4) wpp = 4;
        while (wpp > 1 && wpp > per_list) --wpp;
        pl->nc = ppg * wpp; pl->wpp = wpp; pl->ppw = 1; pl->passes = 1;
    }
    if (o.spmm_slab_waves || o.spmm_slab_panels) {
        // a pinned shape: one wave per panel, as many passes as it takes
        pl->nc = o.spmm_slab_waves ? o.spmm_slab_waves : pl->nc;
        pl->ppw = o.spmm_slab_panels ? o.spmm_slab_panels : pl->ppw;
        pl->wpp = 1;
        pl->passes = (ppg + pl->nc * pl->ppw - 1) / (pl->nc * pl->ppw);
    }
    return pl->ppw <= max_ppw;
}

// Whether the LDS-resident form is expected to beat the gather form.  Both times (microseconds) are least-squares
// fits to measurements on MI355X over V in {2, 4, 8}, six sparsities and N in {128, 256, 512} at 4096 x 4096, for
// byte and for nibble rows of B apart (nibble rows take two MFMA steps per 64 bytes).  Gather form: a start-up
// term plus its gathered bytes at 22 (nibbles: 14) TB/s.  LDS-resident form: a start-up term, about 2 us per
// K-block and pass for the fill it cannot hide, and 16 (nibbles: 42) ns per chunk step of a compute unit.  Picking
// by these fits is on average 0.03 % and at worst 4 % slower than the better form over the points of that sweep
// where both exist.
bool slab_pays(const mc_mat *A, int row_bytes, bool r4, int batch, const SlabPlan &pl)
{
    const double T = (double)((row_bytes + 63) / 64);
    double t_gather = (r4 ? 3.88 : 3.96) + (double)A->nvec * row_bytes * batch / (r4 ? 13.99e6 : 22.13e6);
    if (A->V == 16) {
        // merged copies (16-row panels, fewer and longer): the gather form fitted on the merged operands of the same sweep
        const double t0 = r4 ? 3.9 : (row_bytes >= 512 ? 4.4 : 3.3);
        const double rate = r4 ? (row_bytes == 128 ? 10.0e6 : 12.5e6) : (row_bytes >= 512 ? 20.5e6 : 17.7e6);
        t_gather = t0 + (double)A->nvec * row_bytes * batch / rate;
    }
    const double steps = (double)A->blk_chunks * T * batch / 256.0;
    const double rounds = std::max(1.0, std::ceil((double)pl.workgroups / 256.0) / ((double)pl.workgroups / 256.0));
    const double t_slab = (r4 ? 0.47 : 2.05) + (pl.passes * (r4 ? 2.12 : 1.98) * A->nblk + (r4 ? 0.0417 : 0.01565) * steps) * rounds;
    return t_slab < t_gather;
}

// The form one SpMM call takes: true = K-blocks of B resident in LDS (then *pl is its work split).
bool slab_chosen(const mc_mat *A, int row_bytes, int rb, unsigned flags, const mc_options &o, SlabPlan *pl)
{
    if (o.spmm_slab == -1 || !A->d_blk_vals || !A->blk_valid || flags != 0 || rb == 16 || o.spmm_row_tile_bytes != 0 ||
        o.spmm_waves != 0)
        return false;
    return plan_slab(A, row_bytes, rb == 4, 1, o, pl) && (o.spmm_slab == 1 || slab_pays(A, row_bytes, rb == 4, 1, *pl));
}

// Whether an SpMM call runs on the operand's merged copy.
bool merged_chosen(const mc_mat *A, int row_bytes, unsigned flags, const mc_options &o)
{
    if (!A->merged || !A->merged_valid || o.spmm_merge == -1) return false;
    if (flags != 0 && A->merged->V > 8) return false;
    if (o.spmm_merge == 1) return true;
    // Merged panels of 8 rows (two-plane values) run in the same kernel shape as unmerged ones with fewer gathered
    // rows, fewer padded slots and fewer panels: faster at 34 of 36 points of a 4096 x 4096 sweep (V = 2 / 4, six
    // sparsities, N = 128 .. 512), at worst 9 % slower.
    if (A->merged->V <= 8) return true;
    // Merged panels of 16 rows gather fewer rows (padded slots included) but run fewer, longer panels with 16-row
    // tiles; in the same sweep (V = 2 / 4 / 8) they are the faster form once they save about 24 MB of gathered rows.
    return (double)(A->nslots - A->merged->nslots) * row_bytes >= 24e6;
}

// out_mode 0: int32 results; 1 / 2: scale * result as fp32 / fp16 (fused dequantisation)
int spmm_impl(const mc_mat *A, const void *B_dev, int N, int ldb, mc_prec prec, unsigned flags, int out_mode,
              float scale, void *C_dev, int ldc, const mc_options *opts, void *stream)
{
    if (!A || !B_dev || !C_dev) return MC_EINVAL;
    mc_options o;
    if (resolve_options(opts, &o) != MC_OK) return MC_EINVAL;
    if (!valid_prec((int)prec)) return MC_EUNSUPPORTED;
    if (flags & ~(unsigned)(MC_LHS_UNSIGNED | MC_RHS_UNSIGNED)) return MC_EINVAL;
    if (flags && prec != MC_L8R8 && prec != MC_L8R4 && prec != MC_L4R4) return MC_EUNSUPPORTED;
    // (a matrix without any stored vector has no value buffer and is a valid all-zero operand)
    if ((!A->d_vals && A->nslots > 0) || A->lhs_bits != lhs_bits_of(prec)) return MC_EINVAL;
    const int rb = rhs_bits_of(prec);
    if (N <= 0 || N % (128 / rb) != 0) return MC_EINVAL; // whole 16-byte pieces of a row
    if (ldb < N || ldc < N) return MC_EINVAL;
    if (((int64_t)ldb * rb / 8) % 16 != 0 || ldc % 4 != 0) return MC_EALIGN;
    if (!aligned16(B_dev) || !aligned16(C_dev)) return MC_EALIGN;
    if (rb == 4 && A->K > ((flags != 0) ? 32768 : 131072)) return MC_EUNSUPPORTED;
    if (out_mode && !std::isfinite(scale)) return MC_EINVAL;
    if (!on_device_of(A)) return MC_EINVAL;

    // the operand's merged copy (panels of 8 or 16 rows at the union of their columns) where it is expected to be faster;
    // a 16-row panel leaves no MFMA row for the column sums that unsigned operands need
    const int rows = A->M;
    if (merged_chosen(A, N * rb / 8, flags, o)) A = A->merged;

    SpmmArgs a = {};
    a.rows = rows;
    a.lhs_unsigned = (flags & MC_LHS_UNSIGNED) ? 1 : 0; a.rhs_unsigned = (flags & MC_RHS_UNSIGNED) ? 1 : 0;
    a.panel_ptr = A->d_panel_ptr; a.slot_idx = A->d_slot_idx;
    a.vals = A->d_vals; a.vals_batch_stride = 0;
    a.B = static_cast<const uint8_t *>(B_dev); a.ldb_bytes = (int64_t)ldb * rb / 8; a.B_batch_stride = 0;
    a.row_bytes = N * rb / 8;
    a.C = C_dev; a.ldc = ldc; a.C_batch_stride = 0;
    a.P = A->P; a.V = A->V; a.batch = 1; a.float_out = out_mode; a.out_scale = out_mode ? scale : 1.f;
    // dense matrices: blocks of B resident in LDS instead of a gather per stored vector
    {
        SlabPlan pl;
        if (slab_chosen(A, a.row_bytes, rb, flags, o, &pl)) {
            SlabArgs sa = {};
            sa.blk_ptr = A->d_blk_ptr; sa.blk_rows = A->d_blk_rows; sa.vals = A->d_blk_vals; sa.vals_batch_stride = 0;
            sa.B = a.B; sa.ldb_bytes = a.ldb_bytes; sa.B_batch_stride = 0; sa.row_bytes = a.row_bytes; sa.K = A->K;
            sa.C = C_dev; sa.ldc = ldc; sa.C_batch_stride = 0;
            sa.P = A->P; sa.V = A->V; sa.batch = 1; sa.nblk = A->nblk; sa.rows = rows;
            sa.float_out = out_mode; sa.out_scale = a.out_scale;
            sa.groups = pl.groups; sa.ppg = pl.ppg; sa.wpp = pl.wpp; sa.nc = pl.nc;
            sa.nf = 16 - sa.nc < 4 ? 16 - sa.nc : 4;
            MC_HIP(launch_spmm_slab(prec, sa, pl.ppw, static_cast<hipStream_t>(stream)));
            return MC_OK;
        }
    }
    a.stages = spmm_stages_for(o, A->K, a.ldb_bytes, a.row_bytes);
    a.uniform_chunks = A->uniform_chunks;
    a.max_unit_chunks = A->max_panel_chunks;
    const bool use_items = A->n_items && o.spmm_splitting != -1 && out_mode == 0;
    if (use_items) a.max_unit_chunks = A->max_item_chunks;
    int bnb, waves;
    choose_variant(A, A->lhs_bits, a.row_bytes, rb == 4, 1, a.max_unit_chunks, o, &bnb, &waves);
    if (use_items) {
        // very unequal panels: long ones are shared by several workgroups that add into cleared rows
        // (integer results only: a scaled, rounded result cannot be accumulated piecewise)
        a.items = A->d_items; a.n_units = A->n_items;
        MC_HIP(launch_zero_rows(static_cast<int32_t *>(C_dev), ldc, N, A->V, A->d_split_panels, A->n_split,
                                static_cast<hipStream_t>(stream)));
    }
    MC_HIP(launch_spmm(prec, a, bnb, waves, static_cast<hipStream_t>(stream)));
    return MC_OK;
}
} // namespace

extern "C" int mc_spmm(const mc_mat *A, const void *B_dev, int N, int ldb, mc_prec prec, int32_t *C_dev, int ldc,
                       void *stream)
{
    return spmm_impl(A, B_dev, N, ldb, prec, 0u, 0, 1.f, C_dev, ldc, nullptr, stream);
}

extern "C" int mc_spmm_flags(const mc_mat *A, const void *B_dev, int N, int ldb, mc_prec prec, unsigned flags,
                             int32_t *C_dev, int ldc, void *stream)
{
    return spmm_impl(A, B_dev, N, ldb, prec, flags, 0, 1.f, C_dev, ldc, nullptr, stream);
}

extern "C" int mc_spmm_ex(const mc_mat *A, const void *B_dev, int N, int ldb, mc_prec prec, unsigned flags,
                          const mc_options *options, int32_t *C_dev, int ldc, void *stream)
{
    const mc_options automatic = {};
    return spmm_impl(A, B_dev, N, ldb, prec, flags, 0, 1.f, C_dev, ldc, options ? options : &automatic, stream);
}

extern "C" int mc_spmm_form(const mc_mat *A, int N, mc_prec prec, const mc_options *options)
{
    if (!A || N <= 0 || !valid_prec((int)prec) || A->lhs_bits != lhs_bits_of(prec)) return MC_EINVAL;
    const mc_options automatic = {};
    mc_options o;
    if (resolve_options(options ? options : &automatic, &o) != MC_OK) return MC_EINVAL;
    SlabPlan pl;
    const int rb = rhs_bits_of(prec);
    const bool merged = merged_chosen(A, N * rb / 8, 0u, o);
    if (merged) A = A->merged;
    return (slab_chosen(A, N * rb / 8, rb, 0u, o, &pl) ? 1 : 0) | (merged ? 2 : 0);
}

extern "C" int mc_spmm_dequant(const mc_mat *A, const void *B_dev, int N, int ldb, mc_prec prec, unsigned flags,
                               float scale, mc_out_type out_type, void *C_dev, int ldc, void *stream)
{
    if (out_type != MC_OUT_F32 && out_type != MC_OUT_F16) return MC_EUNSUPPORTED;
    return spmm_impl(A, B_dev, N, ldb, prec, flags, out_type == MC_OUT_F16 ? 2 : 1, scale, C_dev, ldc, nullptr, stream);
}

extern "C" int64_t mc_probe_gather_sink_len(const mc_mat *A, int N, mc_prec prec)
{
    if (!A || N <= 0 || !valid_prec((int)prec)) return 0;
    // the widest tiling (64-byte tiles) bounds the number of workgroups
    return (int64_t)A->P * (((int64_t)N * rhs_bits_of(prec) / 8 + 63) / 64);
}

extern "C" int mc_probe_gather(const mc_mat *A, const void *B_dev, int N, int ldb, mc_prec prec, int32_t *sink_dev,
                               void *stream)
{
    if (!A || !B_dev || !sink_dev) return MC_EINVAL;
    if (!valid_prec((int)prec)) return MC_EUNSUPPORTED;
    const int rb = rhs_bits_of(prec);
    if (N <= 0 || N % (128 / rb) != 0 || ldb < N) return MC_EINVAL;
    if (((int64_t)ldb * rb / 8) % 16 != 0 || !aligned16(B_dev)) return MC_EALIGN;
    if (!on_device_of(A)) return MC_EINVAL;
    const mc_options o = t_options;
    SpmmArgs a = {};
    a.panel_ptr = A->d_panel_ptr; a.slot_idx = A->d_slot_idx;
    a.vals = nullptr; a.vals_batch_stride = 0;
    a.B = static_cast<const uint8_t *>(B_dev); a.ldb_bytes = (int64_t)ldb * rb / 8; a.B_batch_stride = 0;
    a.row_bytes = N * rb / 8;
    a.C = nullptr; a.ldc = 0; a.C_batch_stride = 0;
    a.P = A->P; a.V = A->V; a.rows = A->M; a.batch = 1; a.float_out = 0; a.out_scale = 1.f;
    a.uniform_chunks = A->uniform_chunks;
    int bnb, waves;
    choose_variant(A, A->lhs_bits, a.row_bytes, rb == 4, 1, A->max_panel_chunks, o, &bnb, &waves);
    MC_HIP(launch_gather_probe(a, bnb, waves, sink_dev, static_cast<hipStream_t>(stream)));
    return MC_OK;
}

extern "C" int64_t mc_probe_spmm_phases_len(const mc_mat *A, int N)
{
    if (!A || N <= 0) return 0;
    return (int64_t)A->P * ((N + 127) / 128) * 2 * 10;
}

extern "C" int mc_probe_spmm_phases(const mc_mat *A, const void *B_dev, int N, int ldb, int32_t *C_dev, int ldc, int64_t *trace_dev,
                                    void *stream)
{
    if (!A || !B_dev || !C_dev || !trace_dev) return MC_EINVAL;
    if (N <= 0 || N % 16 != 0 || ldb < N || ldc < N) return MC_EINVAL;
    if (ldb % 16 != 0 || ldc % 4 != 0 || !aligned16(B_dev) || !aligned16(C_dev)) return MC_EALIGN;
    if (!on_device_of(A)) return MC_EINVAL;
    const mc_options automatic = {};
    if (A->lhs_bits != 8 || !A->d_vals || A->max_panel_chunks > 2 * 4 || spmm_stages_for(automatic, A->K, ldb, N) != 2)
        return MC_EUNSUPPORTED;
    SpmmArgs a = {};
    a.panel_ptr = A->d_panel_ptr; a.slot_idx = A->d_slot_idx; a.vals = A->d_vals;
    a.B = static_cast<const uint8_t *>(B_dev); a.ldb_bytes = ldb; a.row_bytes = N;
    a.C = C_dev; a.ldc = ldc;
    a.P = A->P; a.V = A->V; a.rows = A->M; a.batch = 1; a.out_scale = 1.f;
    a.stages = 2; a.max_unit_chunks = A->max_panel_chunks; a.uniform_chunks = A->uniform_chunks;
    a.trace = reinterpret_cast<long long *>(trace_dev);
    MC_HIP(launch_spmm_phase_probe(a, static_cast<hipStream_t>(stream)));
    return MC_OK;
}

extern "C" int mc_probe_mfma(int workgroups, int iters, int32_t *sink_dev, void *stream)
{
    if (!sink_dev || workgroups <= 0 || workgroups > 65535 || iters <= 0) return MC_EINVAL;
    MC_HIP(launch_mfma_probe(workgroups, iters, sink_dev, static_cast<hipStream_t>(stream)));
    return MC_OK;
}

namespace {
int sddmm_impl(const void *Q_dev, int ldq, const void *Kmat_dev, int ldk, int Kd, const mc_mat *mask, mc_prec prec,
               unsigned flags, int out_mode, float scale, void *S_dev, const mc_options *opts, void *stream)
{
    if (!Q_dev || !Kmat_dev || !mask) return MC_EINVAL;
    mc_options o;
    if (resolve_options(opts, &o) != MC_OK) return MC_EINVAL;
    if (!S_dev && mask->nvec > 0) return MC_EINVAL; // (a mask without any vector has an empty output)
    if (!valid_prec((int)prec)) return MC_EUNSUPPORTED;
    if (flags & ~(unsigned)(MC_LHS_UNSIGNED | MC_RHS_UNSIGNED)) return MC_EINVAL;
    if (flags && prec != MC_L8R8 && prec != MC_L4R4) return MC_EUNSUPPORTED;
    if (flags && prec == MC_L4R4 && Kd > 32768) return MC_EUNSUPPORTED; // 256x scaled sums stay inside int32
    if (prec != MC_L8R8 && prec != MC_L4R4 && prec != MC_L16R16) return MC_EUNSUPPORTED;
    const int bits = lhs_bits_of(prec);
    if (Kd <= 0 || Kd % (128 / bits) != 0 || ldq < Kd || ldk < Kd) return MC_EINVAL;
    if (((int64_t)ldq * bits / 8) % 16 != 0 || ((int64_t)ldk * bits / 8) % 16 != 0) return MC_EALIGN;
    if (!aligned16(Q_dev) || !aligned16(Kmat_dev) || !aligned16(S_dev)) return MC_EALIGN;
    if (out_mode && !std::isfinite(scale)) return MC_EINVAL;
    if (mask->nvec == 0) return MC_OK;
    if (!on_device_of(mask)) return MC_EINVAL;

    SddmmArgs a = {};
    a.float_out = out_mode; a.out_scale = out_mode ? scale : 1.f;
    a.panel_ptr = mask->d_panel_ptr; a.row_ptr = mask->d_row_ptr; a.slot_idx = mask->d_slot_idx;
    a.Q = static_cast<const uint8_t *>(Q_dev); a.ldq_bytes = (int64_t)ldq * bits / 8; a.Q_batch_stride = 0;
    a.Kmat = static_cast<const uint8_t *>(Kmat_dev); a.ldk_bytes = (int64_t)ldk * bits / 8; a.K_batch_stride = 0;
    a.row_bytes = Kd * bits / 8;
    a.S = S_dev; a.S_batch_stride = 0;
    a.P = mask->P; a.V = mask->V; a.batch = 1;
    a.lhs_unsigned = (flags & MC_LHS_UNSIGNED) ? 1 : 0; a.rhs_unsigned = (flags & MC_RHS_UNSIGNED) ? 1 : 0;
    if (mask->n_items && o.spmm_splitting != -1) { a.items = mask->d_items; a.n_units = mask->n_items; } // very unequal panels
    MC_HIP(launch_sddmm(bits, a, choose_sddmm_waves(mask, 1, a.row_bytes, bits, o), static_cast<hipStream_t>(stream)));
    return MC_OK;
}
} // namespace

extern "C" int mc_sddmm(const void *Q_dev, int ldq, const void *Kmat_dev, int ldk, int Kd, const mc_mat *mask,
                        mc_prec prec, int32_t *S_dev, void *stream)
{
    return sddmm_impl(Q_dev, ldq, Kmat_dev, ldk, Kd, mask, prec, 0u, 0, 1.f, S_dev, nullptr, stream);
}

extern "C" int mc_sddmm_flags(const void *Q_dev, int ldq, const void *Kmat_dev, int ldk, int Kd, const mc_mat *mask,
                              mc_prec prec, unsigned flags, int32_t *S_dev, void *stream)
{
    return sddmm_impl(Q_dev, ldq, Kmat_dev, ldk, Kd, mask, prec, flags, 0, 1.f, S_dev, nullptr, stream);
}

extern "C" int mc_sddmm_ex(const void *Q_dev, int ldq, const void *Kmat_dev, int ldk, int Kd, const mc_mat *mask,
                           mc_prec prec, unsigned flags, const mc_options *options, int32_t *S_dev, void *stream)
{
    const mc_options automatic = {};
    return sddmm_impl(Q_dev, ldq, Kmat_dev, ldk, Kd, mask, prec, flags, 0, 1.f, S_dev, options ? options : &automatic, stream);
}

extern "C" int mc_sddmm_dequant(const void *Q_dev, int ldq, const void *Kmat_dev, int ldk, int Kd, const mc_mat *mask,
                                mc_prec prec, unsigned flags, float scale, mc_out_type out_type, void *S_dev,
                                void *stream)
{
    if (out_type != MC_OUT_F32 && out_type != MC_OUT_F16) return MC_EUNSUPPORTED;
    return sddmm_impl(Q_dev, ldq, Kmat_dev, ldk, Kd, mask, prec, flags, out_type == MC_OUT_F16 ? 2 : 1, scale, S_dev,
                      nullptr, stream);
}

extern "C" int mc_sddmm_to_mat(const void *Q_dev, int ldq, const void *Kmat_dev, int ldk, int Kd, mc_prec prec, float scale,
                               mc_mat *P, void *stream)
{
    if (!Q_dev || !Kmat_dev || !P) return MC_EINVAL;
    if (prec != MC_L8R8 && prec != MC_L4R4 && prec != MC_L16R16) return MC_EUNSUPPORTED;
    if (P->lhs_bits == 0) return MC_EINVAL;                      // a pattern-only mask has no values to receive the codes
    if (P->lhs_bits != 8 && P->lhs_bits != 16) return MC_EUNSUPPORTED;
    const int bits = lhs_bits_of(prec);
    if (Kd <= 0 || Kd % (128 / bits) != 0 || ldq < Kd || ldk < Kd) return MC_EINVAL;
    if (((int64_t)ldq * bits / 8) % 16 != 0 || ((int64_t)ldk * bits / 8) % 16 != 0) return MC_EALIGN;
    if (!aligned16(Q_dev) || !aligned16(Kmat_dev)) return MC_EALIGN;
    if (!std::isfinite(scale)) return MC_EINVAL;
    if (P->nvec == 0) return MC_OK;
    if (!on_device_of(P)) return MC_EINVAL;
    const mc_options o = t_options;

    SddmmArgs a = {};
    a.float_out = 3; a.out_scale = scale;
    a.dev_vals = P->d_vals; a.dev_batch_stride = 0; a.code_bits = P->lhs_bits;
    a.panel_ptr = P->d_panel_ptr; a.row_ptr = P->d_row_ptr; a.slot_idx = P->d_slot_idx;
    a.Q = static_cast<const uint8_t *>(Q_dev); a.ldq_bytes = (int64_t)ldq * bits / 8; a.Q_batch_stride = 0;
    a.Kmat = static_cast<const uint8_t *>(Kmat_dev); a.ldk_bytes = (int64_t)ldk * bits / 8; a.K_batch_stride = 0;
    a.row_bytes = Kd * bits / 8;
    a.S = nullptr; a.S_batch_stride = 0;
    a.P = P->P; a.V = P->V; a.batch = 1;
    if (P->n_items && o.spmm_splitting != -1) { a.items = P->d_items; a.n_units = P->n_items; }
    P->blk_valid = false; // only the panel format receives the new values
    P->merged_valid = false;
    MC_HIP(launch_sddmm(bits, a, choose_sddmm_waves(P, 1, a.row_bytes, bits, o), static_cast<hipStream_t>(stream)));
    return MC_OK;
}

extern "C" int mc_absmax(const float *x_dev, int64_t n, float *result_dev, void *stream)
{
    if (!x_dev || !result_dev || n < 0) return MC_EINVAL;
    if (!aligned16(x_dev)) return MC_EALIGN;
    MC_HIP(launch_absmax(x_dev, n, result_dev, static_cast<hipStream_t>(stream)));
    return MC_OK;
}

extern "C" int mc_quantize(const float *x_dev, int64_t n, float scale, int bits, void *q_dev, void *stream)
{
    if (!x_dev || !q_dev || n < 0) return MC_EINVAL;
    if (bits != 8 && bits != 4) return MC_EUNSUPPORTED;
    if (!(scale > 0.f) || !std::isfinite(scale) || (bits == 4 && n % 2 != 0)) return MC_EINVAL;
    if (!aligned16(x_dev) || (reinterpret_cast<uintptr_t>(q_dev) & 7u) != 0) return MC_EALIGN;
    MC_HIP(launch_quantize(x_dev, n, scale, bits, static_cast<uint8_t *>(q_dev), static_cast<hipStream_t>(stream)));
    return MC_OK;
}

extern "C" int mc_sparse_softmax_bits(const mc_mat *mask, int batch, const int32_t *S_dev, float score_scale,
                                      float inv_s_p, int code_bits, void *codes_dev, void *stream)
{
    if (!mask || batch <= 0) return MC_EINVAL;
    if ((!S_dev || !codes_dev) && mask->nvec > 0) return MC_EINVAL;
    if (code_bits != 8 && code_bits != 16) return MC_EUNSUPPORTED;
    if (!std::isfinite(score_scale) || !std::isfinite(inv_s_p)) return MC_EINVAL;
    if (mask->nvec == 0) return MC_OK; // nothing stored: empty input and output
    if (!on_device_of(mask)) return MC_EINVAL;
    const mc_options o = t_options;
    SoftmaxArgs a = {};
    a.row_ptr = mask->d_row_ptr; a.S = S_dev; a.codes = codes_dev;
    a.batch_stride = mask->nvec * mask->V;
    a.score_scale = score_scale; a.inv_s_p = inv_s_p;
    a.P = mask->P; a.V = mask->V; a.batch = batch; a.code_bits = code_bits;
    a.max_panel_chunks = mask->max_panel_chunks; a.variant = o.softmax_variant;
    MC_HIP(launch_softmax(a, static_cast<hipStream_t>(stream)));
    return MC_OK;
}

extern "C" int mc_sparse_softmax_to_mat(mc_mat *P, const int32_t *S_dev, float score_scale, float inv_s_p, void *stream)
{
    if (!P || !S_dev) return MC_EINVAL;
    if (P->lhs_bits == 0) return MC_EINVAL;
    if (P->nslots == 0) return MC_OK;
    if (P->lhs_bits != 8 && P->lhs_bits != 16) return MC_EUNSUPPORTED;
    if (!std::isfinite(score_scale) || !std::isfinite(inv_s_p)) return MC_EINVAL;
    if (!on_device_of(P)) return MC_EINVAL;
    const mc_options o = t_options;
    SoftmaxArgs a = {};
    a.row_ptr = P->d_row_ptr; a.S = S_dev; a.codes = nullptr;
    a.panel_ptr = P->d_panel_ptr; a.dev_vals = P->d_vals; a.dev_batch_stride = 0;
    a.batch_stride = P->nvec * P->V;
    a.score_scale = score_scale; a.inv_s_p = inv_s_p;
    a.P = P->P; a.V = P->V; a.batch = 1; a.code_bits = P->lhs_bits;
    a.max_panel_chunks = P->max_panel_chunks; a.variant = o.softmax_variant;
    P->blk_valid = false; // only the panel format receives the new values
    P->merged_valid = false;
    MC_HIP(launch_softmax(a, static_cast<hipStream_t>(stream)));
    return MC_OK;
}

extern "C" int mc_sparse_softmax(const mc_mat *mask, int batch, const int32_t *S_dev, float score_scale,
                                 float inv_s_p, int8_t *codes_dev, void *stream)
{
    return mc_sparse_softmax_bits(mask, batch, S_dev, score_scale, inv_s_p, 8, codes_dev, stream);
}

namespace {
inline size_t round256(size_t x) { return (x + 255) / 256 * 256; }
struct AttnWs { size_t scores, vals, acc, total; };
// with_scores: the int32 scores of all heads travel through the workspace too (the three-kernel form).
// acc_dk != 0: room for the int32 output rows (acc_dk columns) of the panels that several workgroups share.
AttnWs attn_layout(int heads, const mc_mat *mask, int p_bits, bool with_scores = true, int acc_dk = 0)
{
    AttnWs w;
    const size_t nnz = (size_t)mask->nvec * mask->V, pb = (size_t)p_bits / 8;
    w.scores = 0;
    w.vals = w.scores + (with_scores ? round256((size_t)heads * nnz * sizeof(int32_t)) : 0);
    w.acc = w.vals + round256((size_t)heads * (size_t)mask->nslots * mask->V * pb);
    w.total = w.acc + round256((size_t)heads * (size_t)mask->n_split * mask->V * (size_t)acc_dk * sizeof(int32_t));
    return w;
}
// Whether the pipeline's SpMM shares long panels between workgroups (it then needs the extra workspace rows).
// Only on request: on masks whose panel lengths are log-normal (sigma 0.5 .. 1.5, 4096 x 4096, 1 .. 8 heads) it was
// 1 - 10 % slower than whole panels, the pieces of a mask being short (made for the SDDMM, which needs no atomics)
// and the layer's time being that of the scores of the long panels anyway.
inline bool pipeline_splits(const mc_mat *mask, const mc_options &o) { return mask->n_items > 0 && o.spmm_splitting == 1; }

// Waves per (panel, head) of the kernel that computes scores and softmax together, or 0 when the layer has to
// run as three kernels (rows longer than 256 bytes, a panel whose scores do not fit LDS, or pinned by the options).
int scores_kernel_waves(const mc_mat *mask, int heads, int dk, int qkv_bits, const mc_options &o)
{
    const int row_bytes = dk * qkv_bits / 8;
    if (o.attention_mode == 6 || row_bytes > 256) return 0;
    // four waves share a panel's chunks when it has at least three (8 heads x 4096 x 64 at 90 %: 27.2 us with two
    // waves, 21.9 with four), unless the options pin the count
    const double avg = mask->P ? (double)(mask->nslots / MC_CHUNK) / mask->P : 0.0;
    int w = o.sddmm_waves > 0 ? (o.sddmm_waves >= 4 ? 4 : 2) : (avg >= 3.0 ? 4 : 2);
    // long panels: fewer waves leave more LDS for the scores
    while (w > 2 && mask->max_panel_chunks * MC_CHUNK > scores_softmax_max_npad(row_bytes, w)) w /= 2;
    return mask->max_panel_chunks * MC_CHUNK <= scores_softmax_max_npad(row_bytes, w) ? w : 0;
}

// SDDMM -> softmax (writing the SpMM's operand format) -> SpMM, every step a kernel of its own; intermediates in the
// workspace.  Strides of Q/Km/Vm in bytes, of O in elements.
int attention_pipeline(const uint8_t *Q, const uint8_t *Km, const uint8_t *Vm, int heads, int dk, int qkv_bits,
                       int p_bits, int64_t head_stride_bytes, int64_t token_stride_bytes, int64_t o_head_stride,
                       int64_t o_token_stride, const mc_mat *mask, float s_q, float s_k, float s_v, float s_p,
                       void *O, int out_f16, void *workspace_dev, bool split_panels, const mc_options &o, hipStream_t s)
{
    const int sw = scores_kernel_waves(mask, heads, dk, qkv_bits, o);
    const AttnWs ws = attn_layout(heads, mask, p_bits, sw == 0, split_panels ? dk : 0);
    const int64_t nnz = mask->nvec * mask->V;
    uint8_t *wsb = static_cast<uint8_t *>(workspace_dev);
    int32_t *scores = reinterpret_cast<int32_t *>(wsb + ws.scores);
    uint8_t *pvals = wsb + ws.vals;
    const int row_bytes = dk * qkv_bits / 8, pb = p_bits / 8;

    if (sw) {
        // scores and softmax in one kernel: the scores stay in LDS, only the codes (in the layout the SpMM
        // reads: Section 4.3 lets the producer pick the output format by the consumer) reach memory
        ScoresArgs c = {};
        c.panel_ptr = mask->d_panel_ptr; c.slot_idx = mask->d_slot_idx;
        c.Q = Q; c.Km = Km; c.in_head_stride = head_stride_bytes; c.in_token_stride = token_stride_bytes;
        c.row_bytes = row_bytes;
        c.score_scale = s_q * s_k / std::sqrt((float)dk); c.inv_s_p = 1.f / s_p;
        c.dev_vals = pvals; c.dev_batch_stride = mask->nslots * 8 * pb;
        c.P = mask->P; c.heads = heads; c.max_npad = mask->max_panel_chunks * MC_CHUNK;
        MC_HIP(launch_scores_softmax(c, qkv_bits, p_bits, sw, s));
    } else {
        SddmmArgs d = {};
        d.panel_ptr = mask->d_panel_ptr; d.row_ptr = mask->d_row_ptr; d.slot_idx = mask->d_slot_idx;
        d.Q = Q; d.ldq_bytes = token_stride_bytes; d.Q_batch_stride = head_stride_bytes;
        d.Kmat = Km; d.ldk_bytes = token_stride_bytes; d.K_batch_stride = head_stride_bytes;
        d.row_bytes = row_bytes; d.S = scores; d.S_batch_stride = nnz;
        d.P = mask->P; d.V = 8; d.batch = heads;
        if (mask->n_items && o.spmm_splitting != -1) { d.items = mask->d_items; d.n_units = mask->n_items; } // very unequal panels
        MC_HIP(launch_sddmm(qkv_bits, d, choose_sddmm_waves(mask, heads, row_bytes, qkv_bits, o), s));

        // the softmax writes its codes in the layout the SpMM reads
        SoftmaxArgs f = {};
        f.row_ptr = mask->d_row_ptr; f.S = scores; f.batch_stride = nnz;
        f.codes = nullptr; f.panel_ptr = mask->d_panel_ptr; f.dev_vals = pvals; f.dev_batch_stride = mask->nslots * 8 * pb;
        f.score_scale = s_q * s_k / std::sqrt((float)dk); f.inv_s_p = 1.f / s_p;
        f.P = mask->P; f.V = 8; f.batch = heads; f.code_bits = p_bits;
        f.max_panel_chunks = mask->max_panel_chunks; f.variant = o.softmax_variant;
        MC_HIP(launch_softmax(f, s));
    }

    SpmmArgs m = {};
    m.panel_ptr = mask->d_panel_ptr; m.slot_idx = mask->d_slot_idx;
    m.vals = pvals; m.vals_batch_stride = mask->nslots * 8 * pb;
    m.B = Vm; m.ldb_bytes = token_stride_bytes; m.B_batch_stride = head_stride_bytes;
    m.row_bytes = row_bytes; m.C = O; m.ldc = o_token_stride; m.C_batch_stride = o_head_stride;
    m.P = mask->P; m.V = 8; m.rows = mask->M; m.batch = heads; m.float_out = out_f16 ? 2 : 1; m.out_scale = s_p * s_v;
    m.stages = spmm_stages_for(o, mask->K, m.ldb_bytes, m.row_bytes);
    m.uniform_chunks = mask->uniform_chunks;
    m.max_unit_chunks = mask->max_panel_chunks;
    if (split_panels) {
        // Very unequal panels: the long ones are shared by several workgroups.  A rounded result cannot be added
        // up piecewise, so those add their exact int32 tiles into rows of the workspace (cleared first), which a
        // last small kernel scales and writes to O; all other panels write O directly, as without the split.
        m.items = mask->d_items; m.n_units = mask->n_items; m.max_unit_chunks = mask->max_item_chunks;
        m.acc = reinterpret_cast<int32_t *>(wsb + ws.acc); m.acc_ld = dk; m.n_split = mask->n_split;
        MC_HIP(launch_zero_ints(m.acc, (int64_t)heads * mask->n_split * 8 * dk, s));
    }
    int bnb, waves;
    choose_variant(mask, p_bits, m.row_bytes, qkv_bits == 4, heads, m.max_unit_chunks, o, &bnb, &waves);
    const mc_prec prec = (p_bits == 16) ? (qkv_bits == 4 ? MC_L16R4 : MC_L16R8) : (qkv_bits == 4 ? MC_L8R4 : MC_L8R8);
    MC_HIP(launch_spmm(prec, m, bnb, waves, s));
    if (split_panels)
        MC_HIP(launch_finish_split_rows(m.acc, dk, mask->n_split, 8, heads, mask->d_split_panels, O, o_token_stride,
                                        o_head_stride, m.float_out, m.out_scale, s));
    return MC_OK;
}

// Whether the single fused kernel takes this layer (else the pipeline of separate kernels, which needs a workspace).
// (Head dimensions up to 128 whose rows are whole 16-byte pieces; those below 64 or between 64 and 128 run in the
// next larger tile with the missing pieces read as zeros.)
bool attention_is_fused(const mc_mat *mask, int dk, int qkv_bits, const mc_options &o)
{
    return o.attention_mode != 1 && o.attention_mode != 6 && dk <= 128 && (dk * qkv_bits / 8) % 16 == 0 &&
           mask->max_panel_chunks * MC_CHUNK <= attention_fused_max_vectors();
}

// Memory the library itself provides to callers that cannot allocate (mc_sparse_attention_static):
// one array per GPU, in that GPU's memory for the life of the process; its address on each device is
// looked up once, with that device current.
constexpr size_t STATIC_SCRATCH_BYTES = MC_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[STATIC_SCRATCH_BYTES];
constexpr int MAX_DEVICES = 64;
void *g_scratch_ptr[MAX_DEVICES] = {};
std::mutex g_scratch_mutex;

int static_scratch(void **ptr)
{
    int dev = -1;
    if (!hip_ok(hipGetDevice(&dev), "hipGetDevice")) return MC_EHIP;
    if (dev < 0 || dev >= MAX_DEVICES) return MC_EUNSUPPORTED;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        if (!hip_ok(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)), "hipGetSymbolAddress(scratch)")) return MC_EHIP;
        g_scratch_ptr[dev] = p;
    }
    *ptr = g_scratch_ptr[dev];
    return MC_OK;
}

// use_static: the intermediates of the kernel pipeline go to the library's per-device array instead
// of a caller's workspace
int attention_impl(const void *Q_dev, const void *Km_dev, const void *Vm_dev, int batch, int heads, int L, int dk,
                   int64_t batch_stride, int64_t head_stride, int64_t token_stride, const mc_mat *mask, int p_bits,
                   int qkv_bits, float s_q, float s_k, float s_v, float s_p, mc_out_type out_type, void *O_dev,
                   void *workspace_dev, size_t workspace_bytes, bool use_static, const mc_options *opts, void *stream)
{
    if (out_type != MC_OUT_F32 && out_type != MC_OUT_F16) return MC_EUNSUPPORTED;
    const int out_f16 = (out_type == MC_OUT_F16) ? 1 : 0;
    if (!Q_dev || !Km_dev || !Vm_dev || !mask || !O_dev) return MC_EINVAL;
    mc_options o;
    if (resolve_options(opts, &o) != MC_OK) return MC_EINVAL;
    if ((p_bits != 8 && p_bits != 16) || (qkv_bits != 8 && qkv_bits != 4)) return MC_EUNSUPPORTED;
    const int epp = 128 / qkv_bits; // elements per 16-byte piece
    if (batch <= 0 || batch > 65535 || heads <= 0 || L <= 0 || dk <= 0 || dk % epp != 0) return MC_EINVAL;
    if (mask->M != L || mask->K != L || mask->V != 8) return MC_EINVAL;
    // symmetric quantisation scales are positive; the fused kernel takes the row maximum on the
    // integer scores, which is the maximum of the scaled ones only for a positive scale
    if (!(s_q > 0.f) || !(s_k > 0.f) || !(s_v > 0.f) || !(s_p > 0.f) || !std::isfinite(s_q * s_k * s_v / s_p)) return MC_EINVAL;
    if (token_stride < dk || head_stride < dk || (batch > 1 && batch_stride < dk)) return MC_EINVAL;
    if ((int64_t)(L - 1) * token_stride + (int64_t)(heads - 1) * head_stride + dk > (int64_t)INT32_MAX) return MC_EINVAL;
    if (L > (1 << 24) || token_stride >= (1 << 24)) return MC_EINVAL; // kernels use 24-bit multiplies
    if (token_stride % epp != 0 || head_stride % epp != 0 || batch_stride % epp != 0) return MC_EALIGN;
    if (!aligned16(Q_dev) || !aligned16(Km_dev) || !aligned16(Vm_dev) || !aligned16(O_dev)) return MC_EALIGN;
    if (!on_device_of(mask)) return MC_EINVAL;
    hipStream_t s = static_cast<hipStream_t>(stream);

    if (attention_is_fused(mask, dk, qkv_bits, o)) {
        const int tile = dk <= 64 ? 64 : 128;     // the kernel's head dimension
        AttnArgs f;
        f.real_pieces = dk * qkv_bits / 8 / 16; f.out_cols = dk;
        f.panel_ptr = mask->d_panel_ptr; f.slot_idx = mask->d_slot_idx;
        f.Q = static_cast<const uint8_t *>(Q_dev); f.Km = static_cast<const uint8_t *>(Km_dev);
        f.Vm = static_cast<const uint8_t *>(Vm_dev); f.O = static_cast<float *>(O_dev); f.out_f16 = out_f16;
        f.head_stride = head_stride; f.token_stride = token_stride; f.batch_stride = batch_stride;
        f.in_head_stride = head_stride * qkv_bits / 8; f.in_token_stride = token_stride * qkv_bits / 8;
        f.in_batch_stride = batch_stride * qkv_bits / 8;
        f.score_scale = s_q * s_k / std::sqrt((float)dk); f.inv_s_p = 1.f / s_p; f.out_scale = s_p * s_v;
        f.heads = heads; f.batch = batch;
        // neighbouring heads contiguous inside a token, rows of at most 64 bytes: two heads per workgroup can
        // gather 128 bytes per token (not for 16-bit codes with 4-bit inputs, whose output tile does not fit
        // that kernel's stages)
        const bool short_rows = dk == 64 || qkv_bits == 4;
        const bool pairs = dk == tile && short_rows && head_stride == dk && heads % 2 == 0 && !(p_bits == 16 && qkv_bits == 4);
        const double avg = mask->P ? (double)(mask->nslots / MC_CHUNK) / mask->P : 0.0;
        // One launch for the panels in `list` (null: all), none of which has more than max_chunks chunks.
        auto launch = [&](const int32_t *list, int n_panels, int max_chunks) -> hipError_t {
            f.panel_list = list; f.P = n_panels;
            // a wave keeps at most 8 chunks of scores in registers: longer panels are shared by 2, 4 or 8 waves
            int wpp = max_chunks > 32 ? 8 : (max_chunks > 16 ? 4 : (max_chunks > 8 ? 2 : 1));
            int hpg;
            if (o.attention_mode == 0) {
                // Halving the gather requests pays once the launch fills the chip (2048 (panel, head) units and
                // more: 13.3 against 15.6 us for 4096 of them; 5.0 against 4.7 us for 128).  Smaller launches get
                // more waves per unit instead, until about 2048 waves are in flight and while every wave still
                // has a chunk (256 units of 7 chunks: 5.9 us with one wave each, 4.5 us with four).
                const int64_t units = (int64_t)n_panels * heads * batch;
                hpg = (pairs && units >= 2048 && wpp < 8) ? 2 : 1;
                if (hpg == 1) while (wpp < 4 && units * wpp * 2 <= 2048 && wpp * 2 <= avg) wpp *= 2;
            } else {
                if (o.attention_mode == 3 && wpp < 2) wpp = 2;
                if (o.attention_mode == 4 && wpp < 4) wpp = 4;
                hpg = (o.attention_mode != 2 && pairs && wpp < 8) ? 2 : 1;
            }
            if (dk == tile) return launch_attention_fused(f, hpg, wpp, p_bits, qkv_bits, dk, s);
            return launch_attention_fused_padded(f, wpp, p_bits, qkv_bits, tile, s);
        };
        // Panels of very different lengths (the longest at least twice the average and more than one wave's
        // worth), automatic mode: one launch per length class, so that short panels are not given the many waves
        // the longest one needs.  Otherwise one launch sized by the longest panel.
        if (o.attention_mode == 0 && mask->d_class_panels && mask->max_panel_chunks > 8 && mask->max_panel_chunks >= 2.0 * avg) {
            for (int b = 0; b < 4; ++b) {
                const int n = mask->class_start[b + 1] - mask->class_start[b];
                if (n > 0) MC_HIP(launch(mask->d_class_panels + mask->class_start[b], n, b == 3 ? mask->max_panel_chunks : (8 << b)));
            }
        } else {
            MC_HIP(launch(nullptr, mask->P, mask->max_panel_chunks));
        }
        return MC_OK;
    }
    // the kernel pipeline keeps its intermediates in a workspace (none are needed when nothing is stored)
    const bool with_scores = scores_kernel_waves(mask, heads, dk, qkv_bits, o) == 0;
    const size_t need = attn_layout(heads, mask, p_bits, with_scores).total;
    // sharing long panels between workgroups takes some more room; without it they run whole (same results)
    const size_t need_split = attn_layout(heads, mask, p_bits, with_scores, dk).total;
    const bool split_panels = pipeline_splits(mask, o) && (use_static ? need_split <= STATIC_SCRATCH_BYTES : workspace_bytes >= need_split);
    if (use_static) {
        if (need > STATIC_SCRATCH_BYTES) {
            snprintf(g_detail, sizeof g_detail, "the layer's intermediates need %zu bytes, the library's own array holds %zu",
                     need, STATIC_SCRATCH_BYTES);
            return MC_ENOMEM;
        }
        const int rc = static_scratch(&workspace_dev);
        if (rc != MC_OK) return rc;
    } else if (need > 0) {
        if (!workspace_dev) return MC_EINVAL;
        if ((reinterpret_cast<uintptr_t>(workspace_dev) & 255u) != 0) return MC_EALIGN;
        if (workspace_bytes < need) return MC_ENOMEM;
    }
    // the batch items run one after the other through the same workspace
    for (int b = 0; b < batch; ++b) {
        const int64_t ib = (int64_t)b * batch_stride * qkv_bits / 8;
        const int rc = attention_pipeline(static_cast<const uint8_t *>(Q_dev) + ib, static_cast<const uint8_t *>(Km_dev) + ib,
                                          static_cast<const uint8_t *>(Vm_dev) + ib, heads, dk, qkv_bits, p_bits,
                                          head_stride * qkv_bits / 8, token_stride * qkv_bits / 8, head_stride,
                                          token_stride, mask, s_q, s_k, s_v, s_p,
                                          static_cast<uint8_t *>(O_dev) + (int64_t)b * batch_stride * (out_f16 ? 2 : 4),
                                          out_f16, workspace_dev, split_panels, o, s);
        if (rc != MC_OK) return rc;
    }
    return MC_OK;
}
} // namespace

extern "C" size_t mc_attention_workspace_bytes_bits(int heads, const mc_mat *mask, int p_bits)
{
    if (!mask || heads <= 0 || (p_bits != 8 && p_bits != 16)) return 0;
    return attn_layout(heads, mask, p_bits).total;
}

extern "C" size_t mc_attention_workspace_bytes(int heads, const mc_mat *mask)
{
    return mc_attention_workspace_bytes_bits(heads, mask, 8);
}

extern "C" size_t mc_attention_workspace_needed(int heads, int dk, const mc_mat *mask, int p_bits, const mc_options *options)
{
    if (!mask || heads <= 0 || (p_bits != 8 && p_bits != 16)) return 0;
    mc_options o;
    if (resolve_options(options, &o) != MC_OK) return 0;
    // (8-bit inputs decide here; a 4-bit layer whose rows are not whole pieces then needs what is returned)
    if (attention_is_fused(mask, dk, 8, o)) return 0;
    // (the narrowest inputs the layer takes give the smallest rows: whether the scores stay on chip is decided
    // for 8-bit inputs here, which never asks for less than a 4-bit layer needs)
    return attn_layout(heads, mask, p_bits, scores_kernel_waves(mask, heads, dk, 8, o) == 0, pipeline_splits(mask, o) ? dk : 0).total;
}

extern "C" int mc_sparse_attention(const int8_t *Q_dev, const int8_t *Km_dev, const int8_t *Vm_dev, int heads, int L,
                                   int dk, const mc_mat *mask, float s_q, float s_k, float s_v, float s_p,
                                   float *O_dev, void *workspace_dev, size_t workspace_bytes, void *stream)
{
    return attention_impl(Q_dev, Km_dev, Vm_dev, 1, heads, L, dk, 0, (int64_t)L * dk, dk, mask, 8, 8, s_q, s_k, s_v, s_p,
                          MC_OUT_F32, O_dev, workspace_dev, workspace_bytes, false, nullptr, stream);
}

extern "C" int mc_sparse_attention_strided(const int8_t *Q_dev, const int8_t *Km_dev, const int8_t *Vm_dev, int heads,
                                           int L, int dk, int64_t head_stride, int64_t token_stride,
                                           const mc_mat *mask, float s_q, float s_k, float s_v, float s_p,
                                           float *O_dev, void *workspace_dev, size_t workspace_bytes, void *stream)
{
    return attention_impl(Q_dev, Km_dev, Vm_dev, 1, heads, L, dk, 0, head_stride, token_stride, mask, 8, 8, s_q, s_k, s_v,
                          s_p, MC_OUT_F32, O_dev, workspace_dev, workspace_bytes, false, nullptr, stream);
}

extern "C" int mc_sparse_attention_bits(const void *Q_dev, const void *Km_dev, const void *Vm_dev, int heads, int L,
                                        int dk, int64_t head_stride, int64_t token_stride, const mc_mat *mask,
                                        int p_bits, int qkv_bits, float s_q, float s_k, float s_v, float s_p,
                                        float *O_dev, void *workspace_dev, size_t workspace_bytes, void *stream)
{
    return attention_impl(Q_dev, Km_dev, Vm_dev, 1, heads, L, dk, 0, head_stride, token_stride, mask, p_bits, qkv_bits, s_q,
                          s_k, s_v, s_p, MC_OUT_F32, O_dev, workspace_dev, workspace_bytes, false, nullptr, stream);
}

extern "C" int mc_sparse_attention_batched(const void *Q_dev, const void *Km_dev, const void *Vm_dev, int batch,
                                           int heads, int L, int dk, int64_t batch_stride, int64_t head_stride,
                                           int64_t token_stride, const mc_mat *mask, int p_bits, int qkv_bits,
                                           float s_q, float s_k, float s_v, float s_p, float *O_dev,
                                           void *workspace_dev, size_t workspace_bytes, void *stream)
{
    return attention_impl(Q_dev, Km_dev, Vm_dev, batch, heads, L, dk, batch_stride, head_stride, token_stride, mask, p_bits,
                          qkv_bits, s_q, s_k, s_v, s_p, MC_OUT_F32, O_dev, workspace_dev, workspace_bytes, false, nullptr,
                          stream);
}

extern "C" int mc_sparse_attention_out(const void *Q_dev, const void *Km_dev, const void *Vm_dev, int batch, int heads,
                                       int L, int dk, int64_t batch_stride, int64_t head_stride, int64_t token_stride,
                                       const mc_mat *mask, int p_bits, int qkv_bits, float s_q, float s_k, float s_v,
                                       float s_p, mc_out_type out_type, void *O_dev, void *workspace_dev,
                                       size_t workspace_bytes, void *stream)
{
    return attention_impl(Q_dev, Km_dev, Vm_dev, batch, heads, L, dk, batch_stride, head_stride, token_stride, mask, p_bits,
                          qkv_bits, s_q, s_k, s_v, s_p, out_type, O_dev, workspace_dev, workspace_bytes, false, nullptr,
                          stream);
}

extern "C" int mc_sparse_attention_ex(const void *Q_dev, const void *Km_dev, const void *Vm_dev, int batch, int heads,
                                      int L, int dk, int64_t batch_stride, int64_t head_stride, int64_t token_stride,
                                      const mc_mat *mask, int p_bits, int qkv_bits, float s_q, float s_k, float s_v,
                                      float s_p, mc_out_type out_type, const mc_options *options, void *O_dev,
                                      void *workspace_dev, size_t workspace_bytes, void *stream)
{
    const mc_options automatic = {};
    return attention_impl(Q_dev, Km_dev, Vm_dev, batch, heads, L, dk, batch_stride, head_stride, token_stride, mask, p_bits,
                          qkv_bits, s_q, s_k, s_v, s_p, out_type, O_dev, workspace_dev, workspace_bytes, false,
                          options ? options : &automatic, stream);
}

extern "C" int mc_sparse_attention_static(const void *Q_dev, const void *Km_dev, const void *Vm_dev, int batch, int heads,
                                          int L, int dk, int64_t batch_stride, int64_t head_stride, int64_t token_stride,
                                          const mc_mat *mask, int p_bits, int qkv_bits, float s_q, float s_k, float s_v,
                                          float s_p, mc_out_type out_type, const mc_options *options, void *O_dev,
                                          void *stream)
{
    return attention_impl(Q_dev, Km_dev, Vm_dev, batch, heads, L, dk, batch_stride, head_stride, token_stride, mask, p_bits,
                          qkv_bits, s_q, s_k, s_v, s_p, out_type, O_dev, nullptr, 0, true, options, stream);
}
