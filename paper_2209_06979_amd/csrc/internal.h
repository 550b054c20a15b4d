// Internal declarations shared by the translation units of the library (not installed).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/magicube.h"

struct mc_mat {
    int M, K, V, lhs_bits, P;
    int64_t nvec, nslots, vals_bytes;
    int max_panel_chunks;      // longest panel, in chunks of 64 vectors
    int uniform_chunks;        // chunks of every panel when all panels have the same number (and at least one), else 0
    int device;                // HIP device the buffers live on
    int32_t *d_panel_ptr;      // 2*P: chunk-aligned first slot, real end slot
    int32_t *d_row_ptr;        // P+1: interchange row pointers (vector offsets)
    int32_t *d_slot_idx;       // nslots
    uint8_t *d_vals;           // vals_bytes (null for a pattern-only mask)
    // Work items for matrices with very unequal panel lengths (null / 0 otherwise): panels longer
    // than a cap are cut into several items of at most `cap` chunks, so that no single
    // workgroup is left with a tail many times the average.
    int32_t *d_items;          // n_items x 4: panel, first chunk, end chunk, 1 if the panel has several items
    int32_t *d_split_panels;   // n_split: the panels that have several items
    int n_items, n_split;
    int max_item_chunks;       // chunks of the longest item
    // K-blocked copy of the operand for the SpMM that keeps blocks of B resident in LDS (null when not
    // built: pattern-only masks, very sparse or very unequal matrices, more than 63 K-blocks)
    int nblk;                  // K-blocks of MC_KBLOCK rows
    int64_t blk_chunks;        // chunks over all (panel, block) lists
    int32_t *d_blk_ptr;        // P*nblk + 1
    uint16_t *d_blk_rows;      // blk_chunks * 64
    uint8_t *d_blk_vals;       // blk_chunks * chunk bytes
    int32_t *d_blk_src;        // blk_chunks * 64: interchange vector of each slot, -1 for padding
    bool blk_valid;            // false once the values were replaced in the panel format only
    // Panels sorted by length class for kernels that give a panel 1, 2, 4 or 8 waves (V = 8 only; null when every
    // panel falls into one class): class b holds the panels of at most 8 << b chunks that class b - 1 does not
    // hold; class 3 also takes what is longer still.
    int32_t *d_class_panels;   // P panel numbers, class after class
    int class_start[5];        // first entry of each class in d_class_panels; [4] = P
    // Merged copy for the SpMM (null when not built): `merge_group` consecutive panels as one panel of
    // V * merge_group rows at the union of their columns (see mc_merge_host); a complete operand of its own
    // (work items, K-blocked copy), never merged again.  Its rows may run past M: launches on it pass M as the
    // number of output rows.
    mc_mat *merged;
    int merge_group;
    int32_t *d_merge_src;      // merged nvec * merge_group: interchange vector of each panel's share, -1 = zeros
    uint8_t *d_merge_vals;     // staging for mc_mat_set_values_device: the merged operand's values in interchange order
    bool merged_valid;         // false once the values were replaced in the panel format only
};

// Builders that also take V = 16 (4- and 8-bit values): the library's merged copies only.
int mc_layout_query_wide(int M, int K, int V, int lhs_bits, const int32_t *row_ptr, mc_layout *out);
int mc_pack_host_wide(int M, int K, int V, int lhs_bits, const int32_t *row_ptr, const int32_t *col_idx, const void *values,
                      int32_t *panel_ptr, int32_t *slot_idx, void *slot_vals);
int mc_blocked_query_wide(int M, int K, int V, int lhs_bits, const int32_t *row_ptr, const int32_t *col_idx, mc_blocked_layout *out);
int mc_pack_blocked_host_wide(int M, int K, int V, int lhs_bits, const int32_t *row_ptr, const int32_t *col_idx, const void *values,
                              int32_t *blk_ptr, uint16_t *blk_rows, void *blk_vals, int32_t *blk_src);

// One SpMM launch (optionally a batch of problems sharing the sparsity pattern).
struct SpmmArgs {
    const int32_t *panel_ptr;
    const int32_t *slot_idx;
    const uint8_t *vals;
    int64_t vals_batch_stride; // bytes
    const uint8_t *B;
    int64_t ldb_bytes;
    int64_t B_batch_stride;    // bytes
    int row_bytes;             // bytes of one B row that take part (N * bits / 8)
    void *C;                   // int32, float or half (see float_out)
    int64_t ldc;               // elements
    int64_t C_batch_stride;    // elements
    int P, V, batch;
    int rows;                  // rows of C (a merged operand's last panel may run past them); V up to 16
    int float_out;             // 0: int32; 1: float(acc) * out_scale as fp32; 2: the same rounded to fp16
    float out_scale;
    int lhs_unsigned, rhs_unsigned; // 4- and 8-bit operands read as non-negative values
    // optional work items (see mc_mat): null = one unit of work per panel.  Items of a split panel
    // add their int32 results into C with atomics; C's rows of those panels are cleared first.
    const int32_t *items;
    int n_units;               // items, or P
    int stages;                // chunks in flight per wave: 1 or 2 (2 needs B to span less than 4 GiB)
    int uniform_chunks;        // > 0: every panel has this many chunks and starts at panel * uniform_chunks * 64 (panel_ptr is not read)
    int ntiles, tile_shift;    // filled by the launcher: column tiles (workgroups) per unit, and their log2 (-1: not a power of two)
    int max_unit_chunks;       // chunks of the longest unit of work (panel or work item)
    // optional: items of a split panel add their int32 results here instead of into C (which may then be float or
    // half): cleared rows [batch][split panel][V][acc_ld], finished by launch_finish_split_rows
    int32_t *acc;
    int acc_ld, n_split;
    long long *trace;          // measurement aid (launch_spmm_phase_probe only): time stamps per wave
};

// One launch of the SpMM that keeps K-blocks of B resident in LDS (see spmm_slab_kernels.hip).
struct SlabArgs {
    const int32_t *blk_ptr;
    const uint16_t *blk_rows;
    const uint8_t *vals;
    int64_t vals_batch_stride; // bytes
    const uint8_t *B;
    int64_t ldb_bytes, B_batch_stride;
    int row_bytes, K;
    void *C;
    int64_t ldc, C_batch_stride;
    int P, V, batch, nblk;
    int rows;                  // rows of C (see SpmmArgs)
    int float_out;
    float out_scale;
    int groups;                // panel groups (workgroups per column tile)
    int ppg;                   // consecutive panels per workgroup (taken in passes of (nc / wpp) * panels-per-wave)
    int wpp;                   // waves sharing a panel (its chunks dealt round-robin)
    int nc;                    // computing waves per workgroup; nc / wpp panels at a time
    int nf;                    // filling waves (after the computing ones); nc + nf <= 16
};

struct SddmmArgs {
    const int32_t *panel_ptr;
    const int32_t *row_ptr;
    const int32_t *slot_idx;
    const uint8_t *Q;
    int64_t ldq_bytes, Q_batch_stride;
    const uint8_t *Kmat;
    int64_t ldk_bytes, K_batch_stride;
    int row_bytes;             // Kd * bits / 8
    void *S;                   // int32, float or half (see float_out)
    int64_t S_batch_stride;    // elements
    int float_out;             // 0: int32; 1: float(score) * out_scale as fp32; 2: the same rounded to fp16;
                               // 3: integer codes clamp(rint(score * out_scale)) into a sparse operand's device format
    float out_scale;
    uint8_t *dev_vals;         // float_out 3: the operand's value array, its bytes per batch item, its code width (8 / 16)
    int64_t dev_batch_stride;
    int code_bits;
    int P, V, batch;
    int lhs_unsigned, rhs_unsigned; // 4- and 8-bit operands read as non-negative values
    const int32_t *items;      // optional work items (see mc_mat): null = one workgroup per panel
    int n_units;               // items, or P
};

// Scores + softmax of the attention layer in one kernel (attention_scores_kernels.hip): V = 8, one mask for all heads.
struct ScoresArgs {
    const int32_t *panel_ptr;
    const int32_t *slot_idx;
    const uint8_t *Q, *Km;
    int64_t in_head_stride, in_token_stride; // bytes
    int row_bytes;             // dk * bits / 8, a multiple of 16, at most 256
    float score_scale, inv_s_p;
    uint8_t *dev_vals;         // codes in the device panel format, one block of dev_batch_stride bytes per head
    int64_t dev_batch_stride;
    int P, heads;
    int max_npad;              // longest panel of the mask, padded to whole chunks, in vectors
};

struct SoftmaxArgs {
    const int32_t *row_ptr;
    const int32_t *S;
    void *codes;               // int8 (code_bits 8) or int16 (code_bits 16), interchange order; or null:
    // the codes go straight into the device panel format of a sparse operand (padded slots zeroed)
    const int32_t *panel_ptr;
    uint8_t *dev_vals;
    int64_t dev_batch_stride;  // bytes
    int64_t batch_stride;      // elements (nvec * V)
    float score_scale, inv_s_p;
    int P, V, batch, code_bits;
    int max_panel_chunks;      // longest panel of the mask, in chunks of 64 vectors
    int variant;               // 0: automatic; 1: a workgroup per panel even for short panels; 2: the any-length kernel
};

struct RepackArgs {
    const int32_t *panel_ptr;
    const int32_t *row_ptr;
    const uint8_t *src;        // interchange order values
    int64_t src_batch_stride;  // bytes
    uint8_t *dst;              // device-format values
    int64_t dst_batch_stride;  // bytes
    int P, V, bits, batch;
};

// Fused attention for head dimension 64.  Element (head h, token l, d) of Q, Km, Vm (int8)
// and O (fp32) sits at h*head_stride + l*token_stride + d.
struct AttnArgs {
    const int32_t *panel_ptr;
    const int32_t *slot_idx;
    const uint8_t *Q, *Km, *Vm;
    float *O;                                // fp32, or half when out_f16 is set
    int64_t head_stride, token_stride;       // elements of O
    int64_t in_head_stride, in_token_stride; // bytes of Q, Km, Vm
    int64_t batch_stride, in_batch_stride;   // between batch items: elements of O, bytes of Q, Km, Vm
    float score_scale, inv_s_p, out_scale;
    int P, heads, batch;                     // P: panels of this launch
    const int32_t *panel_list;               // their numbers (null: 0 .. P-1)
    int out_f16;                             // 1: O holds fp16 (the fp32 result rounded to nearest even)
    // head dimensions below the kernel's tile (launch_attention_fused_padded): 16-byte pieces a Q / Kmat / V row
    // really has, and columns of O
    int real_pieces, out_cols;
};

hipError_t launch_spmm(mc_prec prec, const SpmmArgs &a, int bnb, int waves, hipStream_t s);
// the L8-R8 SpMM (128-byte tiles, 2 waves per panel, two chunks in flight; every panel at most 8 chunks, whole panels,
// B below 4 GiB) with 10 time stamps per wave written to a.trace
hipError_t launch_spmm_phase_probe(const SpmmArgs &a, hipStream_t s);
// ppw: panels per computing wave (1, 2 or 4; 4 only with an 8-bit B).  Precisions with a 16-bit B are not built.
hipError_t launch_spmm_slab(mc_prec prec, const SlabArgs &a, int ppw, hipStream_t s);
hipError_t launch_repack_blocked(const int32_t *blk_src, const uint8_t *src, uint8_t *dst, int64_t nchunks, int V, int bits,
                                 hipStream_t s);
// clears the C rows (int32, n columns) of the listed panels
hipError_t launch_zero_rows(int32_t *C, int64_t ldc, int n, int V, const int32_t *panels, int n_panels, hipStream_t s);
hipError_t launch_zero_ints(int32_t *p, int64_t n, hipStream_t s); // n a multiple of 4, p 16-byte aligned
// C rows of the split panels = scale * float(acc rows) (float_out 1: fp32, 2: fp16); acc as in SpmmArgs, n columns
hipError_t launch_finish_split_rows(const int32_t *acc, int n, int n_split, int V, int batch, const int32_t *panels, void *C,
                                    int64_t ldc, int64_t C_batch_stride, int float_out, float scale, hipStream_t s);
// the gather of launch_spmm alone (same tile variant); sink: one int32 per workgroup (P * row tiles)
hipError_t launch_gather_probe(const SpmmArgs &a, int bnb, int waves, int32_t *sink, hipStream_t s);
// `workgroups` x 4 waves x `iters` x 8 MFMAs (16x16x64 i8); sink: workgroups * 256 int32
hipError_t launch_mfma_probe(int workgroups, int iters, int32_t *sink, hipStream_t s);
// waves: 0 = the direct-load kernel; 1, 2, 4, 8 = waves per panel of the LDS-staged kernel
// (used when a row has 64, 128, 256, 512 or 1024 bytes)
hipError_t launch_sddmm(int bits, const SddmmArgs &a, int waves, hipStream_t s);
hipError_t launch_softmax(const SoftmaxArgs &a, hipStream_t s);
// waves: 2 or 4 per (panel, head); the longest padded panel must not exceed scores_softmax_max_npad(row_bytes, waves)
hipError_t launch_scores_softmax(const ScoresArgs &a, int qkv_bits, int code_bits, int waves, hipStream_t s);
int scores_softmax_max_npad(int row_bytes, int waves);
hipError_t launch_absmax(const float *x, int64_t n, float *result, hipStream_t s);
hipError_t launch_quantize(const float *x, int64_t n, float scale, int bits, uint8_t *q, hipStream_t s);
hipError_t launch_repack(const RepackArgs &a, hipStream_t s);
// values of a merged operand in interchange order from the original operand's: share (i, g) of vb bytes = vector
// merge_src[i * group + g] of src, or zeros
hipError_t launch_merge_values(const int32_t *merge_src, const uint8_t *src, uint8_t *dst, int64_t shares, int vb, hipStream_t s);
// dk is 64 or 128.  heads_per_group 2 needs head_stride == dk (token-major layout), rows of at most 64
// bytes and an even head count, and is not available for 16-bit codes with 4-bit inputs
hipError_t launch_attention_fused(const AttnArgs &a, int heads_per_group, int waves_per_panel, int p_bits, int qkv_bits,
                                  int dk, hipStream_t s);
// the same kernel for head dimensions below its tile (64 or 128): one head per workgroup; a.real_pieces, a.out_cols set
hipError_t launch_attention_fused_padded(const AttnArgs &a, int waves_per_panel, int p_bits, int qkv_bits, int tile, hipStream_t s);
int attention_fused_max_vectors(); // longest panel (in vectors) the fused kernel accepts
