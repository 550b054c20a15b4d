/*
 * magicube.h -- C ABI of the MI355X (gfx950) library for quantized sparse matrix
 * operations with 1-D block ("column vector") sparsity.
 *
 * Operations (all integer results are exact int32):
 *   SpMM   C[M x N] = A_sparse[M x K] * B[K x N]           (paper, Section 4.2)
 *   SDDMM  S = (Q[M x Kd] * Kmat[Nc x Kd]^T) at a mask     (paper, Section 4.3)
 *   mixed precision Lx-Ry: x-bit sparse/left operand, y-bit dense/right operand
 *          (paper, Section 4.4 and its table of supported precisions)
 *   quantized sparse self-attention: SDDMM -> softmax -> int8 -> SpMM
 *          (paper, Section 5.3)
 *
 * Sparse operand, interchange form ("BCRS with 1-D blocks", Section 4.1):
 *   V          block length, 2, 4 or 8; rows p*V .. p*V+V-1 form row panel p, P = M / V
 *   row_ptr    P + 1 int32; panel p owns vectors row_ptr[p] .. row_ptr[p+1]-1
 *   col_idx    one int32 column per stored vector, strictly ascending inside a panel
 *   values     the V elements of each vector consecutively (vector-major):
 *              8-bit: int8; 16-bit: little-endian int16; 12-bit: int16 restricted to
 *              [-2048, 2047]; 4-bit: two's-complement
 *              nibbles, element 2j in bits 3:0 and element 2j+1 in bits 7:4 of byte j
 * The library converts it into its own device format (a strided row-major layout in
 * the spirit of SR-BCRS, Section 4.1): vectors of a panel are grouped in chunks of 64
 * (the reduction depth of one gfx950 i8 MFMA), the last chunk zero-padded, values
 * row-major inside sub-strides of 16 vectors, two pointers per panel (chunk-aligned
 * start and real end).
 *
 * Conventions
 *   - "dev" pointers are device (HBM) addresses owned by the caller, "host" pointers
 *     are ordinary host memory.  The library owns only mc_mat handles.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Compute
 *     calls are asynchronous on it and never synchronise or allocate.
 *   - Every int-returning function returns MC_OK (0) or a negative mc_status; nothing
 *     throws or aborts.  Argument checks are done on the host before any launch.
 *   - Dense operands are row-major.  int4 dense operands hold two elements per byte
 *     along a row (same nibble order as above); leading dimensions are in ELEMENTS.
 *   - A compute call must be made with the device current on which its mc_mat was created
 *     (MC_EINVAL otherwise; mc_last_error_detail() names both devices).
 *   - The library keeps no process-wide mutable state.  Kernel-variant choices are automatic;
 *     a caller that wants to pin them passes an mc_options to an ..._ex entry point, or sets
 *     defaults for its own thread (mc_set_thread_options).  Calls from different host threads
 *     never influence each other.
 */
#ifndef MAGICUBE_H
#define MAGICUBE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    MC_OK = 0,
    MC_EINVAL = -1,       /* bad size, V, pattern (unsorted / out of range), null pointer   */
    MC_EUNSUPPORTED = -2, /* precision / operation pair outside the supported table         */
    MC_EALIGN = -3,       /* device pointer or leading dimension not 16-byte aligned        */
    MC_EHIP = -4,         /* a HIP runtime call failed                                       */
    MC_ENOMEM = -5,       /* host or device allocation failed / workspace too small         */
    MC_ERANGE = -6        /* a value cannot be represented (16-bit value above 32639, ...)  */
} mc_status;

/* Lx-Ry: bits of the left (sparse for SpMM) and right operands. */
typedef enum {
    MC_L8R8 = 0, MC_L8R4 = 1, MC_L4R4 = 2, MC_L16R8 = 3,
    MC_L16R16 = 4, MC_L16R4 = 5, MC_L12R4 = 6
} mc_prec;

/* Type of a dequantised (real-valued) output: IEEE binary32 or binary16. */
typedef enum { MC_OUT_F32 = 0, MC_OUT_F16 = 1 } mc_out_type;

/* Vectors per chunk of the device format (= reduction depth of v_mfma_i32_16x16x64_i8). */
#define MC_CHUNK 64

typedef struct mc_mat mc_mat; /* opaque: device-resident sparse matrix or mask */

const char *mc_strerror(int status);
/* "major.minor+<source id> gfx950": build identification; the source id (12 hex digits) changes with any
 * source file or compiler flag of the library, so a stored measurement can name the build it belongs to. */
const char *mc_version(void);
/* After a call returned MC_EHIP on this thread: which HIP call failed and its message
 * (empty string if none yet).  The pointer stays valid for the thread's lifetime. */
const char *mc_last_error_detail(void);

/* ------------------------------------------------------------------------------------
 * Kernel-variant choices of one call.  All zero (mc_options_init) = automatic everywhere; the
 * result of a computation never depends on them (softmax-based results: up to fp32 summation
 * order).  They exist for tests and measurements.
 * ---------------------------------------------------------------------------------- */
typedef struct mc_options {
    int spmm_row_tile_bytes; /* 0 automatic, else 64, 128 or 256 bytes of a B row per workgroup            */
    int spmm_waves;          /* 0 automatic, else 1, 2, 4 or 8 wavefronts sharing a panel's chunks         */
    int spmm_stages;         /* 0 automatic (two chunks of gathered rows in flight per wave when B spans
                                less than 4 GiB and no wave has more than 4 chunks), 1 or 2               */
    int spmm_splitting;      /* 0 automatic (very unequal panels are cut into work items, see
                                mc_set_spmm_splitting), -1 never, 1 as 0 and also in the last SpMM of the
                                attention layer's kernel pipeline (see mc_attention_workspace_needed)      */
    int spmm_slab;           /* the SpMM form that keeps blocks of B resident in LDS and reads the gathered
                                rows from there: 0 automatic (when it is expected to be faster: dense
                                matrices), -1 never (also: mc_mat_create on this thread does not build the
                                K-blocked copy of the operand that form needs), 1 whenever the operand has
                                that copy and the precision has an 8- or 4-bit B without unsigned flags    */
    int spmm_slab_waves;     /* that form's computing waves per workgroup: 0 automatic, else 1 .. 15           */
    int spmm_slab_panels;    /* that form's panels per computing wave: 0 automatic, else 1, 2 or 4 (4 only with
                                an 8-bit B)                                                                */
    int sddmm_waves;         /* 0 automatic, -1 the kernel that loads operands straight from memory,
                                1, 2, 4 or 8 waves per panel of the kernel that stages Kmat rows in LDS   */
    int softmax_variant;     /* 0 automatic, 1 a workgroup per panel also for short panels, 2 always the
                                any-length kernel                                                          */
    int attention_mode;      /* 0 automatic, 1..6 as described at mc_set_attention_mode                    */
    int spmm_merge;          /* the SpMM on the operand's merged copy (see mc_merge_host): 0 automatic (when
                                the copy exists and is expected to be faster), -1 never (also: mc_mat_create on
                                this thread does not build the copy), 1 whenever the copy exists (and
                                mc_mat_create on this thread builds it whatever the shape)                  */
} mc_options;
/* Sets every field to automatic. */
void mc_options_init(mc_options *o);
/* Defaults of the CALLING THREAD for entry points that take no options argument (NULL: back to
 * automatic).  MC_EINVAL if a field holds a value outside its list; nothing changes then. */
int mc_set_thread_options(const mc_options *o);
int mc_get_thread_options(mc_options *o);

/* ------------------------------------------------------------------------------------
 * Host-side format builder (Section 4.1).  Pure host code: usable without a GPU.
 * ---------------------------------------------------------------------------------- */
typedef struct {
    int32_t P;           /* row panels = M / V                                       */
    int64_t nvec;        /* stored vectors = row_ptr[P]                              */
    int64_t nslots;      /* vector slots after padding each panel to a multiple of 64 */
    int64_t vals_bytes;  /* bytes of the packed value array (0 for lhs_bits == 0)    */
} mc_layout;

/* Checks M, K, V, lhs_bits (0 = pattern only, 4, 8, 12, 16) and row_ptr (host, P+1,
 * non-decreasing from 0) and fills *out.  MC_EINVAL on any violation. */
int mc_layout_query(int M, int K, int V, int lhs_bits, const int32_t *row_ptr, mc_layout *out);

/* Converts interchange data (host) into the device format (host buffers the caller
 * sized with mc_layout_query):
 *   panel_ptr  2*P int32: [2p] first slot of panel p (multiple of 64), [2p+1] = [2p] +
 *              number of real vectors (the "two row pointers" of Section 4.1)
 *   slot_idx   nslots int32: column of each slot; padded slots repeat the panel's last
 *              real column (their values are zero, so they add nothing)
 *   slot_vals  vals_bytes bytes (ignored when lhs_bits == 0 or values == NULL):
 *              chunk-major; inside a chunk 4 sub-strides of 16 slots; inside a
 *              sub-stride row-major: 8-bit  [row v][16 slots]
 *                                    16-bit [plane hi,lo][row v][16 slots] with the
 *                                           balanced split a = 256*hi + lo, both int8
 *                                    4-bit  [row v][8 bytes], byte b = slot b (low
 *                                           nibble) and slot b + 8 (high nibble)
 * Validates col_idx (ascending per panel, 0 <= c < K): MC_EINVAL; 16-bit values above
 * 32639 cannot be split into two signed bytes: MC_ERANGE; lhs_bits == 12 is stored like
 * 16 and additionally requires every value in [-2048, 2047]: MC_ERANGE. */
int mc_pack_host(int M, int K, int V, int lhs_bits, const int32_t *row_ptr, const int32_t *col_idx,
                 const void *values, int32_t *panel_ptr, int32_t *slot_idx, void *slot_vals);

/* Inverse of mc_pack_host (for round-trip checks): rebuilds row_ptr, col_idx and the
 * vector-major values from device-format host buffers.  Output buffers are sized for
 * P+1, nvec and nvec*V elements of the given width. */
int mc_unpack_host(int M, int K, int V, int lhs_bits, const int32_t *panel_ptr, const int32_t *slot_idx,
                   const void *slot_vals, int32_t *row_ptr, int32_t *col_idx, void *values);

/* K-blocked variant of the device format (Section 4.1 leaves the stride to the kernel; Section 4.2
 * notes that rows of the dense operand have no reuse in on-chip memory when every panel gathers
 * them anew -- this layout is what lets a workgroup keep a block of rows resident instead): the
 * vectors of a panel are also grouped by the block of MC_KBLOCK consecutive columns they fall in,
 * each (panel, block) list zero-padded to whole chunks of 64, so that a chunk only names rows of
 * one block.  nblk = ceil(K / MC_KBLOCK).
 *   blk_ptr   P*nblk + 1 int32: first chunk of (panel p, block b) at [p*nblk + b]; the chunks of a
 *             panel are consecutive over its blocks
 *   blk_rows  nchunks*64 uint16: row of each slot inside its block (column - b*MC_KBLOCK); padded
 *             slots repeat the list's last real row.  Inside a chunk, slot s sits at position
 *             (s/16)*16 + (s%8)*2 + (s%16)/8: slots s and s+8 of a sub-stride of 16 are neighbours
 *             (one lane of the kernel addresses exactly these two and reads them as one word)
 *   blk_vals  vals_bytes bytes, chunk by chunk in the layout of mc_pack_host's slot_vals
 *   blk_src   nchunks*64 int32: interchange index of the vector in each slot, -1 for padding
 * Same validation and error codes as mc_pack_host.  Pure host code. */
#define MC_KBLOCK 1024
typedef struct {
    int32_t nblk;        /* K-blocks                                                  */
    int64_t nchunks;     /* chunks over all (panel, block) lists                      */
    int64_t vals_bytes;  /* bytes of the packed value array (0 for lhs_bits == 0)     */
} mc_blocked_layout;
int mc_blocked_query(int M, int K, int V, int lhs_bits, const int32_t *row_ptr, const int32_t *col_idx,
                     mc_blocked_layout *out);
int mc_pack_blocked_host(int M, int K, int V, int lhs_bits, const int32_t *row_ptr, const int32_t *col_idx,
                         const void *values, int32_t *blk_ptr, uint16_t *blk_rows, void *blk_vals, int32_t *blk_src);

/* ------------------------------------------------------------------------------------
 * Merged panels: a second copy of an SpMM operand with vectors of V * group rows.
 *
 * The MFMA's row operand has 16 rows, a panel of the format fills V of them, and every panel
 * fetches the rows of the dense operand its own vectors name (Section 4.2).  `group`
 * consecutive panels can share both: merged into one panel of V * group rows (8, or 16 for 4-
 * and 8-bit values) whose vectors sit at the union of the panels' columns, with zeros where a
 * panel holds no vector -- explicit zeros are legal inside stored vectors, so the product is
 * unchanged.  A row of the dense operand is then fetched once per group instead of once per
 * panel that names it (random patterns at 50 % sparsity, V = 2, group 8: a quarter of the
 * fetches), padding to whole chunks shrinks, and the matrix unit does useful work in every row.
 *
 * mc_merged_query: panels and vectors of the merged operand.  group must be 2, 4 or 8 with
 * V * group == 8 or (lhs_bits 4 / 8 only) 16; the last merged panel may cover fewer panels.
 * mc_merge_host writes the merged operand as interchange arrays:
 *   m_row_ptr  P_merged + 1,  m_col_idx  nvec_merged (ascending per merged panel)
 *   m_values   nvec_merged * V * group elements of the operand's width (NULL: pattern only);
 *              rows g*V .. g*V+V-1 of a merged vector belong to panel p0 + g of its group
 *   m_src      nvec_merged * group int32: interchange vector that fills those rows, -1 = zeros
 * Same validation and error codes as mc_pack_host.  Pure host code.
 * ---------------------------------------------------------------------------------- */
typedef struct {
    int32_t group;       /* panels per merged panel                                   */
    int32_t P;           /* merged panels = ceil(P / group)                           */
    int64_t nvec;        /* vectors of the merged operand                             */
} mc_merged_layout;
int mc_merged_query(int M, int K, int V, int lhs_bits, const int32_t *row_ptr, const int32_t *col_idx, int group,
                    mc_merged_layout *out);
int mc_merge_host(int M, int K, int V, int lhs_bits, const int32_t *row_ptr, const int32_t *col_idx, const void *values,
                  int group, int32_t *m_row_ptr, int32_t *m_col_idx, void *m_values, int32_t *m_src);

/* ------------------------------------------------------------------------------------
 * Device-resident sparse operand.
 * ---------------------------------------------------------------------------------- */
/* Builds the device format from HOST interchange arrays and uploads it on `stream`
 * (the call returns after the upload has completed).  values == NULL or lhs_bits == 0
 * gives a pattern-only mask (for SDDMM / attention).  *out is owned by the caller
 * until mc_mat_destroy.  Errors as mc_pack_host, plus MC_EHIP / MC_ENOMEM. */
int mc_mat_create(int M, int K, int V, int lhs_bits, const int32_t *row_ptr, const int32_t *col_idx,
                  const void *values, void *stream, mc_mat **out);
/* Replaces the values from a DEVICE array in interchange order (nvec*V elements of the
 * matrix's width; e.g. the output of a softmax).  Asynchronous on `stream`.
 * Device data cannot be range-checked on the host: a 16-bit value must not exceed 32639 (it is
 * split into two signed bytes) and a 12-bit operand must lie in [-2048, 2047]; values outside
 * these ranges are not detected and give a wrong product (mc_mat_create returns MC_ERANGE for
 * the same data on the host). */
int mc_mat_set_values_device(mc_mat *A, const void *values_dev, void *stream);
void mc_mat_destroy(mc_mat *A);
/* Shape queries; return MC_EINVAL on a null handle. */
int mc_mat_info(const mc_mat *A, int *M, int *K, int *V, int *lhs_bits, int64_t *nvec, int64_t *nslots);
/* The operand's merged copy (see mc_merge_host), which mc_mat_create builds for operands with values and
 * V < 16 rows to share: *group = panels per merged panel (0: no such copy), *nvec = its vectors. */
int mc_mat_merged_info(const mc_mat *A, int *group, int64_t *nvec);

/* ------------------------------------------------------------------------------------
 * SpMM (Section 4.2): C = A * B, exact int32.
 *   A      sparse M x K, width must match prec (L8: 8, L4: 4, L12: 12, L16: 16 bits)
 *   B_dev  dense K x N row-major, int8 (R8), packed int4 (R4) or little-endian int16 (R16);
 *          ldb in elements
 *   C_dev  dense M x N row-major int32; ldc in elements
 * Requirements: B_dev, C_dev 16-byte aligned; N a multiple of 16 (R8), 32 (R4) or 8 (R16);
 * ldb*bits/8 a multiple of 16 and >= the row bytes; ldc a multiple of 4 and >= N.
 * R4 paths keep 16x (L8-R4, L16-R4, L12-R4) or 256x (L4-R4) scaled plane sums in int32, so
 * they require K <= 131072.  A 16-bit (12-bit) A is computed as two signed int8 planes in one
 * MFMA and recombined as (C_hi << 8) + C_lo; a 16-bit B is read as its high (signed) and low
 * (unsigned) bytes, any int16 value, and recombined the same way (Section 4.4).
 * Results that do not fit int32 wrap (two's complement).
 * ---------------------------------------------------------------------------------- */
int mc_spmm(const mc_mat *A, const void *B_dev, int N, int ldb, mc_prec prec, int32_t *C_dev, int ldc,
            void *stream);

/* Operand signedness (Section 4.4.1, unsigned integers): with a flag set, the bytes (nibbles) of
 * that operand are read as values in [0, 255] ([0, 15]) instead of two's complement.  The matrix
 * unit multiplies signed bytes, so an unsigned value enters as u - 128 (u - 8) and the difference
 * is put back exactly from row sums of A and column sums of the gathered B rows.
 * Supported for MC_L8R8, MC_L8R4 and MC_L4R4 (other precisions: MC_EUNSUPPORTED); the 4-bit
 * right operand then requires K <= 32768.  flags = 0 is mc_spmm / mc_sddmm. */
#define MC_LHS_UNSIGNED 1u
#define MC_RHS_UNSIGNED 2u
int mc_spmm_flags(const mc_mat *A, const void *B_dev, int N, int ldb, mc_prec prec, unsigned flags, int32_t *C_dev,
                  int ldc, void *stream);
/* mc_spmm_flags with the kernel variant given per call (options == NULL: automatic, whatever the
 * thread's defaults are).  MC_EINVAL for an option value outside its list. */
int mc_spmm_ex(const mc_mat *A, const void *B_dev, int N, int ldb, mc_prec prec, unsigned flags,
               const mc_options *options, int32_t *C_dev, int ldc, void *stream);
/* Which form mc_spmm_ex would run for this operand, width and options (host only, launches nothing):
 * bit 0: 0 = rows of B gathered per stored vector, 1 = K-blocks of B resident in LDS; bit 1 (value 2): on the
 * operand's merged copy (see mc_merge_host).  Negative: an error code. */
int mc_spmm_form(const mc_mat *A, int N, mc_prec prec, const mc_options *options);

/* SpMM with fused dequantisation (Section 5.3: the integer product is turned into real values
 * in the kernel's epilogue): C = scale * (A * B), each element computed as float(int32 result) *
 * scale in fp32 and, for MC_OUT_F16, rounded to nearest even (magnitudes beyond the fp16 range
 * become infinity).  C_dev: M x N row-major float or half, 16-byte aligned, ldc a multiple of 4.
 * scale must be finite.  Other arguments and limits as mc_spmm_flags.  Panels of very unequal
 * length are not shared between workgroups here (a rounded result cannot be added up piecewise, and
 * this call has no workspace for exact partial sums; the attention layer's last SpMM has one). */
int mc_spmm_dequant(const mc_mat *A, const void *B_dev, int N, int ldb, mc_prec prec, unsigned flags, float scale,
                    mc_out_type out_type, void *C_dev, int ldc, void *stream);

/* Measurement aid (Section 4.2.1 names the gather of B rows by column index as the step the
 * kernel is built around): performs ONLY the gather of mc_spmm(A, B_dev, N, ldb, prec, ...) --
 * same tile variant, index loads and row copies into on-chip memory, no arithmetic, no C.
 * Its time is the floor the memory system sets for that launch shape.
 *   sink_dev   int32 array, at least mc_probe_gather_sink_len(A, N, prec) entries; entry
 *              w receives bytes 0..3 of workgroup w's first staged row piece (0 for an empty panel)
 * Same argument checks as mc_spmm. */
int64_t mc_probe_gather_sink_len(const mc_mat *A, int N, mc_prec prec);
int mc_probe_gather(const mc_mat *A, const void *B_dev, int N, int ldb, mc_prec prec, int32_t *sink_dev,
                    void *stream);

/* Measurement aid (the paper's Algorithm 1 and Section 4.2.4 are about hiding the latency between the steps of
 * one thread block; this shows where that latency sits here): the L8-R8 SpMM kernel on 128-byte row tiles, two
 * waves per panel, two chunks in flight -- the form the 4096 x 4096, 90 % sparse, N = 256 problem runs in --
 * computes C exactly as mc_spmm does and also records, per wave, ten readings of the device's constant 100 MHz
 * clock: 0 wave started, 1 kernel arguments and panel pointers arrived, 2 column indices and A operands arrived
 * (first row copies issued next), 3 rows of the wave's first chunk landed, 4 all chunks in the accumulators,
 * 5 partial tile written, 6 workgroup barrier passed, 7 the thread's output pieces summed, 8 stores issued,
 * 9 stores acknowledged.
 *   trace_dev  int64 array of mc_probe_spmm_phases_len(A, N) entries: wave w of workgroup g (= panel *
 *              tiles + tile) writes entries (2 g + w) * 10 .. + 9
 * MC_EUNSUPPORTED unless A holds 8-bit values in panels of at most 8 chunks, none of them cut into work
 * items, and B spans less than 4 GiB with rows below 16 MiB.  Other checks as mc_spmm. */
int64_t mc_probe_spmm_phases_len(const mc_mat *A, int N);
int mc_probe_spmm_phases(const mc_mat *A, const void *B_dev, int N, int ldb, int32_t *C_dev, int ldc, int64_t *trace_dev,
                         void *stream);

/* Measurement aid (Section 5 reports its kernels against the peak of the matrix unit): the matrix unit
 * alone.  `workgroups` workgroups of four waves each issue iters * 8 independent 16x16x64 int8 MFMAs on
 * registers, i.e. workgroups * 4 * iters * 8 * 32768 operations without any memory traffic; timing it gives
 * the int8 rate this device sustains in practice, to set beside the published peak.
 *   sink_dev   workgroups * 256 int32, receives the (meaningless) sums, except that the first wave reports
 *              its own loop in the first two: shader-clock cycles, and ticks of the constant 100 MHz clock
 *              (so cycles per MFMA and the clock frequency under this load can be told apart). */
int mc_probe_mfma(int workgroups, int iters, int32_t *sink_dev, void *stream);

/* ------------------------------------------------------------------------------------
 * SDDMM (Section 4.3): for every stored vector i of the mask (panel p, column c):
 *   S[i*V + v] = sum_k Q[p*V + v][k] * Kmat[c][k],  v = 0..V-1
 *   Q_dev     M x Kd row-major, Kmat_dev  Nc x Kd row-major (the paper's column-major
 *             right operand), int8 (MC_L8R8), packed int4 (MC_L4R4) or int16 (MC_L16R16,
 *             every value <= 32639: both operands are split into signed byte planes);
 *             ldq/ldk in elements
 *   mask      pattern of an M x Nc matrix (values ignored)
 *   S_dev     nvec*V int32 in interchange (vector-major) order
 * Requirements: 16-byte aligned pointers; Kd*bits/8 a multiple of 16; ld*bits/8 a
 * multiple of 16.  Other precisions: MC_EUNSUPPORTED.
 * ---------------------------------------------------------------------------------- */
int mc_sddmm(const void *Q_dev, int ldq, const void *Kmat_dev, int ldk, int Kd, const mc_mat *mask,
             mc_prec prec, int32_t *S_dev, void *stream);
/* The same with operand signedness flags (MC_LHS_UNSIGNED: Q, MC_RHS_UNSIGNED: Kmat; see
 * mc_spmm_flags).  Supported for MC_L8R8 and MC_L4R4 (the latter with Kd <= 32768). */
int mc_sddmm_flags(const void *Q_dev, int ldq, const void *Kmat_dev, int ldk, int Kd, const mc_mat *mask,
                   mc_prec prec, unsigned flags, int32_t *S_dev, void *stream);
/* mc_sddmm_flags with the kernel variant given per call (options == NULL: automatic). */
int mc_sddmm_ex(const void *Q_dev, int ldq, const void *Kmat_dev, int ldk, int Kd, const mc_mat *mask,
                mc_prec prec, unsigned flags, const mc_options *options, int32_t *S_dev, void *stream);

/* SDDMM with fused dequantisation (Section 5.3): S_dev receives scale * score as nvec*V floats
 * or halves (rounded as in mc_spmm_dequant) in the same order.  Other arguments as mc_sddmm_flags. */
int mc_sddmm_dequant(const void *Q_dev, int ldq, const void *Kmat_dev, int ldk, int Kd, const mc_mat *mask,
                     mc_prec prec, unsigned flags, float scale, mc_out_type out_type, void *S_dev, void *stream);

/* SDDMM that writes the operand format of a following SpMM (Section 4.3: the output is stored in the
 * strided format when the next operator is SpMM): the scores are re-quantised in the kernel's epilogue,
 *   code = clamp(rint(score * scale), -qmax, qmax),  qmax = 127 (8-bit P) or 32639 (16-bit P),
 * -- the int32 score converted to fp32, one fp32 product, rounded to nearest even -- and written
 * straight into the device-resident values of P, whose pattern is the mask (padded slots: zeros), so
 * that mc_spmm(P, ...) can follow without an interchange-order round trip.
 *   P       a matrix created with values (e.g. zeros) of 8 or 16 bits; all its values are replaced.
 *           Pattern-only mask: MC_EINVAL; other widths: MC_EUNSUPPORTED.
 *   prec    width of Q and Kmat: MC_L8R8, MC_L4R4 or MC_L16R16 (as mc_sddmm; signed operands)
 * Other arguments and requirements as mc_sddmm; scale must be finite.  Kernel variants: the calling
 * thread's options. */
int mc_sddmm_to_mat(const void *Q_dev, int ldq, const void *Kmat_dev, int ldk, int Kd, mc_prec prec, float scale,
                    mc_mat *P, void *stream);

/* ------------------------------------------------------------------------------------
 * Sparse softmax with fused (de)quantisation (Section 5.3): for each row (p, v) over its
 * stored entries i:  x_i = S[i*V+v] * score_scale;  p_i = exp(x_i - max) / sum;
 * code_i = clamp(rint(p_i * inv_s_p), 0, 127) as int8, in interchange order.  fp32 math.
 *   batch     number of independent score sets sharing the mask (heads)
 *   S_dev     batch * nvec*V int32;  codes_dev  batch * nvec*V int8
 * ---------------------------------------------------------------------------------- */
int mc_sparse_softmax(const mc_mat *mask, int batch, const int32_t *S_dev, float score_scale,
                      float inv_s_p, int8_t *codes_dev, void *stream);
/* The same with code_bits = 8 (int8 codes, as above) or 16: int16 codes clamped to
 * [0, 32639], the largest value that still splits into two signed bytes (Section 4.4) and
 * can therefore feed a 16-bit SpMM operand.  Other widths: MC_EUNSUPPORTED. */
int mc_sparse_softmax_bits(const mc_mat *mask, int batch, const int32_t *S_dev, float score_scale,
                           float inv_s_p, int code_bits, void *codes_dev, void *stream);

/* ------------------------------------------------------------------------------------
 * Quantisation of the layer's inputs (Section 5.3, first step): symmetric, one scale per tensor.
 *   mc_absmax    *result_dev (device float) = max |x_dev[i]|, i < n; the caller takes
 *                scale = max / 127 (8 bits) or max / 7 (4 bits), or uses a calibrated constant
 *   mc_quantize  q[i] = clamp(rint(x[i] / scale), -qmax, qmax), ties to even, decided as in double
 *                precision; bits = 8: int8 codes; bits = 4: two codes per byte (element 2j in bits
 *                3:0 of byte j), n even.  x_dev 16-byte aligned, q_dev 8-byte aligned.
 * Other widths: MC_EUNSUPPORTED; scale must be finite and positive.
 * ---------------------------------------------------------------------------------- */
int mc_absmax(const float *x_dev, int64_t n, float *result_dev, void *stream);
int mc_quantize(const float *x_dev, int64_t n, float scale, int bits, void *q_dev, void *stream);

/* The sparse softmax for ONE score set, written straight into the device-resident values of a
 * sparse operand (Section 4.3: the producer writes the format its consumer reads), so that
 * mc_spmm(P, ...) can follow without mc_mat_set_values_device:
 *   P   a matrix with the mask's pattern that holds 8- or 16-bit values (created with values,
 *       e.g. zeros; a pattern-only mask: MC_EINVAL; other widths: MC_EUNSUPPORTED).  Its width
 *       selects the code range as in mc_sparse_softmax_bits; all its values are replaced. */
int mc_sparse_softmax_to_mat(mc_mat *P, const int32_t *S_dev, float score_scale, float inv_s_p, void *stream);

/* ------------------------------------------------------------------------------------
 * Quantized sparse self-attention layer (Section 5.3), one mask shared by all heads:
 *   O[h] = ( P_q[h] * Vm[h] ) * (s_p * s_v),
 *   P_q[h] = int8( softmax( SDDMM(Q[h], Km[h]; mask) * s_q*s_k/sqrt(dk) ) / s_p )
 *   Q_dev, Km_dev, Vm_dev   heads x L x dk int8, contiguous (see the strided variant below)
 *   mask                    L x L pattern, V = 8
 *   O_dev                   heads x L x dk fp32
 *   workspace_dev           at least mc_attention_workspace_bytes(heads, mask) bytes,
 *                           256-byte aligned, caller-owned; contents undefined after
 * Requirements: dk a multiple of 16; all four scales positive (symmetric quantisation scales
 * are; MC_EINVAL otherwise).  Entries excluded by the mask do not take part in the softmax.
 * Empty rows give zeros.  The workspace is only needed, checked and touched when the layer
 * runs as the pipeline of separate kernels (see mc_set_attention_mode): NULL / 0 is accepted
 * whenever mc_attention_workspace_needed(...) is 0 -- the fused kernel takes the layer, or the
 * mask stores nothing.
 * ---------------------------------------------------------------------------------- */
size_t mc_attention_workspace_bytes(int heads, const mc_mat *mask);
/* Bytes of workspace the layer makes use of for this head dimension and these options (NULL: the
 * calling thread's defaults): 0 when the fused kernel runs; else the codes of all heads, plus the
 * int32 scores when they travel through memory (three kernels), plus -- for a mask with panels many
 * times longer than the average and with spmm_splitting = 1 -- int32 output rows of those panels,
 * which several workgroups of the last SpMM then share (exact partial sums, scaled and rounded by a
 * last small kernel: the same values as with whole panels).  mc_attention_workspace_bytes[_bits] (codes
 * and scores) is always enough to run; with less than the figure returned here the long panels are
 * simply not shared (same results, a longer tail). */
size_t mc_attention_workspace_needed(int heads, int dk, const mc_mat *mask, int p_bits, const mc_options *options);
/* The same layer for any regular layout: element (head h, token l, d) of Q, Km, Vm (int8)
 * and of O (fp32) sits at h*head_stride + l*token_stride + d (strides in elements, both
 * multiples of 16).  mc_sparse_attention is the case head_stride = L*dk, token_stride = dk.
 * The token-major layout a QKV projection produces (head_stride = dk, token_stride =
 * heads*dk) is the fast one: with rows of at most 64 bytes (dk = 64, or dk = 128 of 4-bit
 * values in the variants below) and an even number of heads, two neighbouring heads are
 * gathered with one 128-byte request per token. */
int mc_sparse_attention_strided(const int8_t *Q_dev, const int8_t *Km_dev, const int8_t *Vm_dev, int heads, int L,
                                int dk, int64_t head_stride, int64_t token_stride, const mc_mat *mask, float s_q,
                                float s_k, float s_v, float s_p, float *O_dev, void *workspace_dev,
                                size_t workspace_bytes, void *stream);
int mc_sparse_attention(const int8_t *Q_dev, const int8_t *Km_dev, const int8_t *Vm_dev, int heads, int L,
                        int dk, const mc_mat *mask, float s_q, float s_k, float s_v, float s_p,
                        float *O_dev, void *workspace_dev, size_t workspace_bytes, void *stream);

/* The "xb-yb" variants of the layer (Section 5.3 and the end-to-end latency figure): the
 * softmax output is quantised to p_bits = x (8 or 16; 16-bit codes are clamped to 32639 and
 * multiplied as two signed byte planes) and Q, Km, Vm hold qkv_bits = y bit integers (8, or 4
 * packed two per byte along dk).  Strides are in ELEMENTS for all four tensors and must make
 * whole 16-byte pieces (multiples of 16 for 8-bit, of 32 for 4-bit inputs); dk likewise.
 * p_bits = 8, qkv_bits = 8 is mc_sparse_attention_strided.  Every combination has the fused
 * kernel (dk == 64 or dk == 128; panels of at most 2048 vectors) and the
 * kernel pipeline behind it, as selected by mc_set_attention_mode; the workspace must hold
 * mc_attention_workspace_bytes_bits(heads, mask, p_bits) bytes.
 * Unsupported widths: MC_EUNSUPPORTED. */
size_t mc_attention_workspace_bytes_bits(int heads, const mc_mat *mask, int p_bits);
int mc_sparse_attention_bits(const void *Q_dev, const void *Km_dev, const void *Vm_dev, int heads, int L, int dk,
                             int64_t head_stride, int64_t token_stride, const mc_mat *mask, int p_bits,
                             int qkv_bits, float s_q, float s_k, float s_v, float s_p, float *O_dev,
                             void *workspace_dev, size_t workspace_bytes, void *stream);

/* The layer for a batch of inputs that share the mask (the end-to-end runs of Section 5.3 use
 * batches of 2 and 8): element (b, h, l, d) sits at b*batch_stride + h*head_stride +
 * l*token_stride + d in all four tensors (strides in elements, whole 16-byte pieces), batch
 * <= 65535.  One launch of the fused kernel covers the whole batch; the kernel pipeline runs
 * the items one after the other through the same workspace (sized for ONE item). */
int mc_sparse_attention_batched(const void *Q_dev, const void *Km_dev, const void *Vm_dev, int batch, int heads, int L,
                                int dk, int64_t batch_stride, int64_t head_stride, int64_t token_stride,
                                const mc_mat *mask, int p_bits, int qkv_bits, float s_q, float s_k, float s_v,
                                float s_p, float *O_dev, void *workspace_dev, size_t workspace_bytes, void *stream);

/* The batched layer with a typed output (Section 5.3 dequantises the layer's result to fp16):
 * O_dev holds floats (MC_OUT_F32: identical to mc_sparse_attention_batched) or halves
 * (MC_OUT_F16: the same fp32 results rounded to nearest even); strides stay in elements. */
int mc_sparse_attention_out(const void *Q_dev, const void *Km_dev, const void *Vm_dev, int batch, int heads, int L,
                            int dk, int64_t batch_stride, int64_t head_stride, int64_t token_stride,
                            const mc_mat *mask, int p_bits, int qkv_bits, float s_q, float s_k, float s_v, float s_p,
                            mc_out_type out_type, void *O_dev, void *workspace_dev, size_t workspace_bytes,
                            void *stream);
/* mc_sparse_attention_out with the kernel variants given per call (options == NULL: automatic). */
int mc_sparse_attention_ex(const void *Q_dev, const void *Km_dev, const void *Vm_dev, int batch, int heads, int L,
                           int dk, int64_t batch_stride, int64_t head_stride, int64_t token_stride,
                           const mc_mat *mask, int p_bits, int qkv_bits, float s_q, float s_k, float s_v, float s_p,
                           mc_out_type out_type, const mc_options *options, void *O_dev, void *workspace_dev,
                           size_t workspace_bytes, void *stream);

/* For callers that cannot allocate device memory or hand over a workspace (code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc): mc_sparse_attention_ex without the
 * workspace arguments.  When the layer runs as the pipeline of separate kernels, its intermediates
 * go to an array the library itself holds in device memory -- MC_STATIC_SCRATCH_BYTES per GPU the
 * library has run on, from the first such call on that GPU until the process ends.  A layer whose
 * intermediates (mc_attention_workspace_bytes_bits(heads, mask, p_bits) bytes) exceed that size is
 * refused with MC_ENOMEM before anything is launched (mc_last_error_detail() gives both sizes).  The
 * call allocates nothing and frees nothing; the first call on a device looks up the array's address
 * (make it once outside a graph capture).  All calls on one GPU share the array: every call
 * overwrites all of it that it reads, so nothing has to be cleared between calls, but two calls that
 * overlap in time on the same GPU (different streams, different threads) race on it.  options ==
 * NULL: the calling thread's defaults.  Results equal mc_sparse_attention_ex's. */
#define MC_STATIC_SCRATCH_BYTES (16u << 20)
int mc_sparse_attention_static(const void *Q_dev, const void *Km_dev, const void *Vm_dev, int batch, int heads, int L,
                               int dk, int64_t batch_stride, int64_t head_stride, int64_t token_stride,
                               const mc_mat *mask, int p_bits, int qkv_bits, float s_q, float s_k, float s_v,
                               float s_p, mc_out_type out_type, const mc_options *options, void *O_dev, void *stream);

/* ------------------------------------------------------------------------------------
 * One-knob setters kept for existing callers, tests and measurements.  Each changes one field of
 * the CALLING THREAD's default options (see mc_set_thread_options); none is needed for
 * correctness, and none affects other threads or the ..._ex entry points.
 *   bytes_per_row_tile  0 = automatic, else 64, 128 or 256 bytes of a B row per workgroup
 *   waves               0 = automatic, else 1, 2, 4 or 8 wavefronts sharing a panel's chunks
 * Returns MC_EINVAL for other values.
 * ---------------------------------------------------------------------------------- */
int mc_set_spmm_variant(int bytes_per_row_tile, int waves);
/* Chunks of gathered rows in flight per wave of the SpMM kernel: 2 (default; used when B spans
 * less than 4 GiB and no wave has more than 4 chunks) or 1.  Same results.  MC_EINVAL for other
 * values. */
int mc_set_spmm_stages(int stages);
/* Matrices whose longest panel is far above the average (more than six times the average and
 * more than 16 chunks) get, at mc_mat_create, a list of work items that cuts long panels into
 * pieces of at most three times the average (at least 8 chunks); mc_spmm then lets several workgroups add their exact int32 partial results into the
 * (first cleared) rows of such panels.  enable = 0 turns this off (one workgroup per panel and
 * row tile, as for regular matrices); the result is the same either way. */
int mc_set_spmm_splitting(int enable);
/* (The switch also governs the work items of mc_sddmm.  There every item writes its own outputs,
 * so a pattern-only mask is cut finer: into pieces of at most the average panel length, at least
 * 8 chunks, as soon as one panel is longer than that; a mask with fewer than 256 panels into
 * pieces short enough to make 256 of them, again at least 8 chunks.) */
/* SDDMM variant: -1 = automatic, 0 = the kernel that loads operands straight from memory
 * (any row length), 1, 2, 4 or 8 = waves per panel of the kernel that stages Kmat rows in
 * LDS (used when a row has 64, 128, 256, 512 or 1024 bytes, or 32 bytes of 4-bit values, else
 * ignored). */
int mc_set_sddmm_variant(int waves);
/* Softmax variant: 0 = automatic (panels of up to 4096 scores, padding included, are kept in
 * the registers of one wave, up to 16384 in those of a workgroup: one pass over the scores),
 * 1 = a workgroup per panel also for short panels, 2 = always the kernel for panels of any
 * length (three passes).  Same codes up to fp32 summation order. */
int mc_set_softmax_variant(int variant);
/* Attention path: 0 = automatic (a single fused kernel when dk is 64 or 128 and no panel holds
 * more than 2048 vectors -- one, two or four waves per (panel, head) for panels of up to 512,
 * 1024, 2048 vectors, more waves than that when the launch is small; two neighbouring heads per
 * workgroup for token-major tensors once the launch has 2048 (panel, head) units -- else the
 * pipeline of kernels), 1 = always the pipeline: one kernel that computes the scores of a panel,
 * keeps them in on-chip memory, takes the softmax and writes the integer codes in the SpMM's operand
 * format, then the SpMM (rows of Q / Km of up to 256 bytes and panels of up to about 4700 vectors;
 * beyond that, or with 6 = always, three kernels: SDDMM, softmax, SpMM, with the int32 scores in the
 * workspace).  The remaining modes pin parts of the automatic choice (for tests and measurements):
 * 2 = the fused kernel with one head per workgroup even for token-major tensors, waves by panel
 * length alone; 3 / 4 = the fused kernel with at least two / with four waves per (panel, head)
 * whatever the panel length, 5 = waves by panel length alone -- 3, 4 and 5 with two heads per
 * workgroup wherever the layout allows it, whatever the size of the launch.  All give the same
 * result up to fp32 summation order in the softmax.  MC_EINVAL for other values. */
int mc_set_attention_mode(int mode);

#ifdef __cplusplus
}
#endif
#endif /* MAGICUBE_H */
