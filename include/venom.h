/*
 * venom.h -- C ABI of the MI355X (gfx950) V:N:M sparse x dense product library.
 *
 * The operation is C = A . B with A (R x K, fp16) stored in the V:N:M format of the paper's
 * section 3 ("The V:N:M format"), B dense K x C_cols fp16, fp32 accumulation (section 4,
 * "Spatha").  N is always 2: the innermost pattern is the hardware's 2:4.
 *
 * Conventions that hold for every entry point
 *   - every pointer named *_dev is DEVICE memory owned by the caller; the library never
 *     allocates or frees device memory.  Pointers without that suffix are HOST memory.
 *   - matrices are row-major; leading dimensions (lda, ldm, ldb, ldc) are in ELEMENTS.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *   - every call returns a venom_status_t; nothing aborts or throws across the boundary.
 *   - a handle is a small HOST object holding NON-owning pointers into the caller's workspace;
 *     it stays valid while that workspace is alive and unmodified.  venom_destroy frees the host
 *     object only.
 *
 * Canonical V:N:M arrays (what venom_export returns and venom_import accepts), G = K / M:
 *   values  uint16 [R][G][2]        fp16 bit patterns of the kept entries, 0x0000 in padded slots
 *   columns uint16 [R/V][G][4]      column-loc: which 4 of the M columns each V x M block keeps,
 *                                   relative ids in [0, M), strictly increasing
 *   meta    uint32 [R][ceil(G/8)]   per (row, group) a nibble idx0 | idx1 << 2 with idx0 < idx1, the
 *                                   two 2-bit m-indices, each addressing one of the block's 4
 *                                   SELECTED columns; group g sits in bits [4(g%8), 4(g%8)+3] of
 *                                   word g/8, unused nibbles are 0.
 * Where the paper leaves a choice open the library follows these rules (the CPU oracle states
 * the same ones): column-loc ascending; a block using fewer than 4 columns is padded with its
 * smallest unused column ids; a (row, group) keeping fewer than 2 entries is padded with its
 * smallest unused positions and stores +0 there; structure follows the mask, not the values.
 */
#ifndef VENOM_H_
#define VENOM_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  VENOM_OK = 0,
  VENOM_ERR_INVALID_ARG = 1, /* NULL where a pointer is required, negative size, bad enum value      */
  VENOM_ERR_SHAPE = 2,       /* R % V, K % M, M < 4, V < 1, C_cols < 1, leading dimension too small  */
  VENOM_ERR_UNSUPPORTED = 3, /* N != 2; misaligned pointer / leading dimension; shape the kernels do
                                not cover (venom_spmm needs V in {32,64,96,128} -- any V at M = 4 when
                                R % 128 == 0 --, C_cols % 8 == 0, K > 0; every call needs R/V <= 65535,
                                M <= 1024 and R * K <= 2^38)                                         */
  VENOM_ERR_MASK_COLS = 4,   /* illegal mask: a V x M block uses more than 4 columns                 */
  VENOM_ERR_MASK_ROW = 5,    /* illegal mask: a row keeps more than 2 entries in a group of M        */
  VENOM_ERR_WORKSPACE = 6,   /* workspace NULL, misaligned (256 B) or smaller than required          */
  VENOM_ERR_HIP = 7          /* a HIP runtime call or kernel launch failed                           */
} venom_status_t;

/* First offending block of an illegal mask, in row-major (block_row, group) order.  `row` is the
 * first offending absolute row for VENOM_ERR_MASK_ROW and -1 for VENOM_ERR_MASK_COLS (a block
 * that breaks both rules reports the column rule). */
typedef struct {
  int64_t block_row, group, row;
} venom_violation_t;

typedef struct venom_handle venom_handle_t;

/* Bytes of device workspace a handle for an R x K matrix in V:2:M needs (canonical arrays, the
 * kernel's packed copies and a status word).  Section 3 fixes the array shapes. */
venom_status_t venom_workspace_bytes(int64_t R, int64_t K, int V, int N, int M, size_t* bytes);

/* Section 3 / the sparsifier call of the paper's PyTorch integration listing: dense matrix plus
 * mask -> values, column-loc, m-indices; checks that the mask is V:N:M-legal.
 *   A_f16_dev   R x K fp16 (bit patterns are copied, never interpreted), lda >= K
 *   mask_dev    R x K bytes, nonzero = keep, ldm >= K
 *   workspace_dev / workspace_bytes   >= venom_workspace_bytes(...), 256-byte aligned
 *   out         receives the handle on VENOM_OK, NULL otherwise
 *   viol        optional (may be NULL); filled on VENOM_ERR_MASK_*
 * Synchronises `stream` once (to read the legality word back). */
venom_status_t venom_compress(const void* A_f16_dev, int64_t lda, const uint8_t* mask_dev, int64_t ldm,
                              int64_t R, int64_t K, int V, int N, int M, void* workspace_dev,
                              size_t workspace_bytes, void* stream, venom_handle_t** out,
                              venom_violation_t* viol);

/* Section 3, the three arrays of the format as the persistent form of a compressed matrix: build
 * a handle from canonical arrays already on the device (layout above).  The arrays are copied into
 * the workspace and CHECKED there: column ids strictly increasing and below M, idx0 < idx1 in every
 * nibble, unused nibbles zero; anything else returns VENOM_ERR_INVALID_ARG, no handle, and nothing
 * is ever gathered from such arrays (value bits are free).  Synchronises `stream` once. */
venom_status_t venom_import(const uint16_t* values_dev, const uint16_t* columns_dev, const uint32_t* meta_dev,
                            int64_t R, int64_t K, int V, int N, int M, void* workspace_dev,
                            size_t workspace_bytes, void* stream, venom_handle_t** out);

/* Section 3: the canonical arrays (values R x K/M x 2, m-indices R x K/M x 2 two-bit, column-loc
 * R/V x K/M x 4) copied out; any of the three destinations may be NULL to skip it.
 * Asynchronous on `stream`. */
venom_status_t venom_export(const venom_handle_t* h, uint16_t* values_dev, uint16_t* columns_dev,
                            uint32_t* meta_dev, void* stream);

/* Section 3, the two pruning stages, as one-shot magnitude pruning (the policy of the energy
 * study of section 5): for every V x M block keep the 4 columns of largest L1 mass over the V rows,
 * then in every row the 2 entries of largest magnitude among those 4; ties go to the smaller
 * index.  Writes mask (R x K bytes, 1 = keep, exactly 2 per row and group: always legal for
 * venom_compress).  Optionally accumulates, per block row, the kept and the total L1 mass as exact
 * integers in units of 2^-24 (every fp16 is a multiple of it; Inf/NaN count as 2^40):
 * energy = sum(kept) / sum(total).  kept_mass_dev / total_mass_dev: R/V uint64 each, or NULL.
 * Asynchronous on `stream`. */
venom_status_t venom_prune(const void* A_f16_dev, int64_t lda, int64_t R, int64_t K, int V, int N, int M,
                           uint8_t* mask_dev, int64_t ldm, uint64_t* kept_mass_dev, uint64_t* total_mass_dev,
                           void* stream);

/* Section 3 read backwards: expand to the dense masked R x K fp16 matrix (+0 outside the
 * structure), lda >= K.  Reads the KERNEL's packed copies, so it also checks the packing.
 * Needs V in {32, 64, 96, 128} (else VENOM_ERR_UNSUPPORTED).  Asynchronous on `stream`. */
venom_status_t venom_decompress(const venom_handle_t* h, void* A_f16_dev, int64_t lda, void* stream);

/* Section 4 (stages 1-3 of the kernel design; figure 4 for the mapping onto the 2:4 matrix
 * instruction): C = A . B.
 *   B_f16_dev   K x C_cols fp16, ldb >= C_cols
 *   C_dev       R x C_cols, fp16 (c_dtype 0, rounded once from the fp32 accumulator, nearest-even)
 *               or fp32 (c_dtype 1), ldc >= C_cols; must not overlap B
 * B, C and both leading dimensions must be 16-byte aligned; V in {32, 64, 96, 128}; C_cols % 8 == 0;
 * K < 2^24, ldb < 2^23 and K * ldb < 2^31 (32-bit gather offsets).
 * Asynchronous on `stream`, allocates nothing, bitwise repeatable (no atomics, no split K). */
venom_status_t venom_spmm(const venom_handle_t* h, const void* B_f16_dev, int64_t ldb, int64_t C_cols,
                          void* C_dev, int64_t ldc, int c_dtype, void* stream);

/* Section 4, the template parameters of the kernel (thread-block tile with BS_r = V, pipeline
 * depth): the same product with an explicit kernel variant, for tuning sweeps.
 * variant < 0 selects automatically as venom_spmm does; an unknown or unsuitable variant returns
 * VENOM_ERR_UNSUPPORTED.  venom_spmm_variant_count() variants exist, numbered from 0. */
venom_status_t venom_spmm_variant(const venom_handle_t* h, const void* B_f16_dev, int64_t ldb, int64_t C_cols,
                                  void* C_dev, int64_t ldc, int c_dtype, int variant, void* stream);
/* The product with the layer's epilogue fused into the output stage (the paper's library call
 * takes the bias of the linear layer it replaces: section 7.2, the spmm(values, columns,
 * metadata, input, bias) call): C = act(A . B + bias), bias one fp16 entry per ROW of C (row =
 * output feature), added in fp32 before the single rounding; NULL = no bias.  `activation` is a
 * venom_activation_t: GELU by its definition x * Phi(x), or its tanh form.  bias must be 8-byte
 * aligned.  Everything else as venom_spmm_variant (variant < 0 = automatic). */
typedef enum { VENOM_ACT_NONE = 0, VENOM_ACT_GELU = 1, VENOM_ACT_GELU_TANH = 2 } venom_activation_t;
venom_status_t venom_spmm_bias_act(const venom_handle_t* h, const void* B_f16_dev, int64_t ldb, int64_t C_cols,
                                   const void* bias_f16_dev, int activation, void* C_dev, int64_t ldc, int c_dtype,
                                   int variant, void* stream);
/* The sparse layer as a linear layer sees it (section 7.2: the V:N:M weight replaces the weight of
 * a linear layer): activations token-major, X = tokens x K fp16 (ldx >= K), output token-major,
 * Y = tokens x R (ldy >= R), fp16 (y_dtype 0) or fp32 (1):
 *     Y = act(X . A^T + bias),  bias one fp16 entry per output feature (R), or NULL.
 * The gather needs rows of X^T, so X is first transposed into `scratch_dev` (caller-owned device
 * memory, 16-byte aligned, at least venom_linear_scratch_bytes() bytes, overwritten); the product
 * kernel then writes Y transposed itself, no second transpose pass.  tokens % 8 == 0; Y and ldy
 * aligned to 4 elements (fp16 output is fastest with Y and ldy * 2 bytes 16-byte aligned: whole
 * 128-byte lines per token are then stored); V in {32, 64, 96, 128}.  Asynchronous on `stream`,
 * allocates nothing. */
venom_status_t venom_linear_scratch_bytes(const venom_handle_t* h, int64_t tokens, size_t* bytes);
venom_status_t venom_linear(const venom_handle_t* h, const void* X_f16_dev, int64_t ldx, int64_t tokens,
                            const void* bias_f16_dev, int activation, void* Y_dev, int64_t ldy, int y_dtype,
                            void* scratch_dev, size_t scratch_bytes, void* stream);
/* venom_linear for callers that cannot allocate device memory (code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc): the transposed activations go into an array
 * the library itself holds on every GPU it runs on (venom_linear_static_max_bytes() = 64 MiB per
 * GPU, for the life of the process) instead of caller-owned scratch.  Needs K * tokens * 2 bytes
 * <= that size, else VENOM_ERR_WORKSPACE; every other argument, restriction and status as
 * venom_linear.  Calls no allocating routine.  All calls on one GPU share the one array: calls
 * that overlap in time on the same GPU (different streams or threads) race on it; the array is
 * fully rewritten by each call before it is read, so nothing needs clearing between calls. */
size_t venom_linear_static_max_bytes(void);
venom_status_t venom_linear_static(const venom_handle_t* h, const void* X_f16_dev, int64_t ldx, int64_t tokens,
                                   const void* bias_f16_dev, int activation, void* Y_dev, int64_t ldy, int y_dtype,
                                   void* stream);
int venom_spmm_variant_count(void);
/* Name of a variant ("v128_c512", ...) or NULL. */
const char* venom_spmm_variant_name(int variant);

/* Section 5, the energy metric: sum of the kept L1 mass over the sum of the total L1 mass, from
 * the per-block-row masses venom_prune wrote (exact integers, summed exactly on the host, divided
 * once).  `energy` is a HOST pointer; 1.0 when the total mass is zero.  Synchronises `stream`. */
venom_status_t venom_energy(const uint64_t* kept_mass_dev, const uint64_t* total_mass_dev, int64_t block_rows,
                            double* energy, void* stream);

/* Measurement aid (section 7 reports throughput against the hardware's matrix-instruction peak):
 * launches a register-only loop of the 2:4 matrix instruction, 2 workgroups x 8 waves per compute
 * unit, every wave issuing iterations x 8 instructions of 32768 useful FLOP each on pseudo-random
 * operands.  The caller times it: the rate it finds is the instruction peak at the clock the GPU
 * holds under that load.  sink_dev: 4 bytes of device memory (practically never written). */
venom_status_t venom_probe_smfmac_rate(int iterations, void* sink_dev, void* stream);

/* The shape a handle was built for (section 3: R x K in V:N:M); any output may be NULL. */
venom_status_t venom_get_info(const venom_handle_t* h, int64_t* R, int64_t* K, int* V, int* N, int* M);
void venom_destroy(venom_handle_t* h);
const char* venom_status_string(venom_status_t s);

#ifdef __cplusplus
}
#endif
#endif /* VENOM_H_ */
