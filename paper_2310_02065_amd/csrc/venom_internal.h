// Internal declarations shared by the library's translation units (not part of the ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "venom.h"

namespace venom {

constexpr int kSelCols = 4;    // columns kept per V x M block (section 3)
constexpr int kTileRows = 32;  // rows of one matrix-instruction tile (v_smfmac_f32_32x32x32_f16)
constexpr int kStepGroups = 8; // groups of M columns consumed per k-step: 8 groups x 4 columns = 32
constexpr int kStepRows = kStepGroups * kSelCols;  // gathered rows of B per k-step
constexpr int kTileValBytes = 1024;                // packed values of one 32-row tile for one k-step
constexpr int kMaxTiles = 4;                       // the product kernel serves V = 32, 64, 96, 128
constexpr int kTailBytes = 512;                    // record tail: the index words, 64 lanes x 4 tiles x 16 bits

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// Where each array lives inside the caller's workspace (byte offsets, all 256-byte aligned).
struct Layout {
  int64_t R, K, G, Rb, W;  // G = K/M groups per row, Rb = R/V block rows, W = ceil(G/8) meta words per row
  int64_t steps;           // k-steps = ceil(G/8)
  int vt;                  // 32-row tiles per block row of the PACKED copy (its block height / 32)
  int64_t Rbp;             // block rows of the packed copy: R / (32 * vt).  Its block height is V, except at
                           // M = 4, where every block selects all four columns, V plays no role in the arrays,
                           // and the copy is packed 128 rows high whenever R allows
  int64_t rec_bytes;       // bytes of one (block row, k-step) record of the packed A stream
  bool packed;             // the kernel's packed copies exist (block height 32, 64, 96 or 128)
  size_t off_values, off_columns, off_meta;      // canonical
  size_t off_arec, off_rowidx;                   // packed for the kernel
  size_t off_status;                             // 8-byte legality word
  size_t total;
};

Layout make_layout(int64_t R, int64_t K, int V, int M);

}  // namespace venom

struct venom_handle {
  int64_t R, K;
  int V, N, M;
  venom::Layout lay;
  char* ws;  // borrowed device pointer
};

namespace venom {

// ---- format kernels (venom_format.hip)
hipError_t launch_compress(const uint16_t* A, int64_t lda, const uint8_t* mask, int64_t ldm, const venom_handle& h,
                           hipStream_t st);
hipError_t launch_pack(const venom_handle& h, hipStream_t st);
// checks the canonical arrays in the workspace; the legality word reads ~0 afterwards iff they are well formed
hipError_t launch_validate(const venom_handle& h, hipStream_t st);
hipError_t launch_decompress(const venom_handle& h, uint16_t* A, int64_t lda, hipStream_t st);

// ---- pruning (venom_prune.hip)
hipError_t launch_prune(const uint16_t* A, int64_t lda, int64_t R, int64_t K, int V, int M, uint8_t* mask, int64_t ldm,
                        unsigned long long* kept_mass, unsigned long long* total_mass, hipStream_t st);

// ---- product kernels (venom_spmm.hip)
int spmm_variant_count();
const char* spmm_variant_name(int v);
// returns VENOM_OK / VENOM_ERR_UNSUPPORTED / VENOM_ERR_HIP
// tokens_major != 0: C is written transposed (C[column][row], leading dimension ldc counts rows of A)
venom_status_t launch_spmm(const venom_handle& h, const void* B, int64_t ldb, int64_t Ccols, const void* bias, int act,
                           void* C, int64_t ldc, int c_dtype, int tokens_major, int variant, hipStream_t st);
// register-only loop of 2:4 matrix instructions, for the measured instruction peak (grid = one workgroup of 8 waves per
// compute unit x 2)
hipError_t launch_smfmac_probe(int iters, float* sink, hipStream_t st);
hipError_t launch_transpose_tokens(const uint16_t* X, int64_t ldx, int64_t tokens, int64_t K, uint16_t* BT, int64_t ldbt,
                                   hipStream_t st);

}  // namespace venom
