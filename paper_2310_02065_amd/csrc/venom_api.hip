// The C ABI: argument validation, workspace carving, handle lifetime.  All device work is in
// venom_format.hip / venom_spmm.hip; nothing here allocates device memory.
#include <mutex>
#include <new>

#include "venom_internal.h"

using venom::Layout;

// Scratch of venom_linear_static: the transposed activations of one call, held inside the library
// for callers that cannot allocate.  One copy per GPU, loaded with the code object and kept until
// the process ends.  In host code this name only stands for the symbol: the memory is reached
// through the per-device address that hipGetSymbolAddress returns.
constexpr size_t kStaticScratchBytes = (size_t)64 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {

// Device address of `scratch` on the current device, looked up once per device (each GPU holds its
// own copy at its own address); null if the lookup fails.
void* static_scratch_of_current_device() {
  constexpr int kMaxDev = 64;
  static std::mutex mu;
  static void* addr[kMaxDev] = {};
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDev) return nullptr;
  std::lock_guard<std::mutex> lock(mu);
  if (!addr[dev]) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess) return nullptr;
    addr[dev] = p;
  }
  return addr[dev];
}

bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

venom_status_t check_shape(int64_t R, int64_t K, int V, int N, int M) {
  if (R < 0 || K < 0) return VENOM_ERR_INVALID_ARG;
  if (N != 2) return VENOM_ERR_UNSUPPORTED;
  if (V < 1 || M < venom::kSelCols) return VENOM_ERR_SHAPE;
  if (R % V != 0 || K % M != 0) return VENOM_ERR_SHAPE;
  if (M > 1024 || V >= (1 << 23)) return VENOM_ERR_UNSUPPORTED;
  if (K >= ((int64_t)1 << 31)) return VENOM_ERR_UNSUPPORTED;  // gathered row ids are 32-bit
  // block rows ride on the y dimension of the compression grid; the element-wise format kernels
  // number their threads with 32-bit block ids
  if (R / V > 65535 || R > ((int64_t)1 << 38) / (K > 0 ? K : 1)) return VENOM_ERR_UNSUPPORTED;
  return VENOM_OK;
}

venom_status_t make_handle(int64_t R, int64_t K, int V, int N, int M, void* ws, size_t ws_bytes,
                           venom_handle_t** out) {
  const Layout L = venom::make_layout(R, K, V, M);
  if (ws == nullptr || !aligned(ws, 256) || ws_bytes < L.total) return VENOM_ERR_WORKSPACE;
  venom_handle_t* h = new (std::nothrow) venom_handle_t;
  if (!h) return VENOM_ERR_INVALID_ARG;
  h->R = R; h->K = K; h->V = V; h->N = N; h->M = M;
  h->lay = L;
  h->ws = static_cast<char*>(ws);
  *out = h;
  return VENOM_OK;
}

}  // namespace

extern "C" {

venom_status_t venom_workspace_bytes(int64_t R, int64_t K, int V, int N, int M, size_t* bytes) {
  if (!bytes) return VENOM_ERR_INVALID_ARG;
  *bytes = 0;
  venom_status_t s = check_shape(R, K, V, N, M);
  if (s != VENOM_OK) return s;
  *bytes = venom::make_layout(R, K, V, M).total;
  return VENOM_OK;
}

venom_status_t venom_prune(const void* A_f16_dev, int64_t lda, int64_t R, int64_t K, int V, int N, int M,
                           uint8_t* mask_dev, int64_t ldm, uint64_t* kept_mass_dev, uint64_t* total_mass_dev,
                           void* stream) {
  venom_status_t s = check_shape(R, K, V, N, M);
  if (s != VENOM_OK) return s;
  if ((R > 0 && K > 0) && (!A_f16_dev || !mask_dev)) return VENOM_ERR_INVALID_ARG;
  if (lda < K || ldm < K) return VENOM_ERR_SHAPE;
  if (!aligned(A_f16_dev, 2) || !aligned(kept_mass_dev, 8) || !aligned(total_mass_dev, 8)) return VENOM_ERR_UNSUPPORTED;
  static_assert(sizeof(unsigned long long) == sizeof(uint64_t), "64-bit masses");
  const hipError_t e = venom::launch_prune(static_cast<const uint16_t*>(A_f16_dev), lda, R, K, V, M, mask_dev, ldm,
                                           reinterpret_cast<unsigned long long*>(kept_mass_dev),
                                           reinterpret_cast<unsigned long long*>(total_mass_dev),
                                           static_cast<hipStream_t>(stream));
  return e == hipSuccess ? VENOM_OK : VENOM_ERR_HIP;
}

venom_status_t venom_compress(const void* A_f16_dev, int64_t lda, const uint8_t* mask_dev, int64_t ldm, int64_t R,
                              int64_t K, int V, int N, int M, void* workspace_dev, size_t workspace_bytes,
                              void* stream, venom_handle_t** out, venom_violation_t* viol) {
  if (!out) return VENOM_ERR_INVALID_ARG;
  *out = nullptr;
  if (viol) { viol->block_row = viol->group = viol->row = -1; }
  venom_status_t s = check_shape(R, K, V, N, M);
  if (s != VENOM_OK) return s;
  if ((R > 0 && K > 0) && (!A_f16_dev || !mask_dev)) return VENOM_ERR_INVALID_ARG;
  if (lda < K || ldm < K) return VENOM_ERR_SHAPE;
  if (!aligned(A_f16_dev, 2)) return VENOM_ERR_UNSUPPORTED;
  venom_handle_t* h = nullptr;
  s = make_handle(R, K, V, N, M, workspace_dev, workspace_bytes, &h);
  if (s != VENOM_OK) return s;
  hipStream_t st = static_cast<hipStream_t>(stream);
  hipError_t e = venom::launch_compress(static_cast<const uint16_t*>(A_f16_dev), lda, mask_dev, ldm, *h, st);
  unsigned long long key = ~0ull;
  if (e == hipSuccess)
    e = hipMemcpyAsync(&key, h->ws + h->lay.off_status, sizeof(key), hipMemcpyDeviceToHost, st);
  if (e == hipSuccess) e = hipStreamSynchronize(st);
  if (e != hipSuccess) { delete h; return VENOM_ERR_HIP; }
  if (key != ~0ull) {
    const int64_t G = h->lay.G;
    const int64_t blk = (int64_t)(key >> 24);
    const bool row_rule = (key >> 23) & 1;
    if (viol) {
      viol->block_row = blk / G;
      viol->group = blk % G;
      viol->row = row_rule ? (blk / G) * V + (int64_t)(key & ((1u << 23) - 1)) : -1;
    }
    delete h;
    return row_rule ? VENOM_ERR_MASK_ROW : VENOM_ERR_MASK_COLS;
  }
  e = venom::launch_pack(*h, st);
  if (e != hipSuccess) { delete h; return VENOM_ERR_HIP; }
  *out = h;
  return VENOM_OK;
}

venom_status_t venom_import(const uint16_t* values_dev, const uint16_t* columns_dev, const uint32_t* meta_dev,
                            int64_t R, int64_t K, int V, int N, int M, void* workspace_dev, size_t workspace_bytes,
                            void* stream, venom_handle_t** out) {
  if (!out) return VENOM_ERR_INVALID_ARG;
  *out = nullptr;
  venom_status_t s = check_shape(R, K, V, N, M);
  if (s != VENOM_OK) return s;
  if ((R > 0 && K > 0) && (!values_dev || !columns_dev || !meta_dev)) return VENOM_ERR_INVALID_ARG;
  venom_handle_t* h = nullptr;
  s = make_handle(R, K, V, N, M, workspace_dev, workspace_bytes, &h);
  if (s != VENOM_OK) return s;
  const Layout& L = h->lay;
  hipStream_t st = static_cast<hipStream_t>(stream);
  hipError_t e = hipSuccess;
  if (R > 0 && K > 0) {
    e = hipMemcpyAsync(h->ws + L.off_values, values_dev, (size_t)R * L.G * 4, hipMemcpyDeviceToDevice, st);
    if (e == hipSuccess)
      e = hipMemcpyAsync(h->ws + L.off_columns, columns_dev, (size_t)L.Rb * L.G * 8, hipMemcpyDeviceToDevice, st);
    if (e == hipSuccess)
      e = hipMemcpyAsync(h->ws + L.off_meta, meta_dev, (size_t)R * L.W * 4, hipMemcpyDeviceToDevice, st);
    // the arrays come from outside: nothing is packed (or later gathered) from malformed ones
    unsigned long long word = 0;
    if (e == hipSuccess) e = venom::launch_validate(*h, st);
    if (e == hipSuccess) e = hipMemcpyAsync(&word, h->ws + L.off_status, sizeof(word), hipMemcpyDeviceToHost, st);
    if (e == hipSuccess) e = hipStreamSynchronize(st);
    if (e == hipSuccess && word != ~0ull) { delete h; return VENOM_ERR_INVALID_ARG; }
    if (e == hipSuccess) e = venom::launch_pack(*h, st);
  }
  if (e != hipSuccess) { delete h; return VENOM_ERR_HIP; }
  *out = h;
  return VENOM_OK;
}

venom_status_t venom_export(const venom_handle_t* h, uint16_t* values_dev, uint16_t* columns_dev, uint32_t* meta_dev,
                            void* stream) {
  if (!h) return VENOM_ERR_INVALID_ARG;
  const Layout& L = h->lay;
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (h->R == 0 || h->K == 0) return VENOM_OK;
  hipError_t e = hipSuccess;
  if (values_dev)
    e = hipMemcpyAsync(values_dev, h->ws + L.off_values, (size_t)h->R * L.G * 4, hipMemcpyDeviceToDevice, st);
  if (e == hipSuccess && columns_dev)
    e = hipMemcpyAsync(columns_dev, h->ws + L.off_columns, (size_t)L.Rb * L.G * 8, hipMemcpyDeviceToDevice, st);
  if (e == hipSuccess && meta_dev)
    e = hipMemcpyAsync(meta_dev, h->ws + L.off_meta, (size_t)h->R * L.W * 4, hipMemcpyDeviceToDevice, st);
  return e == hipSuccess ? VENOM_OK : VENOM_ERR_HIP;
}

venom_status_t venom_decompress(const venom_handle_t* h, void* A_f16_dev, int64_t lda, void* stream) {
  if (!h) return VENOM_ERR_INVALID_ARG;
  if (h->R > 0 && h->K > 0 && !A_f16_dev) return VENOM_ERR_INVALID_ARG;
  if (lda < h->K) return VENOM_ERR_SHAPE;
  if (!h->lay.packed || !aligned(A_f16_dev, 2)) return VENOM_ERR_UNSUPPORTED;
  hipError_t e = venom::launch_decompress(*h, static_cast<uint16_t*>(A_f16_dev), lda, static_cast<hipStream_t>(stream));
  return e == hipSuccess ? VENOM_OK : VENOM_ERR_HIP;
}

venom_status_t venom_spmm_bias_act(const venom_handle_t* h, const void* B_f16_dev, int64_t ldb, int64_t C_cols,
                                   const void* bias_f16_dev, int activation, void* C_dev, int64_t ldc, int c_dtype,
                                   int variant, void* stream) {
  if (!h) return VENOM_ERR_INVALID_ARG;
  if (activation != VENOM_ACT_NONE && activation != VENOM_ACT_GELU && activation != VENOM_ACT_GELU_TANH)
    return VENOM_ERR_INVALID_ARG;
  if (bias_f16_dev && !aligned(bias_f16_dev, 8)) return VENOM_ERR_UNSUPPORTED;
  if (c_dtype != 0 && c_dtype != 1) return VENOM_ERR_INVALID_ARG;
  if (C_cols < 0) return VENOM_ERR_INVALID_ARG;
  if (C_cols < 1) return VENOM_ERR_SHAPE;
  if (ldb < C_cols || ldc < C_cols) return VENOM_ERR_SHAPE;
  if ((h->K > 0 && !B_f16_dev) || (h->R > 0 && !C_dev)) return VENOM_ERR_INVALID_ARG;
  if (!h->lay.packed || C_cols % 8 != 0) return VENOM_ERR_UNSUPPORTED;
  const size_t esz = c_dtype == 1 ? 4 : 2;
  if (!aligned(B_f16_dev, 16) || !aligned(C_dev, 16) || (ldb * 2) % 16 != 0 || (ldc * esz) % 16 != 0)
    return VENOM_ERR_UNSUPPORTED;
  return venom::launch_spmm(*h, B_f16_dev, ldb, C_cols, bias_f16_dev, activation, C_dev, ldc, c_dtype, 0, variant,
                            static_cast<hipStream_t>(stream));
}

venom_status_t venom_linear_scratch_bytes(const venom_handle_t* h, int64_t tokens, size_t* bytes) {
  if (!h || !bytes || tokens < 0) return VENOM_ERR_INVALID_ARG;
  *bytes = (size_t)h->K * (size_t)((tokens + 7) / 8 * 8) * 2;
  return VENOM_OK;
}

venom_status_t venom_linear(const venom_handle_t* h, const void* X_f16_dev, int64_t ldx, int64_t tokens,
                            const void* bias_f16_dev, int activation, void* Y_dev, int64_t ldy, int y_dtype,
                            void* scratch_dev, size_t scratch_bytes, void* stream) {
  if (!h) return VENOM_ERR_INVALID_ARG;
  if (y_dtype != 0 && y_dtype != 1) return VENOM_ERR_INVALID_ARG;
  if (activation != VENOM_ACT_NONE && activation != VENOM_ACT_GELU && activation != VENOM_ACT_GELU_TANH)
    return VENOM_ERR_INVALID_ARG;
  if (tokens < 0) return VENOM_ERR_INVALID_ARG;
  if (tokens < 1) return VENOM_ERR_SHAPE;
  if (ldx < h->K || ldy < h->R) return VENOM_ERR_SHAPE;
  if ((h->K > 0 && !X_f16_dev) || (h->R > 0 && !Y_dev)) return VENOM_ERR_INVALID_ARG;
  if (!h->lay.packed || tokens % 8 != 0) return VENOM_ERR_UNSUPPORTED;
  if (tokens > 65535 * 64) return VENOM_ERR_UNSUPPORTED;   // token tiles ride on the transpose grid's y dimension
  const size_t esz = y_dtype == 1 ? 4 : 2;
  // a lane stores runs of 4 consecutive features: 8 bytes (fp16) or 16 bytes (fp32)
  if (!aligned(X_f16_dev, 2) || !aligned(Y_dev, 4 * esz) || (ldy * esz) % (4 * esz) != 0) return VENOM_ERR_UNSUPPORTED;
  if (bias_f16_dev && !aligned(bias_f16_dev, 8)) return VENOM_ERR_UNSUPPORTED;
  size_t need = 0;
  venom_linear_scratch_bytes(h, tokens, &need);
  if (!scratch_dev || !aligned(scratch_dev, 16) || scratch_bytes < need) return VENOM_ERR_WORKSPACE;
  hipStream_t st = static_cast<hipStream_t>(stream);
  const int64_t ldbt = (tokens + 7) / 8 * 8;
  if (venom::launch_transpose_tokens(static_cast<const uint16_t*>(X_f16_dev), ldx, tokens, h->K,
                                     static_cast<uint16_t*>(scratch_dev), ldbt, st) != hipSuccess)
    return VENOM_ERR_HIP;
  return venom::launch_spmm(*h, scratch_dev, ldbt, tokens, bias_f16_dev, activation, Y_dev, ldy, y_dtype, 1, -1, st);
}

size_t venom_linear_static_max_bytes(void) { return kStaticScratchBytes; }

venom_status_t venom_linear_static(const venom_handle_t* h, const void* X_f16_dev, int64_t ldx, int64_t tokens,
                                   const void* bias_f16_dev, int activation, void* Y_dev, int64_t ldy, int y_dtype,
                                   void* stream) {
  if (!h || tokens < 0) return VENOM_ERR_INVALID_ARG;
  size_t need = 0;
  venom_linear_scratch_bytes(h, tokens, &need);
  if (need > kStaticScratchBytes) return VENOM_ERR_WORKSPACE;   // K * tokens * 2 bytes beyond the array
  void* ptr = static_scratch_of_current_device();
  if (!ptr) return VENOM_ERR_HIP;
  return venom_linear(h, X_f16_dev, ldx, tokens, bias_f16_dev, activation, Y_dev, ldy, y_dtype, ptr,
                      kStaticScratchBytes, stream);
}

venom_status_t venom_spmm_variant(const venom_handle_t* h, const void* B_f16_dev, int64_t ldb, int64_t C_cols,
                                  void* C_dev, int64_t ldc, int c_dtype, int variant, void* stream) {
  return venom_spmm_bias_act(h, B_f16_dev, ldb, C_cols, nullptr, VENOM_ACT_NONE, C_dev, ldc, c_dtype, variant, stream);
}

venom_status_t venom_spmm(const venom_handle_t* h, const void* B_f16_dev, int64_t ldb, int64_t C_cols, void* C_dev,
                          int64_t ldc, int c_dtype, void* stream) {
  return venom_spmm_variant(h, B_f16_dev, ldb, C_cols, C_dev, ldc, c_dtype, -1, stream);
}

venom_status_t venom_energy(const uint64_t* kept_mass_dev, const uint64_t* total_mass_dev, int64_t block_rows,
                            double* energy, void* stream) {
  if (!energy || block_rows < 0 || (block_rows > 0 && (!kept_mass_dev || !total_mass_dev))) return VENOM_ERR_INVALID_ARG;
  *energy = 1.0;
  if (block_rows == 0) return VENOM_OK;
  uint64_t* host = new (std::nothrow) uint64_t[2 * (size_t)block_rows];
  if (!host) return VENOM_ERR_INVALID_ARG;
  hipStream_t st = static_cast<hipStream_t>(stream);
  hipError_t e = hipMemcpyAsync(host, kept_mass_dev, (size_t)block_rows * 8, hipMemcpyDeviceToHost, st);
  if (e == hipSuccess)
    e = hipMemcpyAsync(host + block_rows, total_mass_dev, (size_t)block_rows * 8, hipMemcpyDeviceToHost, st);
  if (e == hipSuccess) e = hipStreamSynchronize(st);
  if (e == hipSuccess) {
    // the masses are exact integers: sum them exactly (128 bits), divide once
    unsigned __int128 kept = 0, total = 0;
    for (int64_t b = 0; b < block_rows; ++b) { kept += host[b]; total += host[block_rows + b]; }
    if (total != 0) *energy = (double)((long double)kept / (long double)total);
  }
  delete[] host;
  return e == hipSuccess ? VENOM_OK : VENOM_ERR_HIP;
}

venom_status_t venom_probe_smfmac_rate(int iterations, void* sink_dev, void* stream) {
  if (iterations < 1 || !sink_dev) return VENOM_ERR_INVALID_ARG;
  return venom::launch_smfmac_probe(iterations, static_cast<float*>(sink_dev), static_cast<hipStream_t>(stream)) == hipSuccess
             ? VENOM_OK : VENOM_ERR_HIP;
}

int venom_spmm_variant_count(void) { return venom::spmm_variant_count(); }
const char* venom_spmm_variant_name(int variant) { return venom::spmm_variant_name(variant); }

venom_status_t venom_get_info(const venom_handle_t* h, int64_t* R, int64_t* K, int* V, int* N, int* M) {
  if (!h) return VENOM_ERR_INVALID_ARG;
  if (R) *R = h->R;
  if (K) *K = h->K;
  if (V) *V = h->V;
  if (N) *N = h->N;
  if (M) *M = h->M;
  return VENOM_OK;
}

void venom_destroy(venom_handle_t* h) { delete h; }

const char* venom_status_string(venom_status_t s) {
  switch (s) {
    case VENOM_OK: return "ok";
    case VENOM_ERR_INVALID_ARG: return "invalid argument";
    case VENOM_ERR_SHAPE: return "shape not V:N:M-tileable or leading dimension too small";
    case VENOM_ERR_UNSUPPORTED: return "unsupported configuration or alignment";
    case VENOM_ERR_MASK_COLS: return "illegal mask: a V x M block uses more than 4 columns";
    case VENOM_ERR_MASK_ROW: return "illegal mask: a row keeps more than 2 entries in a group of M";
    case VENOM_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case VENOM_ERR_HIP: return "HIP runtime error";
  }
  return "unknown status";
}

}  // extern "C"
