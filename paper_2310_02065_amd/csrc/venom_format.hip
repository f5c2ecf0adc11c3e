// Format kernels: dense + mask -> canonical V:N:M arrays (section 3 of the paper), canonical ->
// the product kernel's packed copies, and packed -> dense (the format read backwards).
// Pure data movement: fp16 payloads are handled as 16-bit patterns and never interpreted.
#include "venom_internal.h"

namespace venom {

Layout make_layout(int64_t R, int64_t K, int V, int M) {
  Layout L{};
  L.R = R; L.K = K; L.G = K / M; L.Rb = R / V;
  L.W = (L.G + 7) / 8;
  L.steps = (L.G + kStepGroups - 1) / kStepGroups;
  int Vp = V;                                       // block height of the packed copy
  if (M == kSelCols && R % (kMaxTiles * kTileRows) == 0) Vp = kMaxTiles * kTileRows;
  L.packed = (Vp % kTileRows) == 0 && Vp / kTileRows <= kMaxTiles;
  L.vt = L.packed ? Vp / kTileRows : 0;
  L.Rbp = L.packed ? R / Vp : 0;
  L.rec_bytes = (int64_t)L.vt * kTileValBytes + kTailBytes;
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes, 256); return o; };
  L.off_values = take((size_t)R * L.G * 2 * sizeof(uint16_t));
  L.off_columns = take((size_t)L.Rb * L.G * kSelCols * sizeof(uint16_t));
  L.off_meta = take((size_t)R * L.W * sizeof(uint32_t));
  if (L.packed) {
    L.off_arec = take((size_t)L.Rbp * L.steps * L.rec_bytes);
    L.off_rowidx = take((size_t)L.Rbp * L.steps * kStepRows * sizeof(int32_t));
  }
  L.off_status = take(8);
  L.total = off;
  return L;
}

// ---------------------------------------------------------------------------------------------
// Legality word: the smallest key wins, so the first offending block in row-major order is
// reported, the column rule before the row rule inside one block, and the first row for the
// row rule.  key = (block_linear << 24) | (kind << 23) | row_in_block.
constexpr unsigned long long kNoViolation = ~0ull;

__global__ void init_status_kernel(unsigned long long* status) { *status = kNoViolation; }

// One workgroup per (block row b, metadata word w) = V rows x 8 groups x M columns.
//   phase 1: which columns of each group are used by any row of the block (coalesced mask read)
//   phase 2: eight threads pick the 4 columns of their group: the used ones ascending, padded with
//            the smallest unused ids, sorted
//   phase 3: one thread per row: positions kept inside the 4 selected columns, padded with the
//            smallest unused positions, sorted -> nibble; values copied as bits
constexpr int kMaxM = 1024;

__global__ void __launch_bounds__(256) compress_kernel(const uint16_t* __restrict__ A, int64_t lda,
                                                       const uint8_t* __restrict__ mask, int64_t ldm, int V, int M,
                                                       int64_t G, int64_t W, int vec_ok,
                                                       uint32_t* __restrict__ values, uint16_t* __restrict__ columns,
                                                       uint32_t* __restrict__ meta, unsigned long long* status) {
  __shared__ uint8_t used[kStepGroups][kMaxM];
  __shared__ int sel[kStepGroups][kSelCols];
  __shared__ int cols_ok[kStepGroups];
  const int64_t w = blockIdx.x, b = blockIdx.y;
  const int tid = threadIdx.x;
  const int64_t g0 = w * 8;
  const int ng = (int)((G - g0) < 8 ? (G - g0) : 8);  // groups of this word that exist
  const int span = ng * M;

  for (int i = tid; i < kStepGroups * M; i += blockDim.x) used[i / M][i % M] = 0;
  __syncthreads();
  // a thread owns 8 neighbouring columns (one 8-byte mask load per row) and a slice of the rows;
  // columns past the last multiple of 8 and unaligned masks take the byte loop
  const int units = vec_ok ? span / 8 : 0;
  if (units > 0) {
    const int slices = blockDim.x / units > 0 ? blockDim.x / units : 1;
    for (int u0 = 0; u0 < units; u0 += blockDim.x) {
      const int u = u0 + (slices > 1 ? tid % units : tid);
      const int slice = slices > 1 ? tid / units : 0;
      if (u < units && slice < slices) {
        unsigned long long seen = 0;               // OR of the 8 mask bytes over this thread's rows
        for (int v = slice; v < V; v += slices)
          seen |= *reinterpret_cast<const unsigned long long*>(mask + (b * V + v) * ldm + g0 * M + 8 * u);
        for (int e = 0; e < 8; ++e)
          if ((seen >> (8 * e)) & 0xffull) { const int c = 8 * u + e; used[c / M][c % M] = 1; }
      }
    }
  }
  const int tail0 = units * 8, tail = span - tail0;
  for (int64_t i = tid; i < (int64_t)V * tail; i += blockDim.x) {
    const int v = (int)(i / tail), c = tail0 + (int)(i % tail);
    if (mask[(b * V + v) * ldm + g0 * M + c]) used[c / M][c % M] = 1;  // benign: every writer stores 1
  }
  __syncthreads();
  if (tid < ng) {
    int cnt = 0, s[kSelCols];
    for (int c = 0; c < M; ++c)
      if (used[tid][c]) { if (cnt < kSelCols) s[cnt] = c; ++cnt; }
    const bool ok = cnt <= kSelCols;
    if (!ok) atomicMin(status, ((unsigned long long)(b * G + g0 + tid) << 24));
    // pad with the smallest unused ids, keeping the list sorted
    for (int c = 0; cnt < kSelCols && c < M; ++c) {
      if (used[tid][c]) continue;
      int pos = cnt;
      while (pos > 0 && s[pos - 1] > c) { s[pos] = s[pos - 1]; --pos; }
      s[pos] = c; ++cnt;
    }
    cols_ok[tid] = ok;
    for (int p = 0; p < kSelCols; ++p) {
      sel[tid][p] = s[p];
      columns[((b * G) + g0 + tid) * kSelCols + p] = (uint16_t)s[p];
    }
  }
  __syncthreads();
  // one thread per (row, group): eight neighbouring lanes hold the eight nibbles of a metadata word
  // and combine them with three lane exchanges
  for (int i = tid; i < ((V * 8 + 255) / 256) * 256; i += blockDim.x) {
    const int v = i >> 3, t = i & 7;
    uint32_t nib = 0;
    if (v < V && t < ng) {
      const int64_t r = b * V + v;
      const int64_t base = g0 + t;
      const uint8_t* mrow = mask + r * ldm + base * M;
      int kept[kSelCols], nk = 0;
      for (int p = 0; p < kSelCols; ++p) { kept[p] = mrow[sel[t][p]] != 0; nk += kept[p]; }
      if (cols_ok[t] && nk > 2)
        atomicMin(status, ((unsigned long long)(b * G + base) << 24) | (1ull << 23) | (unsigned long long)v);
      // first two kept positions, then the smallest unused ones, sorted
      int p0 = -1, p1 = -1;
      for (int p = 0; p < kSelCols; ++p)
        if (kept[p]) { if (p0 < 0) p0 = p; else if (p1 < 0) p1 = p; }
      bool k0 = p0 >= 0, k1 = p1 >= 0;
      if (!k0) { p0 = 0; p1 = 1; }                     // nothing kept: positions (0, 1)
      else if (!k1) {                                   // one kept: add the smallest other position
        if (p0 == 0) { p1 = 1; }
        else { p1 = p0; p0 = 0; k1 = true; k0 = false; }
      }
      const uint16_t* arow = A + r * lda + base * M;
      const uint32_t v0 = k0 ? arow[sel[t][p0]] : 0u;
      const uint32_t v1 = k1 ? arow[sel[t][p1]] : 0u;
      values[r * G + base] = v0 | (v1 << 16);
      nib = (uint32_t)(p0 | (p1 << 2)) << (4 * t);
    }
    nib |= __shfl_xor(nib, 1);
    nib |= __shfl_xor(nib, 2);
    nib |= __shfl_xor(nib, 4);
    if (v < V && t == 0) meta[(b * V + v) * W + w] = nib;
  }
}

// Absolute row of B for every gathered row: [R/V][steps][32], entry 4*t + p of a step is
// (8*step + t)*M + column_loc[p]; groups past the end point at row 0 (their values are zero).
// (Vp, V: block heights of the packed copy and of the canonical arrays; they differ only at M = 4,
// where all canonical block rows hold the same column ids.)
__global__ void __launch_bounds__(256) pack_rowidx_kernel(const uint16_t* __restrict__ columns, int64_t G, int M,
                                                          int64_t steps, int64_t total, int Vp, int V,
                                                          int32_t* __restrict__ rowidx) {
  const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= total) return;
  const int rho = (int)(idx % kStepRows);
  const int64_t s = (idx / kStepRows) % steps, b = idx / kStepRows / steps;
  const int64_t g = s * 8 + rho / 4;
  const int64_t cb = b * Vp / V;                   // canonical block row that holds the packed block's first row
  rowidx[idx] = (g < G) ? (int32_t)(g * M + columns[(cb * G + g) * kSelCols + (rho % 4)]) : 0;
}

// canonical -> the kernel's packed A stream.  One record per (block row, k-step):
//   [V/32 tiles x 1024 B of values][512 B tail]
// values of a tile: 64 lanes x 8 halfs; lane = 32*h + i holds row 32*tile + i and the two kept
// values of groups 8*step + 4*h .. +3 -- the A operand of v_smfmac_f32_32x32x32_f16.
// tail: 64 lanes x 4 x uint16, entry [lane][tile] = the lane's four canonical nibbles for that tile
//       (a lane reads its 8 bytes with one LDS load; the matrix instruction picks the 16-bit field
//       with its ABID operand).
// One thread per lane-slot: (block row, step, tile, lane) for tile < vt; tile == vt clears the
// index words of the tiles that do not exist.
__global__ void __launch_bounds__(256) pack_arec_kernel(const uint32_t* __restrict__ values,
                                                        const uint32_t* __restrict__ meta, int64_t G, int64_t W,
                                                        int64_t steps, int vt, int V, int64_t total,
                                                        char* __restrict__ arec) {
  const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= total) return;
  const int lane = (int)(idx % 64);
  const int tile = (int)((idx / 64) % (vt + 1));
  const int64_t s = (idx / 64 / (vt + 1)) % steps, b = idx / 64 / (vt + 1) / steps;
  char* rec = arec + (b * steps + s) * ((int64_t)vt * kTileValBytes + kTailBytes);
  char* tail = rec + vt * kTileValBytes;
  if (tile == vt) {
    for (int t = vt; t < kMaxTiles; ++t) reinterpret_cast<uint16_t*>(tail)[lane * kMaxTiles + t] = 0;
    return;
  }
  const int64_t r = b * V + tile * kTileRows + (lane % 32);
  const int h = lane / 32;
  const int64_t g = s * 8 + 4 * h;
  uint32_t v[4];
  for (int e = 0; e < 4; ++e) v[e] = (g + e < G) ? values[r * G + g + e] : 0u;
  reinterpret_cast<uint4*>(rec + tile * kTileValBytes)[lane] = make_uint4(v[0], v[1], v[2], v[3]);
  const uint32_t word = (s < W) ? (meta[r * W + s] >> (16 * h)) & 0xffffu : 0u;
  reinterpret_cast<uint16_t*>(tail)[lane * kMaxTiles + tile] = (uint16_t)word;
}

// packed -> dense: one thread per output element.
__global__ void __launch_bounds__(256) decompress_kernel(const char* __restrict__ arec,
                                                         const int32_t* __restrict__ rowidx, int64_t R, int64_t K, int V,
                                                         int M, int64_t steps, int vt, uint16_t* __restrict__ A,
                                                         int64_t lda) {
  const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= R * K) return;
  const int64_t r = idx / K, k = idx % K;
  const int64_t g = k / M, s = g / 8, b = r / V;
  const int t = (int)(g % 8), h = t / 4, ge = t % 4;
  const int tile = (int)((r % V) / kTileRows);
  const int lane = 32 * h + (int)(r % kTileRows);
  const char* rec = arec + (b * steps + s) * ((int64_t)vt * kTileValBytes + kTailBytes);
  const uint32_t word = reinterpret_cast<const uint16_t*>(rec + vt * kTileValBytes)[lane * kMaxTiles + tile];
  const uint32_t nib = (word >> (4 * ge)) & 0xfu;
  const int32_t* ri = rowidx + (b * steps + s) * kStepRows + 4 * t;
  const uint16_t* pv = reinterpret_cast<const uint16_t*>(rec + tile * kTileValBytes) + lane * 8 + 2 * ge;
  uint16_t out = 0;
  if (ri[nib & 3] == k) out = pv[0];
  if (ri[nib >> 2] == k) out = pv[1];
  A[r * lda + k] = out;
}

// Imported canonical arrays are data from outside: one thread per (row, group) checks what the
// gather and the matrix instruction rely on -- column ids strictly increasing and below M (rows of
// the block's first row only), the two m-indices of a nibble ordered idx0 < idx1, unused nibbles of
// the last metadata word zero.  Any offence sets the flag; nothing is gathered from such arrays.
__global__ void __launch_bounds__(256) validate_kernel(const uint16_t* __restrict__ columns,
                                                       const uint32_t* __restrict__ meta, int64_t R, int64_t G,
                                                       int64_t W, int V, int M, unsigned long long* status) {
  const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= R * W * 8) return;
  const int64_t r = idx / (W * 8), g = idx % (W * 8);
  const uint32_t nib = (meta[r * W + g / 8] >> (4 * (g % 8))) & 0xfu;
  bool bad = false;
  if (g < G) {
    bad = (nib & 3u) >= (nib >> 2);
    if (r % V == 0) {
      const uint16_t* c = columns + ((r / V) * G + g) * kSelCols;
      bad = bad || !(c[0] < c[1] && c[1] < c[2] && c[2] < c[3] && c[3] < M);
    }
  } else bad = nib != 0;
  if (bad) *status = 0;
}

static inline unsigned blocks_for(int64_t total) { return (unsigned)((total + 255) / 256); }

hipError_t launch_validate(const venom_handle& h, hipStream_t st) {
  const Layout& L = h.lay;
  auto* status = reinterpret_cast<unsigned long long*>(h.ws + L.off_status);
  hipLaunchKernelGGL(init_status_kernel, dim3(1), dim3(1), 0, st, status);
  if (L.R > 0 && L.G > 0)
    hipLaunchKernelGGL(validate_kernel, dim3(blocks_for(L.R * L.W * 8)), dim3(256), 0, st,
                       reinterpret_cast<const uint16_t*>(h.ws + L.off_columns),
                       reinterpret_cast<const uint32_t*>(h.ws + L.off_meta), L.R, L.G, L.W, h.V, h.M, status);
  return hipGetLastError();
}

hipError_t launch_compress(const uint16_t* A, int64_t lda, const uint8_t* mask, int64_t ldm, const venom_handle& h,
                           hipStream_t st) {
  const Layout& L = h.lay;
  auto* status = reinterpret_cast<unsigned long long*>(h.ws + L.off_status);
  hipLaunchKernelGGL(init_status_kernel, dim3(1), dim3(1), 0, st, status);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  if (L.R > 0 && L.G > 0) {
    dim3 grid((unsigned)L.W, (unsigned)L.Rb);
    // wide mask loads need every 8-group chunk of every row to start on an 8-byte boundary
    const int vec_ok = ldm % 8 == 0 && reinterpret_cast<uintptr_t>(mask) % 8 == 0;
    hipLaunchKernelGGL(compress_kernel, grid, dim3(256), 0, st, A, lda, mask, ldm, h.V, h.M, L.G, L.W, vec_ok,
                       reinterpret_cast<uint32_t*>(h.ws + L.off_values),
                       reinterpret_cast<uint16_t*>(h.ws + L.off_columns),
                       reinterpret_cast<uint32_t*>(h.ws + L.off_meta), status);
    e = hipGetLastError();
  }
  return e;
}

hipError_t launch_pack(const venom_handle& h, hipStream_t st) {
  const Layout& L = h.lay;
  if (!L.packed || L.R == 0 || L.G == 0) return hipSuccess;
  const int Vp = L.vt * kTileRows;
  int64_t total = L.Rbp * L.steps * kStepRows;
  hipLaunchKernelGGL(pack_rowidx_kernel, dim3(blocks_for(total)), dim3(256), 0, st,
                     reinterpret_cast<const uint16_t*>(h.ws + L.off_columns), L.G, h.M, L.steps, total, Vp, h.V,
                     reinterpret_cast<int32_t*>(h.ws + L.off_rowidx));
  total = L.Rbp * L.steps * (L.vt + 1) * 64;
  hipLaunchKernelGGL(pack_arec_kernel, dim3(blocks_for(total)), dim3(256), 0, st,
                     reinterpret_cast<const uint32_t*>(h.ws + L.off_values),
                     reinterpret_cast<const uint32_t*>(h.ws + L.off_meta), L.G, L.W, L.steps, L.vt, Vp, total,
                     h.ws + L.off_arec);
  return hipGetLastError();
}

hipError_t launch_decompress(const venom_handle& h, uint16_t* A, int64_t lda, hipStream_t st) {
  const Layout& L = h.lay;
  if (L.R == 0 || L.K == 0) return hipSuccess;
  const int64_t total = L.R * L.K;
  hipLaunchKernelGGL(decompress_kernel, dim3(blocks_for(total)), dim3(256), 0, st, h.ws + L.off_arec,
                     reinterpret_cast<const int32_t*>(h.ws + L.off_rowidx), L.R, L.K, L.vt * kTileRows, h.M, L.steps, L.vt,
                     A, lda);
  return hipGetLastError();
}

}  // namespace venom
