// One-shot magnitude pruning of a dense fp16 matrix to V:N:M (paper section 3: per V x M block keep
// the four most significant columns, then per row the two most meaningful of those four) and the
// masses the energy metric of section 5 is made of.
//
// "Most significant" is read as the column's L1 mass over the V rows; ties go to the smaller
// index.  Every fp16 is an integer multiple of 2^-24, so magnitudes are handled as integers in
// that unit (Inf and NaN count as 2^40, above any finite value): the masses are exact, no
// summation order exists, and the mask is a pure function of the bits.
#include "venom_internal.h"

namespace venom {

constexpr int kPruneMaxCols = 1024;   // columns (groups x M) one workgroup looks at

__device__ __forceinline__ unsigned long long magnitude_units(uint16_t bits) {
  const unsigned e = (bits >> 10) & 31u, f = bits & 1023u;
  if (e == 0) return f;
  if (e == 31) return 1ull << 40;
  return (unsigned long long)(1024u + f) << (e - 1);
}

__global__ void zero_u64_kernel(unsigned long long* a, unsigned long long* b, int64_t n) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) {
    if (a) a[i] = 0;
    if (b) b[i] = 0;
  }
}

// Ordering key of a magnitude that fits 16 bits: |bits|, with every non-finite value mapped to
// the one key above all finite ones (same order as magnitude_units, ties included).
__device__ __forceinline__ unsigned magnitude_key(uint16_t bits) {
  const unsigned a = bits & 0x7fffu;
  return a > 0x7c00u ? 0x7c00u : a;
}

// One workgroup per (block row b, chunk of `gpw` groups): V rows x gpw*M columns.
//   phase 1: column masses into LDS (64-bit integer adds), the block's total mass.  A thread owns
//            8 neighbouring columns (one 16-byte load) and a slice of the rows, sums in registers
//            and adds once per column; columns past the last multiple of 8 and unaligned inputs
//            take the element-wise loop.
//   phase 2: one thread per group picks the 4 columns: largest mass first, smaller index on ties,
//            then sorted ascending
//   phase 3: one thread per (row, group): the 2 largest magnitudes among the 4, smaller position on
//            ties; writes the M mask bytes of its row and group, two of them 1, with the widest
//            stores the alignment allows (`mask_word`: 16, 8, 4 or 1 bytes), so the mask is written once
__global__ void __launch_bounds__(256) prune_kernel(const uint16_t* __restrict__ A, int64_t lda, int V, int M,
                                                    int64_t G, int gpw, int vec_ok, int mask_word, uint8_t* __restrict__ mask,
                                                    int64_t ldm, unsigned long long* __restrict__ kept_mass,
                                                    unsigned long long* __restrict__ total_mass) {
  __shared__ unsigned long long mass[kPruneMaxCols];
  __shared__ int sel[kPruneMaxCols / kSelCols][kSelCols];
  __shared__ unsigned long long wg_total, wg_kept;
  const int64_t chunk = blockIdx.x, b = blockIdx.y;
  const int tid = threadIdx.x;
  const int64_t g0 = chunk * gpw;
  const int ng = (int)((G - g0) < gpw ? (G - g0) : gpw);
  const int span = ng * M;

  for (int i = tid; i < span; i += blockDim.x) mass[i] = 0;
  if (tid == 0) { wg_total = 0; wg_kept = 0; }
  __syncthreads();
  unsigned long long my_total = 0;
  const int units = vec_ok ? span / 8 : 0;         // 8-column units handled with wide accesses
  if (units > 0) {
    const int slices = blockDim.x / units > 0 ? blockDim.x / units : 1;   // row slices working side by side
    for (int u0 = 0; u0 < units; u0 += blockDim.x) {                        // (more than 256 units: several sweeps)
      const int u = u0 + (slices > 1 ? tid % units : tid);
      const int slice = slices > 1 ? tid / units : 0;
      if (u < units && slice < slices) {
        unsigned long long m8[8] = {0, 0, 0, 0, 0, 0, 0, 0};
        for (int v = slice; v < V; v += slices) {
          const uint4 w = *reinterpret_cast<const uint4*>(A + (b * V + v) * lda + g0 * M + 8 * u);
          const uint32_t ws[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            m8[2 * e] += magnitude_units((uint16_t)ws[e]);
            m8[2 * e + 1] += magnitude_units((uint16_t)(ws[e] >> 16));
          }
        }
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          if (m8[e]) atomicAdd(&mass[8 * u + e], m8[e]);
          my_total += m8[e];
        }
      }
    }
  }
  const int tail0 = units * 8;                     // columns not covered above
  const int tail = span - tail0;
  for (int64_t i = tid; i < (int64_t)V * tail; i += blockDim.x) {
    const int v = (int)(i / tail), c = tail0 + (int)(i % tail);
    const unsigned long long m = magnitude_units(A[(b * V + v) * lda + g0 * M + c]);
    if (m) atomicAdd(&mass[c], m);
    my_total += m;
  }
  if (my_total) atomicAdd(&wg_total, my_total);
  __syncthreads();
  if (tid < ng) {
    const unsigned long long* mg = mass + tid * M;
    int s[kSelCols];
    for (int k = 0; k < kSelCols; ++k) {
      int best = -1;
      for (int c = 0; c < M; ++c) {
        bool taken = false;
        for (int j = 0; j < k; ++j) taken |= s[j] == c;
        if (!taken && (best < 0 || mg[c] > mg[best])) best = c;   // strict >: the smaller index wins ties
      }
      s[k] = best;
    }
    for (int i = 1; i < kSelCols; ++i)                             // ascending order
      for (int j = i; j > 0 && s[j - 1] > s[j]; --j) { const int t = s[j]; s[j] = s[j - 1]; s[j - 1] = t; }
    for (int k = 0; k < kSelCols; ++k) sel[tid][k] = s[k];
  }
  __syncthreads();
  unsigned long long my_kept = 0;
  for (int i = tid; i < V * ng; i += blockDim.x) {
    const int v = i / ng, t = i % ng;
    const int64_t base = (b * V + v) * lda + (g0 + t) * M;
    uint16_t w[kSelCols];
    unsigned key[kSelCols];
    for (int p = 0; p < kSelCols; ++p) { w[p] = A[base + sel[t][p]]; key[p] = magnitude_key(w[p]); }
    int p0 = 0;
    for (int p = 1; p < kSelCols; ++p) if (key[p] > key[p0]) p0 = p;
    int p1 = p0 == 0 ? 1 : 0;
    for (int p = 0; p < kSelCols; ++p) if (p != p0 && key[p] > key[p1]) p1 = p;
    uint8_t* mrow = mask + (b * V + v) * ldm + (g0 + t) * M;
    const int c0 = sel[t][p0], c1 = sel[t][p1];
    auto word8 = [&](int j) {   // mask bytes of columns j .. j+7
      return ((unsigned)(c0 - j) < 8u ? 1ull << (8 * (c0 - j)) : 0ull) | ((unsigned)(c1 - j) < 8u ? 1ull << (8 * (c1 - j)) : 0ull);
    };
    if (mask_word == 16) {
      for (int j = 0; j < M; j += 16) {
        const unsigned long long lo = word8(j), hi = word8(j + 8);
        *reinterpret_cast<uint4*>(mrow + j) = make_uint4((unsigned)lo, (unsigned)(lo >> 32), (unsigned)hi, (unsigned)(hi >> 32));
      }
    } else if (mask_word == 8) {
      for (int j = 0; j < M; j += 8) {
        *reinterpret_cast<unsigned long long*>(mrow + j) = word8(j);
      }
    } else if (mask_word == 4) {
      for (int j = 0; j < M; j += 4) {
        const unsigned word = ((unsigned)(c0 - j) < 4u ? 1u << (8 * (c0 - j)) : 0u) |
                              ((unsigned)(c1 - j) < 4u ? 1u << (8 * (c1 - j)) : 0u);
        *reinterpret_cast<unsigned*>(mrow + j) = word;
      }
    } else {
      for (int c = 0; c < M; ++c) mrow[c] = (c == c0 || c == c1) ? 1 : 0;
    }
    my_kept += magnitude_units(w[p0]) + magnitude_units(w[p1]);
  }
  if (my_kept) atomicAdd(&wg_kept, my_kept);
  __syncthreads();
  if (tid == 0) {
    if (total_mass && wg_total) atomicAdd(&total_mass[b], wg_total);
    if (kept_mass && wg_kept) atomicAdd(&kept_mass[b], wg_kept);
  }
}

hipError_t launch_prune(const uint16_t* A, int64_t lda, int64_t R, int64_t K, int V, int M, uint8_t* mask, int64_t ldm,
                        unsigned long long* kept_mass, unsigned long long* total_mass, hipStream_t st) {
  const int64_t Rb = R / V, G = K / M;
  if (kept_mass || total_mass)
    hipLaunchKernelGGL(zero_u64_kernel, dim3((unsigned)((Rb + 255) / 256)), dim3(256), 0, st, kept_mass, total_mass, Rb);
  if (Rb == 0 || G == 0) return hipGetLastError();
  int gpw = kPruneMaxCols / M;
  if (gpw > kStepGroups) gpw = kStepGroups;
  if (gpw < 1) gpw = 1;
  const int64_t chunks = (G + gpw - 1) / gpw;
  // wide loads need every chunk of every row of A to start on a 16-byte boundary
  const int vec_ok = ((int64_t)gpw * M) % 8 == 0 && lda % 8 == 0 && reinterpret_cast<uintptr_t>(A) % 16 == 0;
  // every (row, group) of the mask starts at row * ldm + group * M: the widest word that always divides that
  const uintptr_t ma = reinterpret_cast<uintptr_t>(mask);
  const int mask_word = (M % 16 == 0 && ldm % 16 == 0 && ma % 16 == 0) ? 16 : (M % 8 == 0 && ldm % 8 == 0 && ma % 8 == 0) ? 8
                        : (M % 4 == 0 && ldm % 4 == 0 && ma % 4 == 0) ? 4 : 1;
  hipLaunchKernelGGL(prune_kernel, dim3((unsigned)chunks, (unsigned)Rb), dim3(256), 0, st, A, lda, V, M, G, gpw, vec_ok,
                     mask_word, mask, ldm, kept_mass, total_mass);
  return hipGetLastError();
}

}  // namespace venom
