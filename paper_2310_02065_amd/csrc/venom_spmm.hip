// The product kernel: C = A . B with A in V:N:M form (paper section 4: stage 1 loads column-loc,
// the gathered rows of B and the A tile; stage 2 runs the 2:4 matrix instruction; stage 3 stores
// the output through on-chip memory).  Written for gfx950:
//   * the 2:4 inner pattern maps onto v_smfmac_f32_32x32x32_f16: A operand = 8 kept halfs per lane
//     (row = lane%32, four groups), 16 index bits per lane (= four canonical nibbles), B operand =
//     16 halfs per lane (column = lane%32, four groups x the 4 selected rows);
//   * one workgroup of NW waves owns a V x (64*NW) block of C (BS_r = V as in the paper, so every
//     gathered row of B serves all V rows); wave w owns the 64-column strip w; a k-step is 8 groups
//     = 32 gathered rows of B;
//   * EVERYTHING a k-step needs travels global -> LDS by direct-to-LDS loads through one multi-stage
//     ring: the 32 gathered rows of B (XOR-swizzled per row so the transposing LDS reads
//     ds_read_b64_tr_b16 that build the B operand spread over the banks), the packed values and
//     index words of the block row, and the row ids of the k-step that will be issued STAGES-1
//     steps later (so the gather addresses never wait on a dependent global load);
//   * the loads are issued from inline assembly and retired with exact `s_waitcnt vmcnt(n)` counts,
//     so STAGES-1 k-steps stay in flight while one is being multiplied;
//   * the block index is remapped so that each XCD (one L2 each) walks a contiguous range of the
//     column-tile-major work list and keeps its slab of B hot.
#include <cstdlib>
#include <type_traits>

#include "venom_internal.h"

namespace venom {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half16 __attribute__((ext_vector_type(16)));
typedef _Float16 half4 __attribute__((ext_vector_type(4)));
typedef short short4v __attribute__((ext_vector_type(4)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

#define LDS_PTR(T) T __attribute__((address_space(3)))*

struct SpmmParams {
  const char* arec;        // packed A stream, one record per (block row, k-step)
  const int32_t* rowidx;   // absolute B row of every gathered row, [block row][k-step][32]
  const char* B;           // fp16, row-major
  void* C;
  int64_t ldb_bytes, ldc, Ccols, rec_bytes;
  int steps;
  int nbr, nct;            // block rows, column tiles
  int per_xcd;             // ceil(nbr*nct / 8)
#ifdef VENOM_ABLATE
  int ablate;              // experiment switches (never compiled into the product library)
#endif
};

constexpr int kNumXcd = 8;

// ---- direct-to-LDS loads and their retirement, outside the compiler's wait-count bookkeeping.
// LDS destination of lane l is lds_addr + l*16 (resp. l*4); M0 carries lds_addr and needs one
// wait state before the load reads it.
__device__ __forceinline__ void dma16(const void* gptr, uint32_t lds_addr) {
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(gptr), "s"(lds_addr) : "memory");
}
__device__ __forceinline__ void dma4(const void* gptr, uint32_t lds_addr) {
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dword %0, off" ::"v"(gptr), "s"(lds_addr) : "memory");
}
// wait until at most N of this wave's loads are outstanding, then meet the other waves
template <int N>
__device__ __forceinline__ void wait_loads_and_barrier() {
  asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" ::"n"(N) : "memory");
}
template <int CNT>
__device__ __forceinline__ void wait_steps_and_barrier(int steps_in_flight) {
  static_assert(2 * CNT <= 63, "vmcnt is a 6-bit counter");
  if (steps_in_flight == 0) wait_loads_and_barrier<0>();
  else if (steps_in_flight == 1) wait_loads_and_barrier<CNT>();
  else wait_loads_and_barrier<2 * CNT>();
}

// 16-byte slot swizzle of gathered row rho inside its LDS row
__device__ __forceinline__ int slot_swizzle(int rho) { return 4 * (rho & 3); }

template <int VT, int NW, int STAGES, bool OUT_F32>
__global__ void __launch_bounds__(NW * 64, 2) spmm_kernel(SpmmParams p) {
  static_assert(NW == 2 || NW == 4 || NW == 8, "waves per workgroup");
  static_assert(STAGES >= 2 && STAGES <= 4, "ring depth");
  constexpr int BSC = 64 * NW;                     // columns of C per workgroup
  constexpr int ROW_BYTES = 2 * BSC;               // one gathered row of B in LDS
  constexpr int RPI = 1024 / ROW_BYTES;            // rows written by one wave-wide 16-byte load
  constexpr int LPR = 64 / RPI;                    // lanes (= 16-byte slots) per row
  constexpr int IPW = 4;                           // B loads per wave per k-step (32 rows / RPI / NW)
  constexpr int B_BYTES = kStepRows * ROW_BYTES;
  constexpr int A_OFF = B_BYTES;                   // packed values, VT tiles x 1 KB
  constexpr int I_OFF = A_OFF + VT * kTileValBytes;  // index words, VT tiles x 256 B
  constexpr int R_OFF = I_OFF + VT * kTileIdxBytes;  // row ids of the step issued P steps later (64 words)
  constexpr int STAGE_BYTES = R_OFF + 256;
  constexpr int P = STAGES - 1;                    // k-steps in flight ahead of the one being multiplied
  constexpr int NJOBS = 2 * VT + 1;                // A-side loads per k-step: VT values, VT index, 1 row ids
  constexpr int JH = (NJOBS + NW - 1) / NW, JL = NJOBS / NW, NHI = NJOBS % NW;
  constexpr int CROW = 64 + 8;                     // halfs per staged output row (padded)
  static_assert(STAGE_BYTES % 256 == 0, "stage alignment");

  extern __shared__ __attribute__((aligned(1024))) char smem[];
  const uint32_t lds0 = (uint32_t)(uintptr_t)(LDS_PTR(char))smem;

  // ---- which block of C: consecutive workgroup ids land on different XCDs; give each XCD a
  // contiguous range of the column-tile-major work list.
  const int xcd = blockIdx.x % kNumXcd;
  const int work = xcd * p.per_xcd + blockIdx.x / kNumXcd;
  if (work >= p.nbr * p.nct) return;
  const int ct = work / p.nbr, br = work % p.nbr;

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);

  // ---- stage 1 addressing.  B load q of this wave covers rows (wave*4+q)*RPI .. +RPI-1 of the
  // k-step; lane l writes 16-byte slot l%LPR of row (l/LPR) and fetches the XOR-swizzled chunk.
  int ld_rho[IPW];
  const char* ld_src[IPW];
#pragma unroll
  for (int q = 0; q < IPW; ++q) {
    const int rho = (wave * IPW + q) * RPI + lane / LPR;
    const int chunk = (lane % LPR) ^ slot_swizzle(rho);
    int64_t col = (int64_t)ct * BSC + chunk * 8;
    if (col + 8 > p.Ccols) col = p.Ccols - 8;      // past the edge: any in-bounds data, never stored
    ld_rho[q] = rho;
    ld_src[q] = p.B + col * 2;
  }
#ifdef VENOM_ABLATE
  const int abr = (p.ablate & 1) ? (br % 4) : br;            // A stream of only 4 block rows (L2 resident)
  const int rbr = (p.ablate & 2) ? (br % 4) : br;            // row ids of only 4 block rows
  const int32_t* ridx = p.rowidx + (int64_t)rbr * p.steps * kStepRows;
  const char* arec = p.arec + (int64_t)abr * p.steps * p.rec_bytes;
#else
  const int32_t* ridx = p.rowidx + (int64_t)br * p.steps * kStepRows;
  const char* arec = p.arec + (int64_t)br * p.steps * p.rec_bytes;
#endif

  auto issue = [&](int u, const int (&rid)[IPW]) {
#ifdef VENOM_ABLATE
    if (p.ablate & 8) return;                                 // no loads at all
#endif
    const uint32_t sb = lds0 + (u % STAGES) * STAGE_BYTES;
#pragma unroll
    for (int q = 0; q < IPW; ++q)
      dma16(ld_src[q] + (int64_t)rid[q] * p.ldb_bytes, sb + (wave * IPW + q) * 1024);
    const char* rec = arec + (int64_t)u * p.rec_bytes;
#pragma unroll
    for (int jj = 0; jj < JH; ++jj) {
      const int j = wave + jj * NW;
      if (j < VT) dma16(rec + j * kTileValBytes + lane * 16, sb + A_OFF + j * kTileValBytes);
      else if (j < 2 * VT) dma4(rec + VT * kTileValBytes + (j - VT) * kTileIdxBytes + lane * 4, sb + I_OFF + (j - VT) * kTileIdxBytes);
      else if (j == 2 * VT) dma4(ridx + (int64_t)(u + P) * kStepRows + lane, sb + R_OFF);
    }
  };

  // ---- stage 2 addressing: transposing LDS reads that build the B operand.
  // Sub-read cb of a 32-column tile: lane block blk = lane/16 reads group t = 4*(cb/2) + 2*(blk/2) + cb%2,
  // 16-column window 2*tile + blk%2; inside the block lane i reads row 4*t + i/4, 8-byte piece i%4.
  int rd_off[2][4];
  {
    const int blk = lane >> 4, i = lane & 15, e = i >> 2, c8 = i & 3;
#pragma unroll
    for (int tc = 0; tc < 2; ++tc)
#pragma unroll
      for (int cb = 0; cb < 4; ++cb) {
        const int t = 4 * (cb >> 1) + 2 * (blk >> 1) + (cb & 1);
        const int rho = 4 * t + e;
        const int win = wave * 4 + tc * 2 + (blk & 1);
        const int slot = (2 * win + (c8 >> 1)) ^ slot_swizzle(rho);
        rd_off[tc][cb] = rho * ROW_BYTES + slot * 16 + (c8 & 1) * 8;
      }
  }

  floatx16 acc[VT][2];
#pragma unroll
  for (int tr = 0; tr < VT; ++tr)
#pragma unroll
    for (int tc = 0; tc < 2; ++tc)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[tr][tc][v] = 0.f;

  auto compute = [&](int stage) {
    const char* sb = smem + stage * STAGE_BYTES;
    half16 bf[2];
#pragma unroll
    for (int tc = 0; tc < 2; ++tc)
#pragma unroll
      for (int cb = 0; cb < 4; ++cb) {
        const short4v piece = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_PTR(short4v))(sb + rd_off[tc][cb]));
        const half4 ph = __builtin_bit_cast(half4, piece);
        bf[tc][4 * cb + 0] = ph[0]; bf[tc][4 * cb + 1] = ph[1]; bf[tc][4 * cb + 2] = ph[2]; bf[tc][4 * cb + 3] = ph[3];
      }
#pragma unroll
    for (int tr = 0; tr < VT; ++tr) {
      const half8 av = *reinterpret_cast<const half8*>(sb + A_OFF + tr * kTileValBytes + lane * 16);
      const int ix = *reinterpret_cast<const int*>(sb + I_OFF + tr * kTileIdxBytes + lane * 4);
#pragma unroll
      for (int tc = 0; tc < 2; ++tc)
        acc[tr][tc] = __builtin_amdgcn_smfmac_f32_32x32x32_f16(av, bf[tc], acc[tr][tc], ix, 0, 0);
    }
  };

  // ---- prologue: fill the ring with the first P k-steps (row ids straight from global memory)
#pragma unroll
  for (int j = 0; j < P; ++j) {
    if (j < p.steps) {
      int rid[IPW];
#pragma unroll
      for (int q = 0; q < IPW; ++q) rid[q] = ridx[j * kStepRows + ld_rho[q]];
      issue(j, rid);
    }
  }

  // ---- main loop: one barrier per k-step
  for (int s = 0; s < p.steps; ++s) {
    const int left = p.steps - 1 - s;
    const int in_flight = left < P - 1 ? left : P - 1;   // later k-steps already issued
    if (NHI != 0 && wave < NHI) wait_steps_and_barrier<IPW + JH>(in_flight);
    else wait_steps_and_barrier<IPW + JL>(in_flight);
    // every wave's part of step s has landed, and every wave is done with step s-1
    const int stage = s % STAGES;
    if (s + P < p.steps) {
      int rid[IPW];
#pragma unroll
      for (int q = 0; q < IPW; ++q)
        rid[q] = *reinterpret_cast<const int*>(smem + stage * STAGE_BYTES + R_OFF + ld_rho[q] * 4);
      issue(s + P, rid);
    }
#ifdef VENOM_ABLATE
    if (!(p.ablate & 4))
#endif
    compute(stage);
  }

  // ---- stage 3: registers -> (LDS) -> global.  Accumulator element v of a 32x32 tile sits at
  // row 8*(v/4) + 4*(lane/32) + v%4, column lane%32.
#ifdef VENOM_ABLATE
  if ((p.ablate & 16) && acc[0][0][0] != 12345.f) return;     // no output stage
#endif
  const int64_t row0 = (int64_t)br * VT * 32;
  const int64_t col0 = (int64_t)ct * BSC + wave * 64;
  if constexpr (OUT_F32) {
    float* Cf = reinterpret_cast<float*>(p.C);
#pragma unroll
    for (int tr = 0; tr < VT; ++tr)
#pragma unroll
      for (int tc = 0; tc < 2; ++tc) {
        const int64_t col = col0 + tc * 32 + (lane & 31);
        if (col < p.Ccols) {
#pragma unroll
          for (int v = 0; v < 16; ++v) {
            const int64_t row = row0 + tr * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
            Cf[row * p.ldc + col] = acc[tr][tc][v];
          }
        }
      }
  } else {
    wait_loads_and_barrier<0>();  // every wave is done reading the ring; reuse it
    _Float16* cl = reinterpret_cast<_Float16*>(smem) + wave * (VT * 32 * CROW);   // this wave's strip
#pragma unroll
    for (int tr = 0; tr < VT; ++tr)
#pragma unroll
      for (int tc = 0; tc < 2; ++tc) {
        const int col = tc * 32 + (lane & 31);
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int row = tr * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
          cl[row * CROW + col] = (_Float16)acc[tr][tc][v];  // one rounding, nearest-even
        }
      }
    // same wave reads its own strip back: 8 lanes x 16 B per row, 8 rows per pass
    _Float16* Ch = reinterpret_cast<_Float16*>(p.C);
    const int chunk = lane & 7, rsub = lane >> 3;
    const int64_t col = col0 + chunk * 8;
    if (col < p.Ccols) {
#pragma unroll 4
      for (int r = rsub; r < VT * 32; r += 8) {
        const uint4 val = *reinterpret_cast<const uint4*>(cl + r * CROW + chunk * 8);
        *reinterpret_cast<uint4*>(Ch + (row0 + r) * p.ldc + col) = val;
      }
    }
  }
}

// ---------------------------------------------------------------------------------------------
struct Variant {
  const char* name;
  int V;       // block height it serves
  int bsc;     // columns per workgroup
  int threads;
  int lds;     // dynamic LDS bytes
  void (*f16)(SpmmParams);
  void (*f32)(SpmmParams);
};

template <int VT, int NW, int STAGES>
constexpr int lds_bytes() {
  const int stage = kStepRows * 128 * NW + VT * (kTileValBytes + kTileIdxBytes) + 256;
  const int ring = STAGES * stage;
  const int epi = NW * VT * 32 * (64 + 8) * 2;
  return ring > epi ? ring : epi;
}

#define VARIANT(NAME, VT, NW, ST) \
  { NAME, (VT) * 32, 64 * (NW), 64 * (NW), lds_bytes<VT, NW, ST>(), spmm_kernel<VT, NW, ST, false>, spmm_kernel<VT, NW, ST, true> }

static const Variant kVariants[] = {
    VARIANT("v128_c256_s3", 4, 4, 3),
    VARIANT("v128_c512_s4", 4, 8, 4),
    VARIANT("v128_c512_s3", 4, 8, 3),
    VARIANT("v128_c256_s2", 4, 4, 2),
    VARIANT("v128_c128_s4", 4, 2, 4),
    VARIANT("v64_c256_s3", 2, 4, 3),
    VARIANT("v64_c512_s4", 2, 8, 4),
    VARIANT("v64_c128_s4", 2, 2, 4),
    VARIANT("v32_c256_s3", 1, 4, 3),
    VARIANT("v32_c128_s4", 1, 2, 4),
};
constexpr int kNumVariants = sizeof(kVariants) / sizeof(kVariants[0]);

int spmm_variant_count() { return kNumVariants; }
const char* spmm_variant_name(int v) { return (v >= 0 && v < kNumVariants) ? kVariants[v].name : nullptr; }

static int pick_variant(int V, int64_t Ccols, int64_t nbr) {
  // first listed variant for this V whose tile is not wider than C needs; else the narrowest
  int narrowest = -1;
  for (int i = 0; i < kNumVariants; ++i) {
    if (kVariants[i].V != V) continue;
    if (narrowest < 0 || kVariants[i].bsc < kVariants[narrowest].bsc) narrowest = i;
  }
  for (int i = 0; i < kNumVariants; ++i) {
    if (kVariants[i].V != V) continue;
    const int64_t nct = (Ccols + kVariants[i].bsc - 1) / kVariants[i].bsc;
    if (Ccols >= kVariants[i].bsc && nct * nbr >= 256) return i;
  }
  return narrowest;
}

venom_status_t launch_spmm(const venom_handle& h, const void* B, int64_t ldb, int64_t Ccols, void* C, int64_t ldc,
                           int c_dtype, int variant, hipStream_t st) {
  const Layout& L = h.lay;
  if (!L.packed) return VENOM_ERR_UNSUPPORTED;
  if (L.R == 0 || Ccols == 0) return VENOM_OK;
  if (variant < 0) variant = pick_variant(h.V, Ccols, L.Rb);
  if (variant < 0 || variant >= kNumVariants || kVariants[variant].V != h.V) return VENOM_ERR_UNSUPPORTED;
  const Variant& var = kVariants[variant];
  SpmmParams p{};
  p.arec = h.ws + L.off_arec;
  p.rowidx = reinterpret_cast<const int32_t*>(h.ws + L.off_rowidx);
  p.B = reinterpret_cast<const char*>(B);
  p.C = C;
  p.ldb_bytes = ldb * 2; p.ldc = ldc; p.Ccols = Ccols; p.rec_bytes = L.rec_bytes;
  p.steps = (int)L.steps;
#ifdef VENOM_ABLATE
  p.ablate = getenv("VENOM_ABLATE") ? atoi(getenv("VENOM_ABLATE")) : 0;
#endif
  const int64_t nct = (Ccols + var.bsc - 1) / var.bsc;
  const int64_t total = nct * L.Rb;
  if (total > (int64_t)1 << 30 || L.steps > (int64_t)1 << 24) return VENOM_ERR_UNSUPPORTED;
  p.nbr = (int)L.Rb; p.nct = (int)nct;
  p.per_xcd = (int)((total + kNumXcd - 1) / kNumXcd);
  const unsigned grid = (unsigned)(p.per_xcd * kNumXcd);
  auto fn = c_dtype == 1 ? var.f32 : var.f16;
  if (var.lds > 64 * 1024) {
    // opting in to more than 64 KB of dynamic LDS is a per-function attribute (set once per device)
    static bool opted_in[kNumVariants][2][16] = {};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return VENOM_ERR_HIP;
    if (dev < 0 || dev >= 16 || !opted_in[variant][c_dtype][dev]) {
      if (hipFuncSetAttribute(reinterpret_cast<const void*>(fn), hipFuncAttributeMaxDynamicSharedMemorySize,
                              var.lds) != hipSuccess)
        return VENOM_ERR_HIP;
      if (dev >= 0 && dev < 16) opted_in[variant][c_dtype][dev] = true;
    }
  }
  hipLaunchKernelGGL(fn, dim3(grid), dim3(var.threads), var.lds, st, p);
  return hipGetLastError() == hipSuccess ? VENOM_OK : VENOM_ERR_HIP;
}

}  // namespace venom
