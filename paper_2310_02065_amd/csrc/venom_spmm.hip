// The product kernel: C = A . B with A in V:N:M form (paper section 4: stage 1 loads column-loc,
// the gathered rows of B and the A tile; stage 2 runs the 2:4 matrix instruction; stage 3 stores
// the output through on-chip memory).  Written for gfx950:
//   * the 2:4 inner pattern maps onto v_smfmac_f32_32x32x32_f16: A operand = 8 kept halfs per lane
//     (row = lane%32, four groups), 16 index bits per lane (= four canonical nibbles), B operand =
//     16 halfs per lane (column = lane%32, four groups x the 4 selected rows);
//   * one workgroup owns a V x (64*NC) block of C (BS_r = V as in the paper, so every gathered row
//     of B serves all V rows); a k-step is 8 groups = 32 gathered rows of B;
//   * the workgroup is split by role.  NC CONSUMER waves each own a 64-column strip: they only read
//     LDS (transposing reads ds_read_b64_tr_b16 build the B operand, plain reads fetch the packed
//     values and index words) and issue matrix instructions.  PRODUCER waves only move data, by
//     direct-to-LDS loads: NPB of them gather the 32 rows of B of every k-step (XOR-swizzled per
//     row so the transposing reads spread over the banks) into a 4-stage ring, three k-steps ahead;
//     one more streams the packed A records into a deeper ring, NA-1 k-steps ahead, because that
//     stream comes from HBM while B is L2-resident.  Loads retire in order per wave, so the two
//     streams live in different waves.  The tail of each A record names the B rows of the k-step
//     three steps later, so the gather addresses are on chip before they are needed.  A producer
//     that has to queue behind the memory pipeline stalls alone; the matrix units keep running;
//   * the loads are issued from inline assembly and retired with exact `s_waitcnt vmcnt(n)` counts;
//     one s_barrier per k-step hands filled stages to the consumers and drained ones back;
//   * the block index is remapped so that each XCD (one L2 each) walks a contiguous range of the
//     column-tile-major work list and keeps its slab of B hot.
#include <cstdio>
#include <cstdlib>

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
  unsigned long long* trace;
#endif
};

#ifdef VENOM_ABLATE
// timestamps of steps 16..23 go to the last 1.5 KB of LDS (no vector-memory traffic), dumped at the end
#define TRACE(slot, step, k) do { if (p.trace && blockIdx.x == 8 && lane == 0 && (step) >= 16 && (step) < 24) \
  reinterpret_cast<unsigned*>(smem + 163840 - 1536)[(((slot) * 8 + (step) - 16) * 4 + (k))] = (unsigned)__builtin_readcyclecounter(); } while (0)
#define TRACE_DUMP() do { if (p.trace && blockIdx.x == 8) { barrier_only(); if (threadIdx.x < 384) p.trace[threadIdx.x] = reinterpret_cast<unsigned*>(smem + 163840 - 1536)[threadIdx.x]; } } while (0)
#else
#define TRACE(slot, step, k) do {} while (0)
#endif
constexpr int kNumXcd = 8;
constexpr int kStages = 4;           // B ring depth; kRidLead == kStages - 1 k-steps are in flight
static_assert(kRidLead == kStages - 1, "the record tail must name the rows of the step being issued");

// ---- direct-to-LDS loads and their retirement, outside the compiler's wait-count bookkeeping.
// LDS destination of lane l is lds_addr + l*16; M0 carries lds_addr and needs one wait state
// before the load reads it.
// The global address is a wave-uniform 64-bit base (SGPR pair) plus an unsigned 32-bit byte offset
// per lane, so address generation costs one vector instruction per load.
__device__ __forceinline__ void dma16(const char* base, uint32_t lane_off, uint32_t lds_addr) {
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(lane_off), "s"(base), "s"(lds_addr)
               : "memory");
}
// wait until at most N of this wave's loads are outstanding, then meet the other waves
// wait until at most N of this wave's loads are outstanding, then meet the other waves
// (ts, experiments only: receives the time between the wait and the barrier)
template <int N>
__device__ __forceinline__ void wait_loads_and_barrier(unsigned* ts = nullptr) {
#ifdef VENOM_ABLATE
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
  if (ts) *ts = (unsigned)__builtin_readcyclecounter();
  asm volatile("s_barrier" ::: "memory");
#else
  asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" ::"n"(N) : "memory");
#endif
}
// the same with N = k * UNIT for a run-time k in [0, MAXK]
template <int UNIT, int MAXK, int K = 0>
__device__ __forceinline__ void wait_units_and_barrier(int k, unsigned* ts = nullptr) {
  static_assert(MAXK * UNIT <= 63, "vmcnt is a 6-bit counter");
  if constexpr (K >= MAXK) {
    wait_loads_and_barrier<MAXK * UNIT>(ts);
  } else {
    if (k == K) wait_loads_and_barrier<K * UNIT>(ts);
    else wait_units_and_barrier<UNIT, MAXK, K + 1>(k, ts);
  }
}
__device__ __forceinline__ void barrier_only() { asm volatile("s_barrier" ::: "memory"); }

// 16-byte slot swizzle of gathered row rho inside its LDS row
__device__ __forceinline__ int slot_swizzle(int rho) { return 4 * (rho & 3); }

template <int ABID>
__device__ __forceinline__ floatx16 smfmac(half8 a, half16 b, floatx16 c, int idx) {
  return __builtin_amdgcn_smfmac_f32_32x32x32_f16(a, b, c, idx, 0, ABID);
}

template <int VT, int NC, int NPB, int NA, bool OUT_F32>
__global__ void __launch_bounds__((NC + NPB + 1) * 64, 3) spmm_kernel(SpmmParams p) {
  static_assert(NC == 2 || NC == 4 || NC == 8, "consumer waves per workgroup");
  static_assert(VT >= 1 && VT <= kMaxTiles, "32-row tiles per block row");
  static_assert(NA >= 4, "the A ring holds the record being read, the next one (row ids), and records in flight");
  constexpr int BSC = 64 * NC;                     // columns of C per workgroup
  constexpr int ROW_BYTES = 2 * BSC;               // one gathered row of B in LDS
  constexpr int RPI = 1024 / ROW_BYTES;            // rows written by one wave-wide 16-byte load
  constexpr int LPR = 64 / RPI;                    // lanes (= 16-byte slots) per row
  constexpr int NI = kStepRows / RPI;              // B loads per k-step (4 * NC)
  constexpr int NBH = (NI + NPB - 1) / NPB, NBL = NI / NPB, NBHI = NI % NPB;  // ... per B producer
  constexpr int B_BYTES = kStepRows * ROW_BYTES;
  constexpr int A_BYTES = VT * kTileValBytes + kTailBytes;   // one A record
  constexpr int T_OFF = VT * kTileValBytes;        // record tail: index words, row ids
  constexpr int ARING = kStages * B_BYTES;         // LDS: [B ring][A ring]
  constexpr int NJ = VT + 1;                       // A loads per k-step: VT value blocks + the tail
  constexpr int PA = NA - 1;                       // k-steps the A stream runs ahead
  constexpr int CROW = 64 + 8;                     // halfs per staged output row (padded)
  static_assert((kStages - 2) * NBH <= 63 && PA * NJ <= 63, "load counts");

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

  if (wave == NC + NPB) {
    // ========================================================================= A producer
    const char* arec = p.arec + (int64_t)br * p.steps * p.rec_bytes;
    const uint32_t lane_off = lane * 16;
    auto issue = [&](int u) {
#ifdef VENOM_ABLATE
      if (p.ablate & 8) return;
#endif
      const uint32_t dst = lds0 + ARING + (u % NA) * A_BYTES;
      const char* rec = arec + (int64_t)u * p.rec_bytes;
#pragma unroll
      for (int j = 0; j < NJ; ++j) dma16(rec + j * 1024, lane_off, dst + j * 1024);
    };
    for (int j = 0; j < PA; ++j)
      if (j < p.steps) issue(j);
    for (int s = 0; s < p.steps; ++s) {
      // records s and s+1 have landed when at most the records of the steps after s+1 are pending
      // (the B producers read the row ids in record s+1 one step early)
      const int left = p.steps - 2 - s;
      TRACE(0, s, 0);
      unsigned ts = 0;
      wait_units_and_barrier<NJ, PA - 2>(left < 0 ? 0 : (left < PA - 2 ? left : PA - 2), &ts);
#ifdef VENOM_ABLATE
      if (p.trace && blockIdx.x == 8 && lane == 0 && s >= 16 && s < 24) reinterpret_cast<unsigned*>(smem + 163840 - 1536)[((0 * 8 + s - 16) * 4 + 3)] = ts;
#endif
      TRACE(0, s, 1);
      // after the barrier everyone is done with record s-1: its slot takes record s+PA
      if (s + PA < p.steps) issue(s + PA);
      TRACE(0, s, 2);
    }
    wait_loads_and_barrier<0>();                   // the consumers' last barrier
#ifdef VENOM_ABLATE
    TRACE_DUMP();
#endif
    return;
  }
  if (wave >= NC) {
    // ========================================================================= B producers
    const int pj = wave - NC;
    // B load q of this producer is load number pj + NPB*q of the k-step; it covers rows
    // (that number)*RPI .. +RPI-1; lane l writes 16-byte slot l%LPR of row l/LPR and fetches the
    // XOR-swizzled chunk of the gathered row.
    // The row ids of a k-step sit in lane order in one register (lane l holds row l%32); the rows
    // of one load are picked out with v_readlane and the byte offset of a lane is
    // row * ldb_bytes + column offset, a 24-bit multiply-add (the host checks the ranges).
    uint32_t ld_col[NBH];
#pragma unroll
    for (int q = 0; q < NBH; ++q) {
      const int rho = ((pj + NPB * q) % NI) * RPI + lane / LPR;
      const int chunk = (lane % LPR) ^ slot_swizzle(rho);
      int64_t col = (int64_t)ct * BSC + chunk * 8;
      if (col + 8 > p.Ccols) col = p.Ccols - 8;    // past the edge: any in-bounds data, never stored
      ld_col[q] = (uint32_t)(col * 2);
    }
    const int rowsel = lane / LPR;                 // which of the RPI rows of a load this lane writes
    const uint32_t ldb24 = (uint32_t)p.ldb_bytes;
    const int32_t* ridx = p.rowidx + (int64_t)br * p.steps * kStepRows;
    const bool hi = NBHI == 0 || pj < NBHI;        // this producer has NBH loads per k-step, else NBL

    auto issue = [&](int u, int ridv) {
#ifdef VENOM_ABLATE
      if (p.ablate & 8) return;
#endif
      const uint32_t sb = lds0 + (u % kStages) * B_BYTES;
#pragma unroll
      for (int q = 0; q < NBH; ++q) {
        if (q < NBL || hi) {
          const int rho0 = ((pj + NPB * q) % NI) * RPI;
          int row = __builtin_amdgcn_readlane(ridv, rho0);
#pragma unroll
          for (int k = 1; k < RPI; ++k) {
            const int rk = __builtin_amdgcn_readlane(ridv, rho0 + k);
            row = rowsel == k ? rk : row;
          }
          dma16(p.B, __umul24((uint32_t)row, ldb24) + ld_col[q], sb + (pj + NPB * q) * 1024);
        }
      }
    };

    // prologue: the first two k-steps (row ids straight from global memory)
#pragma unroll
    for (int j = 0; j < kRidLead; ++j) {
      if (j < p.steps) issue(j, ridx[j * kStepRows + (lane & 31)]);
    }
    int ridv = 0;                                  // row ids of the k-step issued next
    for (int s = 0; s < p.steps; ++s) {
      // this producer's part of k-step s has landed when at most its loads of the later steps
      // (up to two) are pending
      const int left = p.steps - 1 - s;
      const int pend = left < kStages - 2 ? left : kStages - 2;
      TRACE(1 + pj, s, 0);
      unsigned ts = 0;
      if (hi) wait_units_and_barrier<NBH, kStages - 2>(pend, &ts);
      else wait_units_and_barrier<NBL, kStages - 2>(pend, &ts);
      TRACE(1 + pj, s, 1);
      // after the barrier: A records s and s+1 are on chip, and the consumers are done with B stage s-1
      if (s + kRidLead < p.steps) {
        if (s == 0) ridv = *reinterpret_cast<const int*>(smem + ARING + T_OFF + kTailRidOff + (lane & 31) * 4);
        TRACE(1 + pj, s, 2);
        issue(s + kRidLead, ridv);
        if (s + 1 + kRidLead < p.steps)            // row ids for the next iteration, from record s+1
          ridv = *reinterpret_cast<const int*>(smem + ARING + ((s + 1) % NA) * A_BYTES + T_OFF + kTailRidOff +
                                               (lane & 31) * 4);
      }
#ifdef VENOM_ABLATE
      if (p.trace && blockIdx.x == 8 && lane == 0 && s >= 16 && s < 24) reinterpret_cast<unsigned*>(smem + 163840 - 1536)[(((1 + pj) * 8 + s - 16) * 4 + 3)] = ts;
#endif
    }
    wait_loads_and_barrier<0>();                   // the consumers' last barrier
#ifdef VENOM_ABLATE
    TRACE_DUMP();
#endif
    return;
  }

  // ============================================================================= consumer
  // Transposing LDS reads that build the B operand.  Sub-read cb of a 32-column tile: lane block
  // blk = lane/16 reads group t = 4*(cb/2) + 2*(blk/2) + cb%2, 16-column window 2*tile + blk%2;
  // inside the block lane i reads row 4*t + i/4, 8-byte piece i%4.
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

  for (int s = 0; s < p.steps; ++s) {
    TRACE(4 + wave, s, 0);
    barrier_only();                                // stage s is complete
    TRACE(4 + wave, s, 1);
#ifdef VENOM_ABLATE
    if (p.ablate & 4) continue;
#endif
    const char* sb = smem + (s % kStages) * B_BYTES;
    const char* sa = smem + ARING + (s % NA) * A_BYTES;
    half16 bf[2];
#pragma unroll
    for (int tc = 0; tc < 2; ++tc)
#pragma unroll
      for (int cb = 0; cb < 4; ++cb) {
        const short4v piece = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_PTR(short4v))(sb + rd_off[tc][cb]));
        const half4 ph = __builtin_bit_cast(half4, piece);
        bf[tc][4 * cb + 0] = ph[0]; bf[tc][4 * cb + 1] = ph[1]; bf[tc][4 * cb + 2] = ph[2]; bf[tc][4 * cb + 3] = ph[3];
      }
    const uint2 ixw = *reinterpret_cast<const uint2*>(sa + T_OFF + lane * 8);   // 4 x 16 index bits
#pragma unroll
    for (int tr = 0; tr < VT; ++tr) {
      const half8 av = *reinterpret_cast<const half8*>(sa + tr * kTileValBytes + lane * 16);
      const int ix = (int)((tr >> 1) ? ixw.y : ixw.x);
#pragma unroll
      for (int tc = 0; tc < 2; ++tc) {
        if (tr & 1) acc[tr][tc] = smfmac<1>(av, bf[tc], acc[tr][tc], ix);
        else acc[tr][tc] = smfmac<0>(av, bf[tc], acc[tr][tc], ix);
      }
    }
    TRACE(4 + wave, s, 2);
  }
  barrier_only();                                  // every consumer is done reading the ring
#ifdef VENOM_ABLATE
  TRACE_DUMP();
#endif

  // ---- stage 3: registers -> (LDS) -> global.  Accumulator element v of a 32x32 tile sits at
  // row 8*(v/4) + 4*(lane/32) + v%4, column lane%32.
#ifdef VENOM_ABLATE
  if ((p.ablate & 16) && acc[0][0][0] != 12345.f) return;
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
    // the same wave reads its own strip back: 8 lanes x 16 B per row, 8 rows per pass
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

template <int VT, int NC, int NA>
constexpr int lds_bytes() {
  const int ring = kStages * kStepRows * 128 * NC + NA * (VT * kTileValBytes + kTailBytes);
  const int epi = NC * VT * 32 * (64 + 8) * 2;
  return ring > epi ? ring : epi;
}

#define VARIANT(NAME, VT, NC, NPB, NA)                                                         \
  { NAME, (VT) * 32, 64 * (NC), 64 * ((NC) + (NPB) + 1), lds_bytes<VT, NC, NA>(),                \
    spmm_kernel<VT, NC, NPB, NA, false>, spmm_kernel<VT, NC, NPB, NA, true> }

static const Variant kVariants[] = {
    VARIANT("v128_c512", 4, 8, 3, 6), VARIANT("v128_c256", 4, 4, 2, 9), VARIANT("v128_c128", 4, 2, 1, 10),
    VARIANT("v96_c512", 3, 8, 3, 7),  VARIANT("v96_c256", 3, 4, 2, 10), VARIANT("v96_c128", 3, 2, 1, 10),
    VARIANT("v64_c512", 2, 8, 3, 10), VARIANT("v64_c256", 2, 4, 2, 10), VARIANT("v64_c128", 2, 2, 1, 10),
    VARIANT("v32_c512", 1, 8, 3, 10), VARIANT("v32_c256", 1, 4, 2, 10), VARIANT("v32_c128", 1, 2, 1, 10),
};
constexpr int kNumVariants = sizeof(kVariants) / sizeof(kVariants[0]);

int spmm_variant_count() { return kNumVariants; }
const char* spmm_variant_name(int v) { return (v >= 0 && v < kNumVariants) ? kVariants[v].name : nullptr; }

static int pick_variant(int V, int64_t Ccols, int64_t nbr) {
  // the widest column tile that C fills at least half of: wide tiles re-read the A stream least
  // and measured fastest at every shape tried; narrow C takes the narrow tiles
  (void)nbr;
  int best = -1;
  for (int i = 0; i < kNumVariants; ++i) {
    if (kVariants[i].V != V) continue;
    if (best < 0) { best = i; continue; }
    const bool fits_i = 2 * Ccols > kVariants[i].bsc, fits_b = 2 * Ccols > kVariants[best].bsc;
    if (fits_i && (!fits_b || kVariants[i].bsc > kVariants[best].bsc)) best = i;
    else if (!fits_i && !fits_b && kVariants[i].bsc < kVariants[best].bsc) best = i;
  }
  return best;
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
  static unsigned long long* trace_buf = nullptr;
  if (getenv("VENOM_TRACE")) {
    if (!trace_buf) { hipMalloc(&trace_buf, 16 * 64 * 4 * 8); }
    hipMemsetAsync(trace_buf, 0, 16 * 64 * 4 * 8, st);
    p.trace = trace_buf;
  }
#endif
  const int64_t nct = (Ccols + var.bsc - 1) / var.bsc;
  const int64_t total = nct * L.Rb;
  if (total > (int64_t)1 << 30 || L.steps > (int64_t)1 << 24) return VENOM_ERR_UNSUPPORTED;
  // gather offsets are formed as row * ldb_bytes + column bytes in 32 bits with a 24-bit multiply
  if (h.K >= ((int64_t)1 << 24) || ldb * 2 >= ((int64_t)1 << 24) || h.K * ldb * 2 >= ((int64_t)1 << 32))
    return VENOM_ERR_UNSUPPORTED;
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
#ifdef VENOM_ABLATE
  const int launch_lds = 163840;   // room for the timestamp area
  hipFuncSetAttribute(reinterpret_cast<const void*>(fn), hipFuncAttributeMaxDynamicSharedMemorySize, launch_lds);
#else
  const int launch_lds = var.lds;
#endif
  hipLaunchKernelGGL(fn, dim3(grid), dim3(var.threads), launch_lds, st, p);
#ifdef VENOM_ABLATE
  if (p.trace) {
    hipStreamSynchronize(st);
    static unsigned long long host[384];
    hipMemcpy(host, p.trace, sizeof(host), hipMemcpyDeviceToHost);
    FILE* f = fopen(getenv("VENOM_TRACE"), "w");
    if (f) {
      for (int slot = 0; slot < 12; ++slot) for (int st_ = 0; st_ < 8; ++st_) {
        const unsigned long long* e = host + (slot * 8 + st_) * 4;
        if (e[0] | e[1] | e[2] | e[3]) fprintf(f, "%d %d %llu %llu %llu %llu\n", slot, st_ + 16, e[0], e[1], e[2], e[3]);
      }
      fclose(f);
    }
  }
#endif
  return hipGetLastError() == hipSuccess ? VENOM_OK : VENOM_ERR_HIP;
}

}  // namespace venom
