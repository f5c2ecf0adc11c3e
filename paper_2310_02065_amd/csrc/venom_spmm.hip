// The product kernel: C = A . B with A in V:N:M form (paper section 4: stage 1 loads column-loc,
// the gathered rows of B and the A tile; stage 2 runs the 2:4 matrix instruction; stage 3 stores
// the output through on-chip memory).  Written for gfx950:
//   * the 2:4 inner pattern maps onto v_smfmac_f32_32x32x32_f16: A operand = 8 kept halfs per lane
//     (row = lane%32, four groups), 16 index bits per lane (= four canonical nibbles), B operand =
//     16 halfs per lane (column = lane%32, four groups x the 4 selected rows);
//   * a workgroup owns V x (64*NC) blocks of C (BS_r = V as in the paper, so every gathered row of
//     B serves all V rows); a k-step is 8 groups = 32 gathered rows of B;
//   * the workgroup is split by role.  NC CONSUMER waves each own a 64-column strip: they only read
//     LDS (transposing reads ds_read_b64_tr_b16 build the B operand, plain reads fetch the packed
//     values and index words) and issue matrix instructions.  PRODUCER waves only move data, by
//     direct-to-LDS loads: NPB of them gather the 32 rows of B of every k-step (XOR-swizzled per
//     row so the transposing reads spread over the banks) into a 4-stage ring, three k-steps ahead;
//     one more streams the packed A records into a deeper ring, NA-1 k-steps ahead, because that
//     stream comes from HBM while B is mostly L2-resident, and with them the row ids of B that the
//     gather needs.  Loads retire in order per wave, so the streams live in different waves, and a
//     producer that has to queue behind the memory pipeline stalls alone;
//   * the loads are issued from inline assembly and retired with exact `s_waitcnt vmcnt(n)` counts;
//     one s_barrier per k-step hands filled stages to the consumers and drained ones back;
//   * workgroups are persistent (one per compute unit): the k-steps of all tiles of a workgroup
//     form one sequence, so the load pipeline runs on across tile boundaries while the consumers
//     store their output;
//   * each XCD (one L2 each) walks a contiguous range of the column-tile-major tile list and keeps
//     its slab of B hot.
#include <atomic>
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
  int stream_out;          // nonzero: non-temporal stores of C
  int serpentine;          // nonzero: a workgroup's odd tiles run their k-steps backwards, so the end of the
                           // slab of B that the last tile left in L2 is where the next one starts
  int pad_row0;            // first gathered row of a tile's LAST k-step that lies past the end of K (32: none)
  const _Float16* bias;    // one entry per row of C, or null
  int act;                 // venom_activation_t
#ifdef VENOM_ABLATE
  unsigned long long* trace;
  int k_rows;              // rows of B: experiment builds clamp every gathered row id to it
#endif
};

#ifdef VENOM_ABLATE
constexpr int kAbl = VENOM_ABLATE;   // experiment switches, fixed at compile time (never in the product library)
#endif
constexpr int kNumXcd = 8;
constexpr int kMaxDevices = 16;      // devices whose per-device launch state is cached
#ifndef VENOM_STAGES
#define VENOM_STAGES 4
#endif
#ifndef VENOM_NA512
#define VENOM_NA512 6
#endif
constexpr int kStages = VENOM_STAGES;           // B ring depth: three k-steps are in flight
constexpr int kRidSlots = 16;        // row-id ring: 128 bytes per k-step

// ---- direct-to-LDS loads and their retirement, outside the compiler's wait-count bookkeeping.
// LDS destination of lane l is lds_addr + l*16; M0 carries lds_addr and needs one wait state
// before the load reads it.
// The global address is a wave-uniform 64-bit base (SGPR pair) plus an unsigned 32-bit byte offset
// per lane, so address generation costs one vector instruction per load.
__device__ __forceinline__ void dma16(const char* base, uint32_t lane_off, uint32_t lds_addr) {
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(lane_off), "s"(base), "s"(lds_addr)
               : "memory");
}
__device__ __forceinline__ void dma4(const char* base, uint32_t lane_off, uint32_t lds_addr) {  // lane l -> lds_addr + 4*l
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dword %0, %1" ::"v"(lane_off), "s"(base), "s"(lds_addr)
               : "memory");
}
// wait until at most N of this wave's loads are outstanding, then meet the other waves
template <int N>
__device__ __forceinline__ void wait_loads_and_barrier() {
  asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" ::"n"(N) : "memory");
}
// the same with N = min(k, MAXK) * UNIT for a run-time k >= 0; the steady state (k >= MAXK) is the
// first case tested
template <int UNIT, int MAXK>
__device__ __forceinline__ void wait_units_and_barrier(int k) {
  static_assert(MAXK * UNIT <= 63, "vmcnt is a 6-bit counter");
  if (k >= MAXK) wait_loads_and_barrier<MAXK * UNIT>();
  else if constexpr (MAXK > 0) wait_units_and_barrier<UNIT, MAXK - 1>(k);
}
// only the wait, for N = min(k, MAXK) * UNIT
template <int UNIT, int MAXK>
__device__ __forceinline__ void wait_units(int k) {
  static_assert(MAXK * UNIT <= 63, "vmcnt is a 6-bit counter");
  if (k >= MAXK) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(MAXK * UNIT) : "memory");
  else if constexpr (MAXK > 0) wait_units<UNIT, MAXK - 1>(k);
}
__device__ __forceinline__ void barrier_only() { asm volatile("s_barrier" ::: "memory"); }
// the same once every LDS read of this wave has returned (its reads of a stage must be over
// before the barrier that hands the stage back)
__device__ __forceinline__ void lgkm_drained_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

// 16-byte slot swizzle of gathered row rho inside its LDS row
__device__ __forceinline__ int slot_swizzle(int rho) { return 4 * (rho & 3); }

// GELU(x) = x * Phi(x) = x/2 * (1 + erf(x / sqrt 2)).  erf by the rational-times-Gaussian formula
// 7.1.26 of Abramowitz & Stegun (absolute error below 1.5e-7, fp32 noise level), a dozen
// instructions with the hardware exp2 and reciprocal: the output stage evaluates it 128 times per
// lane, fully unrolled, so a library erff would cost more code than the rest of the kernel.
__device__ __forceinline__ float gelu_by_definition(float x) {
  const float z = fabsf(x) * 0.70710678118654752f;
  const float t = __builtin_amdgcn_rcpf(fmaf(0.3275911f, z, 1.f));
  float poly = fmaf(1.061405429f, t, -1.453152027f);
  poly = fmaf(poly, t, 1.421413741f);
  poly = fmaf(poly, t, -0.284496736f);
  poly = fmaf(poly, t, 0.254829592f);
  const float tail = poly * t * __builtin_amdgcn_exp2f(-1.4426950408889634f * z * z);   // 1 - erf(z)
  const float phi = x < 0.f ? 0.5f * tail : 1.f - 0.5f * tail;                           // Phi(x)
  return x * phi;
}
// The tanh form x/2 * (1 + tanh u), u = sqrt(2/pi) (x + 0.044715 x^3), written as x / (1 + e^(-2u)).
__device__ __forceinline__ float gelu_tanh_form(float x) {
  const float u = 0.79788456080286536f * x * fmaf(0.044715f * x, x, 1.f);
  const float e = __builtin_amdgcn_exp2f(-2.f * 1.4426950408889634f * u);
  return x * __builtin_amdgcn_rcpf(1.f + e);
}

template <int ABID>
__device__ __forceinline__ floatx16 smfmac(half8 a, half16 b, floatx16 c, int idx) {
  return __builtin_amdgcn_smfmac_f32_32x32x32_f16(a, b, c, idx, 0, ABID);
}

// This workgroup's share of the tile list.  The grid holds one workgroup per compute unit (the
// host sizes it) and every workgroup walks several tiles: starting a wide workgroup that owns most
// of the LDS costs microseconds, and a persistent one can keep its load pipeline full across tile
// boundaries.  Consecutive workgroup ids land on different XCDs; each XCD takes a contiguous
// range of the column-tile-major list, so the workgroups of one XCD sweep the same slab of B at
// the same time and it stays in that L2.
struct TileWalk {
  int base, first, stride, count;
  __device__ __forceinline__ void locate(const SpmmParams& p, int t, int& ct, int& br) const {
    const int work = base + first + t * stride;
    ct = work / p.nbr;
    br = work - ct * p.nbr;
  }
};

// MODE 0: the plain product; 1: fused bias / activation; 2: the same with C written transposed
// (token-major).  Separate instantiations: the plain kernel carries none of the epilogue code.
// PAIR 2: the workgroup owns TWO neighbouring block rows and half the columns per wave.  Legal only
// where both block rows select the same columns of every group (always at M = 4, where all four are
// selected): the gathered rows of B then serve 2V rows, which halves the gather per matrix
// instruction, the kernel's tightest resource.
template <int VT, int NC, int NPB, int NA, bool OUT_F32, int MODE, int PAIR>
__global__ void __launch_bounds__((NC + NPB + 1) * 64, 3) spmm_kernel(SpmmParams p) {
  static_assert(NC == 2 || NC == 4 || NC == 8, "consumer waves per workgroup");
  static_assert(PAIR == 1 || PAIR == 2, "block rows per workgroup");
  constexpr bool EPI = MODE != 0;
  static_assert(VT >= 1 && VT <= kMaxTiles, "32-row tiles per block row");
  static_assert(NA >= 4, "the A ring holds the record being read, the next one, and records in flight");
  constexpr int RT = PAIR * VT;                    // 32-row tiles a consumer wave accumulates
  constexpr int CT = 2 / PAIR;                     // 32-column tiles a consumer wave accumulates
  constexpr int WCOLS = 32 * CT;                   // columns of C per consumer wave
  constexpr int BSC = WCOLS * NC;                  // columns of C per workgroup
  constexpr int ROW_BYTES = 2 * BSC;               // one gathered row of B in LDS
  constexpr int RPI = 1024 / ROW_BYTES;            // rows written by one wave-wide 16-byte load
  constexpr int LPR = 64 / RPI;                    // lanes (= 16-byte slots) per row
  constexpr int NI = kStepRows / RPI;              // B loads per k-step (4 * NC)
  constexpr int NBH = (NI + NPB - 1) / NPB, NBL = NI / NPB, NBHI = NI % NPB;  // ... per B producer
  constexpr int B_BYTES = kStepRows * ROW_BYTES;
  constexpr int REC = VT * kTileValBytes + kTailBytes;       // one A record
  constexpr int A_BYTES = PAIR * REC;              // the records of one k-step (one per block row)
  constexpr int T_OFF = VT * kTileValBytes;        // record tail: index words
  constexpr int ARING = kStages * B_BYTES;         // LDS: [B ring][A ring][row-id ring]
  constexpr int RIDRING = ARING + NA * A_BYTES;
  constexpr int NJ = PAIR * (VT + 1);              // A loads per k-step: VT value blocks + the tail, per block row
  constexpr int PA = NA - 2;                       // k-steps the A stream runs ahead (a record stays one step
                                                   // longer than its k-step: the late consumers re-read it)
  constexpr int PB = kStages - 1;                  // k-steps the B stream runs ahead
  static_assert((kStages - 2) * NBH <= 63 && PA * NJ <= 63, "load counts fit the 6-bit counter");
  static_assert(NC * 32 * WCOLS * 2 <= B_BYTES, "the output staging of all consumers fits one B stage");
  constexpr int RA = PA + PB + 1;                  // k-steps the row-id stream runs ahead: the ids of step
                                                   // g+PB+1 are then older than record g+1 in the load queue
  static_assert(kRidSlots >= RA - PB + 2, "a row-id slot is rewritten only after its last reader");

  extern __shared__ __attribute__((aligned(1024))) char smem[];
  const uint32_t lds0 = (uint32_t)(uintptr_t)(LDS_PTR(char))smem;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);

#ifdef VENOM_ABLATE
  if (p.trace && threadIdx.x == 0 && blockIdx.x < 16) {
    p.trace[blockIdx.x * 4 + 0] = __builtin_readcyclecounter();
    p.trace[blockIdx.x * 4 + 1] = wall_clock64();
  }
#endif
  TileWalk tw;
  {
    const int xcd = blockIdx.x % kNumXcd;
    tw.base = xcd * p.per_xcd;
    tw.first = blockIdx.x / kNumXcd;
    tw.stride = gridDim.x / kNumXcd;
    int lim = p.nbr * p.nct - tw.base;
    if (lim > p.per_xcd) lim = p.per_xcd;
    tw.count = lim > tw.first ? (lim - tw.first + tw.stride - 1) / tw.stride : 0;
  }
  if (tw.count == 0) return;                       // the whole workgroup leaves together
  // All k-steps of all tiles of this workgroup form one sequence g = 0 .. G-1; the rings and the
  // barriers are indexed by g, so the loads of the next tile start while this one is finishing.
  // Barriers, in order: one before the first step (the first row ids are on chip), one per step
  // ("step g is complete in LDS, step g-1 is consumed"), and one more after the last step of each
  // tile, after which the consumers stage their output in the B stage they have just drained.
  const int G = tw.count * p.steps;

  // the producers' few instructions per k-step go ahead of the consumers' when both are ready
  if (wave >= NC) __builtin_amdgcn_s_setprio(3);
  if (wave == NC + NPB) {
    // ========================================================================= A producer
    // Streams, in one in-order queue: the packed records, PA steps ahead, and the row ids of B
    // that the gather producers need, RA steps ahead, into a ring of kRidSlots x 128 bytes.
    const uint32_t lane_off = lane * 16;
    int ct, br;
    // record stream position
    int a_t = 0, a_s = 0, a_slot = 0;
    tw.locate(p, 0, ct, br);
    // (br numbers groups of PAIR block rows; the records of the second block row of a pair lie
    // pair_gap bytes after those of the first)
    const char* a_ptr = p.arec + (int64_t)br * PAIR * p.steps * p.rec_bytes;
    const int64_t pair_gap = (int64_t)p.steps * p.rec_bytes;
    int64_t a_inc = p.rec_bytes;
    auto next_record = [&]() {
#ifdef VENOM_ABLATE
      if (!(kAbl & (8 | 1024)))
#endif
      {
        const uint32_t dst = lds0 + ARING + a_slot * A_BYTES;
#pragma unroll
        for (int pr = 0; pr < PAIR; ++pr) {
          const char* src = a_ptr + pr * pair_gap;
#pragma unroll
          for (int j = 0; j < VT; ++j) dma16(src + j * 1024, lane_off, dst + pr * REC + j * 1024);
          if (lane < kTailBytes / 16) dma16(src + T_OFF, lane_off, dst + pr * REC + T_OFF);   // the 512-byte tail: half a wave
        }
      }
      a_ptr += a_inc;
      a_slot = a_slot + 1 == NA ? 0 : a_slot + 1;
      if (++a_s == p.steps) {
        a_s = 0;
        if (++a_t < tw.count) {
          tw.locate(p, a_t, ct, br);
          const bool back = p.serpentine && (a_t & 1);       // odd tiles run their k-steps backwards
          a_inc = back ? -p.rec_bytes : p.rec_bytes;
          a_ptr = p.arec + ((int64_t)br * PAIR * p.steps + (back ? p.steps - 1 : 0)) * p.rec_bytes;
        }
      }
    };
    // row-id stream position
    int r_t = 0, r_s = 0, r_slot = 0;
    const char* r_ptr = reinterpret_cast<const char*>(p.rowidx) + (int64_t)br * PAIR * p.steps * (kStepRows * 4);
    int r_inc = kStepRows * 4;
    auto next_rowids = [&]() {
      if (lane < kStepRows) dma4(r_ptr, lane * 4, lds0 + RIDRING + r_slot * (kStepRows * 4));
      r_ptr += r_inc;
      r_slot = (r_slot + 1) % kRidSlots;
      if (++r_s == p.steps) {
        r_s = 0;
        if (++r_t < tw.count) {
          int ct2, br2;
          tw.locate(p, r_t, ct2, br2);
          const bool back = p.serpentine && (r_t & 1);
          r_inc = back ? -(kStepRows * 4) : kStepRows * 4;
          r_ptr = reinterpret_cast<const char*>(p.rowidx) +
                  ((int64_t)br2 * PAIR * p.steps + (back ? p.steps - 1 : 0)) * (kStepRows * 4);
        }
      }
    };
    int first_records = 0;
    for (int j = 0; j < RA && j < G; ++j) next_rowids();
    for (int j = 0; j < PA && j < G; ++j, ++first_records) next_record();
#ifdef VENOM_ABLATE
    if constexpr ((kAbl & (8 | 1024)) != 0) wait_loads_and_barrier<0>();   // no record loads to count behind
    else
#endif
    wait_units_and_barrier<NJ, PA>(first_records);  // the row ids (older than every record) have landed
    int c_s = 0;                                   // step inside the tile the consumers are on
    for (int g = 0; g < G; ++g) {
      // records g and g+1 have landed when at most the records after g+1 are pending; the row-id
      // loads in between only make the wait a little stricter
      const int left = G - 2 - g;
#ifdef VENOM_ABLATE
      if constexpr ((kAbl & (8 | 1024)) != 0) wait_loads_and_barrier<0>();
      else
#endif
      wait_units_and_barrier<NJ, PA - 2>(left < 0 ? 0 : left);
      // after the barrier everyone is done with record g-2: its slot takes record g+PA
      if (g + PA < G) next_record();
      if (g + RA < G) next_rowids();
      if (++c_s == p.steps) { c_s = 0; barrier_only(); }
    }
  } else if (wave >= NC) {
    // ========================================================================= B producers
    const int pj = wave - NC;
    // B load q of this producer is load number pj + NPB*q of the k-step; it covers rows
    // (that number)*RPI .. +RPI-1; lane l writes 16-byte slot l%LPR of row l/LPR and fetches the
    // XOR-swizzled chunk of the gathered row.
    // The row ids of a k-step sit in lane order in one register (lane l holds row l%32); one
    // 24-bit multiply turns them into byte offsets row * ldb_bytes (the host checks the ranges),
    // the rows of one load are picked out with v_readlane, and a lane adds its column offset.
    int chunk_col[NBH];                            // first column of this lane's chunk inside the tile
#pragma unroll
    for (int q = 0; q < NBH; ++q) {
      const int rho = ((pj + NPB * q) % NI) * RPI + lane / LPR;
      chunk_col[q] = ((lane % LPR) ^ slot_swizzle(rho)) * 8;
    }
    uint32_t ld_col[NBH];
    auto set_tile = [&](int t) {
      int ct, br;
      tw.locate(p, t, ct, br);
#pragma unroll
      for (int q = 0; q < NBH; ++q) {
        int64_t col = (int64_t)ct * BSC + chunk_col[q];
        if (col + 8 > p.Ccols) col = p.Ccols - 8;  // past the edge: any in-bounds data, never stored
        ld_col[q] = (uint32_t)(col * 2);
      }
    };
    const int rowsel = lane / LPR;                 // which of the RPI rows of a load this lane writes
    const uint32_t ldb24 = (uint32_t)p.ldb_bytes;
    const bool hi = NBHI == 0 || pj < NBHI;        // this producer has NBH loads per k-step, else NBL
    int b_t = 0, b_s = 0, b_slot = 0;
    set_tile(0);
    auto issue = [&](int ridv) {
#ifdef VENOM_ABLATE
      if (!(kAbl & (8 | 2048)))
#endif
      {
        const uint32_t sb = lds0 + b_slot * B_BYTES;
        // byte offsets of all 32 rows at once (lane l: row l%32), then one v_readlane per row
        const int rowoff = (int)__umul24((uint32_t)ridv, ldb24);
#pragma unroll
        for (int q = 0; q < NBH; ++q) {
          if (q < NBL || hi) {
            const int rho0 = ((pj + NPB * q) % NI) * RPI;
            int off = __builtin_amdgcn_readlane(rowoff, rho0);
#pragma unroll
            for (int k = 1; k < RPI; ++k) {
              const int ok = __builtin_amdgcn_readlane(rowoff, rho0 + k);
              off = rowsel == k ? ok : off;
            }
            dma16(p.B, (uint32_t)off + ld_col[q], sb + (pj + NPB * q) * 1024);
          }
        }
      }
      b_slot = (b_slot + 1) % kStages;
      if (++b_s == p.steps) {
        b_s = 0;
        if (++b_t < tw.count) set_tile(b_t);
      }
    };
    auto rowids_of = [&](int g) {
      int r = *reinterpret_cast<const int*>(smem + RIDRING + (g % kRidSlots) * (kStepRows * 4) + (lane & 31) * 4);
#ifdef VENOM_ABLATE
      r = r < 0 ? 0 : (r >= p.k_rows ? p.k_rows - 1 : r);
#endif
      return r;
    };
    barrier_only();                                // the first row ids are on chip
    for (int j = 0; j < PB && j < G; ++j) issue(rowids_of(j));
    int ridv = PB < G ? rowids_of(PB) : 0;         // row ids of the k-step issued next
    int c_s = 0, c_t = 0;                          // k-step inside the tile / tile the consumers are on
    for (int g = 0; g < G; ++g) {
      // this producer's part of k-step g has landed when at most its loads of the later steps
      // (up to two) are pending
      const int left = G - 1 - g;
      if (p.pad_row0 < kStepRows && c_s == ((p.serpentine && (c_t & 1)) ? 0 : p.steps - 1)) {
        // The last k-step of a tile when K/M is not a multiple of 8: its trailing groups do not
        // exist.  Their values are zero, but 0 x Inf is not, so the rows gathered for them (row 0
        // of B, a valid address that keeps the load count exact) are overwritten with zeros once
        // they have landed; every producer cleans the rows it loaded itself.
        if (hi) wait_units<NBH, kStages - 2>(left);
        else wait_units<NBL, kStages - 2>(left);
        char* stage = smem + (g % kStages) * B_BYTES;
#pragma unroll
        for (int q = 0; q < NBH; ++q)
          if ((q < NBL || hi) && ((pj + NPB * q) % NI) * RPI + rowsel >= p.pad_row0)
            *reinterpret_cast<uint4*>(stage + (pj + NPB * q) * 1024 + lane * 16) = make_uint4(0, 0, 0, 0);
        lgkm_drained_barrier();
      } else if (hi) wait_units_and_barrier<NBH, kStages - 2>(left);
      else wait_units_and_barrier<NBL, kStages - 2>(left);
      // after the barrier the consumers are done with stage g-1: it takes step g+PB
      if (g + PB < G) {
        issue(ridv);
        if (g + PB + 1 < G) ridv = rowids_of(g + PB + 1);
      }
      if (++c_s == p.steps) { c_s = 0; ++c_t; barrier_only(); }
    }
  } else {
    // ========================================================================= consumers
    // Transposing LDS reads that build the B operand.  Sub-read cb of a 32-column tile: lane block
    // blk = lane/16 reads group t = 4*(cb/2) + 2*(blk/2) + cb%2, 16-column window 2*tile + blk%2;
    // inside the block lane i reads row 4*t + i/4, 8-byte piece i%4.
    int rd_off[CT][4];
    {
      const int blk = lane >> 4, i = lane & 15, e = i >> 2, c8 = i & 3;
#pragma unroll
      for (int tc = 0; tc < CT; ++tc)
#pragma unroll
        for (int cb = 0; cb < 4; ++cb) {
          const int t = 4 * (cb >> 1) + 2 * (blk >> 1) + (cb & 1);
          const int rho = 4 * t + e;
          const int win = (wave * CT + tc) * 2 + (blk & 1);
          const int slot = (2 * win + (c8 >> 1)) ^ slot_swizzle(rho);
          rd_off[tc][cb] = rho * ROW_BYTES + slot * 16 + (c8 & 1) * 8;
        }
    }
    // One k-step of matrix work: operands bf (the wave's 32-column B tiles) and ixw are in
    // registers, the A operands stream from the records at `sa` through two alternating registers;
    // av[0] may already hold tile row 0 (`have0`).  Tile row t = block row t / VT of the pair,
    // 32-row tile t % VT of it.
    floatx16 acc[RT][CT];
    half16 bf[CT];
    uint2 ixw[PAIR];                               // 4 x 16 index bits per block row
    half8 av[2];
    auto read_a = [&](const char* sa, int t) {
      return *reinterpret_cast<const half8*>(sa + (t / VT) * REC + (t % VT) * kTileValBytes + lane * 16);
    };
    auto read_b_ix = [&](const char* sb, const char* sa) {
#pragma unroll
      for (int tc = 0; tc < CT; ++tc)
#pragma unroll
        for (int cb = 0; cb < 4; ++cb) {
          const short4v piece = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_PTR(short4v))(sb + rd_off[tc][cb]));
          const half4 ph = __builtin_bit_cast(half4, piece);
          bf[tc][4 * cb + 0] = ph[0]; bf[tc][4 * cb + 1] = ph[1]; bf[tc][4 * cb + 2] = ph[2]; bf[tc][4 * cb + 3] = ph[3];
        }
#pragma unroll
      for (int pr = 0; pr < PAIR; ++pr) ixw[pr] = *reinterpret_cast<const uint2*>(sa + pr * REC + T_OFF + lane * 8);
    };
    auto multiply = [&](const char* sa, bool have0) {
      if (!have0) av[0] = read_a(sa, 0);
      if (RT > 1) av[1] = read_a(sa, 1);
#pragma unroll
      for (int t = 0; t < RT; ++t) {
        const int tr = t % VT;
        const int ix = (int)((tr >> 1) ? ixw[t / VT].y : ixw[t / VT].x);
#pragma unroll
        for (int tc = 0; tc < CT; ++tc) {
          if (tr & 1) acc[t][tc] = smfmac<1>(av[t & 1], bf[tc], acc[t][tc], ix);
          else acc[t][tc] = smfmac<0>(av[t & 1], bf[tc], acc[t][tc], ix);
        }
        if (t + 2 < RT) av[t & 1] = read_a(sa, t + 2);
      }
    };
    // The two consumer waves that share a SIMD work half a k-step apart: the EARLY one reads its
    // operands right after the barrier and multiplies when they arrive; the LATE one first
    // multiplies with the operands it fetched during the previous k-step, then fetches this one's.
    // So one wave's LDS latency hides behind the other's matrix instructions.  Every LDS read of a
    // stage still happens inside that stage's k-step; the late wave re-reads A tile rows of the
    // previous record, which is why the A ring is refilled one step later than it is consumed.
    const bool late = (wave / (NC / 2)) & 1;
    int b_slot = 0, a_slot = 0;
    barrier_only();                                // (the producers' start-up barrier)
    for (int t = 0; t < tw.count; ++t) {
#pragma unroll
      for (int tr = 0; tr < RT; ++tr)
#pragma unroll
        for (int tc = 0; tc < CT; ++tc)
#pragma unroll
          for (int v = 0; v < 16; ++v) acc[tr][tc][v] = 0.f;

      const char* sb = smem;
      const char* sa = smem;
      auto advance = [&]() {
        sb = smem + b_slot * B_BYTES;
        sa = smem + ARING + a_slot * A_BYTES;
        b_slot = (b_slot + 1) % kStages;
        a_slot = a_slot + 1 == NA ? 0 : a_slot + 1;
      };
      if (!late) {
        for (int s = 0; s < p.steps; ++s) {
          barrier_only();                          // this k-step is complete in LDS
          advance();
          read_b_ix(sb, sa);
          multiply(sa, false);
        }
        barrier_only();                            // every consumer has drained the last B stage
      } else {
        lgkm_drained_barrier();
        advance();
        read_b_ix(sb, sa);
        av[0] = read_a(sa, 0);
        for (int s = 1; s < p.steps; ++s) {
          const char* sa_prev = sa;
          lgkm_drained_barrier();                  // this k-step is complete; my reads of the last one are done
          advance();
          multiply(sa_prev, true);
          read_b_ix(sb, sa);
          av[0] = read_a(sa, 0);
        }
        lgkm_drained_barrier();                    // every consumer has drained the last B stage
        multiply(sa, true);
      }

      // ---- stage 3: registers -> (LDS) -> global.  Accumulator element v of a 32x32 tile sits
      // at row 8*(v/4) + 4*(lane/32) + v%4, column lane%32.
#ifdef VENOM_ABLATE
      if ((kAbl & 16) && acc[0][0][0] != 12345.f) continue;
#endif
      // everything below is per-tile work: keep its index arithmetic from being hoisted out of the
      // tile loop, where it would sit in registers the k-loop needs
      int ln = lane;
      asm volatile("" : "+v"(ln));
      int ct, br;
      tw.locate(p, t, ct, br);
#ifdef VENOM_ABLATE
      if (kAbl & 8192) { br = 0; ct = 0; }         // experiment: every tile writes block (0, 0) of C
#endif
      const int64_t row0 = (int64_t)br * RT * 32;   // (the block rows of a pair are neighbours: RT tiles in a row)
      const int64_t col0 = (int64_t)ct * BSC + wave * WCOLS;
      // fused epilogue (the layer's bias, one per output row, then the activation), in fp32 on
      // the accumulators, one 32-row tile at a time right before it is stored: a ln holds rows
      // 8j + 4*(ln/32) + 0..3 of the tile
      auto finish = [&](int tr) {
        if constexpr (!EPI) return;                // the plain product compiles without any of this
        if (p.bias) {
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            const half4 b4 = *reinterpret_cast<const half4*>(p.bias + row0 + tr * 32 + 8 * j + 4 * (ln >> 5));
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
              for (int tc = 0; tc < CT; ++tc) acc[tr][tc][4 * j + i] += (float)b4[i];
            __builtin_amdgcn_sched_barrier(0);
          }
        }
        // (scheduling fences keep the evaluations from being interleaved by the dozen: their
        // temporaries would push accumulators out of registers, for the whole kernel)
        if (p.act == VENOM_ACT_GELU) {
#pragma unroll
          for (int tc = 0; tc < CT; ++tc)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
              acc[tr][tc][v] = gelu_by_definition(acc[tr][tc][v]);
              if ((v & 1) == 1) __builtin_amdgcn_sched_barrier(0);
            }
        } else if (p.act == VENOM_ACT_GELU_TANH) {
#pragma unroll
          for (int tc = 0; tc < CT; ++tc)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
              acc[tr][tc][v] = gelu_tanh_form(acc[tr][tc][v]);
              if ((v & 1) == 1) __builtin_amdgcn_sched_barrier(0);
            }
        }
      };
      if constexpr (MODE == 2) {
        // Token-major output Y[token][feature] = C transposed: a ln owns one column of C (a
        // token) and, per 32-row tile, four runs of 4 consecutive rows (features): each run is one
        // 8-byte (fp16) or 16-byte (fp32) store straight from the accumulators; the two half-waves
        // write neighbouring runs, the tiles of a block row continue the same 2*V bytes of a token.
#pragma unroll
        for (int tr = 0; tr < RT; ++tr) {
          finish(tr);
#pragma unroll
          for (int tc = 0; tc < CT; ++tc) {
            const int64_t tok = col0 + tc * 32 + (ln & 31);
            if (tok < p.Ccols) {
#pragma unroll
              for (int q = 0; q < 4; ++q) {
                const int64_t feat = row0 + tr * 32 + 8 * q + 4 * (ln >> 5);
                if constexpr (OUT_F32) {
                  typedef float f32x4 __attribute__((ext_vector_type(4)));
                  const f32x4 o = {acc[tr][tc][4 * q], acc[tr][tc][4 * q + 1], acc[tr][tc][4 * q + 2], acc[tr][tc][4 * q + 3]};
                  *reinterpret_cast<f32x4*>(reinterpret_cast<float*>(p.C) + tok * p.ldc + feat) = o;
                } else {
                  const half4 o = {(_Float16)acc[tr][tc][4 * q], (_Float16)acc[tr][tc][4 * q + 1],
                                   (_Float16)acc[tr][tc][4 * q + 2], (_Float16)acc[tr][tc][4 * q + 3]};
                  *reinterpret_cast<half4*>(reinterpret_cast<_Float16*>(p.C) + tok * p.ldc + feat) = o;
                }
              }
            }
          }
          __builtin_amdgcn_sched_barrier(0);
        }
      } else if constexpr (OUT_F32) {
        float* Cf = reinterpret_cast<float*>(p.C);
#pragma unroll
        for (int tr = 0; tr < RT; ++tr) {
          finish(tr);
#pragma unroll
          for (int tc = 0; tc < CT; ++tc) {
            const int64_t col = col0 + tc * 32 + (ln & 31);
            if (col < p.Ccols) {
#pragma unroll
              for (int v = 0; v < 16; ++v) {
                const int64_t row = row0 + tr * 32 + 8 * (v >> 2) + 4 * (ln >> 5) + (v & 3);
                Cf[row * p.ldc + col] = acc[tr][tc][v];
              }
            }
          }
          __builtin_amdgcn_sched_barrier(0);
        }
      } else {
        // One 32-row tile of the wave's columns at a time through this wave's share of the drained
        // stage (the producers refill that stage only after the next barrier).  A staged row is
        // 2*WCOLS bytes; its 16-byte chunks are XOR-swizzled by bit 2 of the row so that the two
        // half-waves, which write rows r and r+4, use different banks.
        constexpr int SROW = 2 * WCOLS;            // bytes of a staged row
        constexpr int LPS = SROW / 16;             // lanes (16-byte chunks) per staged row
        constexpr int SWZ = LPS / 2;               // chunk distance that changes the bank group
        char* stg = const_cast<char*>(sb) + wave * (32 * SROW);
        _Float16* Ch = reinterpret_cast<_Float16*>(p.C);
        const int chunk = ln % LPS, rsub = ln / LPS;
        const int64_t col = col0 + chunk * 8;
#pragma unroll
        for (int tr = 0; tr < RT; ++tr) {
          finish(tr);
#pragma unroll
          for (int tc = 0; tc < CT; ++tc) {
            const int c = tc * 32 + (ln & 31);
#pragma unroll
            for (int v = 0; v < 16; ++v) {
              const int r = 8 * (v >> 2) + 4 * (ln >> 5) + (v & 3);
              const int sw = ((c >> 3) ^ (SWZ * ((r >> 2) & 1)));
              *reinterpret_cast<_Float16*>(stg + r * SROW + sw * 16 + (c & 7) * 2) =
                  (_Float16)acc[tr][tc][v];        // one rounding, nearest-even
            }
          }
#pragma unroll
          for (int i = 0; i < 32 / (64 / LPS); ++i) {
            const int r = i * (64 / LPS) + rsub;
            const uint4 val = *reinterpret_cast<const uint4*>(stg + r * SROW + ((chunk ^ (SWZ * ((r >> 2) & 1))) * 16));
            if (col < p.Ccols) {
              typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
              u32x4* dst = reinterpret_cast<u32x4*>(Ch + (row0 + tr * 32 + r) * p.ldc + col);
              const u32x4 v4 = {val.x, val.y, val.z, val.w};
              // streaming stores keep C out of the L2 that holds the slab of B; they drain more
              // slowly, so the host asks for them only where the output is a small share of the traffic
              if (p.stream_out) __builtin_nontemporal_store(v4, dst);
              else *dst = v4;
            }
          }
          __builtin_amdgcn_sched_barrier(0);
        }
      }
    }
  }
#ifdef VENOM_ABLATE
  if (p.trace && threadIdx.x == 0 && blockIdx.x < 16) {
    p.trace[blockIdx.x * 4 + 2] = __builtin_readcyclecounter();
    p.trace[blockIdx.x * 4 + 3] = wall_clock64();
  }
#endif
}

// ---------------------------------------------------------------------------------------------
struct Variant {
  const char* name;
  int V;       // block height it serves
  int pair;    // block rows a workgroup owns (2: only where neighbouring block rows select the same columns)
  int bsc;     // columns per workgroup
  int threads;
  int lds;     // dynamic LDS bytes
  void (*fn[2][3])(SpmmParams);   // [fp32 output][mode]
};

template <int VT, int NC, int NA, int PAIR>
constexpr int lds_bytes() {   // B ring, A ring, row-id ring (the output staging reuses a B stage)
  return kStages * kStepRows * (128 / PAIR) * NC + NA * PAIR * (VT * kTileValBytes + kTailBytes) +
         kRidSlots * kStepRows * 4;
}

#define VARIANT(NAME, VT, NC, NPB, NA, PAIR)                                                            \
  { NAME, (VT) * 32, PAIR, (64 / (PAIR)) * (NC), 64 * ((NC) + (NPB) + 1), lds_bytes<VT, NC, NA, PAIR>(),       \
    { { spmm_kernel<VT, NC, NPB, NA, false, 0, PAIR>, spmm_kernel<VT, NC, NPB, NA, false, 1, PAIR>,         \
        spmm_kernel<VT, NC, NPB, NA, false, 2, PAIR> },                                                   \
      { spmm_kernel<VT, NC, NPB, NA, true, 0, PAIR>, spmm_kernel<VT, NC, NPB, NA, true, 1, PAIR>,           \
        spmm_kernel<VT, NC, NPB, NA, true, 2, PAIR> } } }

static const Variant kVariants[] = {
    VARIANT("v128_c512", 4, 8, 3, VENOM_NA512, 1), VARIANT("v128_c256", 4, 4, 2, 9, 1), VARIANT("v128_c128", 4, 2, 1, 10, 1),
    VARIANT("v96_c512", 3, 8, 3, 7, 1),  VARIANT("v96_c256", 3, 4, 2, 10, 1), VARIANT("v96_c128", 3, 2, 1, 10, 1),
    VARIANT("v64_c512", 2, 8, 3, 10, 1), VARIANT("v64_c256", 2, 4, 2, 10, 1), VARIANT("v64_c128", 2, 2, 1, 10, 1),
    VARIANT("v32_c512", 1, 8, 3, 10, 1), VARIANT("v32_c256", 1, 4, 2, 10, 1), VARIANT("v32_c128", 1, 2, 1, 10, 1),
    // two block rows per workgroup (same selected columns in both: M = 4)
    VARIANT("v128x2_c256", 4, 8, 2, 6, 2), VARIANT("v64x2_c256", 2, 8, 2, 6, 2),
};
constexpr int kNumVariants = sizeof(kVariants) / sizeof(kVariants[0]);

int spmm_variant_count() { return kNumVariants; }
const char* spmm_variant_name(int v) { return (v >= 0 && v < kNumVariants) ? kVariants[v].name : nullptr; }

static int pick_variant(int V, int M, int64_t Ccols, int64_t nbr) {
  // M = 4 selects all four columns in every block, so neighbouring block rows gather the same rows
  // of B: the paired tile halves the gather per matrix instruction (and doubles the passes over
  // the A stream).  Measured at 8192 x 8192 x 2048: +7 % at V = 64, nothing at V = 128, where it is
  // therefore only used on request.
  if (M == kSelCols && V <= 64 && nbr % 2 == 0 && Ccols > 128)
    for (int i = 0; i < kNumVariants; ++i)
      if (kVariants[i].V == V && kVariants[i].pair == 2) return i;
  // The widest column tile that C fills at least half of: wide tiles re-read the A stream least
  // and measured fastest at every large shape tried; narrow C takes the narrow tiles.  When that
  // choice leaves more than half of the compute units without a tile (few block rows), the
  // 256-column tile spreads the work over twice as many units and measured ~12 % faster; the
  // 128-column tile (one gather wave, two consumers) never paid off.
  int best = -1;
  for (int i = 0; i < kNumVariants; ++i) {
    if (kVariants[i].V != V || kVariants[i].pair != 1) continue;
    if (best < 0) { best = i; continue; }
    const bool fits_i = 2 * Ccols > kVariants[i].bsc, fits_b = 2 * Ccols > kVariants[best].bsc;
    if (fits_i && (!fits_b || kVariants[i].bsc > kVariants[best].bsc)) best = i;
    else if (!fits_i && !fits_b && kVariants[i].bsc < kVariants[best].bsc) best = i;
  }
  if (best >= 0 && kVariants[best].bsc == 512) {
    const int64_t tiles = nbr * ((Ccols + 511) / 512);
    if (tiles <= 128)
      for (int i = 0; i < kNumVariants; ++i)
        if (kVariants[i].V == V && kVariants[i].pair == 1 && kVariants[i].bsc == 256) best = i;
  }
  return best;
}

venom_status_t launch_spmm(const venom_handle& h, const void* B, int64_t ldb, int64_t Ccols, const void* bias, int act,
                           void* C, int64_t ldc, int c_dtype, int tokens_major, int variant, hipStream_t st) {
  const Layout& L = h.lay;
  if (!L.packed) return VENOM_ERR_UNSUPPORTED;
  if (L.R == 0 || Ccols == 0) return VENOM_OK;
  if (variant < 0) variant = pick_variant(h.V, h.M, Ccols, L.Rb);
  if (variant < 0 || variant >= kNumVariants || kVariants[variant].V != h.V) return VENOM_ERR_UNSUPPORTED;
  const Variant& var = kVariants[variant];
  // a paired tile is only correct where both block rows of a pair gather the same rows of B
  if (var.pair == 2 && (h.M != kSelCols || L.Rb % 2 != 0)) return VENOM_ERR_UNSUPPORTED;
  SpmmParams p{};
  p.arec = h.ws + L.off_arec;
  p.rowidx = reinterpret_cast<const int32_t*>(h.ws + L.off_rowidx);
  p.B = reinterpret_cast<const char*>(B);
  p.C = C;
  p.ldb_bytes = ldb * 2; p.ldc = ldc; p.Ccols = Ccols; p.rec_bytes = L.rec_bytes;
  p.steps = (int)L.steps;
  p.bias = reinterpret_cast<const _Float16*>(bias);
  p.act = act;
#ifdef VENOM_NO_SERPENTINE
  p.serpentine = 0;
#else
  p.serpentine = 1;
#endif
  p.pad_row0 = (L.G % kStepGroups) ? (int)(L.G % kStepGroups) * kSelCols : kStepRows;
  p.stream_out = L.steps >= 32;   // measured: +3 % at 48 k-steps per tile, -20 % at 8
#ifdef VENOM_ABLATE
  p.k_rows = (int)h.K;
#endif
#ifdef VENOM_ABLATE
  static unsigned long long* trace_buf = nullptr;
  static int trace_calls = 0;
  if (getenv("VENOM_TRACE")) {
    if (!trace_buf) hipMalloc(&trace_buf, 64 * 8);
    p.trace = trace_buf;
  }
#endif
  const int64_t nct = (Ccols + var.bsc - 1) / var.bsc;
  const int64_t nbr = L.Rb / var.pair;
  const int64_t total = nct * nbr;
  if (total > (int64_t)1 << 30 || L.steps > (int64_t)1 << 24) return VENOM_ERR_UNSUPPORTED;
  // gather offsets are formed as row * ldb_bytes + column bytes in 32 bits with a 24-bit multiply
  if (h.K >= ((int64_t)1 << 24) || ldb * 2 >= ((int64_t)1 << 24) || h.K * ldb * 2 >= ((int64_t)1 << 32))
    return VENOM_ERR_UNSUPPORTED;
  p.nbr = (int)nbr; p.nct = (int)nct;
  p.per_xcd = (int)((total + kNumXcd - 1) / kNumXcd);
  // one resident workgroup per compute unit (two where the tile is small enough to share a unit);
  // each walks per_xcd / (grid / 8) tiles
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) return VENOM_ERR_HIP;
  static std::atomic<int> cu_count[kMaxDevices] = {};   // per device, filled on first use
  int cus = (dev >= 0 && dev < kMaxDevices) ? cu_count[dev].load(std::memory_order_relaxed) : 0;
  if (cus == 0) {
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < kNumXcd)
      return VENOM_ERR_HIP;
    if (dev >= 0 && dev < kMaxDevices) cu_count[dev].store(cus, std::memory_order_relaxed);
  }
  const int share = (var.lds <= 80 * 1024 && var.threads <= 512) ? 2 : 1;
  const int64_t resident_per_xcd = (int64_t)(cus / kNumXcd) * share;
  const int64_t wg_per_xcd = p.per_xcd < resident_per_xcd ? p.per_xcd : resident_per_xcd;
  const unsigned grid = (unsigned)(wg_per_xcd * kNumXcd);
  // a workgroup numbers the k-steps of all its tiles with one 32-bit counter
  if ((p.per_xcd + wg_per_xcd - 1) / wg_per_xcd * L.steps >= ((int64_t)1 << 30)) return VENOM_ERR_UNSUPPORTED;
  const int epi = tokens_major ? 2 : ((bias != nullptr || act != VENOM_ACT_NONE) ? 1 : 0);
  auto fn = var.fn[c_dtype == 1 ? 1 : 0][epi];
  if (var.lds > 64 * 1024) {
    // opting in to more than 64 KB of dynamic LDS is a per-function attribute (set once per device)
    // (two threads racing here both set the same attribute: harmless)
    static std::atomic<bool> opted_in[kNumVariants][6][kMaxDevices] = {};
    const bool cached = dev >= 0 && dev < kMaxDevices;
    if (!cached || !opted_in[variant][3 * c_dtype + epi][dev].load(std::memory_order_acquire)) {
      if (hipFuncSetAttribute(reinterpret_cast<const void*>(fn), hipFuncAttributeMaxDynamicSharedMemorySize,
                              var.lds) != hipSuccess)
        return VENOM_ERR_HIP;
      if (cached) opted_in[variant][3 * c_dtype + epi][dev].store(true, std::memory_order_release);
    }
  }
  const int launch_lds = var.lds;
  hipLaunchKernelGGL(fn, dim3(grid), dim3(var.threads), launch_lds, st, p);
#ifdef VENOM_ABLATE
  if (p.trace && ++trace_calls == atoi(getenv("VENOM_TRACE"))) {
    hipStreamSynchronize(st);
    unsigned long long host[64];
    hipMemcpy(host, p.trace, sizeof(host), hipMemcpyDeviceToHost);
    for (int b = 0; b < 16; b += 5) {
      const double cyc = (double)(host[b * 4 + 2] - host[b * 4 + 0]), ref = (double)(host[b * 4 + 3] - host[b * 4 + 1]);
      fprintf(stderr, "wg %d: %.0f shader ticks, %.0f ref ticks (100 MHz) -> %.3f us, %.1f MHz\n", b, cyc, ref, ref / 100.0,
              cyc / ref * 100.0);
    }
  }
#endif
  return hipGetLastError() == hipSuccess ? VENOM_OK : VENOM_ERR_HIP;
}

// ---------------------------------------------------------------------------------------------
// Activations as a linear layer holds them, X[token][k], to the K x tokens row-major operand the
// gather wants: 64 x 64 tiles through LDS, 4-byte accesses on both sides.
__global__ void __launch_bounds__(256) transpose_tokens_kernel(const uint16_t* __restrict__ X, int64_t ldx, int64_t tokens,
                                                               int64_t K, uint16_t* __restrict__ BT, int64_t ldbt) {
  __shared__ uint16_t tile[64][66];                // [k][token], padded
  const int64_t k0 = (int64_t)blockIdx.x * 64, tok0 = (int64_t)blockIdx.y * 64;
  const int pair = threadIdx.x & 31, sub = threadIdx.x >> 5;
  for (int r = sub; r < 64; r += 8) {               // r: token inside the tile, pair: two k
    const int64_t tok = tok0 + r, k = k0 + 2 * pair;
    uint16_t a = 0, b = 0;
    if (tok < tokens) {
      if (k + 1 < K && ((reinterpret_cast<uintptr_t>(X + tok * ldx + k) & 3) == 0)) {
        const uint32_t w = *reinterpret_cast<const uint32_t*>(X + tok * ldx + k);
        a = (uint16_t)w; b = (uint16_t)(w >> 16);
      } else {
        if (k < K) a = X[tok * ldx + k];
        if (k + 1 < K) b = X[tok * ldx + k + 1];
      }
    }
    tile[2 * pair][r] = a;
    tile[2 * pair + 1][r] = b;
  }
  __syncthreads();
  for (int r = sub; r < 64; r += 8) {               // r: k inside the tile, pair: two tokens
    const int64_t k = k0 + r, tok = tok0 + 2 * pair;
    if (k < K && tok < ldbt) {                       // ldbt is even and >= tokens: pad columns get zeros
      const uint32_t w = (uint32_t)tile[r][2 * pair] | ((uint32_t)tile[r][2 * pair + 1] << 16);
      *reinterpret_cast<uint32_t*>(BT + k * ldbt + tok) = w;
    }
  }
}

hipError_t launch_transpose_tokens(const uint16_t* X, int64_t ldx, int64_t tokens, int64_t K, uint16_t* BT, int64_t ldbt,
                                   hipStream_t st) {
  if (tokens == 0 || K == 0) return hipSuccess;
  hipLaunchKernelGGL(transpose_tokens_kernel, dim3((unsigned)((K + 63) / 64), (unsigned)((ldbt + 63) / 64)), dim3(256), 0,
                     st, X, ldx, tokens, K, BT, ldbt);
  return hipGetLastError();
}

}  // namespace venom
