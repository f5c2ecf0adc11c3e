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
//     values and index words) and issue matrix instructions.  Four PRODUCER waves, one per SIMD,
//     only move data, by direct-to-LDS loads.  A SIMD issues one wave-wide 16-byte load (1 KB) per
//     ~69 cycles whatever the rest of the compute unit does (measured), so the loads of a k-step --
//     the gathered rows of B, the packed A record, the row ids -- are dealt round-robin over the
//     four producers: every SIMD's share of the vector-memory issue rate is used;
//   * the loads are issued from inline assembly and retired with exact `s_waitcnt vmcnt(n)` counts
//     (loads retire in order per wave); one s_barrier per k-step hands filled stages to the
//     consumers and drained ones back;
//   * the consumers run one k-step behind the loads and refill each operand register from the new
//     stage right after its last use, so no LDS latency sits between two barriers;
//   * workgroups are persistent (one per compute unit): the k-steps of all tiles of a workgroup
//     form one sequence, so the load pipeline runs on across tile boundaries while the consumers
//     store their output;
//   * each XCD (one L2 each) walks a contiguous range of the column-tile-major tile list, so its
//     workgroups share the gathered rows of one slab of B through that L2.
#include <atomic>
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
  int stream_out;          // nonzero: non-temporal stores of C
  int serpentine;          // nonzero: a workgroup's odd tiles run their k-steps backwards, so the end of the
                           // slab of B that the last tile left in L2 is where the next one starts
  int pad_row0;            // first gathered row of a tile's LAST k-step that lies past the end of K (32: none)
  const _Float16* bias;    // one entry per row of C, or null
  int act;                 // venom_activation_t
};

constexpr int kNumXcd = 8;
constexpr int kMaxDevices = 16;      // devices whose per-device launch state is cached
constexpr int kProducers = 4;        // producer waves per workgroup: one per SIMD
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
// wait until at most n of this wave's loads are outstanding, 0 <= n <= MAXN; the steady state
// (n == MAXN) is the first case tested.  The count is an immediate of the instruction, hence the cascade.
template <int MAXN>
__device__ __forceinline__ void wait_loads(int n) {
  static_assert(MAXN <= 63, "vmcnt is a 6-bit counter");
  if (n >= MAXN) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(MAXN) : "memory");
  else if constexpr (MAXN > 0) wait_loads<MAXN - 1>(n);
}
__device__ __forceinline__ void barrier_only() { asm volatile("s_barrier" ::: "memory"); }
// the same once every LDS access of this wave has completed
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
// range of the column-tile-major list, so the workgroups of one XCD sweep the same slab of B and
// a gathered row is fetched from beyond the L2 once for the workgroups that reach it while it is
// resident (measured: all of them while the workgroups run in lock-step, fewer once they drift).
struct TileWalk {
  int base, first, stride, count;
  __device__ __forceinline__ void locate(const SpmmParams& p, int t, int& ct, int& br) const {
    const int work = base + first + t * stride;
    ct = work / p.nbr;
    br = work - ct * p.nbr;
  }
};

// MODE 0: the plain product; 1: fused bias / activation; 2: the same with C written transposed
// (token-major), straight from the accumulators; 3: token-major fp16 through LDS with 16-byte
// stores (needs the output and its leading dimension 16-byte aligned).  Separate instantiations:
// the plain kernel carries none of the epilogue code, and one kernel holding both token-major
// paths behind a run-time branch does not compile (the compiler then keeps the producers' scalar
// operands in vector registers).
// NS: stages of the B ring; NA: records in the A ring.
// D: barriers after which a consumed stage returns to the producers.  The consumers read stage g
// between barriers g and g+1 but use what they read only after barrier g+1.  D = 2: they do not
// wait for those reads before barrier g+1, so the stage stays theirs until barrier g+2 and the
// loads run NS-2 k-steps ahead.  D = 1: they drain their reads before every barrier and the loads
// run NS-1 k-steps ahead.
template <int VT, int NC, int NS, int NA, int D, bool OUT_F32, int MODE>
__global__ void __launch_bounds__((NC + kProducers) * 64, 3) spmm_kernel(SpmmParams p) {
  static_assert(NC == 2 || NC == 4 || NC == 8, "consumer waves per workgroup");
  static_assert(D == 1 || D == 2, "barriers between the hand-over of a stage and its return");
  constexpr bool EPI = MODE != 0;
  static_assert(VT >= 1 && VT <= kMaxTiles, "32-row tiles per block row");
  constexpr int NP = kProducers;
  constexpr int RT = VT;                           // 32-row tiles a consumer wave accumulates
  constexpr int CT = 2;                            // 32-column tiles a consumer wave accumulates
  constexpr int WCOLS = 32 * CT;                   // columns of C per consumer wave
  constexpr int BSC = WCOLS * NC;                  // columns of C per workgroup
  constexpr int ROW_BYTES = 2 * BSC;               // one gathered row of B in LDS
  constexpr int RPI = 1024 / ROW_BYTES;            // rows written by one wave-wide 16-byte load
  constexpr int LPR = 64 / RPI;                    // lanes (= 16-byte slots) per row
  constexpr int NI = kStepRows / RPI;              // B loads per k-step (4 * NC)
  constexpr int CB = NI / NP;                      // ... per producer
  static_assert(NI % NP == 0, "the B loads of a k-step divide evenly over the producers");
  constexpr int B_BYTES = kStepRows * ROW_BYTES;
  constexpr int REC = VT * kTileValBytes + kTailBytes;       // one A record
  constexpr int T_OFF = VT * kTileValBytes;        // record tail: index words
  constexpr int ARING = NS * B_BYTES;              // LDS: [B ring][A ring][row-id ring]
  constexpr int RIDRING = ARING + NA * REC;
  constexpr int NJ = VT + 1;                       // A loads per k-step: VT value blocks + the tail
  constexpr int PB = NS - D;                       // k-steps the B stream runs ahead
  constexpr int PA = NA - D;                       // k-steps the A stream runs ahead
  constexpr int RA = 2 * PB + 2;                   // k-steps the row-id stream runs ahead: the ids of step g+PB+1 are
                                                   // then older, in their producer's load queue, than its loads of step g
  static_assert(PB >= 1 && PA >= PB, "a record is issued no later than the B rows of its k-step");
  static_assert(kRidSlots >= PB + 2, "a row-id slot is rewritten only after its last reader");
  static_assert(NC * 32 * WCOLS * 2 <= B_BYTES, "the output staging of all consumers fits one B stage");

  extern __shared__ __attribute__((aligned(1024))) char smem[];
  const uint32_t lds0 = (uint32_t)(uintptr_t)(LDS_PTR(char))smem;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);

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
  // ("step g is complete in LDS, step g-D is consumed"), and one more after the last step of each
  // tile, after which the consumers stage their output in the B stage they have just drained.
  const int G = tw.count * p.steps;

  if (wave >= NC) {
    // ========================================================================= producers
    // Iteration i (after barrier i) issues, in this order: the row ids of step i+RA, this
    // producer's part of record i+PA, its part of the B rows of step i+PB.  Before barrier g the
    // producer needs its loads of step g and of record g landed (and the row ids of step g+PB):
    // all of them are at least as old as its B loads of step g, so it waits until only the loads
    // of the PB-1 iterations issued since then are outstanding.
    __builtin_amdgcn_s_setprio(3);                 // their few instructions go ahead of the consumers'
    auto produce = [&](auto pj_const) {
      constexpr int PJ = decltype(pj_const)::value;
      constexpr int CA = PJ < NJ ? (NJ - PJ + NP - 1) / NP : 0;   // A loads per k-step: loads PJ, PJ+NP, ...
      constexpr int CR = PJ == NP - 1 ? 1 : 0;                    // the row ids travel with the last producer
      constexpr int L = CA + CR + CB;
      static_assert((PB - 1) * L <= 63, "load counts fit the 6-bit counter");
      // A producer is never ahead of the barrier it is about to meet: every instruction of its loop
      // body lengthens the k-step (a wave issues nothing else while the address unit takes one of
      // its loads, ~70 cycles, and instructions between two loads are not hidden behind them:
      // measured).  So the streams advance by plain increments, ring positions wrap by compare and
      // select, and everything that depends on the tile is recomputed in a branch taken once per tile.
      const uint32_t lane_off = lane * 16;
      int ct, br;
      // ---- record stream: record pointer, LDS slot address, k-steps left in its tile
      tw.locate(p, 0, ct, br);
      const char* a_ptr = p.arec + (int64_t)br * p.steps * p.rec_bytes;
      int64_t a_inc = p.rec_bytes;
      uint32_t a_lds = lds0 + ARING;
      int a_left = p.steps, a_t = 0;
      auto next_record = [&]() {
#pragma unroll
        for (int a = PJ; a < NJ; a += NP) {
          if (a < VT) dma16(a_ptr + a * 1024, lane_off, a_lds + a * 1024);
          else if (lane < kTailBytes / 16) dma16(a_ptr + T_OFF, lane_off, a_lds + T_OFF);   // the 512-byte tail: half a wave
        }
        a_ptr += a_inc;
        a_lds = a_lds + REC == lds0 + ARING + NA * REC ? lds0 + ARING : a_lds + REC;
        if (--a_left == 0) {
          a_left = p.steps;
          if (++a_t < tw.count) {
            tw.locate(p, a_t, ct, br);
            const bool back = p.serpentine && (a_t & 1);       // odd tiles run their k-steps backwards
            a_inc = back ? -p.rec_bytes : p.rec_bytes;
            a_ptr = p.arec + ((int64_t)br * p.steps + (back ? p.steps - 1 : 0)) * p.rec_bytes;
          }
        }
      };
      // ---- row-id stream (producer NP-1 only)
      const char* r_ptr = reinterpret_cast<const char*>(p.rowidx) + (int64_t)br * p.steps * (kStepRows * 4);
      int r_inc = kStepRows * 4;
      uint32_t r_lds = lds0 + RIDRING;
      int r_left = p.steps, r_t = 0;
      auto next_rowids = [&]() {
        if (lane < kStepRows) dma4(r_ptr, lane * 4, r_lds);
        r_ptr += r_inc;
        r_lds = r_lds + kStepRows * 4 == lds0 + RIDRING + kRidSlots * kStepRows * 4 ? lds0 + RIDRING : r_lds + kStepRows * 4;
        if (--r_left == 0) {
          r_left = p.steps;
          if (++r_t < tw.count) {
            int ct2, br2;
            tw.locate(p, r_t, ct2, br2);
            const bool back = p.serpentine && (r_t & 1);
            r_inc = back ? -(kStepRows * 4) : kStepRows * 4;
            r_ptr = reinterpret_cast<const char*>(p.rowidx) +
                    ((int64_t)br2 * p.steps + (back ? p.steps - 1 : 0)) * (kStepRows * 4);
          }
        }
      };
      // ---- B stream.  Load q of this producer is load number PJ + NP*q of the k-step; it covers
      // rows (that number)*RPI .. +RPI-1; lane l writes 16-byte slot l%LPR of row l/LPR and fetches
      // the XOR-swizzled chunk of the gathered row.  A lane reads the id of its row from the row-id
      // ring (one LDS read per load, all of them before the record loads so that their latency is
      // covered) and forms the byte offset with one multiply-add (the host checks the 24-bit ranges).
      int chunk_col[CB];                           // first column of this lane's chunk inside the tile
#pragma unroll
      for (int q = 0; q < CB; ++q) {
        const int rho = (PJ + NP * q) * RPI + lane / LPR;
        chunk_col[q] = ((lane % LPR) ^ slot_swizzle(rho)) * 8;
      }
      uint32_t ld_col[CB];
      auto set_tile = [&](int t) {
        int ct3, br3;
        tw.locate(p, t, ct3, br3);
#pragma unroll
        for (int q = 0; q < CB; ++q) {
          int64_t col = (int64_t)ct3 * BSC + chunk_col[q];
          if (col + 8 > p.Ccols) col = p.Ccols - 8;  // past the edge: any in-bounds data, never stored
          ld_col[q] = (uint32_t)(col * 2);
        }
      };
      const int rowsel = lane / LPR;               // which of the RPI rows of a load this lane writes
      const uint32_t ldb24 = (uint32_t)p.ldb_bytes;
      uint32_t b_lds = lds0 + PJ * 1024;           // this producer's first row in the stage it fills next
      const char* rid_rd = smem + RIDRING + rowsel * 4;   // this lane's entry of the ring slot it reads next
      int b_left = p.steps, b_t = 0;
      set_tile(0);
      int rid[CB];
      auto read_rowids = [&]() {
#pragma unroll
        for (int q = 0; q < CB; ++q) rid[q] = *reinterpret_cast<const int*>(rid_rd + (PJ + NP * q) * RPI * 4);
        rid_rd = rid_rd + kStepRows * 4 == smem + RIDRING + rowsel * 4 + kRidSlots * kStepRows * 4
                     ? smem + RIDRING + rowsel * 4 : rid_rd + kStepRows * 4;
      };
      auto next_rows = [&]() {
        uint32_t off[CB];
#pragma unroll
        for (int q = 0; q < CB; ++q)   // row id x bytes per row + this lane's column bytes, one instruction
          asm("v_mad_u32_u24 %0, %1, %2, %3" : "=v"(off[q]) : "v"(rid[q]), "s"(ldb24), "v"(ld_col[q]));
#pragma unroll
        for (int q = 0; q < CB; ++q) dma16(p.B, off[q], b_lds + q * (NP * 1024));
        b_lds = b_lds + B_BYTES == lds0 + PJ * 1024 + NS * B_BYTES ? lds0 + PJ * 1024 : b_lds + B_BYTES;
        if (--b_left == 0) {
          b_left = p.steps;
          if (++b_t < tw.count) set_tile(b_t);
        }
      };
      // loads this producer issued in each of the last PB-1 iterations (oldest first)
      int issued[PB > 1 ? PB - 1 : 1] = {};
      auto remember = [&](int n) {
#pragma unroll
        for (int k = 0; k + 1 < PB - 1; ++k) issued[k] = issued[k + 1];
        if (PB > 1) issued[PB - 2] = n;
      };
      auto outstanding_after_step = [&]() {
        int n = 0;
#pragma unroll
        for (int k = 0; k < PB - 1; ++k) n += issued[k];
        return n;
      };
      // start-up: the row ids of the first RA steps, then what iterations -PA .. -1 would have issued
      if constexpr (CR != 0)
        for (int j = 0; j < RA && j < G; ++j) next_rowids();
      asm volatile("s_waitcnt vmcnt(0)\n\ts_barrier" ::: "memory");   // the first row ids are on chip
      for (int i = -PA; i < 0; ++i) {
        int n = 0;
        if (i + PA < G) { next_record(); n += CA; }
        if (i + PB >= 0 && i + PB < G) { read_rowids(); next_rows(); n += CB; }
        remember(n);
      }
      const bool ragged = p.pad_row0 < kStepRows;  // K/M is not a multiple of 8
      int c_left = p.steps, c_t = 0;               // k-steps left in the tile the consumers are on / that tile
      // One iteration.  STEADY: all three streams are inside the sequence and have been for PB
      // iterations, so the loads outstanding after those of step g are a compile-time count.
      auto iteration = [&](int g, auto steady_const) {
        constexpr bool STEADY = decltype(steady_const)::value;
        if constexpr (STEADY) asm volatile("s_waitcnt vmcnt(%0)" ::"n"((PB - 1) * L) : "memory");
        else wait_loads<(PB - 1) * L>(outstanding_after_step());
        if (ragged && c_left == ((p.serpentine && (c_t & 1)) ? p.steps : 1)) {
          // The last k-step of a tile when K/M is not a multiple of 8: its trailing groups do not
          // exist.  Their values are zero, but 0 x Inf is not, so the rows gathered for them (row 0
          // of B, a valid address that keeps the load count exact) are overwritten with zeros once
          // they have landed; every producer cleans the rows it loaded itself.
          char* stage = smem + (g % NS) * B_BYTES;
#pragma unroll
          for (int q = 0; q < CB; ++q)
            if ((PJ + NP * q) * RPI + rowsel >= p.pad_row0)
              *reinterpret_cast<uint4*>(stage + (PJ + NP * q) * 1024 + lane * 16) = make_uint4(0, 0, 0, 0);
          lgkm_drained_barrier();
        } else barrier_only();
        // after barrier g the consumers are done with stage g-D and record g-D
        int n = 0;
        const bool rows = STEADY || g + PB < G;
        if (rows) read_rowids();
        if constexpr (CR != 0)
          if (STEADY || g + RA < G) { next_rowids(); n += 1; }
        if (STEADY || g + PA < G) { next_record(); n += CA; }
        if (rows) { next_rows(); n += CB; }
        if constexpr (!STEADY) remember(n);
        if (--c_left == 0) { c_left = p.steps; ++c_t; barrier_only(); }
      };
      int g = 0;
      for (; g < G && g < PB; ++g) iteration(g, std::false_type{});
      if (g + RA < G) {
        for (; g + RA < G; ++g) iteration(g, std::true_type{});
#pragma unroll
        for (int k = 0; k < PB - 1; ++k) issued[k] = L;   // what the steady iterations issued
      }
      for (; g < G; ++g) iteration(g, std::false_type{});
    };
    switch (wave - NC) {
      case 0: produce(std::integral_constant<int, 0>{}); break;
      case 1: produce(std::integral_constant<int, 1>{}); break;
      case 2: produce(std::integral_constant<int, 2>{}); break;
      default: produce(std::integral_constant<int, 3>{}); break;
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
    floatx16 acc[RT][CT];
    half16 bf[CT];                                 // the wave's two 32-column B operands of one k-step
    uint32_t ixw[2];                               // index words of tile rows (0,1) and (2,3): 2 x 16 bits each
    half8 av[RT];                                  // the A operands of one k-step
    auto read_a = [&](const char* sa, int t) {
      av[t] = *reinterpret_cast<const half8*>(sa + t * kTileValBytes + lane * 16);
    };
    auto read_b = [&](const char* sb, int tc) {
#pragma unroll
      for (int cb = 0; cb < 4; ++cb) {
        const short4v piece = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_PTR(short4v))(sb + rd_off[tc][cb]));
        const half4 ph = __builtin_bit_cast(half4, piece);
        bf[tc][4 * cb + 0] = ph[0]; bf[tc][4 * cb + 1] = ph[1]; bf[tc][4 * cb + 2] = ph[2]; bf[tc][4 * cb + 3] = ph[3];
      }
    };
    auto read_ix = [&](const char* sa, int half) {
      ixw[half] = *reinterpret_cast<const uint32_t*>(sa + T_OFF + lane * 8 + 4 * half);
    };
    auto mma = [&](int t, int tc) {
      const int ix = (int)ixw[t >> 1];
      if (t & 1) acc[t][tc] = smfmac<1>(av[t], bf[tc], acc[t][tc], ix);
      else acc[t][tc] = smfmac<0>(av[t], bf[tc], acc[t][tc], ix);
    };
    // after tile row t of the LAST column pass nothing reads av[t] any more, and an index word is
    // free after the last tile row that uses it
    auto refill_after = [&](const char* sa, int t) {
      read_a(sa, t);
      if ((t & 1) == 1 || t == RT - 1) read_ix(sa, t >> 1);
    };
    // In iteration g (after barrier g: stage g and record g are complete) a wave multiplies step
    // g-1 from registers, one column tile after the other, and refills every operand register from
    // stage g as soon as its last matrix instruction has been issued.
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
        sa = smem + ARING + a_slot * REC;
        b_slot = (b_slot + 1) % NS;
        a_slot = a_slot + 1 == NA ? 0 : a_slot + 1;
      };
      // first k-step of the tile: only fetch (same order of reads as in the steady state)
      barrier_only();
      advance();
      read_b(sb, 0);
#pragma unroll
      for (int tr = 0; tr < RT; ++tr) refill_after(sa, tr);
      read_b(sb, 1);
      for (int s = 1; s < p.steps; ++s) {
        if constexpr (D == 1) lgkm_drained_barrier();   // my reads of the last stage are over; this one is complete
        else barrier_only();                            // stage s and record s are complete
        advance();
#pragma unroll
        for (int tc = 0; tc < CT; ++tc) {
#pragma unroll
          for (int tr = 0; tr < RT; ++tr) {
            mma(tr, tc);
            if (tc == CT - 1) refill_after(sa, tr);
            __builtin_amdgcn_sched_barrier(0);
          }
          read_b(sb, tc);
          __builtin_amdgcn_sched_barrier(0);
        }
      }
#pragma unroll
      for (int tc = 0; tc < CT; ++tc)
#pragma unroll
        for (int tr = 0; tr < RT; ++tr) mma(tr, tc);
      lgkm_drained_barrier();                      // every consumer has drained the last B stage

      // ---- stage 3: registers -> (LDS) -> global.  Accumulator element v of a 32x32 tile sits
      // at row 8*(v/4) + 4*(lane/32) + v%4, column lane%32.
      // everything below is per-tile work: its index arithmetic starts from a lane id computed here,
      // so that none of it is hoisted out of the tile loop into registers the k-loop needs
      int ln;
      asm volatile("v_mbcnt_lo_u32_b32 %0, -1, 0\n\tv_mbcnt_hi_u32_b32 %0, -1, %0" : "=v"(ln));
      int ct, br;
      tw.locate(p, t, ct, br);
      const int64_t row0 = (int64_t)br * RT * 32;
      const int64_t col0 = (int64_t)ct * BSC + wave * WCOLS;
      // fused epilogue (the layer's bias, one per output row, then the activation), in fp32 on
      // the accumulators, one 32-row tile at a time right before it is stored: a ln holds rows
      // 8j + 4*(ln/32) + 0..3 of the tile
      auto finish = [&](int tr, int tc_lo = 0, int tc_hi = CT) {   // column tiles tc_lo .. tc_hi-1 of tile row tr
        if constexpr (!EPI) return;                // the plain product compiles without any of this
        if (p.bias) {
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            const half4 b4 = *reinterpret_cast<const half4*>(p.bias + row0 + tr * 32 + 8 * j + 4 * (ln >> 5));
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
              for (int tc = tc_lo; tc < tc_hi; ++tc) acc[tr][tc][4 * j + i] += (float)b4[i];
            __builtin_amdgcn_sched_barrier(0);
          }
        }
        // (scheduling fences keep the evaluations from being interleaved by the dozen: their
        // temporaries would push accumulators out of registers, for the whole kernel)
        if (p.act == VENOM_ACT_GELU) {
#pragma unroll
          for (int tc = tc_lo; tc < tc_hi; ++tc)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
              acc[tr][tc][v] = gelu_by_definition(acc[tr][tc][v]);
              if ((v & 1) == 1) __builtin_amdgcn_sched_barrier(0);
            }
        } else if (p.act == VENOM_ACT_GELU_TANH) {
#pragma unroll
          for (int tc = tc_lo; tc < tc_hi; ++tc)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
              acc[tr][tc][v] = gelu_tanh_form(acc[tr][tc][v]);
              if ((v & 1) == 1) __builtin_amdgcn_sched_barrier(0);
            }
        }
      };
      if constexpr (MODE >= 2) {
        // Token-major output Y[token][feature] = C transposed: a lane owns one column of C (a token)
        // and, per 32-row tile, four runs of 4 consecutive rows (features).
        auto direct = [&]() {
          // each run is one 8-byte (fp16) or 16-byte (fp32) store straight from the accumulators;
          // the two half-waves write neighbouring runs
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
        };
        if constexpr (OUT_F32 || MODE == 2) {
          direct();
        } else {
          // fp16: the 8-byte runs of FT tile rows go through this wave's 4 KB of the drained stage
          // as [token][32*FT features] and leave as 16-byte stores, 64*FT contiguous bytes per
          // token (a full 128-byte line when the block height allows pairs of tile rows).  The
          // 8-byte slots of a staged row are XOR-swizzled by the token so that neighbouring tokens,
          // whose rows lie 64*FT bytes apart, use different banks.
          constexpr int FT = RT % 2 == 0 ? 2 : 1;  // 32-row tiles per pass
          constexpr int RB = 64 * FT;              // bytes of a staged token row
          constexpr int LPT = RB / 16;             // lanes (16-byte chunks) per token row
          constexpr int TPI = 64 / LPT;            // tokens per wave-wide read
          constexpr int SH = FT == 2 ? 1 : 2;      // tokens 2^SH apart share a bank group
          char* stg = const_cast<char*>(sb) + wave * 4096;
          _Float16* Y = reinterpret_cast<_Float16*>(p.C);
          const int h = ln >> 5;
#pragma unroll
          for (int trg = 0; trg < RT / FT; ++trg) {
#pragma unroll
            for (int ps = 0; ps < FT; ++ps) {      // FT = 2: one column tile per pass; FT = 1: both in one pass
#pragma unroll
              for (int trr = 0; trr < FT; ++trr) {   // the epilogue of exactly what this pass stores
                if constexpr (FT == 2) finish(trg * FT + trr, ps, ps + 1);
                else finish(trg * FT + trr);
              }
#pragma unroll
              for (int tc = (FT == 2 ? ps : 0); tc < (FT == 2 ? ps + 1 : CT); ++tc) {
                const int t = (FT == 2 ? 0 : tc * 32) + (ln & 31);
                const int sw = 2 * ((t >> SH) & (LPT - 1));
#pragma unroll
                for (int trr = 0; trr < FT; ++trr)
#pragma unroll
                  for (int q = 0; q < 4; ++q) {
                    const int tr = trg * FT + trr;
                    const half4 o = {(_Float16)acc[tr][tc][4 * q], (_Float16)acc[tr][tc][4 * q + 1],
                                     (_Float16)acc[tr][tc][4 * q + 2], (_Float16)acc[tr][tc][4 * q + 3]};
                    const int slot = trr * 8 + 2 * q + h;
                    *reinterpret_cast<half4*>(stg + t * RB + ((slot ^ sw) * 8)) = o;
                  }
              }
#pragma unroll
              for (int i = 0; i < (64 / FT) / TPI; ++i) {
                const int tt = i * TPI + ln / LPT, c = ln % LPT;
                const uint4 val = *reinterpret_cast<const uint4*>(stg + tt * RB + ((c ^ ((tt >> SH) & (LPT - 1))) * 16));
                const int64_t tok = col0 + (FT == 2 ? ps * 32 : 0) + tt;
                if (tok < p.Ccols) {
                  typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
                  const u32x4 v4 = {val.x, val.y, val.z, val.w};
                  *reinterpret_cast<u32x4*>(Y + tok * p.ldc + row0 + trg * FT * 32 + c * 8) = v4;
                }
              }
            }
            __builtin_amdgcn_sched_barrier(0);
          }
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
}

// ---------------------------------------------------------------------------------------------
struct Variant {
  const char* name;
  int V;       // block height it serves
  int bsc;     // columns per workgroup
  int threads;
  int lds;     // dynamic LDS bytes
  void (*fn[2][4])(SpmmParams);   // [fp32 output][mode]
};

template <int VT, int NC, int NS, int NA>
constexpr int lds_bytes() {   // B ring, A ring, row-id ring (the output staging reuses a B stage)
  return NS * kStepRows * 128 * NC + NA * (VT * kTileValBytes + kTailBytes) + kRidSlots * kStepRows * 4;
}

#define VARIANT(NAME, VT, NC, NS, NA, D)                                                                  \
  { NAME, (VT) * 32, 64 * (NC), 64 * ((NC) + kProducers), lds_bytes<VT, NC, NS, NA>(),                     \
    { { spmm_kernel<VT, NC, NS, NA, D, false, 0>, spmm_kernel<VT, NC, NS, NA, D, false, 1>,               \
        spmm_kernel<VT, NC, NS, NA, D, false, 2>, spmm_kernel<VT, NC, NS, NA, D, false, 3> },             \
      { spmm_kernel<VT, NC, NS, NA, D, true, 0>, spmm_kernel<VT, NC, NS, NA, D, true, 1>,                 \
        spmm_kernel<VT, NC, NS, NA, D, true, 2>, spmm_kernel<VT, NC, NS, NA, D, true, 2> } } }

constexpr int kD = 2;   // barriers between the hand-over of a stage and its return (1 and 2 measure the same)
static const Variant kVariants[] = {
    VARIANT("v128_c512", 4, 8, 4, 6, kD), VARIANT("v128_c256", 4, 4, 6, 10, kD), VARIANT("v128_c128", 4, 2, 8, 10, kD),
    VARIANT("v96_c512", 3, 8, 4, 8, kD),  VARIANT("v96_c256", 3, 4, 6, 10, kD), VARIANT("v96_c128", 3, 2, 8, 10, kD),
    VARIANT("v64_c512", 2, 8, 4, 10, kD), VARIANT("v64_c256", 2, 4, 6, 10, kD), VARIANT("v64_c128", 2, 2, 8, 10, kD),
    VARIANT("v32_c512", 1, 8, 4, 10, kD), VARIANT("v32_c256", 1, 4, 6, 10, kD), VARIANT("v32_c128", 1, 2, 8, 10, kD),
};
constexpr int kNumVariants = sizeof(kVariants) / sizeof(kVariants[0]);

int spmm_variant_count() { return kNumVariants; }
const char* spmm_variant_name(int v) { return (v >= 0 && v < kNumVariants) ? kVariants[v].name : nullptr; }

static int pick_variant(int V, int64_t Ccols, int64_t nbr) {
  // The widest column tile that C fills at least half of: wide tiles re-read the A stream least
  // and measured fastest at every large shape tried; narrow C takes the narrow tiles.  When that
  // choice leaves more than half of the compute units without a tile (few block rows), the
  // 256-column tile spreads the work over twice as many units.
  int best = -1;
  for (int i = 0; i < kNumVariants; ++i) {
    if (kVariants[i].V != V) continue;
    if (best < 0) { best = i; continue; }
    const bool fits_i = 2 * Ccols > kVariants[i].bsc, fits_b = 2 * Ccols > kVariants[best].bsc;
    if (fits_i && (!fits_b || kVariants[i].bsc > kVariants[best].bsc)) best = i;
    else if (!fits_i && !fits_b && kVariants[i].bsc < kVariants[best].bsc) best = i;
  }
  if (best >= 0 && kVariants[best].bsc == 512) {
    const int64_t tiles = nbr * ((Ccols + 511) / 512);
    if (tiles <= 128)
      for (int i = 0; i < kNumVariants; ++i)
        if (kVariants[i].V == V && kVariants[i].bsc == 256) best = i;
  }
  return best;
}

venom_status_t launch_spmm(const venom_handle& h, const void* B, int64_t ldb, int64_t Ccols, const void* bias, int act,
                           void* C, int64_t ldc, int c_dtype, int tokens_major, int variant, hipStream_t st) {
  const Layout& L = h.lay;
  if (!L.packed) return VENOM_ERR_UNSUPPORTED;
  if (L.R == 0 || Ccols == 0) return VENOM_OK;
  if (L.steps == 0) return VENOM_ERR_UNSUPPORTED;  // K = 0: there is no k-step to run the pipeline on
  const int Vp = L.vt * kTileRows;                 // block height of the packed copy
  if (variant < 0) variant = pick_variant(Vp, Ccols, L.Rbp);
  if (variant < 0 || variant >= kNumVariants || kVariants[variant].V != Vp) return VENOM_ERR_UNSUPPORTED;
  const Variant& var = kVariants[variant];
  SpmmParams p{};
  p.arec = h.ws + L.off_arec;
  p.rowidx = reinterpret_cast<const int32_t*>(h.ws + L.off_rowidx);
  p.B = reinterpret_cast<const char*>(B);
  p.C = C;
  p.ldb_bytes = ldb * 2; p.ldc = ldc; p.Ccols = Ccols; p.rec_bytes = L.rec_bytes;
  p.steps = (int)L.steps;
  p.bias = reinterpret_cast<const _Float16*>(bias);
  p.act = act;
  p.serpentine = 1;
  p.pad_row0 = (L.G % kStepGroups) ? (int)(L.G % kStepGroups) * kSelCols : kStepRows;
  p.stream_out = L.steps >= 32;   // measured: +3 % at 48 k-steps per tile, -20 % at 8
  const int64_t nct = (Ccols + var.bsc - 1) / var.bsc;
  const int64_t nbr = L.Rbp;
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
  // token-major fp16 output takes the staged path when 16-byte stores are possible
  const bool wide = tokens_major && c_dtype == 0 && reinterpret_cast<uintptr_t>(C) % 16 == 0 && ldc % 8 == 0;
  const int epi = tokens_major ? (wide ? 3 : 2) : ((bias != nullptr || act != VENOM_ACT_NONE) ? 1 : 0);
  auto fn = var.fn[c_dtype == 1 ? 1 : 0][epi];
  if (var.lds > 64 * 1024) {
    // opting in to more than 64 KB of dynamic LDS is a per-function attribute (set once per device)
    // (two threads racing here both set the same attribute: harmless)
    static std::atomic<bool> opted_in[kNumVariants][8][kMaxDevices] = {};
    const bool cached = dev >= 0 && dev < kMaxDevices;
    if (!cached || !opted_in[variant][4 * c_dtype + epi][dev].load(std::memory_order_acquire)) {
      if (hipFuncSetAttribute(reinterpret_cast<const void*>(fn), hipFuncAttributeMaxDynamicSharedMemorySize,
                              var.lds) != hipSuccess)
        return VENOM_ERR_HIP;
      if (cached) opted_in[variant][4 * c_dtype + epi][dev].store(true, std::memory_order_release);
    }
  }
  hipLaunchKernelGGL(fn, dim3(grid), dim3(var.threads), var.lds, st, p);
  return hipGetLastError() == hipSuccess ? VENOM_OK : VENOM_ERR_HIP;
}

// ---------------------------------------------------------------------------------------------
// The 2:4 matrix instruction alone: every wave issues `iters` x 8 independent instructions on
// register operands (pseudo-random fp16 values, so the multipliers toggle as they do on real data).
// Timed by the caller, it gives the instruction peak this GPU sustains at the clock it holds under
// that load: iters * 8 * 32768 useful FLOP per wave, 8 waves x 2 workgroups per compute unit.
__global__ void __launch_bounds__(512) smfmac_probe_kernel(int iters, float* sink) {
  const unsigned lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  unsigned x = (blockIdx.x * 8 + wave) * 64 + lane;
  auto next_half = [&]() {
    x = x * 1664525u + 1013904223u;
    return (_Float16)((float)((x >> 9) & 0xfff) * (1.f / 2048.f) - 1.f);      // in [-1, 1)
  };
  half8 a; half16 b;
  for (int e = 0; e < 8; ++e) a[e] = next_half();
  for (int e = 0; e < 16; ++e) b[e] = next_half();
  const int idx = 0x4e944e94 ^ (int)((lane & 1) * 0x00900090);                 // legal nibbles only
  floatx16 acc[8] = {};
  for (int i = 0; i < iters; ++i) {
#pragma unroll
    for (int j = 0; j < 8; ++j) acc[j] = smfmac<0>(a, b, acc[j], idx);
  }
  float s = 0.f;
  for (int j = 0; j < 8; ++j) s += acc[j][0];
  if (s == 12345.678f) sink[0] = s;              // keeps the loop alive; practically never true
}

hipError_t launch_smfmac_probe(int iters, float* sink, hipStream_t st) {
  int dev = 0, cus = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e == hipSuccess) e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(smfmac_probe_kernel, dim3(2 * cus), dim3(512), 0, st, iters, sink);
  return hipGetLastError();
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

// The same with 16-byte accesses on both sides, for X, BT and both leading dimensions 16-byte
// aligned and K a multiple of 8: a thread loads 8 consecutive k of a token, the tile sits in LDS as
// [token][k] with rows of 136 bytes (so that the column reads below spread over the banks), and a
// thread gathers 8 consecutive tokens of one k for its store; 8 lanes write 128 contiguous bytes.
__global__ void __launch_bounds__(256) transpose_tokens_wide_kernel(const uint16_t* __restrict__ X, int64_t ldx,
                                                                    int64_t tokens, int64_t K,
                                                                    uint16_t* __restrict__ BT, int64_t ldbt) {
  constexpr int kPitch = 136;                      // bytes per token row in LDS
  __shared__ __attribute__((aligned(16))) char tile[64 * kPitch];
  const int64_t k0 = (int64_t)blockIdx.x * 64, tok0 = (int64_t)blockIdx.y * 64;
  const int c = threadIdx.x & 7, r = threadIdx.x >> 3;
#pragma unroll
  for (int j = 0; j < 2; ++j) {                    // token r + 32j, k chunk c
    const int64_t tok = tok0 + r + 32 * j, k = k0 + 8 * c;
    uint4 w = make_uint4(0, 0, 0, 0);
    if (tok < tokens && k < K) w = *reinterpret_cast<const uint4*>(X + tok * ldx + k);
    uint2* dst = reinterpret_cast<uint2*>(tile + (r + 32 * j) * kPitch + c * 16);
    dst[0] = make_uint2(w.x, w.y);
    dst[1] = make_uint2(w.z, w.w);
  }
  __syncthreads();
#pragma unroll
  for (int j = 0; j < 2; ++j) {                    // k row r + 32j, token chunk c
    const int kr = r + 32 * j;
    const int64_t k = k0 + kr, tok = tok0 + 8 * c;
    uint32_t o[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const uint32_t lo = *reinterpret_cast<const uint16_t*>(tile + (8 * c + 2 * e) * kPitch + kr * 2);
      const uint32_t hi = *reinterpret_cast<const uint16_t*>(tile + (8 * c + 2 * e + 1) * kPitch + kr * 2);
      o[e] = lo | (hi << 16);
    }
    if (k < K && tok < ldbt) *reinterpret_cast<uint4*>(BT + k * ldbt + tok) = make_uint4(o[0], o[1], o[2], o[3]);
  }
}

hipError_t launch_transpose_tokens(const uint16_t* X, int64_t ldx, int64_t tokens, int64_t K, uint16_t* BT, int64_t ldbt,
                                   hipStream_t st) {
  if (tokens == 0 || K == 0) return hipSuccess;
  if (reinterpret_cast<uintptr_t>(X) % 16 == 0 && reinterpret_cast<uintptr_t>(BT) % 16 == 0 && ldx % 8 == 0 &&
      ldbt % 8 == 0 && K % 8 == 0) {
    hipLaunchKernelGGL(transpose_tokens_wide_kernel, dim3((unsigned)((K + 63) / 64), (unsigned)((ldbt + 63) / 64)), dim3(256),
                       0, st, X, ldx, tokens, K, BT, ldbt);
    return hipGetLastError();
  }
  hipLaunchKernelGGL(transpose_tokens_kernel, dim3((unsigned)((K + 63) / 64), (unsigned)((ldbt + 63) / 64)), dim3(256), 0,
                     st, X, ldx, tokens, K, BT, ldbt);
  return hipGetLastError();
}

}  // namespace venom
