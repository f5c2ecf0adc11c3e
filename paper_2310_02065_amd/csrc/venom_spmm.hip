// The product kernel: C = A . B with A in V:N:M form (paper section 4: stage 1 loads column-loc,
// the gathered rows of B and the A tile; stage 2 runs the 2:4 matrix instruction; stage 3 stores
// the output through on-chip memory).  Written for gfx950:
//   * the 2:4 inner pattern maps onto v_smfmac_f32_32x32x32_f16: A operand = 8 kept halfs per lane
//     (row = lane%32, four groups), 16 index bits per lane (= four canonical nibbles), B operand =
//     16 halfs per lane (column = lane%32, four groups x the 4 selected rows);
//   * one workgroup owns a V x BSC block of C (BS_r = V as in the paper, so every gathered row of B
//     is shared by all V rows); a k-step is 8 groups = 32 gathered rows of B;
//   * gathered B rows go global -> LDS with 16-byte direct-to-LDS loads, XOR-swizzled per row so the
//     transposing LDS reads (ds_read_b64_tr_b16) that build the B operand do not collide on banks;
//   * values and index words stream from the packed arrays straight into registers, one coalesced
//     16-byte (resp. 4-byte) load per lane;
//   * the block index is remapped so that the 8 XCDs (one L2 each) each walk one column slab of B.
#include "venom_internal.h"

namespace venom {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half16 __attribute__((ext_vector_type(16)));
typedef _Float16 half4 __attribute__((ext_vector_type(4)));
typedef short short4v __attribute__((ext_vector_type(4)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

#define LDS_PTR(T) T __attribute__((address_space(3)))*

struct SpmmParams {
  const uint4* pvalues;
  const uint32_t* pmeta;
  const int32_t* rowidx;
  const _Float16* B;
  void* C;
  int64_t ldb, ldc, Ccols;
  int steps, steps2;
  int nbr, nct;  // block rows, column tiles
  int per_xcd;   // ceil(nbr*nct / 8)
};

constexpr int kNumXcd = 8;

template <int ABID>
__device__ __forceinline__ floatx16 smfmac(half8 a, half16 b, floatx16 c, int idx) {
  return __builtin_amdgcn_smfmac_f32_32x32x32_f16(a, b, c, idx, 0, ABID);
}

// 16-byte slot swizzle of gathered row rho inside its LDS row (slots_per_row is a power of two).
__device__ __forceinline__ int slot_swizzle(int rho, int slots_per_row) { return (4 * (rho & 3)) & (slots_per_row - 1); }

template <int VT, int BSC, int WAVES_R, int WAVES_C, bool OUT_F32>
__global__ void __launch_bounds__(256, 2) spmm_kernel(SpmmParams p) {
  static_assert(WAVES_R * WAVES_C == 4, "four waves per workgroup");
  constexpr int TR = VT / WAVES_R;                 // 32-row tiles per wave
  constexpr int TC = BSC / WAVES_C / 32;           // 32-column tiles per wave
  constexpr int ROW_BYTES = BSC * 2;               // one gathered row of B in LDS
  constexpr int SLOTS = BSC / 8;                   // 16-byte slots per row
  constexpr int RPI = 1024 / ROW_BYTES;            // rows written by one wave-wide direct-to-LDS load
  constexpr int LPR = 64 / RPI;                    // lanes per row (== SLOTS)
  constexpr int NI = kStepRows / RPI;              // loads per k-step for the workgroup
  constexpr int IPW = NI / 4;                      // ... per wave
  static_assert(TR >= 1 && TC >= 1 && IPW >= 1 && LPR == SLOTS, "tile shape");
  constexpr int STAGE_BYTES = kStepRows * ROW_BYTES;
  constexpr int CPAD = 8;                          // halfs of padding per staged output row
  constexpr int CROW = BSC + CPAD;
  constexpr int EPI_BYTES = OUT_F32 ? 0 : VT * 32 * CROW * 2;
  constexpr int LDS_BYTES = (2 * STAGE_BYTES > EPI_BYTES) ? 2 * STAGE_BYTES : EPI_BYTES;
  __shared__ __attribute__((aligned(1024))) char lds[LDS_BYTES];

  // ---- which block of C: consecutive workgroup ids go to different XCDs, so give each XCD a
  // contiguous range of the column-tile-major work list (its L2 then keeps one slab of B hot).
  const int xcd = blockIdx.x % kNumXcd;
  const int work = xcd * p.per_xcd + blockIdx.x / kNumXcd;
  if (work >= p.nbr * p.nct) return;
  const int ct = work / p.nbr, br = work % p.nbr;

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int wr = wave / WAVES_C, wc = wave % WAVES_C;

  // ---- stage-1 addressing: gathered rows of B -> LDS
  const int32_t* ridx = p.rowidx + (int64_t)br * p.steps * kStepRows;
  int ld_rho[IPW];
  int64_t ld_col[IPW];
#pragma unroll
  for (int q = 0; q < IPW; ++q) {
    const int rho = (wave * IPW + q) * RPI + lane / LPR;
    const int chunk = (lane % LPR) ^ slot_swizzle(rho, SLOTS);
    int64_t col = (int64_t)ct * BSC + chunk * 8;
    if (col + 8 > p.Ccols) col = p.Ccols - 8;      // past the edge: any in-bounds data, never stored
    ld_rho[q] = rho;
    ld_col[q] = col;
  }
  auto issue_B = [&](int s, int stage) {
#pragma unroll
    for (int q = 0; q < IPW; ++q) {
      const int64_t row = ridx[s * kStepRows + ld_rho[q]];
      const _Float16* src = p.B + row * p.ldb + ld_col[q];
      LDS_PTR(char) dst = (LDS_PTR(char))(lds + stage * STAGE_BYTES + (wave * IPW + q) * 1024);
      __builtin_amdgcn_global_load_lds((const void*)src, (LDS_PTR(void))dst, 16, 0, 0);
    }
  };

  // ---- stage-1 addressing: A tile (values + index words) -> registers
  const int64_t rt0 = (int64_t)br * VT + wr * TR;
  auto load_A = [&](int s, half8 (&av)[TR]) {
#pragma unroll
    for (int tr = 0; tr < TR; ++tr) {
      const uint4 raw = p.pvalues[((rt0 + tr) * p.steps + s) * 64 + lane];
      av[tr] = __builtin_bit_cast(half8, raw);
    }
  };
  auto load_idx = [&](int s2, int (&ix)[TR]) {
#pragma unroll
    for (int tr = 0; tr < TR; ++tr) ix[tr] = (int)p.pmeta[((rt0 + tr) * p.steps2 + s2) * 64 + lane];
  };

  // ---- stage-2 addressing: transposing LDS reads that build the B operand.
  // Sub-read cb of a 32-column tile: lane block blk = lane/16 reads group t = 4*(cb/2) + 2*(blk/2) + cb%2,
  // 16-column window 2*tile + blk%2; inside the block lane i reads row 4*t + i/4, 8-byte piece i%4.
  int rd_off[TC][4];
  {
    const int blk = lane >> 4, i = lane & 15, e = i >> 2, c8 = i & 3;
#pragma unroll
    for (int tc = 0; tc < TC; ++tc)
#pragma unroll
      for (int cb = 0; cb < 4; ++cb) {
        const int t = 4 * (cb >> 1) + 2 * (blk >> 1) + (cb & 1);
        const int rho = 4 * t + e;
        const int win = (wc * (BSC / WAVES_C) + tc * 32) / 16 + (blk & 1);
        const int slot = (2 * win + (c8 >> 1)) ^ slot_swizzle(rho, SLOTS);
        rd_off[tc][cb] = rho * ROW_BYTES + slot * 16 + (c8 & 1) * 8;
      }
  }

  floatx16 acc[TR][TC];
#pragma unroll
  for (int tr = 0; tr < TR; ++tr)
#pragma unroll
    for (int tc = 0; tc < TC; ++tc)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[tr][tc][v] = 0.f;

  auto compute = [&](int stage, const half8 (&av)[TR], const int (&ix)[TR], auto abid_tag) {
    constexpr int ABID = decltype(abid_tag)::value;
#pragma unroll
    for (int tc = 0; tc < TC; ++tc) {
      half16 bf;
#pragma unroll
      for (int cb = 0; cb < 4; ++cb) {
        const short4v piece = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
            (LDS_PTR(short4v))(lds + stage * STAGE_BYTES + rd_off[tc][cb]));
        const half4 ph = __builtin_bit_cast(half4, piece);
        bf[4 * cb + 0] = ph[0]; bf[4 * cb + 1] = ph[1]; bf[4 * cb + 2] = ph[2]; bf[4 * cb + 3] = ph[3];
      }
#pragma unroll
      for (int tr = 0; tr < TR; ++tr) acc[tr][tc] = smfmac<ABID>(av[tr], bf, acc[tr][tc], ix[tr]);
    }
  };

  // ---- main loop: two LDS stages, the loads of step s+1 in flight while step s computes
  half8 a0[TR], a1[TR];
  int ix[TR];
  issue_B(0, 0);
  load_A(0, a0);
  load_idx(0, ix);
  for (int s = 0; s < p.steps; s += 2) {
    // even step
    __builtin_amdgcn_s_waitcnt(0);  // this wave's direct-to-LDS loads have landed ...
    __syncthreads();                // ... and so have everyone else's; the other stage is free again
    if (s + 1 < p.steps) { issue_B(s + 1, 1); load_A(s + 1, a1); }
    compute(0, a0, ix, std::integral_constant<int, 0>{});
    if (s + 1 >= p.steps) break;
    // odd step
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();
    int ixn[TR];
    if (s + 2 < p.steps) { issue_B(s + 2, 0); load_A(s + 2, a0); load_idx(s / 2 + 1, ixn); }
    compute(1, a1, ix, std::integral_constant<int, 1>{});
    if (s + 2 < p.steps) {
#pragma unroll
      for (int tr = 0; tr < TR; ++tr) ix[tr] = ixn[tr];
    }
  }

  // ---- stage 3: registers -> (LDS) -> global.  Accumulator element v of a 32x32 tile sits at
  // row 8*(v/4) + 4*(lane/32) + v%4, column lane%32.
  const int64_t row0 = (int64_t)br * VT * 32;
  const int64_t col0 = (int64_t)ct * BSC;
  if constexpr (OUT_F32) {
    float* Cf = reinterpret_cast<float*>(p.C);
#pragma unroll
    for (int tr = 0; tr < TR; ++tr)
#pragma unroll
      for (int tc = 0; tc < TC; ++tc) {
        const int64_t col = col0 + wc * (BSC / WAVES_C) + tc * 32 + (lane & 31);
        if (col < p.Ccols) {
#pragma unroll
          for (int v = 0; v < 16; ++v) {
            const int64_t row = row0 + (wr * TR + tr) * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
            Cf[row * p.ldc + col] = acc[tr][tc][v];
          }
        }
      }
  } else {
    __syncthreads();  // every wave is done reading the B stages; reuse the memory
    _Float16* cl = reinterpret_cast<_Float16*>(lds);
#pragma unroll
    for (int tr = 0; tr < TR; ++tr)
#pragma unroll
      for (int tc = 0; tc < TC; ++tc) {
        const int col = wc * (BSC / WAVES_C) + tc * 32 + (lane & 31);
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int row = (wr * TR + tr) * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
          cl[row * CROW + col] = (_Float16)acc[tr][tc][v];  // one rounding, nearest-even
        }
      }
    __syncthreads();
    _Float16* Ch = reinterpret_cast<_Float16*>(p.C);
    constexpr int CHUNKS = BSC / 8;             // 16-byte pieces per row
    constexpr int ROWS_PER_PASS = 256 / CHUNKS;
    const int chunk = threadIdx.x % CHUNKS, rsub = threadIdx.x / CHUNKS;
    const int64_t col = col0 + chunk * 8;
    if (col < p.Ccols) {
#pragma unroll 4
      for (int r = rsub; r < VT * 32; r += ROWS_PER_PASS) {
        const uint4 val = *reinterpret_cast<const uint4*>(cl + r * CROW + chunk * 8);
        *reinterpret_cast<uint4*>(Ch + (row0 + r) * p.ldc + col) = val;
      }
    }
  }
}

// ---------------------------------------------------------------------------------------------
struct Variant {
  const char* name;
  int V;    // block height it serves
  int bsc;  // columns per workgroup
  void (*f16)(SpmmParams);
  void (*f32)(SpmmParams);
};

#define VARIANT(NAME, VT, BSC, WR, WC) \
  { NAME, (VT) * 32, BSC, spmm_kernel<VT, BSC, WR, WC, false>, spmm_kernel<VT, BSC, WR, WC, true> }

static const Variant kVariants[] = {
    VARIANT("v128_c256_w2x2", 4, 256, 2, 2),
    VARIANT("v128_c128_w2x2", 4, 128, 2, 2),
    VARIANT("v64_c256_w2x2", 2, 256, 2, 2),
    VARIANT("v64_c128_w2x2", 2, 128, 2, 2),
    VARIANT("v32_c256_w1x4", 1, 256, 1, 4),
    VARIANT("v32_c128_w1x4", 1, 128, 1, 4),
};
constexpr int kNumVariants = sizeof(kVariants) / sizeof(kVariants[0]);

int spmm_variant_count() { return kNumVariants; }
const char* spmm_variant_name(int v) { return (v >= 0 && v < kNumVariants) ? kVariants[v].name : nullptr; }

static int pick_variant(int V, int64_t Ccols, int64_t nbr) {
  // widest column tile that still gives every CU work; narrow tiles for narrow C
  int best = -1;
  for (int i = 0; i < kNumVariants; ++i) {
    if (kVariants[i].V != V) continue;
    if (best < 0) best = i;
    const int64_t nct = (Ccols + kVariants[i].bsc - 1) / kVariants[i].bsc;
    if (kVariants[i].bsc == 256 && (Ccols >= 256 && nct * nbr >= 512)) return i;
    if (kVariants[i].bsc == 128) return i;
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
  p.pvalues = reinterpret_cast<const uint4*>(h.ws + L.off_pvalues);
  p.pmeta = reinterpret_cast<const uint32_t*>(h.ws + L.off_pmeta);
  p.rowidx = reinterpret_cast<const int32_t*>(h.ws + L.off_rowidx);
  p.B = reinterpret_cast<const _Float16*>(B);
  p.C = C;
  p.ldb = ldb; p.ldc = ldc; p.Ccols = Ccols;
  p.steps = (int)L.steps; p.steps2 = (int)L.steps2;
  const int64_t nct = (Ccols + var.bsc - 1) / var.bsc;
  const int64_t total = nct * L.Rb;
  if (total > (int64_t)1 << 30 || L.steps > (int64_t)1 << 24) return VENOM_ERR_UNSUPPORTED;
  p.nbr = (int)L.Rb; p.nct = (int)nct;
  p.per_xcd = (int)((total + kNumXcd - 1) / kNumXcd);
  const unsigned grid = (unsigned)(p.per_xcd * kNumXcd);
  hipLaunchKernelGGL(c_dtype == 1 ? var.f32 : var.f16, dim3(grid), dim3(256), 0, st, p);
  return hipGetLastError() == hipSuccess ? VENOM_OK : VENOM_ERR_HIP;
}

}  // namespace venom
