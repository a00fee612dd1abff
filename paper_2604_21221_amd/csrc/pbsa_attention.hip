// PBSA fine stage (Eq. 3-5) for gfx950: block-sparse flash attention on bf16 MFMA.
//
// One workgroup = 2 waves = 128 consecutive query tokens of one head (one query block when B = 128,
// two when B = 64).  Wave w owns rows 64 w .. 64 w + 63 of the workgroup as two row groups of 32, so
// with B = 64 a wave is exactly one query block.  Two workgroups share a CU, one wave per SIMD, so a
// wave has the whole 512-entry register file of its SIMD.
//
// The workgroup walks a list of 64-key tiles: every non-empty persistent slot (the dense part of the
// mask, visible to all rows) and the union of the local blocks selected by its query blocks, sorted by
// who attends a tile:
//   shared  full tiles both waves attend, then the ragged tiles (fewer than 64 valid keys, masked per
//           wave).  The waves stage each tile together, two tiles per operand in flight, and meet at a
//           barrier once per tile.
//   solo    full tiles only one wave attends (B = 64: a block one query block selected and its
//           neighbour did not).  After the shared part each wave streams its own tiles through its own
//           half of the LDS in 32-key halves, with no barrier: both waves run at full width on different
//           tiles, and since every query block selects the same number of blocks the two waves, and all
//           workgroups, have the same amount of work however the selections overlap.
// The order of keys does not matter to an online softmax.  K/V tiles go from global memory straight
// into LDS (global_load_lds, no register round trip).
//
// MFMA arrangement (v_mfma_f32_32x32x16_bf16, wave64):
//   S^T = K Q^T   A = K tile rows (32 keys x 16 dims), B = Q^T (16 dims x 32 query rows).
//                 The accumulator then holds, per lane, 16 keys of ONE query row (column lane%32),
//                 so the softmax row reductions are in-lane plus one exchange with lane^32.
//   O^T = V^T P^T A = V^T (32 dims x 16 keys), B = P^T (16 keys x 32 query rows) taken straight
//                 from the S^T accumulators: the contraction index (key) is enumerated in the order
//                 the accumulator holds it, and V^T is read from LDS with the same enumeration.
//   A K or V^T fragment read from LDS feeds the MFMAs of both row groups, which halves the LDS
//   traffic per flop.  (At one fragment per MFMA -- 32 rows per wave, two waves per SIMD -- four matrix
//   pipes ask the LDS for 128 bytes per clock, about half of what it delivers to reads alone; with the
//   staging loads and the barrier beside them that arrangement measured no faster in a probe, and it
//   needs the whole step in 256 registers.)
//
// Software pipeline.  The unit is a sub-tile of 32 keys.  In step u a wave runs, as one straight
// stretch of code cut into slots (one MFMA plus a slice of vector work each), the softmax of
// sub-tile u (one fma and one exp2 per score, one conversion per pair; S^T(u) -> P^T(u)) together with
// the MFMAs that do not depend on it: O^T += V^T P^T of sub-tile u-1 and S^T = K Q^T of sub-tile u+1.
// S^T and P^T are double buffered.  Each part of the list (shared full, shared ragged, solo) is one
// pipelined run with its own template instance; the pipeline drains between them.  Softmax is online,
// fp32, base 2 (scale and log2 e folded into one fma), against a reference that a step takes as given.
// The row sums (over the bf16-rounded probabilities, the numbers the second product uses) are four small
// MFMAs per step whose A operand selects the rows (sum_mfma); the check that the reference still serves is
// one OR per two pairs inside the slots and one compare at the end of the step, and the rare step that
// fails it is redone in place (softmax_redo).  A step loads the first operand fragments of the step after
// it during its last slots and hands them over in registers, so no step starts by waiting for LDS; the
// barrier that turns the rings over sits in the middle of a tile's second step, under its MFMAs.
#include <type_traits>

#include "pbsa_internal.h"
#include "pbsa_plan_device.h"

namespace pbsa {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

constexpr int kThreads = 128;
constexpr int kRowsPerWg = 128;
constexpr int kTile = 64;                 // keys per staged tile
// persistent + local 64-key tiles: of the plain attention call, and of the variants that also score or take decisions
constexpr int kMaxTiles = 2 * (PBSA_MAX_C_ATTEND + 1) + 2 * PBSA_MAX_N_LOC;
constexpr int kMaxTilesAux = 2 * (PBSA_MAX_C_AUX + 1) + 2 * PBSA_MAX_N_LOC_AUX;
constexpr float kMasked = -1.0e30f;        // score of a key that does not exist
constexpr float kInitMax = -1.0e29f;       // reference of a row that has seen no key: above kMasked, below any score
// The softmax reference of a row is not its running max: probabilities only have to stay inside the
// exponent range of bf16 / fp32, whose precision is relative.  The reference is set kLift base-2
// exponent units above the row max of the sub-tile that sets it and is then used as it stands: a step
// computes no row maximum.  Whether a reference still serves is read off the exponent fields of the rounded
// probabilities: as long as every probability is below 2, the top exponent bit of every bf16 pattern is
// clear, so the bitwise OR of all the pairs of a sub-tile has it clear in both halves; a probability of 2 or
// more, an infinity or a NaN sets it (one three-input OR per two pairs, no false alarms).  Only then is the
// sub-tile's softmax redone with a new reference and the output accumulators rescaled (softmax_redo).
// Probabilities thus lie between 2^-126 and 2, a key more than 126 - kLift units below the score that set
// the reference contributes nothing (less than 2^-46 of that score's weight), and after the first sub-tile
// of a row a new reference needs scores that rise by a factor of 2^kLift.
constexpr float kLift = 80.0f;
constexpr uint32_t kTooBig = 0x40004000u;  // the top exponent bit of both halves of a bf16 pair

__device__ __forceinline__ int lanes_below(unsigned long long mask) {   // set bits of `mask` below this lane
  return __builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0u));
}

struct AttnArgs {
  int H, Nq, nqb, n_loc, n_loc_cap, C, k;
  float scale;
  long q_stride_h, q_stride_t, o_stride_h, o_stride_t;
  const bf16_t* Q;
  const bf16_t* Kp;
  const bf16_t* Vp;
  const int32_t* p_len;
  const bf16_t* Kl;
  const bf16_t* Vl;
  const int32_t* l_len;
  const int32_t* l_map;
  const int32_t* sel;
  bf16_t* O;
  float* lse;
  // mass variant only: per workgroup the tile list, per wave and sub-tile the row sums (see MassOut)
  float* R;
  int32_t* Rlist;
  int r_slots, list_cap;
};

// LDS layout of a 64-key tile: unpadded rows of D bf16 whose 16-byte chunks are permuted within the
// row (logical chunk c of row r sits at chunk c ^ f(r)).  The permutation is applied on the way in
// by choosing which global chunk each lane of a global_load_lds fetches (a wave instruction fills
// 1 KiB of consecutive LDS bytes), and again when the MFMA operands are read:
//  K (ds_read_b128, 16 consecutive rows at one logical chunk per quarter wave): f(r) = r mod (D/8),
//    so the 16 reads land in 16 distinct chunks.
//  V (ds_read_b64_tr_b16: within 16 lanes, lane s supplies the address of row s/4, columns
//    4(s%4)..+3, and lane j receives column j of those 4 rows): the 4 rows x 64 bytes a half wave
//    reads must cover all 64 banks: D = 128: f(r) = 4 (r mod 4); D = 64: f(r) = 4 ((r/2) mod 2).
// Both f are unchanged by adding a multiple of 8 to the row, so a lane's address within a tile is one
// per-lane base plus compile-time offsets for the sub-tile, the k-step and the row pair.
template <int D>
__device__ __forceinline__ int k_swz(int row) { return row & (D / 8 - 1); }
template <int D>
__device__ __forceinline__ int v_swz(int row) {
  if constexpr (D == 128) return (row & 3) << 2;
  else return ((row >> 1) & 1) << 2;
}

// One wave-wide global -> LDS load of 16 bytes per lane: LDS bytes [lds_off, lds_off + 1024) receive
// lane i's 16 bytes at lds_off + 16 i.  Completion is tracked by the issuing wave's vmcnt.
// The global address is a scalar base plus a 32-bit per-lane byte offset.
__device__ __forceinline__ void dma16(const void* base, uint32_t lane_off, uint32_t lds_off) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
               :
               : "s"(lds_off), "v"(lane_off), "s"(base)
               : "memory", "m0");
}
// Four such loads of consecutive KiB: the instruction's offset field moves the LDS address and the
// global address alike, so one setting of M0 and one scalar base serve four loads whose sources are
// 1 KiB apart like their destinations (lane offsets o0..o3 are relative to those steps).  A load costs
// the issuing wave about 20 cycles with its own M0 setting and base, which is why they come in fours.
template <int LDS_IMM>
__device__ __forceinline__ void dma16x4(const void* base, uint32_t o0, uint32_t o1, uint32_t o2, uint32_t o3,
                                        uint32_t lds_base) {
  asm volatile("s_add_u32 m0, %0, %6\n\ts_nop 0\n\t"
               "global_load_lds_dwordx4 %1, %5\n\t"
               "global_load_lds_dwordx4 %2, %5 offset:1024\n\t"
               "global_load_lds_dwordx4 %3, %5 offset:2048\n\t"
               "global_load_lds_dwordx4 %4, %5 offset:3072"
               :
               : "s"(lds_base), "v"(o0), "v"(o1), "v"(o2), "v"(o3), "s"(base), "n"(LDS_IMM)
               : "memory", "scc", "m0");
}

template <int D>
struct Geo {
  static constexpr int KS = D / 16;                 // MFMA k-steps of Q K^T
  static constexpr int DT = D / 32;                 // 32-wide output tiles of O^T
  static constexpr int ROW = D * 2;                 // bytes of a tile row
  static constexpr int TILE_BYTES = kTile * D * 2;  // one K or V tile in LDS
  static constexpr int SUB_BYTES = 32 * D * 2;      // a 32-key sub-tile
};

typedef __attribute__((address_space(3))) const bf16x8* lds_b128_t;
typedef __attribute__((address_space(3))) bf16x4* lds_tr_t;

__device__ __forceinline__ bf16x8 lds_read_k(uint32_t addr) { return *(lds_b128_t)(uintptr_t)addr; }
// V^T fragment of 16 keys: two transposing reads, rows r and r + 8 of the 16
template <int ROW>
__device__ __forceinline__ bf16x8 lds_read_vt(uint32_t addr) {
  const bf16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_tr_t)(uintptr_t)addr);
  const bf16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_tr_t)(uintptr_t)(addr + 8 * ROW));
  return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
}
// P^T is kept as single registers (a bf16 pair each), put together into an operand where an MFMA uses them: the
// rare redo of a sub-tile's softmax rewrites them, and whole-vector values merged after that branch cost the common
// path a register copy per element
typedef uint32_t PTile[2][2][4];
__device__ __forceinline__ bf16x8 as_bf16x8(const uint32_t (&w)[4]) {
  const u32x4 v = {w[0], w[1], w[2], w[3]};
  return __builtin_bit_cast(bf16x8, v);
}

// O^T accumulators live in the accumulator half of the register file for the whole kernel: the
// second product is issued as an instruction with an accumulator-register destination, so the
// architectural half is left to S^T, P^T, the operand fragments and the softmax.  The compiler does
// not see a matrix instruction here: code that reads or rewrites these accumulators with vector
// instructions waits out the matrix pipeline itself (acc_settle).
__device__ __forceinline__ void pv_mfma(f32x16& acc, const bf16x8& a, const bf16x8& b) {
  asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+a"(acc) : "v"(a), "v"(b));
}
// The wait is tied to the accumulators it protects, so their reads and writes cannot be moved across it.
template <int DT>
__device__ __forceinline__ void acc_settle(f32x16 (&o)[DT]) {
  static_assert(DT == 2 || DT == 4, "two or four output tiles per row group");
  if constexpr (DT == 4)
    asm volatile("s_nop 15\n\ts_nop 15" : "+a"(o[0]), "+a"(o[1]), "+a"(o[2]), "+a"(o[3]));
  else
    asm volatile("s_nop 15\n\ts_nop 15" : "+a"(o[0]), "+a"(o[1]));
}

// max over the 16 keys a lane holds of one row, then with the other half-wave's 16.  The three-input
// maximum is written as the instruction: fmaxf would first quiet each input (a move per input), and no
// NaN can be here -- scores of existing keys are finite and the others have been replaced.
__device__ __forceinline__ float max3(float a, float b, float c) {
  float r;
  asm("v_max3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
  return r;
}
__device__ __forceinline__ float row_max(const f32x16& s) {
  float t = max3(s[0], s[1], s[2]);
#pragma unroll
  for (int v = 3; v < 15; v += 2) t = max3(t, s[v], s[v + 1]);
  t = max3(t, s[15], s[15]);
  const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(t), __float_as_uint(t), false, false);
  return max3(__uint_as_float(r[0]), __uint_as_float(r[1]), __uint_as_float(r[1]));
}

// The probabilities of two neighbouring keys: exp2 of each score, then the two rounded to a bf16 pair.
// The pipeline steps issue the stages in different slots so that none waits for the one before.
__device__ __forceinline__ float prob_exp(float s, float c2, float mc) { return __builtin_amdgcn_exp2f(__builtin_fmaf(s, c2, mc)); }
__device__ __forceinline__ uint32_t prob_round(float e0, float e1) {
  bf16x2 pk;
  pk[0] = (__bf16)e0;
  pk[1] = (__bf16)e1;
  return __builtin_bit_cast(uint32_t, pk);
}
// Row sums are taken over the rounded values, the numbers the second product uses, by the matrix pipe: one
// v_mfma_f32_16x16x32_bf16 per row group and 16 keys, whose B operand is the P^T operand of the second product
// as it stands and whose A operand selects.  That instruction reads lane L's eight values as column L % 16,
// contraction indices 8 (L / 16) ..: of the 32 query rows of a row group (row = L % 32, keys split over the two
// half waves) rows r and r + 16 fall into the same column r % 16, on contraction groups {0, 2} and {1, 3}.  With
// A[m0][k] = 1 on groups 0 and 2, A[m0 + 4][k] = 1 on groups 1 and 3 and zero elsewhere, output row m0 holds the
// sums of rows 0..15 and output row m0 + 4 those of rows 16..31, and the instruction leaves output row m in element
// m % 4 of lanes 16 (m / 4) ..+15: with m0 = 8 g for row group g, element 0 of the result holds, in lane L, the
// complete sum (all 16 keys, both half waves) of row L % 32 of row group L / 32 -- one register for the wave's 64
// rows, the other three elements stay zero.  Four instructions of 16 cycles per 32-key sub-tile, against sixteen
// v_dot2c_f32_bf16 (which also run in the matrix pipe and stall the wave) or thirty-two additions the vector unit
// has no slots for.
typedef __attribute__((ext_vector_type(4))) float f32x4;
__device__ __forceinline__ bf16x8 sum_selector(int lane, int g) {
  const int m = lane & 15, kg = lane >> 4;
  const bool on = (m == 8 * g && (kg & 1) == 0) || (m == 8 * g + 4 && (kg & 1) == 1);
  const uint32_t w = on ? 0x3F803F80u : 0u;
  const u32x4 v = {w, w, w, w};
  return __builtin_bit_cast(bf16x8, v);
}
// The instruction is written out so that its result register is its accumulator input (an MFMA's destination
// must be the same registers as its addend or none of them; with the addend in the architectural half of the
// register file the compiler's register assignment has let the two overlap by part).  The compiler does not
// see a matrix instruction here: vector code that reads or rewrites the sums waits out the matrix pipe itself
// (sum_settle).
__device__ __forceinline__ void sum_mfma(f32x4& acc, const bf16x8& sel, const bf16x8& p) {
  asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+v"(acc) : "v"(sel), "v"(p));
}
__device__ __forceinline__ void sum_settle(f32x4& l) {
  asm volatile("s_nop 15\n\ts_nop 7" : "+v"(l));
}
__device__ __forceinline__ uint32_t or3(uint32_t a, uint32_t b, uint32_t c) {
  uint32_t r;
  asm("v_or3_b32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
  return r;
}
template <int DT>
__device__ __forceinline__ void rescale(f32x16 (&o)[2][DT], const float (&alpha)[2]) {
#pragma unroll
  for (int g = 0; g < 2; ++g) {
    if (__any(alpha[g] != 1.0f)) {
      acc_settle<DT>(o[g]);
#pragma unroll
      for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int v = 0; v < 16; ++v) o[g][dt][v] *= alpha[g];
      acc_settle<DT>(o[g]);
    }
  }
}

// ------------------------------------------------------------------------------------------------
// One pipeline step: up to three parts on three different sub-tiles, for both row groups of the wave.
//   SM  softmax of the current sub-tile: s_cur -> p_cur (RAGGED: keys at or beyond lim[g] are masked)
//   PV  O^T += V^T P^T of the previous sub-tile (p_prev, V fragments at vaddr + V_OFF)
//   QK  S^T = K Q^T of the next sub-tile (s_next, K fragments at kaddr + K_OFF)
// The step is a sequence of MFMA pairs, PV and QK alternating when both are present; the MFMAs of a
// pair (one per row group) share one LDS fragment, read kAhead pairs earlier.  After every MFMA comes
// a slice of the softmax, so the matrix pipe works while the VALU computes.  Nothing is allowed to
// move across slot boundaries.
// ------------------------------------------------------------------------------------------------
// Staging loads that ride along a pipeline step, in bursts of four wave instructions (4 KiB: 16 rows at
// D = 128) at a few slots of the step's first half; spread out like this they travel while the wave
// computes.  A plan names what one wave loads during one step, always 32 tile rows per operand:
//   shared part: this wave's half (rows 32 w ..) of K of tile t+2 and of V of tile t+1
//   solo part:   the 32-key halves K(u+2) and V(u) of its own tiles, into its own ring entries
template <int D>
struct DmaPlan {
  static constexpr int CH = D / 8, RPI = 64 / CH;   // 16-byte chunks per row, rows per wave instruction
  static constexpr int NIW = 32 / RPI;               // wave instructions (1 KiB pieces) per 32 rows
  static constexpr int NW = NIW / 4;                 // bursts per operand
  static constexpr int NB = 2 * NW;                  // bursts per step: K and V of each 4 KiB window
  const unsigned char* kp;    // source of the first of the 32 rows
  const unsigned char* vp;
  const unsigned char* vtile; // ragged V tile: its first row
  uint32_t klds, vlds;        // LDS address the first row goes to
  int kpat[4];                // per lane: source byte offset within piece k of a window (the K permutation has
                              // a period of 16 rows, at most the window)
  int vpat;                   // per lane: source byte offset within any V piece
  bool vragged;               // the V tile has fewer than 64 valid rows: rows past them must not reach LDS
  int voff[NIW];              // then, per lane: source byte offset from vtile of each piece, rows past the
                              // valid length replaced by the last valid row.  Computed when the plan is made
                              // and left alone until every load has been issued: an address register rewritten
                              // shortly after the load that uses it has produced wrong loads here.
};

template <int D, int B>
__device__ __forceinline__ void dma_burst(const DmaPlan<D>& p) {
  constexpr int win = B / 2;
  if constexpr (B % 2 == 0) {
    dma16x4<win * 4096>(p.kp + win * 4096, p.kpat[0], p.kpat[1], p.kpat[2], p.kpat[3], p.klds);
  } else {
    if (__builtin_expect(p.vragged, 0)) {
      dma16(p.vtile, p.voff[4 * win + 0], p.vlds + (4 * win + 0) * 1024);
      dma16(p.vtile, p.voff[4 * win + 1], p.vlds + (4 * win + 1) * 1024);
      dma16(p.vtile, p.voff[4 * win + 2], p.vlds + (4 * win + 2) * 1024);
      dma16(p.vtile, p.voff[4 * win + 3], p.vlds + (4 * win + 3) * 1024);
    } else {
      dma16x4<win * 4096>(p.vp + win * 4096, p.vpat, p.vpat, p.vpat, p.vpat, p.vlds);
    }
  }
}
// all of a plan at once (before a pipelined run starts)
template <int D, int B = 0>
__device__ __forceinline__ void dma_all(const DmaPlan<D>& p, bool k_too, bool v_too) {
  if constexpr (B < DmaPlan<D>::NB) {
    if (B % 2 == 0 ? k_too : v_too) dma_burst<D, B>(p);
    dma_all<D, B + 1>(p, k_too, v_too);
  }
}

constexpr bool kLoads = true, kNoLoads = false;   // whether a step carries its plan's loads
// Operand fragments.  A step finds the fragments of its first kPre MFMA pairs in registers: the step before it
// read them from LDS under its last pairs (or, where a run of steps starts, a preload does).  The fragment of a
// later pair r is read while pair max(0, r - kOwn) is issued.  So the matrix pipe never waits for LDS at the
// start of a step, and a step has issued all its own LDS reads kOwn - kPre pairs before it starts reading
// for the next one.
constexpr int kPre = 4;
constexpr int kOwn = 6;
constexpr int issue_pair(int r) { return r - kOwn > 0 ? r - kOwn : 0; }

// Which products a step has and where its sub-tiles lie: byte offsets of the K and V sub-tiles from the
// tile the address registers point at.
template <bool PV_, bool QK_, int K_OFF_, int V_OFF_>
struct StepKind {
  static constexpr bool PV = PV_, QK = QK_;
  static constexpr int K_OFF = K_OFF_, V_OFF = V_OFF_;
};
// What a step does for the one that follows it: nothing; read its first fragments (same tile addresses); or
// end the tile -- move the address registers to the next ring entries once their last read is issued, wait for
// the staged tile and meet the other wave, then read the next tile's first fragments.
constexpr int kNextNone = 0, kNextSame = 1, kNextTile = 2;
constexpr int kMidPieces = 5;   // pieces of the caller's work inside a step (run_slots)

template <int D, bool PV, bool QK, bool SM, bool RAGGED>
struct StepCtx {
  static constexpr int NP = (PV ? Geo<D>::KS : 0) + (QK ? Geo<D>::KS : 0);   // MFMA pairs (PV has 2 DT = KS)
  static constexpr int NC = 2 * NP;                 // slots
  static constexpr int PRE = SM && RAGGED ? 2 : 0;  // slots that mask the keys that do not exist
  uint32_t (&vaddr)[Geo<D>::DT];
  uint32_t (&kaddr)[Geo<D>::KS];
  float c2;                      // log2(e) * softmax scale
  const bf16x8 (&qf)[2][Geo<D>::KS];
  f32x16 (&o)[2][Geo<D>::DT];
  f32x16 (&s_cur)[2];
  f32x16 (&s_next)[2];
  PTile& p_cur;
  const PTile& p_prev;
  const float (&mc)[2];          // minus the softmax reference of each row group, times c2
  const int (&lim)[2];           // RAGGED: valid keys of the current sub-tile minus 4 * half, per row group
  const DmaPlan<D>& dma;
  bf16x8 (&frag)[2 * Geo<D>::KS];   // operand fragment of each MFMA pair
  int dk, dv;                    // kNextTile: what moves kaddr / vaddr to the next tile's ring entries
  float ex[32];                  // exp2 of the scores, row group g element v at 16 g + v, until they are rounded
  f32x4& lsum;                   // PV: the running row sums, which take those of p_prev (see sum_selector)
  f32x4& ltile;                  // PV, mass variant: the row sums of p_prev alone
  const bf16x8 (&sel)[2];        // the selecting operands of the row-sum instruction, per row group
  uint32_t por;                  // SM: bitwise OR of the pairs of p_cur
  uint32_t phold;                // SM: a pair waiting for the next one to share a three-input OR
};

// pair q: with both products, even q is PV pair q/2 and odd q is QK pair q/2
template <bool PV, bool QK>
constexpr bool pair_is_pv(int q) { return PV && (!QK || q % 2 == 0); }
template <bool PV, bool QK>
constexpr int pair_index(int q) { return (PV && QK) ? q / 2 : q; }

// reads the operand fragment of pair R of a step of kind KIND
template <int D, class KIND, int R>
__device__ __forceinline__ void load_pair(bf16x8 (&frag)[2 * Geo<D>::KS], const uint32_t (&vaddr)[Geo<D>::DT],
                                          const uint32_t (&kaddr)[Geo<D>::KS]) {
  constexpr int NP = (KIND::PV ? Geo<D>::KS : 0) + (KIND::QK ? Geo<D>::KS : 0);
  if constexpr (R < NP) {
    constexpr int i = pair_index<KIND::PV, KIND::QK>(R);
    if constexpr (pair_is_pv<KIND::PV, KIND::QK>(R)) {
      constexpr int j = i / Geo<D>::DT, dt = i % Geo<D>::DT;
      frag[R] = lds_read_vt<Geo<D>::ROW>(vaddr[dt] + KIND::V_OFF + 16 * j * Geo<D>::ROW);
    } else {
      frag[R] = lds_read_k(kaddr[i] + KIND::K_OFF);
    }
  }
}
template <int D, class KIND, int R = 0>
__device__ __forceinline__ void preload_frags(bf16x8 (&frag)[2 * Geo<D>::KS], const uint32_t (&vaddr)[Geo<D>::DT],
                                              const uint32_t (&kaddr)[Geo<D>::KS]) {
  if constexpr (R < kPre) {
    load_pair<D, KIND, R>(frag, vaddr, kaddr);
    preload_frags<D, KIND, R + 1>(frag, vaddr, kaddr);
  }
}
// the reads a step issues under pair Q for its own later pairs
template <int D, class KIND, int Q, int R = kPre>
__device__ __forceinline__ void own_loads(bf16x8 (&frag)[2 * Geo<D>::KS], const uint32_t (&vaddr)[Geo<D>::DT],
                                          const uint32_t (&kaddr)[Geo<D>::KS]) {
  constexpr int NP = (KIND::PV ? Geo<D>::KS : 0) + (KIND::QK ? Geo<D>::KS : 0);
  if constexpr (R < NP) {
    if constexpr (issue_pair(R) == Q) load_pair<D, KIND, R>(frag, vaddr, kaddr);
    own_loads<D, KIND, Q, R + 1>(frag, vaddr, kaddr);
  }
}
// the pair under which a step of kind KIND issues its last read through kaddr[ks] / vaddr[dt] (-1: only in a preload)
template <int D, class KIND>
constexpr int last_read_k(int ks) {
  if (!KIND::QK) return -1;
  const int r = KIND::PV ? 2 * ks + 1 : ks;
  return r < kPre ? -1 : issue_pair(r);
}
template <int D, class KIND>
constexpr int last_read_v(int dt) {
  if (!KIND::PV) return -1;
  const int i = Geo<D>::DT + dt, r = KIND::QK ? 2 * i : i;
  return r < kPre ? -1 : issue_pair(r);
}

template <int D, bool PV, bool QK, bool SM, bool RAGGED, int Q, int GRP>
__device__ __forceinline__ void mfma_slot(StepCtx<D, PV, QK, SM, RAGGED>& c) {
  constexpr int i = pair_index<PV, QK>(Q);
  if constexpr (pair_is_pv<PV, QK>(Q)) {
    constexpr int j = i / Geo<D>::DT, dt = i % Geo<D>::DT;
    pv_mfma(c.o[GRP][dt], c.frag[Q], as_bf16x8(c.p_prev[GRP][j]));
  } else {
    const f32x16 zero = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
    c.s_next[GRP] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(c.frag[Q], c.qf[GRP][i], i == 0 ? zero : c.s_next[GRP], 0, 0, 0);
  }
}

// Slice C of the softmax of s_cur.  In a ragged step the first two slices mask the row groups.  The
// other NS slices share the 32 scores of a lane (score e in slice e NS / 32) and the 16 pairs: the
// exponential of a score is issued in its slice and a pair is rounded one slice after its second
// exponential (the last slice takes what would fall behind it), so every slice has about the same few
// instructions and none of them waits for the previous one.  Every second pair is OR-ed, with the one before
// it, into the word that decides in the last slice whether the reference served (returned as a wave mask of the
// lanes that saw a probability of 2 or more, an infinity or a NaN).
template <int D, bool PV, bool QK, bool SM, bool RAGGED, int C>
__device__ __forceinline__ void valu_slot(StepCtx<D, PV, QK, SM, RAGGED>& c, unsigned long long& bad) {
  using S = StepCtx<D, PV, QK, SM, RAGGED>;
  if constexpr (!SM) {
  } else if constexpr (C < S::PRE) {
#pragma unroll
    for (int v = 0; v < 16; ++v)           // accumulator element v is key 8 (v/4) + 4 half + v%4
      if (8 * (v / 4) + (v % 4) >= c.lim[C]) c.s_cur[C][v] = kMasked;
  } else {
    constexpr int NS = S::NC - S::PRE, j = C - S::PRE;
    constexpr bool last = j == NS - 1;
#pragma unroll
    for (int e = 0; e < 32; ++e) {
      if (e * NS / 32 == j) {
        c.ex[e] = prob_exp(c.s_cur[e / 16][e % 16], c.c2, c.mc[e / 16]);
        // a use that cannot move keeps the work of a slice in its slot
        asm volatile("" ::"v"(c.ex[e]));
      }
    }
#pragma unroll
    for (int n = 0; n < 16; ++n) {         // pair n: scores 2n, 2n+1 of row group n / 8
      const int jr = (2 * n + 1) * NS / 32 + 1;
      if (jr == j || (last && jr > j)) {
        const uint32_t w = prob_round(c.ex[2 * n], c.ex[2 * n + 1]);
        if (n % 2 == 0) {
          c.phold = w;
          asm volatile("" : "+v"(c.phold));          // keeps the conversion in this slot
        } else {
          c.por = n == 1 ? (c.phold | w) : or3(c.por, c.phold, w);
          asm volatile("" : "+v"(c.por));
        }
        c.p_cur[n / 8][(n % 8) / 4][n % 4] = w;
      }
    }
    if constexpr (last) {
      uint32_t top;
      asm volatile("v_and_b32 %0, %3, %2\n\tv_cmp_ne_u32 %1, 0, %0" : "=&v"(top), "=s"(bad) : "v"(c.por), "s"(kTooBig));
    }
  }
}

// Everything a step needs of the running softmax: per row group the reference (m_ref, and mc = -m_ref c2),
// the running sum, and whether anything has been added to the output accumulators yet.
struct SoftmaxRun {
  float m_ref[2], mc[2];
  f32x4 l_run;              // running row sums as the row-sum instruction leaves them: element 0 of lane L is row
                            // L % 32 of row group L / 32 (see sum_selector)
  bf16x8 sel[2];            // sum_selector of this lane, per row group
  unsigned long long bad;   // lanes in which the sub-tile whose softmax ran last needs another reference
  float c2, lift;
  bool o_live;
};

// The mass variant of the kernel also leaves, for every 64-key tile a wave walks and every one of its 64 rows,
// the base-2 logarithm of the row's share of the softmax normaliser that falls on that tile, in absolute units
// (independent of the reference in force at the time): log2(sum of the tile's probabilities) minus mc.  A later
// pass turns them into attention mass per key block: 2^(that - log2 normaliser), summed over rows.  The sum of
// a tile's first sub-tile is held until the second is summed; one 256-byte store per tile: lanes 0..31 hold
// rows 0..31, lanes 32..63 rows 32..63.
struct MassOut {
  float* rp;        // where this wave's next 64 values go (uniform)
  int lane;
  bool hi;          // lane >= 32
  float hold, hold_mc;   // the first sub-tile's row sum and the mc it is relative to
};

// What the slots of a step do beside the MFMA and the softmax slice.
//  first slot of pair Q, before the MFMA: the LDS reads of the step's own later fragments.
//  second slot of each of the last kPre pairs, after the MFMA: the read of one of the first fragments of the step
//    that follows (NEXT); a step that ends a tile first waits for the staged tile and for its own reads and meets
//    the other wave: from then on the ring entries it has been reading may be refilled, and the next tile's read.
//  after the MFMA: staging loads (DMA), a piece of the caller's work for the next tile (MID, slots 2, 4, ...), the move of
//    the address registers to the next tile (each right after the pair that issued its last read), the slice
//    of the softmax, and in four slots of the step a row-sum instruction of p_prev.
template <int D, bool MASSV, bool PV, bool QK, bool SM, bool RAGGED, bool DMA, class KIND, int NEXT, class NKIND, int I, class MID>
__device__ __forceinline__ void run_slots(StepCtx<D, PV, QK, SM, RAGGED>& c, unsigned long long& bad, MID& mid) {
  using S = StepCtx<D, PV, QK, SM, RAGGED>;
  if constexpr (I < S::NC) {
    constexpr int Q = I / 2, k = I % 2;
    if constexpr (k == 0) own_loads<D, KIND, Q>(c.frag, c.vaddr, c.kaddr);
    mfma_slot<D, PV, QK, SM, RAGGED, Q, k>(c);
    __builtin_amdgcn_sched_barrier(0);         // the MFMA first, then the slot's vector work
    if constexpr (k == 1 && NEXT != kNextNone && Q >= S::NP - kPre) {
      // after both MFMAs of the pair: in a short step the fragment register read here may be this pair's own
      if constexpr (NEXT == kNextTile && Q == S::NP - kPre) {
        asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
      }
      load_pair<D, NKIND, Q - (S::NP - kPre)>(c.frag, c.vaddr, c.kaddr);
    }
    if constexpr (DMA) {
      constexpr int every = (S::NC < 16 ? S::NC : 16) / DmaPlan<D>::NB;     // a burst every few slots of the first 16
      static_assert(every >= 1, "a slot for every burst");
      if constexpr (I % every == 0 && I / every < DmaPlan<D>::NB) dma_burst<D, I / every>(c.dma);
    }
    // the caller's work for the next tile comes in kMidPieces pieces, one in each of the slots 2, 4, ...: scalar
    // instructions issued in a lump hold the wave up for four to five cycles each, spread out for one or two
    if constexpr (I >= 2 && I % 2 == 0 && (I - 2) / 2 < kMidPieces) mid(std::integral_constant<int, (I - 2) / 2>{});
    if constexpr (NEXT == kNextTile && k == 1) {
      static_assert(NEXT != kNextTile || S::NP - kPre > issue_pair(S::NP - 1), "every address is free before the turnover");
#pragma unroll
      for (int ks = 0; ks < Geo<D>::KS; ++ks)
        if (last_read_k<D, KIND>(ks) == Q || (Q == 0 && last_read_k<D, KIND>(ks) < 0)) {
          c.kaddr[ks] += c.dk;
          asm volatile("" : "+v"(c.kaddr[ks]));
        }
#pragma unroll
      for (int dt = 0; dt < Geo<D>::DT; ++dt)
        if (last_read_v<D, KIND>(dt) == Q || (Q == 0 && last_read_v<D, KIND>(dt) < 0)) {
          c.vaddr[dt] += c.dv;
          asm volatile("" : "+v"(c.vaddr[dt]));
        }
    }
    valu_slot<D, PV, QK, SM, RAGGED, I>(c, bad);
    if constexpr (PV) {
      // the four row-sum instructions of p_prev (row group g, keys 16 j ..), spread over the step
#pragma unroll
      for (int q = 0; q < 4; ++q)
        if ((2 * q + 1) * S::NC / 8 == I) {
          sum_mfma(c.lsum, c.sel[q / 2], as_bf16x8(c.p_prev[q / 2][q % 2]));
          // the mass variant wants the sub-tile's own sums as well, and the running sums exactly as without it
          if constexpr (MASSV) sum_mfma(c.ltile, c.sel[q / 2], as_bf16x8(c.p_prev[q / 2][q % 2]));
        }
    }
    __builtin_amdgcn_sched_barrier(0);
    run_slots<D, MASSV, PV, QK, SM, RAGGED, DMA, KIND, NEXT, NKIND, I + 1, MID>(c, bad, mid);
  }
}

// A sub-tile whose probabilities cannot be used (its step left sr.bad set: some probability came out above
// 2, or the reference was never set: a row's first keys) gets its softmax redone here, outside the
// pipeline and before anything uses it, for both row groups: row maxima, references raised to kLift above them
// where that is higher than the old reference, the probabilities again, and the running sums and output
// accumulators rescaled to the new references.  s is the sub-tile's S^T, which the coming step will overwrite,
// p its P^T.  What this rare branch changes it changes in place (instructions whose result register is their
// input's): values that merely merge with new ones after a branch cost the common path a register copy each.
template <int D>
__device__ __forceinline__ void softmax_redo(const f32x16 (&s)[2], PTile& p, SoftmaxRun& sr, f32x16 (&o)[2][Geo<D>::DT]) {
  float alpha[2];
#pragma unroll
  for (int g = 0; g < 2; ++g) {
    const float tmax = row_max(s[g]);
    // every row takes the occasion to move its reference up to kLift above what it sees now: the redo and the
    // rescale cost the same, and a row that was drifting towards its own limit will not ask for another
    const float m_new = tmax + sr.lift > sr.m_ref[g] ? tmax + sr.lift : sr.m_ref[g];
    alpha[g] = __builtin_amdgcn_exp2f((sr.m_ref[g] - m_new) * sr.c2);
    const float mc_new = -m_new * sr.c2;
#pragma unroll
    for (int v = 0; v < 16; v += 2) {
      const float e0 = prob_exp(s[g][v], sr.c2, mc_new), e1 = prob_exp(s[g][v + 1], sr.c2, mc_new);
      // (the wait states a vector instruction needs before it reads the result of a transcendental one are the
      // compiler's business, but it cannot see what this instruction reads)
      asm volatile("s_nop 3\n\tv_cvt_pk_bf16_f32 %0, %1, %2" : "+v"(p[g][v / 8][(v % 8) / 2]) : "v"(e0), "v"(e1));
    }
    asm volatile("v_mov_b32 %0, %1" : "+v"(sr.m_ref[g]) : "v"(m_new));
    asm volatile("v_mov_b32 %0, %1" : "+v"(sr.mc[g]) : "v"(mc_new));
  }
  // the running sum of lane L is that of row L % 32 of row group L / 32: this lane's own alpha of that group
  sum_settle(sr.l_run);
  sr.l_run[0] *= __lane_id() < 32 ? alpha[0] : alpha[1];
  sum_settle(sr.l_run);
  if (sr.o_live) rescale<Geo<D>::DT>(o, alpha);
}

// Before the first softmax of a run: a row that has no reference yet -- and so nothing accumulated: whatever it has
// met so far was masked -- takes kLift above the row maximum of the scores just computed.  Without this the first
// sub-tile of every wave would be computed against the initial reference, overflow, and be redone.
__device__ __forceinline__ void seed_reference(const f32x16 (&s)[2], SoftmaxRun& sr) {
#pragma unroll
  for (int g = 0; g < 2; ++g) {
    const float tmax = row_max(s[g]);
    const bool fresh = sr.m_ref[g] == kInitMax && tmax > kInitMax;     // (false for a NaN as well)
    const float m_new = fresh ? tmax + sr.lift : sr.m_ref[g];
    sr.m_ref[g] = m_new;
    sr.mc[g] = -m_new * sr.c2;
  }
}

// One step.  KIND: its products and sub-tile offsets.  PRELOADED: the fragments of its first kPre pairs are in
// frag already.  NEXT / NKIND: what it does for the step after it (see run_slots).  mid() is called once, early
// in the step.  dk, dv: kNextTile only.
template <int D, bool MASS, bool SM, bool RAGGED, bool DMA, class KIND, bool PRELOADED, int NEXT, class NKIND, class MID>
__device__ __forceinline__ void step(uint32_t (&vaddr)[Geo<D>::DT], uint32_t (&kaddr)[Geo<D>::KS],
                                     const bf16x8 (&qf)[2][Geo<D>::KS], f32x16 (&o)[2][Geo<D>::DT], f32x16 (&s_cur)[2],
                                     f32x16 (&s_next)[2], PTile& p_cur, PTile& p_prev, SoftmaxRun& sr,
                                     const int (&lim)[2], const DmaPlan<D>& dma, MassOut& mo,
                                     bf16x8 (&frag)[2 * Geo<D>::KS], int dk, int dv, MID& mid) {
  static_assert(2 * Geo<D>::DT == Geo<D>::KS, "PV and QK pairs alternate one to one");
  constexpr bool PV = KIND::PV, QK = KIND::QK;
  // the row sums of p_prev go straight into the running sums; the mass variant takes them per sub-tile as well
  f32x4 pt = {0.0f, 0.0f, 0.0f, 0.0f};
  StepCtx<D, PV, QK, SM, RAGGED> c{vaddr, kaddr, sr.c2, qf, o, s_cur, s_next, p_cur, p_prev, sr.mc, lim, dma, frag, dk, dv, {}, sr.l_run, pt, sr.sel, 0u, 0u};
  if constexpr (!PRELOADED) preload_frags<D, KIND>(frag, vaddr, kaddr);
  if constexpr (PV) {
    // p_prev is the softmax of the sub-tile whose S^T still sits in s_next
    if (__builtin_expect(sr.bad != 0ull, 0)) softmax_redo<D>(s_next, p_prev, sr, o);
    sr.bad = 0ull;
  }
  __builtin_amdgcn_sched_barrier(0);
  unsigned long long bad = 0ull;
  run_slots<D, MASS, PV, QK, SM, RAGGED, DMA, KIND, NEXT, NKIND, 0, MID>(c, bad, mid);
  if constexpr (SM) sr.bad = bad;
  if constexpr (PV) {
    sr.o_live = true;
    if constexpr (MASS) {
      sum_settle(pt);
      // lanes 0..31 hold the sums of rows 0..31 (row group 0), lanes 32..63 those of row group 1
      const float tot = pt[0];
      const float mc_now = mo.hi ? sr.mc[1] : sr.mc[0];
      if constexpr (KIND::V_OFF == 0) {    // the sub-tile summed is the one whose V the step multiplied: a tile's first
        mo.hold = tot;
        mo.hold_mc = mc_now;
      } else {
        // the held sum in today's units (the factor is 1 unless the reference moved in between)
        const float both = __builtin_fmaf(mo.hold, __builtin_amdgcn_exp2f(mc_now - mo.hold_mc), tot);
        mo.rp[mo.lane] = __builtin_amdgcn_logf(both) - mc_now;
        mo.rp += 64;
      }
    }
  }
}
struct NoMid {
  template <class PIECE>
  __device__ __forceinline__ void operator()(PIECE) const {}
};
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Wuninitialized"
// What the extra workgroups of a launch with PLAN need: the argument blocks of the update's decisions.
template <bool PLAN>
struct PlanArgs {};
template <>
struct PlanArgs<true> {
  plan_dev::ScoreArgs sa;
  plan_dev::RetainArgs ra;
};

// PLAN: the grid has H more workgroups ahead of those of the attention, one per head, which take the decisions of
// the memory update (Eq. 7-9: scoring, retention, slot assignment) while the attention runs.  They read the
// cache's metadata and pooled keys and what the selection call left, never K / V or the attention's output, and
// a one-round launch leaves them SIMDs to run on (two workgroups per CU, 128 rows each: at 4680 rows and 12
// heads 444 of 512 places are taken).
template <int D, int B, bool MASS, bool PLAN>
__global__ void __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(1, 1)))
attention_kernel(AttnArgs a, PlanArgs<PLAN> pl) {
  constexpr int G = kRowsPerWg / B;        // query blocks per workgroup
  constexpr int SUB = B / kTile;           // 64-key tiles per block
  constexpr int KS = Geo<D>::KS, DT = Geo<D>::DT, TILE = Geo<D>::TILE_BYTES, ROW = Geo<D>::ROW;
  constexpr int SUB1 = Geo<D>::SUB_BYTES;
  constexpr int CH = D / 8, RPI = 64 / CH;          // 16-byte chunks per row, rows per wave instruction
  constexpr int NIW = (kTile / RPI) / 2;            // global_load_lds instructions per wave per tile
  constexpr int SMEM = 4 * TILE;                    // K ring (2 tiles), V ring (2 tiles)
  static_assert((3 * PBSA_MAX_N_LOC + PBSA_MAX_C_ATTEND + 1) * 4 <= SMEM, "setup scratch must fit");
  // the plain call takes the larger limits and keeps the list within two workgroups' share of a CU's LDS by
  // storing 16-bit descriptors (the mass variant's carry the key block as well)
  constexpr bool kAux = MASS || PLAN;
  constexpr int kTilesMax = kAux ? kMaxTilesAux : kMaxTiles;
  constexpr int kLocMax = kAux ? PBSA_MAX_N_LOC_AUX : PBSA_MAX_N_LOC;
  using meta_t = std::conditional_t<kAux, int, uint16_t>;

  __shared__ __align__(1024) unsigned char smem[SMEM];
  __shared__ int t_src[kTilesMax];         // bit 31: local, bits 0..: (slot * SUB + sub)
  __shared__ meta_t t_meta[kTilesMax];     // valid keys (bits 0..7) | waves that attend (bits 8, 9)
  int* lflag = reinterpret_cast<int*>(smem);        // setup scratch, dead before the first tile is staged

  // XCD-aware mapping: consecutive workgroup ids go round-robin to the 8 XCDs, so give XCD x the
  // contiguous range [x * per, (x+1) * per) of (head, query tile) pairs: neighbours share K/V in L2.
  const int n_qt = (a.Nq + kRowsPerWg - 1) / kRowsPerWg;
  const int n_wg = a.H * n_qt;
  const int per = (n_wg + 7) / 8;
  // the workgroups that take the decisions come first in the grid (whole rows of 8, so that the XCD of the others is
  // still their index mod 8): they start with the launch however many rounds the attention needs
  const int n_plan = PLAN ? 8 * ((a.H + 7) / 8) : 0;
  if constexpr (PLAN) {
    if ((int)blockIdx.x < n_plan) {
      const int hp = (int)blockIdx.x;
      if (hp >= a.H) return;
      static_assert(plan_dev::score_head_lds_bytes<D, kThreads>(PBSA_MAX_N_LOC_AUX) <= SMEM, "scoring scratch must fit");
      static_assert(sizeof(plan_dev::RetainLds) <= SMEM, "retention scratch must fit");
      plan_dev::score_head_body<D, kThreads>(pl.sa, hp, smem);
      __syncthreads();                     // the head's rows are written, and the scoring scratch is dead
      plan_dev::retain_body<kThreads>(pl.ra, hp, *reinterpret_cast<plan_dev::RetainLds*>(smem));
      return;
    }
  }
  const int bx = (int)blockIdx.x - n_plan;
  const int logical = (bx % 8) * per + bx / 8;
  if (logical >= n_wg) return;
  const int h = logical / n_qt;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int T0 = (logical % n_qt) * kRowsPerWg;
  const int i0 = T0 / B;
  const int qn = lane & 31, half = lane >> 5;

  // ---- tile list --------------------------------------------------------------------------------
  // Everything the list needs is fetched from global memory in one parallel round into LDS scratch:
  // per local block the set of waves whose query block selected it, its length and its physical slot;
  // per persistent slot its length.  The candidates -- the 64-key tiles of the persistent slots, then
  // of the local blocks, in ascending order -- are then classified by every wave, candidate i by lane
  // i mod 64 in round i / 64: full tiles of both waves, ragged tiles, full tiles of wave 0 only, of
  // wave 1 only.  Every part of the list is in ascending candidate order.
  int* llen_s = lflag + kLocMax;
  int* lmap_s = llen_s + kLocMax;
  int* plen_s = lmap_s + kLocMax;
  for (int l = tid; l < a.n_loc; l += kThreads) {
    lflag[l] = 0;
    llen_s[l] = a.l_len[l];
    lmap_s[l] = a.l_map[l];
  }
  for (int c = tid; c <= a.C; c += kThreads) plen_s[c] = a.p_len[(size_t)h * (a.C + 1) + c];
  // the selections of this workgroup's query blocks, fetched now (loads return in order: anything asked
  // for after the queries would wait for them) and turned into flags once the flags are zeroed
  constexpr int kSelPer = (2 * (kAux ? PBSA_MAX_K_AUX : PBSA_MAX_K) + kThreads - 1) / kThreads;
  int selv[kSelPer];
#pragma unroll
  for (int u = 0; u < kSelPer; ++u) {
    const int idx = tid + u * kThreads;
    const int g = idx / max(a.k, 1), j = idx % max(a.k, 1);
    selv[u] = idx < G * a.k && i0 + g < a.nqb ? a.sel[((size_t)h * a.nqb + i0 + g) * a.k + j] : -1;
  }

  // ---- Q fragments (B operand of S^T = K Q^T): row group g, query row lane % 32, dims 16 ks + 8 (lane/32) ..+8.
  // Issued after the few loads the tile list waits for and not touched until the list is built: the
  // chunk's queries come from HBM while every workgroup of the launch asks for its own at the same time.
  const int tok0 = T0 + wave * 64 + qn;                 // row group g holds token tok0 + 32 g
  bf16x8 qf[2][KS];
#pragma unroll
  for (int g = 0; g < 2; ++g) {
    const int tok_c = min(tok0 + 32 * g, a.Nq - 1);
    const bf16_t* qrow = a.Q + (size_t)h * a.q_stride_h + (size_t)tok_c * a.q_stride_t + 8 * half;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) qf[g][ks] = *reinterpret_cast<const bf16x8*>(qrow + 16 * ks);
  }
  __syncthreads();
#pragma unroll
  for (int u = 0; u < kSelPer; ++u) {
    const int l = selv[u], g = (tid + u * kThreads) / max(a.k, 1);
    // with one query block per workgroup both waves belong to it
    if (l >= 0 && l < a.n_loc) atomicOr(&lflag[l], G == 1 ? 3 : 1 << g);
  }
  __syncthreads();
  const int n_pers = (a.C + 1) * SUB, n_cand = n_pers + a.n_loc * SUB;
  // candidate i -> its class (-1: no tile) and its list entry
  auto classify = [&](int i, int& src, int& meta) -> int {
    if (i >= n_cand) return -1;
    if (i < n_pers) {
      const int c = i / SUB, sub = i % SUB;
      const int tl = min(max(min(max(plen_s[c], 0), B) - sub * kTile, 0), kTile);
      src = i;
      meta = tl | (3 << 8);
      if constexpr (MASS) meta |= (c << 10) | (sub << 20);       // the key block the tile belongs to, and which tile of it
      return tl == 0 ? -1 : tl == kTile ? 0 : 1;
    }
    const int l = (i - n_pers) / SUB, sub = (i - n_pers) % SUB;
    const int f = lflag[l], slot = lmap_s[l];
    if (f == 0 || slot < 0 || slot >= a.n_loc_cap) return -1;
    const int tl = min(max(min(max(llen_s[l], 0), B) - sub * kTile, 0), kTile);
    src = (int)(0x80000000u | (uint32_t)(slot * SUB + sub));
    meta = tl | (f << 8);
    if constexpr (MASS) meta |= ((a.C + 1 + l) << 10) | (sub << 20);
    return tl == 0 ? -1 : tl < kTile ? 1 : f == 3 ? 0 : f + 1;      // f is 1 or 2 otherwise
  };
  // Every wave classifies every candidate, 64 per round, twice: the first sweep gives the sizes of the four parts, the
  // second the places, with the running counts in scalar registers (ballots only: no barrier and no LDS traffic
  // between the sweeps).  The waves take turns writing the rounds.
  const int n_rounds = (n_cand + 63) / 64;
  int tot[4] = {0, 0, 0, 0};
  for (int r = 0; r < n_rounds; ++r) {
    int src, meta;
    const int cls = classify(r * 64 + lane, src, meta);
#pragma unroll
    for (int c = 0; c < 4; ++c) tot[c] += __popcll(__ballot(cls == c));
  }
  int base[4] = {0, tot[0], tot[0] + tot[1], tot[0] + tot[1] + tot[2]};
  const int cls_end[4] = {base[1], base[2], base[3], base[3] + tot[3]};
  for (int r = 0; r < n_rounds; ++r) {
    int src = 0, meta = 0;
    const int cls = classify(r * 64 + lane, src, meta);
    const bool mine = (r & 1) == wave;
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      const unsigned long long m = __ballot(cls == c);
      if (cls == c && mine) {
        const int pos = base[c] + lanes_below(m);
        t_src[pos] = src;
        t_meta[pos] = (meta_t)meta;
      }
      base[c] += __popcll(m);
    }
  }
  __syncthreads();
  // The Q fragments are only ever MFMA operands, which may come from the accumulator half of the
  // register file: define them there, leaving the architectural half to the softmax and the outputs.
#pragma unroll
  for (int g = 0; g < 2; ++g)
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) asm volatile("" : "+a"(qf[g][ks]));

  MassOut mo{nullptr, lane, lane >= 32, 0.0f, 0.0f};
  if constexpr (MASS) {
    // the later pass walks the same list: the ends of its four parts, then a descriptor per tile
    int32_t* out = a.Rlist + (size_t)logical * a.list_cap;
    if (tid == 0) {
      out[0] = cls_end[0]; out[1] = cls_end[1]; out[2] = cls_end[2]; out[3] = cls_end[3];
    }
    for (int i = tid; i < cls_end[3] && i < a.list_cap - 4; i += kThreads) out[4 + i] = t_meta[i];
    mo.rp = a.R + ((size_t)logical * 2 + wave) * a.r_slots * 64;
  }
  const int e0 = cls_end[0];               // shared full tiles [0, e0)
  const int n_tiles = cls_end[1];          // shared ragged tiles [e0, n_tiles): the end of the shared list
  const int solo_b = wave == 0 ? n_tiles : cls_end[2];         // this wave's solo tiles [solo_b, solo_e)
  const int solo_e = wave == 0 ? cls_end[2] : cls_end[3];

  f32x16 o[2][DT];
#pragma unroll
  for (int g = 0; g < 2; ++g)
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) {
#pragma unroll
      for (int v = 0; v < 16; ++v) o[g][dt][v] = 0.0f;
      asm volatile("" : "+a"(o[g][dt]));
    }
  f32x16 sA[2], sB[2];                     // S^T of even / odd sub-tiles
  PTile pA, pB;                            // P^T of even / odd sub-tiles (bf16 pairs)
  const float c2 = a.scale * 1.4426950408889634f, lift = kLift / c2;
  SoftmaxRun sr{{kInitMax, kInitMax}, {-kInitMax * c2, -kInitMax * c2}, {0.0f, 0.0f, 0.0f, 0.0f},
                {sum_selector(lane, 0), sum_selector(lane, 1)}, 0ull, c2, lift, false};
  bf16x8 frag[2 * KS];                     // operand fragments, handed from step to step
  NoMid nomid;

  // ---- operand addresses ------------------------------------------------------------------------
  // this lane's fragment addresses inside ring entry 0, sub-tile 0 (LDS byte addresses)
  const uint32_t smem_lds = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)smem;
  uint32_t ka0[KS], va0[DT];
  {
    const int kb = qn * ROW + ((half ^ k_swz<D>(qn)) << 4);        // chunk (2 ks + half) ^ f = (half ^ f) ^ 2 ks
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) ka0[ks] = smem_lds + (uint32_t)(kb ^ (ks << 5));
    const int s16 = lane & 15, q16 = (lane >> 4) & 1;
    const int v_row0 = 4 * half + (s16 >> 2);                      // address row within 16 keys
    const int v_sub = 2 * q16 + ((s16 & 3) >> 1), v_lo = (s16 & 1) * 8;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
      va0[dt] = smem_lds + 2 * TILE + (uint32_t)(v_row0 * ROW + (((4 * dt + v_sub) ^ v_swz<D>(v_row0)) << 4) + v_lo);
  }

  // ---- staging --------------------------------------------------------------------------------
  // A wave instruction fills one KiB of a tile: RPI consecutive rows, lane i -> row i / CH, physical
  // chunk i % CH, i.e. the logical chunk (i % CH) ^ f(row) of that row.  Since f has period 16 in the row
  // (K) or depends on the row within the piece only (V), the per-lane source offsets within a piece are
  // four patterns for K (the pieces of 16 rows) and one for V, whatever rows a load brings.  In the
  // shared part wave w brings rows 32 w .. 32 w + 31 of every tile.  A ragged V tile must not bring rows
  // past its valid length into LDS (they meet p = 0 in the MFMA, and 0 x NaN-or-Inf pattern is NaN): the
  // lanes of such rows fetch the last valid row instead.
  const int rl = lane / CH, vchk = ((lane % CH) ^ v_swz<D>(rl)) << 4;
  DmaPlan<D> plan;
#pragma unroll
  for (int k = 0; k < 4; ++k) plan.kpat[k] = rl * ROW + (((lane % CH) ^ k_swz<D>(RPI * k + rl)) << 4);
  plan.vpat = rl * ROW + vchk;
  plan.vragged = false;
#pragma unroll
  for (int i = 0; i < NIW; ++i) plan.voff[i] = 0;
  const uint32_t smem_s = __builtin_amdgcn_readfirstlane(smem_lds);
  const size_t head_l = (size_t)h * a.n_loc_cap * B * D * 2, head_p = (size_t)h * (a.C + 1) * B * D * 2;
#define PBSA_TILE_PTR(SRC, BASE_L, BASE_P)                                                              \
  ((SRC) < 0 ? reinterpret_cast<const unsigned char*>(BASE_L) + head_l + (size_t)((SRC) & 0x7FFFFFFF) * (kTile * D * 2) \
             : reinterpret_cast<const unsigned char*>(BASE_P) + head_p + (size_t)(SRC) * (kTile * D * 2))
  // the plan that brings this wave's half of K tile KSRC into K ring entry KENTRY and of V tile VSRC
  // (descriptor words of the list) into V ring entry VENTRY
#define PBSA_PLAN_K(KSRC, KENTRY)                                                                       \
  {                                                                                                     \
    const int ksrc_ = __builtin_amdgcn_readfirstlane(KSRC);                                             \
    plan.kp = PBSA_TILE_PTR(ksrc_, a.Kl, a.Kp) + wave * (TILE / 2);                                     \
    plan.klds = smem_s + (KENTRY) * TILE + wave * (TILE / 2);                                           \
  }
#define PBSA_PLAN_V(VSRC, VENTRY)                                                                       \
  {                                                                                                     \
    const int vsrc_ = __builtin_amdgcn_readfirstlane(VSRC);                                             \
    plan.vtile = PBSA_TILE_PTR(vsrc_, a.Vl, a.Vp);                                                      \
    plan.vp = plan.vtile + wave * (TILE / 2);                                                           \
    plan.vlds = smem_s + (2 + (VENTRY)) * TILE + wave * (TILE / 2);                                     \
  }
#define PBSA_PLAN_VRAGGED(VMETA)                                                                        \
  {                                                                                                     \
    const int vlast_ = (__builtin_amdgcn_readfirstlane(VMETA) & 0xFF) - 1;                              \
    plan.vragged = vlast_ < kTile - 1;                                                                  \
    if (plan.vragged) {                                                                                 \
      _Pragma("unroll") for (int i_ = 0; i_ < NIW; ++i_)                                                \
        plan.voff[i_] = min(32 * wave + RPI * i_ + rl, vlast_) * ROW + vchk;                            \
    }                                                                                                   \
  }
#define PBSA_PLAN_SHARED(KSRC, VSRC, VMETA, KENTRY, VENTRY)                                             \
  PBSA_PLAN_K(KSRC, KENTRY)                                                                             \
  PBSA_PLAN_V(VSRC, VENTRY)                                                                             \
  PBSA_PLAN_VRAGGED(VMETA)

  // One part of the shared list, tiles [TB, TE), as one pipelined run.  Tile t is sub-tiles 2t (buffers
  // A) and 2t+1 (buffers B):
  //   before   : QK(TB,0)
  //   step 2t  : softmax(t,0)  with  PV(t-1,1) (not for t = TB)  and  QK(t,1)
  //   step 2t+1: softmax(t,1)  with  PV(t,0)                     and  QK(t+1,0) (not for t = TE-1)
  //   after    : PV(TE-1,1)
  // Between the two steps of a tile the tiles K(t) and V(t-1) are dead: their ring entries are refilled
  // with K(t+2) and V(t+1), which have until the same point of the next tile to arrive.  Steps 2t+1 and
  // 2t+2 read the same two ring entries (V of t, K of t+1), so the loop body is that pair and takes one
  // set of addresses.  The ragged run masks, per tile, the keys that do not exist and the wave that does
  // not attend.
  // The addresses are computed once per tile and kept in registers (the empty asm stops the compiler from
  // recomputing them next to each use): an address made by a vector instruction right before the LDS read
  // that uses it stalls the wave for about ten cycles per read.
#define PBSA_ADDR_K(T_)                                                                                 \
  _Pragma("unroll") for (int ks = 0; ks < KS; ++ks) {                                                   \
    kx[ks] = ka0[ks] + ((T_) & 1) * TILE;                                                               \
    asm volatile("" : "+v"(kx[ks]));                                                                    \
  }
#define PBSA_ADDR_V(T_)                                                                                 \
  _Pragma("unroll") for (int dt = 0; dt < DT; ++dt) {                                                   \
    vx[dt] = va0[dt] + ((T_) & 1) * TILE;                                                               \
    asm volatile("" : "+v"(vx[dt]));                                                                    \
  }
#define PBSA_LIMITS(T_, RAGGED)                                                                         \
  if (RAGGED) {                                                                                         \
    const int meta_ = __builtin_amdgcn_readfirstlane(t_meta[T_]);                                       \
    const int len_ = meta_ & 0xFF;                                                                      \
    const bool on_ = (meta_ >> (8 + wave)) & 1;                                                         \
    lim0[0] = lim0[1] = (on_ ? min(len_, 32) : 0) - 4 * half;                                           \
    lim1[0] = lim1[1] = (on_ ? max(len_ - 32, 0) : 0) - 4 * half;                                       \
  }
  // The loads of K(T_+2) and V(T_+1) ride along the step that follows.  Past the end of the list the
  // last tile is fetched again: the ring entries it lands in are dead and never read.  The descriptors
  // of those tiles were read from LDS one tile earlier (d_ksrc, d_vsrc, d_vmeta), so that no LDS latency
  // sits between the barrier and the first load; the reads for the next turnover are issued here.
#define PBSA_FETCH_DESC(T_)                                                                             \
  {                                                                                                     \
    d_ksrc = t_src[min((T_) + 2, n_tiles - 1)];                                                         \
    d_vsrc = t_src[min((T_) + 1, n_tiles - 1)];                                                         \
    d_vmeta = t_meta[min((T_) + 1, n_tiles - 1)];                                                       \
  }
#define PBSA_NEXT_PLAN(T_)                                                                              \
  PBSA_PLAN_SHARED(d_ksrc, d_vsrc, d_vmeta, (T_) & 1, ((T_) + 1) & 1)                                   \
  PBSA_FETCH_DESC((T_) + 1)
#define PBSA_TURNOVER(T_)                                                                               \
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); /* K(T_+1), V(T_) have landed */                     \
  __syncthreads();
  /* the query fragments stay in the accumulator half of the register file (only MFMAs read them) */
#define PBSA_PIN_Q                                                                                      \
  _Pragma("unroll") for (int g_ = 0; g_ < 2; ++g_)                                                      \
    _Pragma("unroll") for (int ks_ = 0; ks_ < KS; ++ks_) asm volatile("" : "+a"(qf[g_][ks_]));
#define PBSA_RUN_SHARED(RAGGED, TB, TE)                                                                 \
  if ((TB) < (TE)) {                                                                                    \
    uint32_t kx[KS], vx[DT];                                                                            \
    int lim0[2] = {0, 0}, lim1[2] = {0, 0};                                                             \
    typedef StepKind<true, true, 0, 0> KindA;              /* the loop's first step of a tile */      \
    typedef StepKind<true, true, SUB1, SUB1> KindB;        /* and its second */                        \
    PBSA_ADDR_K(TB)                                                                                     \
    PBSA_ADDR_V(TB)                                                                                     \
    step<D, MASS, false, false, kNoLoads, StepKind<false, true, 0, 0>, false, kNextNone, void, NoMid>(  \
        vx, kx, qf, o, sB, sA, pB, pA, sr, lim0, plan, mo, frag, 0, 0, nomid);                          \
    if (!(RAGGED)) seed_reference(sA, sr);   /* (a ragged tile's scores are not masked yet) */          \
    PBSA_LIMITS(TB, RAGGED)                                                                             \
    PBSA_NEXT_PLAN(TB)                                                                                  \
    step<D, MASS, true, RAGGED, kNoLoads, StepKind<false, true, SUB1, 0>, false, kNextNone, void, NoMid>( \
        vx, kx, qf, o, sA, sB, pA, pB, sr, lim0, plan, mo, frag, 0, 0, nomid);                          \
    PBSA_TURNOVER(TB)                                                                                   \
    PBSA_ADDR_V(TB)                                                                                     \
    PBSA_ADDR_K((TB) + 1)                                                                               \
    /* (unconditional: fragments defined on one path only cost registers on all of them) */            \
    preload_frags<D, KindA>(frag, vx, kx);                                                              \
    for (int t = (TB); t < (TE) - 1; ++t) {                                                             \
      /* the tile's second step ends by moving the address registers to the other ring entries */       \
      const int dv_ = (t & 1) ? -TILE : TILE;                                                           \
      step<D, MASS, true, RAGGED, kLoads, KindA, true, kNextSame, KindB, NoMid>(                        \
          vx, kx, qf, o, sB, sA, pB, pA, sr, lim1, plan, mo, frag, 0, 0, nomid);                        \
      PBSA_LIMITS(t + 1, RAGGED)                                                                        \
      /* the plan of the next tile's loads is made inside the second step, which issues no loads */     \
      auto mid_ = [&](auto piece_) {                                                                    \
        constexpr int pc_ = decltype(piece_)::value;                                                    \
        if constexpr (pc_ == 0) PBSA_PLAN_K(d_ksrc, (t + 1) & 1)                                        \
        if constexpr (pc_ == 1) PBSA_PLAN_V(d_vsrc, (t + 2) & 1)                                        \
        if constexpr (pc_ == 2) PBSA_PLAN_VRAGGED(d_vmeta)                                              \
        if constexpr (pc_ == 3) d_ksrc = t_src[min(t + 4, n_tiles - 1)];                                \
        if constexpr (pc_ == 4) {                                                                       \
          d_vsrc = t_src[min(t + 3, n_tiles - 1)];                                                      \
          d_vmeta = t_meta[min(t + 3, n_tiles - 1)];                                                    \
        }                                                                                               \
      };                                                                                                \
      step<D, MASS, true, RAGGED, kNoLoads, KindB, true, kNextTile, KindA, decltype(mid_)>(             \
          vx, kx, qf, o, sA, sB, pA, pB, sr, lim0, plan, mo, frag, -dv_, dv_, mid_);                    \
    }                                                                                                   \
    /* the address registers now point at V(TE-1) */                                                    \
    step<D, MASS, true, RAGGED, kLoads, StepKind<true, false, 0, 0>, false, kNextSame,                  \
         StepKind<true, false, 0, SUB1>, NoMid>(vx, kx, qf, o, sB, sA, pB, pA, sr, lim1, plan, mo, frag, 0, 0, nomid); \
    step<D, MASS, false, false, kNoLoads, StepKind<true, false, 0, SUB1>, true, kNextNone, void, NoMid>( \
        vx, kx, qf, o, sA, sB, pA, pB, sr, lim0, plan, mo, frag, 0, 0, nomid);                          \
    /* between runs the compiler may copy the accumulators to other registers: let the matrix pipe drain first */ \
    acc_settle<DT>(o[0]);                                                                               \
    acc_settle<DT>(o[1]);                                                                               \
  }

  if (n_tiles > 0) {
    __syncthreads();                       // the setup scratch (aliasing the rings) is dead
    PBSA_PLAN_SHARED(t_src[0], t_src[0], t_meta[0], 0, 0)
    dma_all<D>(plan, true, true);
    if (n_tiles > 1) {
      PBSA_PLAN_SHARED(t_src[1], t_src[0], t_meta[0], 1, 0)
      dma_all<D>(plan, true, false);
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    int d_ksrc, d_vsrc, d_vmeta;
    PBSA_FETCH_DESC(0)
    PBSA_RUN_SHARED(false, 0, e0)
    PBSA_RUN_SHARED(true, e0, n_tiles)
  }

  // ---- solo part ----------------------------------------------------------------------------------
  // Wave w streams its own full local tiles [solo_b, solo_e) through ring entry w of K and of V, which
  // it treats as two 32-key halves.  Sub-tile u = 2t + h lives in half h; in step u the wave computes
  // softmax(u), PV(u-1) from the other V half and QK(u+1) from the other K half, while the halves it
  // has finished with are refilled with K(u+2) and V(u), which must have landed when the step ends.
  //   before   : QK(2 TB)
  //   step 2t  : softmax(2t)    PV(2t-1) (not for t = TB)   QK(2t+1)        loads K(t+1, half 0), V(t, half 0)
  //   step 2t+1: softmax(2t+1)  PV(2t)                      QK(2t+2) (not for t = TE-1)   K(t+1, half 1), V(t, half 1)
  //   after    : PV(2 TE - 1)
  // These are the step instances of the shared loop with another load plan.  Past the end of the list
  // the last tile's K is fetched again into halves that are never read.
  if constexpr (G > 1) {
    // the other wave may still read the rings, and the shared part's trailing loads may still land in them
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (solo_b < solo_e) {
      const unsigned char* kl_h = reinterpret_cast<const unsigned char*>(a.Kl) + head_l;
      const unsigned char* vl_h = reinterpret_cast<const unsigned char*>(a.Vl) + head_l;
      const uint32_t kring = smem_s + wave * TILE, vring = smem_s + (2 + wave) * TILE;
      plan.vragged = false;
      uint32_t kx[KS], vx[DT];
      const int lim0[2] = {0, 0};
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        kx[ks] = ka0[ks] + wave * TILE;
        asm volatile("" : "+v"(kx[ks]));
      }
#pragma unroll
      for (int dt = 0; dt < DT; ++dt) {
        vx[dt] = va0[dt] + wave * TILE;
        asm volatile("" : "+v"(vx[dt]));
      }
      int d_cur = t_src[solo_b], d_next, d_nn;
      // sources of the loads of the steps of tile t: K from tile t+1, V from tile t; HALF picks the rows
#define PBSA_SOLO_PLAN(HALF)                                                                            \
  plan.kp = kl_h + (size_t)(__builtin_amdgcn_readfirstlane(d_next) & 0x7FFFFFFF) * (kTile * D * 2) + (HALF) * SUB1; \
  plan.vp = vl_h + (size_t)(__builtin_amdgcn_readfirstlane(d_cur) & 0x7FFFFFFF) * (kTile * D * 2) + (HALF) * SUB1;  \
  plan.klds = kring + (HALF) * SUB1;                                                                    \
  plan.vlds = vring + (HALF) * SUB1;
#define PBSA_SOLO_LANDED asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      d_next = d_cur;                     // the whole K tile of the first solo tile, half by half
      PBSA_SOLO_PLAN(0)
      dma_all<D>(plan, true, false);
      PBSA_SOLO_PLAN(1)
      dma_all<D>(plan, true, false);
      d_next = t_src[min(solo_b + 1, solo_e - 1)];
      PBSA_SOLO_LANDED
      step<D, MASS, false, false, kNoLoads, StepKind<false, true, 0, 0>, false, kNextNone, void, NoMid>(vx, kx, qf, o, sB, sA, pB, pA, sr, lim0, plan, mo, frag, 0, 0, nomid);
      seed_reference(sA, sr);
      PBSA_SOLO_PLAN(0)
      step<D, MASS, true, false, kLoads, StepKind<false, true, SUB1, 0>, false, kNextNone, void, NoMid>(vx, kx, qf, o, sA, sB, pA, pB, sr, lim0, plan, mo, frag, 0, 0, nomid);
      PBSA_SOLO_LANDED
      for (int t = solo_b; t < solo_e - 1; ++t) {
        d_nn = t_src[min(t + 2, solo_e - 1)];
        PBSA_SOLO_PLAN(1)
        step<D, MASS, true, false, kLoads, StepKind<true, true, 0, 0>, false, kNextNone, void, NoMid>(vx, kx, qf, o, sB, sA, pB, pA, sr, lim0, plan, mo, frag, 0, 0, nomid);
        PBSA_SOLO_LANDED
        d_cur = d_next;
        d_next = d_nn;
        PBSA_SOLO_PLAN(0)
        step<D, MASS, true, false, kLoads, StepKind<true, true, SUB1, SUB1>, false, kNextNone, void, NoMid>(vx, kx, qf, o, sA, sB, pA, pB, sr, lim0, plan, mo, frag, 0, 0, nomid);
        PBSA_SOLO_LANDED
      }
      PBSA_SOLO_PLAN(1)
      step<D, MASS, true, false, kLoads, StepKind<true, false, 0, 0>, false, kNextNone, void, NoMid>(vx, kx, qf, o, sB, sA, pB, pA, sr, lim0, plan, mo, frag, 0, 0, nomid);
      PBSA_SOLO_LANDED
      step<D, MASS, false, false, kNoLoads, StepKind<true, false, 0, SUB1>, false, kNextNone, void, NoMid>(vx, kx, qf, o, sA, sB, pA, pB, sr, lim0, plan, mo, frag, 0, 0, nomid);
    }
  }

  // ---- epilogue ---------------------------------------------------------------------------------
  acc_settle<DT>(o[0]);
  acc_settle<DT>(o[1]);
  sum_settle(sr.l_run);
#pragma unroll
  for (int g = 0; g < 2; ++g) {
    // row r of the group: lane 32 g + r of the running sums
    const float l_tot = __shfl(sr.l_run[0], 32 * g + qn, 64);
    const float inv = l_tot > 0.0f ? 1.0f / l_tot : 0.0f;
    const int tok = tok0 + 32 * g;
    if (tok < a.Nq) {
      bf16_t* orow = a.O + (size_t)h * a.o_stride_h + (size_t)tok * a.o_stride_t;
#pragma unroll
      for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
          bf16x4 w;
#pragma unroll
          for (int e = 0; e < 4; ++e) w[e] = (__bf16)(o[g][dt][4 * q4 + e] * inv);
          *reinterpret_cast<bf16x4*>(orow + 32 * dt + 8 * q4 + 4 * half) = w;
        }
      if (a.lse && half == 0)
        a.lse[(size_t)h * a.Nq + tok] = l_tot > 0.0f ? sr.m_ref[g] * a.scale + __logf(l_tot) : -INFINITY;
    }
  }
}
#pragma clang diagnostic pop

}  // namespace

template <bool MASS, bool PLAN>
static void launch_attention_t(const pbsa_params& p, const AttnArgs& a, const PlanArgs<PLAN>& pl, dim3 grid,
                               hipStream_t stream) {
  const dim3 block(kThreads);
  if (p.d == 128 && p.B == 128) hipLaunchKernelGGL((attention_kernel<128, 128, MASS, PLAN>), grid, block, 0, stream, a, pl);
  else if (p.d == 128 && p.B == 64) hipLaunchKernelGGL((attention_kernel<128, 64, MASS, PLAN>), grid, block, 0, stream, a, pl);
  else if (p.d == 64 && p.B == 128) hipLaunchKernelGGL((attention_kernel<64, 128, MASS, PLAN>), grid, block, 0, stream, a, pl);
  else hipLaunchKernelGGL((attention_kernel<64, 64, MASS, PLAN>), grid, block, 0, stream, a, pl);
}

static AttnArgs attn_args(const pbsa_params& p, const bf16_t* Q, const bf16_t* Kp, const bf16_t* Vp, const int32_t* p_len,
                          const bf16_t* Kl, const bf16_t* Vl, const int32_t* l_len, const int32_t* l_map,
                          const int32_t* sel, bf16_t* O, float* lse, const MassRows* rows) {
  return AttnArgs{p.H, p.Nq, p.nqb, p.n_loc, p.n_loc_cap, p.C, p.k, p.scale, p.q_stride_h, p.q_stride_t,
                  p.o_stride_h, p.o_stride_t, Q, Kp, Vp, p_len, Kl, Vl, l_len, l_map, sel, O, lse,
                  rows ? rows->R : nullptr, rows ? rows->list : nullptr, rows ? rows->r_slots : 0,
                  rows ? rows->list_cap : 0};
}

hipError_t launch_attention(const pbsa_params& p, const bf16_t* Q, const bf16_t* Kp, const bf16_t* Vp,
                            const int32_t* p_len, const bf16_t* Kl, const bf16_t* Vl, const int32_t* l_len,
                            const int32_t* l_map, const int32_t* sel, bf16_t* O, float* lse, const MassRows* rows,
                            hipStream_t stream) {
  const AttnArgs a = attn_args(p, Q, Kp, Vp, p_len, Kl, Vl, l_len, l_map, sel, O, lse, rows);
  const int n_wg = p.H * ((p.Nq + kRowsPerWg - 1) / kRowsPerWg);
  const dim3 grid(8 * ((n_wg + 7) / 8));
  if (rows) launch_attention_t<true, false>(p, a, PlanArgs<false>{}, grid, stream);
  else launch_attention_t<false, false>(p, a, PlanArgs<false>{}, grid, stream);
  return hipGetLastError();
}

hipError_t launch_attention_plan(const pbsa_params& p, const bf16_t* Q, const bf16_t* Kp, const bf16_t* Vp,
                                 const int32_t* p_len, const bf16_t* Kl, const bf16_t* Vl, const int32_t* l_len,
                                 const int32_t* l_map, const int32_t* sel, bf16_t* O, float* lse, const float* Qc,
                                 const float* Kc_l, const float* Zl, float* Kc_p, int64_t* p_id, int32_t* S_cnt, int fold,
                                 const int64_t* l_id, float* scores, int32_t* slot_src, const UpdateWs& ws,
                                 hipStream_t stream) {
  const AttnArgs a = attn_args(p, Q, Kp, Vp, p_len, Kl, Vl, l_len, l_map, sel, O, lse, nullptr);
  PlanArgs<true> pl;
  pl.sa = plan_dev::make_score_args(p, Qc, Kc_l, Zl, Kc_p, p_len, l_map, ws);
  pl.ra = plan_dev::make_retain_args(p, ws.A, p.C + p.n_loc, 0, Kc_l, Kc_p, p_len, p_id, S_cnt, fold, l_len, l_map, l_id,
                                     scores, slot_src, ws);
  const int n_wg = p.H * ((p.Nq + kRowsPerWg - 1) / kRowsPerWg);
  const dim3 grid(8 * ((n_wg + 7) / 8) + 8 * ((p.H + 7) / 8));
  launch_attention_t<false, true>(p, a, pl, grid, stream);
  return hipGetLastError();
}

}  // namespace pbsa
