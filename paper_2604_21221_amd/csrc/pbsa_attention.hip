// PBSA fine stage (Eq. 3-5) for gfx950: block-sparse flash attention on bf16 MFMA.
//
// One workgroup = 8 waves = 128 consecutive query tokens of one head (one query block when B = 128,
// two when B = 64).  The workgroup walks a tile list: first every non-empty persistent slot (the
// dense part of the mask, visible to all rows), then the union, in ascending order, of the local
// blocks selected by its query blocks; a wave skips a tile its own query block did not select.
// K/V tiles of 64 keys go from global memory straight into LDS (global_load_lds, no register
// round trip) through rings three tiles deep, so an L2 miss has three slots to arrive.
//
// The 8 waves form two sets of 4 (one wave of each set per SIMD).  Both sets own the same 128 query
// rows (32 per wave) but alternate tiles: set 0 takes the even tiles, set 1 the odd ones, each with
// its own running max / sum / output accumulators, merged at the end.  Time is cut into slots
// separated by workgroup barriers; in slot s the set whose turn it is runs its matrix phase
// (O^T += V^T P^T of its previous tile, then S^T = K Q^T of tile s) while the other set runs the
// softmax of the tile it multiplied one slot earlier.  The two waves sharing a SIMD are thereby
// always in opposite phases, so the MFMA pipe and the VALU (exp2, max, sums, conversions) overlap
// instead of queueing behind each other.
//
// MFMA arrangement (v_mfma_f32_32x32x16_bf16, wave64):
//   S^T = K Q^T   A = K tile rows (32 keys x 16 dims), B = Q^T (16 dims x 32 query rows).
//                 The accumulator then holds, per lane, 16 keys of ONE query row (column lane%32),
//                 so the softmax row reductions are in-lane plus one exchange with lane^32.
//   O^T = V^T P^T A = V^T (32 dims x 16 keys), B = P^T (16 keys x 32 query rows) taken straight
//                 from the S^T accumulators: the contraction index (key) is enumerated in the order
//                 the accumulator holds it, and V^T is read from LDS with the same enumeration.
// Softmax is online, fp32, base 2 (the scale and log2 e are folded into one fma).
#include "pbsa_internal.h"

namespace pbsa {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;

constexpr int kThreads = 512;
constexpr int kRowsPerWg = 128;
constexpr int kTile = 64;                 // keys per staged tile
constexpr int kMaxTiles = 2 * (PBSA_MAX_C + 1) + 2 * PBSA_MAX_K;   // persistent + local 64-key tiles
constexpr float kNegBig = -1.0e30f;

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
template <int D>
__device__ __forceinline__ int k_swz(int row) { return row & (D / 8 - 1); }
template <int D>
__device__ __forceinline__ int v_swz(int row) {
  if constexpr (D == 128) return (row & 3) << 2;
  else return ((row >> 1) & 1) << 2;
}
template <int D>
__device__ __forceinline__ int v_byte_offset(int row, int chunk) {
  return row * (D * 2) + ((chunk ^ v_swz<D>(row)) << 4);
}

// One wave-wide global -> LDS load of 16 bytes per lane: LDS bytes [lds_off, lds_off + 1024) receive
// lane i's 16 bytes at lds_off + 16 i.  Completion is tracked by the issuing wave's vmcnt.
__device__ __forceinline__ void dma16(const void* gptr, uint32_t lds_off) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off"
               :
               : "s"(lds_off), "v"(gptr)
               : "memory");
}

template <int D>
struct Geo {
  static constexpr int KS = D / 16;                 // MFMA k-steps of Q K^T
  static constexpr int DT = D / 32;                 // 32-wide output tiles of O^T
  static constexpr int TILE_BYTES = kTile * D * 2;  // one K or V tile in LDS
  static constexpr int NI = D / 64;                 // global_load_lds instructions per wave per tile
};

// S^T (two 32-key sub-tiles) = K tile x Q^T.
template <int D>
__device__ __forceinline__ void qk_tile(const unsigned char* kbuf, const bf16x8 (&qf)[Geo<D>::KS], int qn, int half,
                                        f32x16& s0, f32x16& s1) {
  const f32x16 zero = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
  // chunk (2 ks + half) ^ f(row) = (half ^ f(row)) ^ 2 ks: one per-lane base, one xor per k-step; rows qn
  // and 32 + qn share the permutation
  const int base = qn * (D * 2) + ((half ^ k_swz<D>(qn)) << 4);
#pragma unroll
  for (int ks = 0; ks < Geo<D>::KS; ++ks) {
    const unsigned char* r0 = kbuf + (base ^ (ks << 5));
    const bf16x8 k0 = *reinterpret_cast<const bf16x8*>(r0);
    const bf16x8 k1 = *reinterpret_cast<const bf16x8*>(r0 + 32 * (D * 2));
    s0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(k0, qf[ks], ks == 0 ? zero : s0, 0, 0, 0);
    s1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(k1, qf[ks], ks == 0 ? zero : s1, 0, 0, 0);
  }
  // operand reads run 4 k-steps (8 MFMAs) ahead of the MFMAs: an LDS read takes several MFMA times
  constexpr int AHEAD = Geo<D>::KS < 4 ? Geo<D>::KS : 4;
  __builtin_amdgcn_sched_group_barrier(0x100, 2 * AHEAD, 0);
#pragma unroll
  for (int ks = 0; ks < Geo<D>::KS - AHEAD; ++ks) {
    __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);
    __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
  }
  __builtin_amdgcn_sched_group_barrier(0x008, 2 * AHEAD, 0);
}

// O^T += V^T P^T: 4 k-steps of 16 keys; V^T fragments by transposing LDS reads.  The fragment of
// k-step j holds keys 16 j + 4 half + {0..3} (lo) and + 8 (hi).
template <int D>
__device__ __forceinline__ void pv_tile(const unsigned char* vbuf, const bf16x8 (&pf)[4], f32x16 (&o)[Geo<D>::DT],
                                        int v_row0, int v_sub, int v_lo) {
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int r0 = 16 * j + v_row0;            // this lane's address rows: r0 and r0 + 8
#pragma unroll
    for (int dt = 0; dt < Geo<D>::DT; ++dt) {
      const bf16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16(
          (bf16x4 __attribute__((address_space(3)))*)(vbuf + v_byte_offset<D>(r0, 4 * dt + v_sub) + v_lo));
      const bf16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16(
          (bf16x4 __attribute__((address_space(3)))*)(vbuf + v_byte_offset<D>(r0 + 8, 4 * dt + v_sub) + v_lo));
      const bf16x8 vf = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
      o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[j], o[dt], 0, 0, 0);
    }
  }
  // operand reads (two per MFMA) run 8 MFMAs ahead: an LDS read takes several MFMA times
  constexpr int N = 4 * Geo<D>::DT, AHEAD = N < 8 ? N : 8;
  __builtin_amdgcn_sched_group_barrier(0x100, 2 * AHEAD, 0);
#pragma unroll
  for (int i = 0; i < N - AHEAD; ++i) {
    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
    __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
  }
  __builtin_amdgcn_sched_group_barrier(0x008, AHEAD, 0);
}

// Online softmax of one tile: S^T accumulators -> bf16 P^T operands; updates the running max and
// the in-lane partial row sum, rescaling the output accumulators only when some row's max moved.
// Accumulator element v of sub-tile st is key 32 st + 8 (v/4) + 4 half + v%4.
template <int DT>
__device__ __forceinline__ void softmax_tile(f32x16& s0, f32x16& s1, int tlen, int half, float c2, float& m_run,
                                             float& l_run, f32x16 (&o)[DT], bf16x8 (&pf)[4]) {
  if (tlen < kTile) {
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      if (8 * (v / 4) + 4 * half + (v % 4) >= tlen) s0[v] = kNegBig;
      if (32 + 8 * (v / 4) + 4 * half + (v % 4) >= tlen) s1[v] = kNegBig;
    }
  }
  float tmax = fmaxf(s0[0], s1[0]);
#pragma unroll
  for (int v = 1; v < 16; ++v) tmax = fmaxf(fmaxf(tmax, s0[v]), s1[v]);
  tmax = fmaxf(tmax, __shfl_xor(tmax, 32, 64));
  const float m_new = fmaxf(m_run, tmax);
  const float mc = -m_new * c2;
  float psum = 0.0f;
#pragma unroll
  for (int v = 0; v < 16; ++v) {
    s0[v] = __builtin_amdgcn_exp2f(__builtin_fmaf(s0[v], c2, mc));
    s1[v] = __builtin_amdgcn_exp2f(__builtin_fmaf(s1[v], c2, mc));
    psum += s0[v] + s1[v];
  }
  if (__any(m_new != m_run)) {
    const float alpha = __builtin_amdgcn_exp2f((m_run - m_new) * c2);
    l_run *= alpha;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
      for (int v = 0; v < 16; ++v) o[dt][v] *= alpha;
    m_run = m_new;
  }
  l_run += psum;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    pf[0][e] = (__bf16)s0[e];
    pf[1][e] = (__bf16)s0[8 + e];
    pf[2][e] = (__bf16)s1[e];
    pf[3][e] = (__bf16)s1[8 + e];
  }
}

// (the kernel marks dead accumulators by assigning an uninitialised value on purpose)
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Wuninitialized"
template <int D, int B>
__global__ void __launch_bounds__(kThreads) attention_kernel(AttnArgs a) {
  constexpr int G = kRowsPerWg / B;        // query blocks per workgroup
  constexpr int SUB = B / kTile;           // 64-key tiles per block
  constexpr int KS = Geo<D>::KS, DT = Geo<D>::DT, TILE = Geo<D>::TILE_BYTES, NI = Geo<D>::NI;
  constexpr int DEPTH = 3;                 // a tile's loads are issued this many slots before its first use
  constexpr int RING = DEPTH + 1;          // ring entries per operand (power of two)
  constexpr int LPS = 2 * NI;              // global_load_lds instructions per wave per slot (K + V)
  constexpr int XROWS = DT * 16 + 2;       // exchange rows per wave pair: O, running max, partial sum
  constexpr int SMEM = 2 * RING * TILE;
  static_assert((RING & (RING - 1)) == 0, "ring size must be a power of two");
  static_assert(4 * XROWS * 256 <= SMEM && PBSA_MAX_N_LOC * 4 <= SMEM, "scratch aliases must fit");

  __shared__ __align__(1024) unsigned char smem[SMEM];   // K ring, then V ring
  __shared__ int t_src[kMaxTiles];         // bit 31: local, bits 0..: (slot * SUB + sub)
  __shared__ int t_meta[kMaxTiles];        // valid keys (bits 0..7) | which of the G query blocks attend (bits 8..)
  __shared__ int n_tiles_s;
  unsigned char* const kring = smem;
  unsigned char* const vring = smem + RING * TILE;
  int* lflag = reinterpret_cast<int*>(smem);        // setup scratch, dead before the first tile is staged

  // XCD-aware mapping: consecutive workgroup ids go round-robin to the 8 XCDs, so give XCD x the
  // contiguous range [x * per, (x+1) * per) of (head, query tile) pairs: neighbours share K/V in L2.
  const int n_qt = (a.Nq + kRowsPerWg - 1) / kRowsPerWg;
  const int n_wg = a.H * n_qt;
  const int per = (n_wg + 7) / 8;
  const int logical = (blockIdx.x % 8) * per + blockIdx.x / 8;
  if (logical >= n_wg) return;
  const int h = logical / n_qt;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int set = wave >> 2, w4 = wave & 3;
  const int T0 = (logical % n_qt) * kRowsPerWg;
  const int i0 = T0 / B;
  const int my_g = (w4 * 32) / B;

  // ---- Q fragments (B operand of S^T = K Q^T): query row = lane % 32, dims 16*ks + 8*(lane/32) ..+8.
  // Issued first so the loads fly while the tile list is built.
  const int qn = lane & 31, half = lane >> 5;
  const int tok = T0 + w4 * 32 + qn;
  const int tok_c = min(tok, a.Nq - 1);
  bf16x8 qf[KS];
  {
    const bf16_t* qrow = a.Q + (size_t)h * a.q_stride_h + (size_t)tok_c * a.q_stride_t + 8 * half;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) qf[ks] = *reinterpret_cast<const bf16x8*>(qrow + 16 * ks);
  }

  // ---- tile list --------------------------------------------------------------------------------
  // Everything the list needs is fetched from global memory in one parallel round into LDS scratch:
  // per local block the set of query blocks that selected it, its length and its physical slot;
  // per persistent slot its length.  Wave 0 then compacts both into the list with ballots.
  int* llen_s = lflag + PBSA_MAX_N_LOC;
  int* lmap_s = llen_s + PBSA_MAX_N_LOC;
  int* plen_s = lmap_s + PBSA_MAX_N_LOC;
  static_assert((3 * PBSA_MAX_N_LOC + PBSA_MAX_C + 1) * 4 <= SMEM, "setup scratch must fit");
  for (int l = tid; l < a.n_loc; l += kThreads) {
    lflag[l] = 0;
    llen_s[l] = a.l_len[l];
    lmap_s[l] = a.l_map[l];
  }
  for (int c = tid; c <= a.C; c += kThreads) plen_s[c] = a.p_len[(size_t)h * (a.C + 1) + c];
  __syncthreads();
  for (int idx = tid; idx < G * a.k; idx += kThreads) {
    const int g = idx / a.k, j = idx % a.k;
    if (i0 + g < a.nqb) {
      const int l = a.sel[((size_t)h * a.nqb + i0 + g) * a.k + j];
      if (l >= 0 && l < a.n_loc) atomicOr(&lflag[l], 1 << g);
    }
  }
  __syncthreads();
  if (wave == 0) {
    int n = 0;
    // a block yields ceil(len / 64) tiles (0, 1 or 2); positions by a wave prefix count
    for (int c0 = 0; c0 <= a.C; c0 += 64) {
      const int c = c0 + lane;
      const int len = c <= a.C ? min(max(plen_s[c], 0), B) : 0;
      const int nt = (len + kTile - 1) / kTile;
      const unsigned long long m1 = __ballot(nt >= 1), m2 = __ballot(nt >= 2);
      const int pos = n + lanes_below(m1) + lanes_below(m2);
      for (int s = 0; s < nt; ++s) {
        t_src[pos + s] = c * SUB + s;
        t_meta[pos + s] = min(kTile, len - s * kTile) | (((1 << G) - 1) << 8);
      }
      n += __popcll(m1) + __popcll(m2);
    }
    for (int l0 = 0; l0 < a.n_loc; l0 += 64) {
      const int l = l0 + lane;
      const int f = l < a.n_loc ? lflag[l] : 0;
      int len = 0, slot = 0;
      if (f) {
        len = min(max(llen_s[l], 0), B);
        slot = lmap_s[l];
        if (slot < 0 || slot >= a.n_loc_cap) len = 0;
      }
      const int nt = f ? (len + kTile - 1) / kTile : 0;
      const unsigned long long m1 = __ballot(nt >= 1), m2 = __ballot(nt >= 2);
      const int pos = n + lanes_below(m1) + lanes_below(m2);
      for (int s = 0; s < nt; ++s) {
        t_src[pos + s] = (int)(0x80000000u | (uint32_t)(slot * SUB + s));
        t_meta[pos + s] = min(kTile, len - s * kTile) | (f << 8);
      }
      n += __popcll(m1) + __popcll(m2);
    }
    if (lane == 0) n_tiles_s = n;
  }
  __syncthreads();
  const int n_tiles = n_tiles_s;

  f32x16 o[DT];
#pragma unroll
  for (int dt = 0; dt < DT; ++dt)
#pragma unroll
    for (int v = 0; v < 16; ++v) o[dt][v] = 0.0f;
  f32x16 s0, s1;
#pragma unroll
  for (int v = 0; v < 16; ++v) { s0[v] = 0.0f; s1[v] = 0.0f; }
  bf16x8 pf[4];
#pragma unroll
  for (int j = 0; j < 4; ++j)
#pragma unroll
    for (int e = 0; e < 8; ++e) pf[j][e] = (__bf16)0.0f;
  float m_run = kNegBig, l_run = 0.0f;
  const float c2 = a.scale * 1.4426950408889634f;

  // ---- staging --------------------------------------------------------------------------------
  // Wave w fills LDS KiB (NI w + n), n < NI, of a tile: rows (64 / (D/8)) (NI w + n) + lane / (D/8),
  // physical chunk lane % (D/8), i.e. the logical chunk (lane % (D/8)) ^ f(row) of that row.
  const uint32_t smem_lds = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)smem;
  constexpr int CH = D / 8, RPI = 64 / CH;          // chunks per row, rows per wave instruction
  // A ragged V tile must not bring rows past its valid length into LDS (they meet p = 0 in the
  // MFMA, and 0 x NaN-or-Inf pattern is NaN): the lanes of such rows fetch the last valid row instead.
  int koff[NI], vrow[NI], vchk[NI];                 // this lane's byte offset / row / chunk offset in a tile
#pragma unroll
  for (int n = 0; n < NI; ++n) {
    const int r = RPI * (NI * wave + n) + lane / CH, c = lane % CH;
    koff[n] = r * (D * 2) + ((c ^ k_swz<D>(r)) << 4);
    vrow[n] = r;
    vchk[n] = (c ^ v_swz<D>(r)) << 4;
  }
  const uint32_t wave_lds = __builtin_amdgcn_readfirstlane(smem_lds + NI * wave * 1024);
  // Byte offset of a tile from the K (or V) base of its cache: descriptor bit 31 picks the cache.
  const size_t head_l = (size_t)h * a.n_loc_cap * B * D * 2, head_p = (size_t)h * (a.C + 1) * B * D * 2;
#define PBSA_TILE_PTR(SRC, BASE_L, BASE_P)                                                              \
  ((SRC) < 0 ? reinterpret_cast<const unsigned char*>(BASE_L) + head_l + (size_t)((SRC) & 0x7FFFFFFF) * (kTile * D * 2) \
             : reinterpret_cast<const unsigned char*>(BASE_P) + head_p + (size_t)(SRC) * (kTile * D * 2))
  // slot S_ issues K(S_ + DEPTH) and V(S_ + DEPTH - 2) given their descriptors.  Indices outside the
  // list are clamped by the caller (the load count per slot stays constant, which the vmcnt
  // arithmetic below relies on; the ring entry such a load lands in is never read).
#define PBSA_ISSUE(S_, SRC_K, SRC_V, LEN_V)                                                             \
  {                                                                                                     \
    const unsigned char* kp_ = PBSA_TILE_PTR(SRC_K, a.Kl, a.Kp);                                        \
    const unsigned char* vp_ = PBSA_TILE_PTR(SRC_V, a.Vl, a.Vp);                                        \
    const uint32_t kl_ = wave_lds + (uint32_t)((((S_) + DEPTH) & (RING - 1)) * TILE);                   \
    const uint32_t vl_ = wave_lds + (uint32_t)((RING + (((S_) + DEPTH - 2) & (RING - 1))) * TILE);      \
    _Pragma("unroll") for (int n_ = 0; n_ < NI; ++n_) dma16(kp_ + koff[n_], kl_ + n_ * 1024);           \
    _Pragma("unroll") for (int n_ = 0; n_ < NI; ++n_)                                                   \
        dma16(vp_ + (min(vrow[n_], (LEN_V) - 1) * (D * 2) + vchk[n_]), vl_ + n_ * 1024);                \
  }
#define PBSA_SRC(IT) __builtin_amdgcn_readfirstlane(t_src[min(max((IT), 0), n_tiles - 1)])
#define PBSA_META(IT) ((IT) >= 0 && (IT) < n_tiles ? __builtin_amdgcn_readfirstlane(t_meta[IT]) : kTile)
  // everything but the loads of the last DEPTH-1 slots has landed
#define PBSA_WAIT_TILES() asm volatile("s_waitcnt vmcnt(%0)" ::"n"(LPS * (DEPTH - 1)) : "memory")

  // per-lane pieces of the V^T operand address: 16-lane group s -> row s/4, chunk pair 2q + (s%4)/2
  const int s16 = lane & 15, q16 = (lane >> 4) & 1;
  const int v_row0 = 4 * half + (s16 >> 2);
  const int v_sub = 2 * q16 + ((s16 & 3) >> 1);
  const int v_lo = (s16 & 1) * 8;

  if (n_tiles > 0) {
    __syncthreads();                       // lflag (aliasing the K ring) is dead
    for (int s = -DEPTH; s < 0; ++s)
      PBSA_ISSUE(s, PBSA_SRC(s + DEPTH), PBSA_SRC(s + DEPTH - 2), PBSA_META(min(max(s + DEPTH - 2, 0), n_tiles - 1)) & 0xFF)
    // Tile descriptors travel in scalar registers and are fetched from LDS one slot before they are
    // needed: src_a/b/c describe tiles s+3, s+2, s+1 (K of s+3 and V of s+1 are issued in slot s);
    // meta_n/0/1/2 are the length/attendance words of tiles s+1, s, s-1, s-2 (a word outside the list
    // has no attendance bit set).
    int src_a = PBSA_SRC(DEPTH), src_b = PBSA_SRC(DEPTH - 1), src_c = PBSA_SRC(DEPTH - 2);
    int meta_n = PBSA_META(1), meta_0 = PBSA_META(0), meta_1 = kTile, meta_2 = kTile;
    PBSA_WAIT_TILES();
    __syncthreads();
    // Slot s: the set whose turn it is multiplies (V(s-2) from its ring entry, then K(s)); the other
    // set runs the softmax of tile s-1.
    for (int s = 0; s < n_tiles + 2; ++s) {
      const int nxt_src_v = t_src[min(s + 1 + DEPTH, n_tiles - 1)];       // consumed at the end of the slot
      const int nxt_meta_v = t_meta[min(s + 2, n_tiles - 1)];
      PBSA_ISSUE(s, src_a, src_c, meta_n & 0xFF)
      if (((s + set) & 1) == 0) {
        {
          // the S^T accumulators are dead here (tile s-2 went through its softmax, tile s is about to be
          // written from zero): say so, or they stay allocated across the whole matrix phase
          f32x16 dead0, dead1;
          s0 = dead0;
          s1 = dead1;
        }
        if ((meta_2 >> (8 + my_g)) & 1) pv_tile<D>(vring + ((s - 2) & (RING - 1)) * TILE, pf, o, v_row0, v_sub, v_lo);
        if ((meta_0 >> (8 + my_g)) & 1) qk_tile<D>(kring + (s & (RING - 1)) * TILE, qf, qn, half, s0, s1);
      } else {
        if ((meta_1 >> (8 + my_g)) & 1) softmax_tile<DT>(s0, s1, meta_1 & 0xFF, half, c2, m_run, l_run, o, pf);
      }
      src_c = src_b; src_b = src_a; src_a = __builtin_amdgcn_readfirstlane(nxt_src_v);
      meta_2 = meta_1; meta_1 = meta_0; meta_0 = meta_n;
      meta_n = s + 2 < n_tiles ? __builtin_amdgcn_readfirstlane(nxt_meta_v) : kTile;
      PBSA_WAIT_TILES();
      __syncthreads();
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // stray clamped loads must not land in the exchange area
  }
  __syncthreads();

  // ---- merge the two sets (same rows, disjoint tiles) and write out ---------------------------
  // exchange layout: per wave pair w4, XROWS rows of 64 floats ([value index][lane]): conflict-free
  float* xch = reinterpret_cast<float*>(smem) + (size_t)w4 * XROWS * 64 + lane;
  if (set == 1) {
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
      for (int v = 0; v < 16; ++v) xch[(dt * 16 + v) * 64] = o[dt][v];
    xch[(DT * 16) * 64] = m_run;
    xch[(DT * 16 + 1) * 64] = l_run;
  }
  __syncthreads();
  if (set == 1) return;
  {
    const float m_b = xch[(DT * 16) * 64], l_b = xch[(DT * 16 + 1) * 64];
    const float m = fmaxf(m_run, m_b);
    const float fa = __builtin_amdgcn_exp2f((m_run - m) * c2), fb = __builtin_amdgcn_exp2f((m_b - m) * c2);
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
      for (int v = 0; v < 16; ++v) o[dt][v] = o[dt][v] * fa + xch[(dt * 16 + v) * 64] * fb;
    l_run = l_run * fa + l_b * fb;
    m_run = m;
  }
  const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
  const float inv = l_tot > 0.0f ? 1.0f / l_tot : 0.0f;
  if (tok < a.Nq) {
    bf16_t* orow = a.O + (size_t)h * a.o_stride_h + (size_t)tok * a.o_stride_t;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        bf16x4 w;
#pragma unroll
        for (int e = 0; e < 4; ++e) w[e] = (__bf16)(o[dt][4 * q4 + e] * inv);
        *reinterpret_cast<bf16x4*>(orow + 32 * dt + 8 * q4 + 4 * half) = w;
      }
    if (a.lse && half == 0)
      a.lse[(size_t)h * a.Nq + tok] = l_tot > 0.0f ? m_run * a.scale + __logf(l_tot) : -INFINITY;
  }
}

#pragma clang diagnostic pop

}  // namespace

hipError_t launch_attention(const pbsa_params& p, const bf16_t* Q, const bf16_t* Kp, const bf16_t* Vp,
                            const int32_t* p_len, const bf16_t* Kl, const bf16_t* Vl, const int32_t* l_len,
                            const int32_t* l_map, const int32_t* sel, bf16_t* O, float* lse, hipStream_t stream) {
  AttnArgs a{p.H, p.Nq, p.nqb, p.n_loc, p.n_loc_cap, p.C, p.k, p.scale, p.q_stride_h, p.q_stride_t,
             p.o_stride_h, p.o_stride_t, Q, Kp, Vp, p_len, Kl, Vl, l_len, l_map, sel, O, lse};
  const int n_wg = p.H * ((p.Nq + kRowsPerWg - 1) / kRowsPerWg);
  const dim3 grid(8 * ((n_wg + 7) / 8)), block(kThreads);
  if (p.d == 128 && p.B == 128) hipLaunchKernelGGL((attention_kernel<128, 128>), grid, block, 0, stream, a);
  else if (p.d == 128 && p.B == 64) hipLaunchKernelGGL((attention_kernel<128, 64>), grid, block, 0, stream, a);
  else if (p.d == 64 && p.B == 128) hipLaunchKernelGGL((attention_kernel<64, 128>), grid, block, 0, stream, a);
  else hipLaunchKernelGGL((attention_kernel<64, 64>), grid, block, 0, stream, a);
  return hipGetLastError();
}

}  // namespace pbsa
