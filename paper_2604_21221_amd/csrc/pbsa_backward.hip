// Backward of the PBSA fine stage for gfx950 (the gradient of Eq. 3-5; the paper's training kernel is
// the block-sparse attention backward).  With P the masked row softmax of Z = scale Q K^T and dO given:
//     dV = P^T dO        dP = dO V^T        dZ = P o (dP - D),  D[q] = dO[q] . O[q]
//     dQ = scale dZ K    dK = scale dZ^T Q
// P is recomputed from the forward's log-sum-exp: exp2(z c2 - lse log2 e); nothing of the forward's
// probabilities is stored.  Three kernels, no atomics, every output element written by exactly one lane:
//   prep   D[h][q] = sum_x dO[q][x] O[q][x]                                      (fp32, from the bf16 tensors)
//   dq     one single-wave workgroup per 64 query rows: their Q and dO fragments stay in registers, the 64-key tiles
//          they attend (persistent slots, then the blocks of their row of sel) stream through LDS
//   dkv    one two-wave workgroup per 64-key tile: its K and V fragments stay in registers, the 64-row tiles of the
//          query blocks that attend it (all of them for a persistent slot; those whose row of sel names the block
//          otherwise, found by scanning sel) stream through LDS
// Both have a fixed side in registers (MFMA B operands) and a streamed side in LDS (A operands):
//   A1 = T1 F1^T, A2 = T2 F2^T   32 streamed rows x 32 fixed rows per MFMA chain (v_mfma_f32_32x32x16_bf16)
//          dq:  T1 = K, T2 = V, F1 = Q, F2 = dO   ->  A1 = Z^T / scale, A2 = dP^T     (keys x queries)
//          dkv: T1 = Q, T2 = dO, F1 = K, F2 = V   ->  A1 = Z / scale,   A2 = dP       (queries x keys)
//   P and dZ, elementwise from A1, A2 and the per-query lse and D, rounded to bf16, are B operands as the
//   accumulators hold them (the contraction index enumerated in accumulator order), and the A operands of the
//   second products are transposing LDS reads of the streamed tiles with the same enumeration:
//          dq:  dQ^T += K^T dZ^T          dkv: dK^T += Q^T dZ,  dV^T += dO^T P
// Tiles go from global memory straight to LDS (global_load_lds), half a tile (32 streamed rows) per ring entry; the
// 16-byte chunks of a row are permuted by the row number so that both the row-wise and the transposing operand
// reads are free of bank conflicts.  Rows past a tile's valid length are never loaded: their lanes fetch the last
// valid row, and the elementwise stage zeroes what belongs to them.  dq holds 64 fixed rows per wave, so every
// fragment read from LDS feeds two MFMAs; dkv cannot at d = 128 (two outputs: 256 accumulator registers for 64
// keys) and holds 32 per wave: it reads one fragment per MFMA and sits at the LDS bandwidth.
#include <type_traits>

#include "pbsa_internal.h"

namespace pbsa {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

constexpr int kThreads = 128;
constexpr int kTile = 64;
constexpr float kLog2e = 1.4426950408889634f;

struct BwdArgs {
  int H, Nq, nqb, n_loc, n_loc_cap, C, k, B;
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
  const bf16_t* O;
  const bf16_t* dO;
  const float* lse;
  float* Dr;          // [H][Nq] rowsum(dO o O)
  float* dQ;
  float* dKp;
  float* dVp;
  float* dKl;
  float* dVl;
};

__device__ __forceinline__ int lanes_below(unsigned long long mask) {
  return __builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0u));
}

// One wave-wide global -> LDS load of 16 bytes per lane: LDS bytes [lds_off, lds_off + 1024) receive lane i's
// 16 bytes at lds_off + 16 i.  Completion is tracked by the issuing wave's vmcnt.
__device__ __forceinline__ void dma16(const void* base, uint32_t lane_off, uint32_t lds_off) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
               :
               : "s"(lds_off), "v"(lane_off), "s"(base)
               : "memory", "m0");
}

// the same with 4 bytes per lane: LDS bytes [lds_off, lds_off + 256)
__device__ __forceinline__ void dma4(const void* base, uint32_t lane_off, uint32_t lds_off) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dword %1, %2"
               :
               : "s"(lds_off), "v"(lane_off), "s"(base)
               : "memory", "m0");
}

// Where the 16-byte chunks of a tile row sit in LDS: logical chunk c of row r at chunk c ^ swz(r).  The row-wise
// operand reads (16 consecutive rows, one logical chunk) need swz distinct over 16 consecutive rows (8 when a row
// has 8 chunks); the transposing reads (4 consecutive rows from a multiple of 4, two adjacent chunks c, c + 1 with
// c even, each) need swz(r) >> 1 distinct over those rows.  The row number rotated left by one bit does both.
template <int CH>
__device__ __forceinline__ int swz(int r) {
  if constexpr (CH == 16) return ((r & 7) << 1) | ((r >> 3) & 1);
  else return ((r & 3) << 1) | ((r >> 2) & 1);
}

typedef __attribute__((address_space(3))) const bf16x8* lds_b128_t;
typedef __attribute__((address_space(3))) bf16x4* lds_tr_t;
__device__ __forceinline__ bf16x8 lds_read_row(uint32_t addr) { return *(lds_b128_t)(uintptr_t)addr; }
// transposed fragment of 16 streamed rows: two transposing reads, rows r and r + 8 of the 16.  HI_XOR: what the
// row permutation does to the byte address when the row goes up by 8.
// off: this lane's byte offset inside the tile (the permutation acts on it), base: LDS address of the tile plus a
// whole number of 16-row groups.
template <int ROW, int HI_XOR>
__device__ __forceinline__ bf16x8 lds_read_tr(uint32_t base, uint32_t off) {
  const bf16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_tr_t)(uintptr_t)(base + off));
  const bf16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_tr_t)(uintptr_t)(base + (off ^ HI_XOR) + 8 * ROW));
  return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
}
__device__ __forceinline__ void acc_mfma(f32x16& acc, const bf16x8& a, const bf16x8& b) {
  asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+a"(acc) : "v"(a), "v"(b));
}
__device__ __forceinline__ uint32_t pack2(float a, float b) {
  bf16x2 pk;
  pk[0] = (__bf16)a;
  pk[1] = (__bf16)b;
  return __builtin_bit_cast(uint32_t, pk);
}
__device__ __forceinline__ bf16x8 as_bf16x8(const u32x4& w) { return __builtin_bit_cast(bf16x8, w); }

// ------------------------------------------------------------------------------------------------
// D[h][q] = dO[q] . O[q]: 16 lanes per row, 8 elements each (d = 128) or 8 lanes (d = 64)
// ------------------------------------------------------------------------------------------------
template <int D>
__global__ void __launch_bounds__(256) bwd_prep_kernel(BwdArgs a) {
  constexpr int LPR = D / 8;               // lanes per row
  const long idx = (long)blockIdx.x * 256 + threadIdx.x;
  const long row = idx / LPR;
  const int part = (int)(idx % LPR);
  float acc = 0.0f;
  const bool ok = row < (long)a.H * a.Nq;
  if (ok) {
    const int h = (int)(row / a.Nq), t = (int)(row % a.Nq);
    const size_t off = (size_t)h * a.o_stride_h + (size_t)t * a.o_stride_t + 8 * part;
    const bf16x8 o = *reinterpret_cast<const bf16x8*>(a.O + off);
    const bf16x8 g = *reinterpret_cast<const bf16x8*>(a.dO + off);
#pragma unroll
    for (int x = 0; x < 8; ++x) acc = __builtin_fmaf((float)o[x], (float)g[x], acc);
  }
#pragma unroll
  for (int s = 1; s < LPR; s <<= 1) acc += __shfl_xor(acc, s, 64);
  if (ok && part == 0) a.Dr[row] = acc;
}

// ------------------------------------------------------------------------------------------------
// dkv: one workgroup (two waves) per 64-key tile
// ------------------------------------------------------------------------------------------------
template <int D>
__global__ void __launch_bounds__(kThreads) bwd_dkv_kernel(BwdArgs a) {
  constexpr int KS = D / 16, DT = D / 32, ROW = D * 2, TILE = kTile * ROW;
  constexpr int CH = D / 8, RPI = 64 / CH;          // 16-byte chunks per row, rows per load instruction
  constexpr int NI = 32 / RPI;                      // load instructions per wave per tile (its 32 rows)
  constexpr int HI_XOR = CH == 16 ? 16 : 0;         // row + 8 flips the lowest bit of the chunk permutation when it has 4 bits
  extern __shared__ __align__(1024) unsigned char smem[];
  __shared__ int cnt_s[2 * 12];
  __shared__ __align__(256) float rows_f[4 * 128];  // per ring entry, lse (64 floats, 32 used) then D of the half tile's rows
  // ring: entry e holds T1 at e * 2 TILE and T2 behind it
  int* lst_a = reinterpret_cast<int*>(smem + 4 * TILE);   // per streamed tile: where it is
  const int SUB = a.B / kTile;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int qn = lane & 31, half = lane >> 5;
  const float c2 = a.scale * kLog2e;

  // ---- what this workgroup is, and the list of streamed tiles ------------------------------------
  int n_cand;
  int* lst_b;                              // per streamed tile: its valid rows
  int* flag_s;                             // query blocks that attend the key block
  // The workgroup's 64-key tile: persistent (slot c) or local (logical block l).  The grid is one line with the
  // persistent tiles of all heads first: every query block attends them, so their workgroups walk the whole chunk
  // and run several times as long as a local block's, and a long workgroup that starts late ends the launch late.
  const int n_pers = (a.C + 1) * SUB, n_locs = a.n_loc * SUB;
  int h, r_tile;
  {
    int b = (int)blockIdx.x;
    if (b < a.H * n_pers) {
      h = b / n_pers;
      r_tile = b % n_pers;
    } else {
      b -= a.H * n_pers;
      h = b / n_locs;
      r_tile = n_pers + b % n_locs;
    }
  }
  int fixed_len = 0, kv_slot_tile = 0;
  bool kv_local = false;
  n_cand = a.nqb * SUB;
  lst_b = lst_a + n_cand;
  flag_s = lst_b + n_cand;
  kv_local = r_tile >= n_pers;
  if (!kv_local) {
    const int c = r_tile / SUB, sub = r_tile % SUB;
    fixed_len = min(max(min(max(a.p_len[(size_t)h * (a.C + 1) + c], 0), a.B) - sub * kTile, 0), kTile);
    kv_slot_tile = r_tile;
  } else {
    const int l = (r_tile - n_pers) / SUB, sub = (r_tile - n_pers) % SUB;
    const int slot = a.l_map[l];
    const bool ok = slot >= 0 && slot < a.n_loc_cap;
    fixed_len = ok ? min(max(min(max(a.l_len[l], 0), a.B) - sub * kTile, 0), kTile) : 0;
    kv_slot_tile = (ok ? slot : 0) * SUB + sub;
    for (int i = tid; i < a.nqb; i += kThreads) flag_s[i] = 0;
    __syncthreads();
    // the head's rows of sel, eight loads in flight per thread (one at a time the scan is a chain of memory latencies)
    const int32_t* sel_h = a.sel + (size_t)h * a.nqb * a.k;
    const int n_sel = a.nqb * a.k;
    for (int e0 = tid; e0 < n_sel; e0 += 8 * kThreads) {
      int v[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) v[j] = e0 + j * kThreads < n_sel ? sel_h[e0 + j * kThreads] : -1;
#pragma unroll
      for (int j = 0; j < 8; ++j)
        if (v[j] == l) flag_s[(e0 + j * kThreads) / a.k] = 1;
    }
    if (!ok) fixed_len = -1;             // a block that is nowhere: nothing to write either
  }
  __syncthreads();
  if (fixed_len < 0) return;
  auto classify = [&](int i, int& where, int& rows) -> bool {
    if (i >= n_cand) return false;
    const int ib = i / SUB;
    if (fixed_len <= 0 || (kv_local && !flag_s[ib])) return false;
    rows = min(kTile, a.Nq - i * kTile);            // row tile i covers tokens 64 i ..
    where = i;
    return rows > 0;
  };
  constexpr int kMaxRounds = 12;           // (2 (C_max + 1) + 2 k_max) / 128 rounded up; dkv needs 8
  const int n_rounds = min((n_cand + kThreads - 1) / kThreads, kMaxRounds);
  // every candidate is looked at once (a look is a chain of dependent loads); what it found stays in registers
  // until the counts of all rounds are known
  int c_where[kMaxRounds], c_rows[kMaxRounds];
  unsigned long long c_mask[kMaxRounds];
#pragma unroll
  for (int r = 0; r < kMaxRounds; ++r) {
    c_where[r] = 0;
    c_rows[r] = 0;
    const bool on = r < n_rounds && classify(r * kThreads + tid, c_where[r], c_rows[r]);
    c_mask[r] = __ballot(on);
    if (r < n_rounds && lane == 0) cnt_s[r * 2 + wave] = __popcll(c_mask[r]);
  }
  __syncthreads();
  int n_tiles = 0;
  for (int q = 0; q < 2 * n_rounds; ++q) n_tiles += cnt_s[q];
#pragma unroll
  for (int r = 0; r < kMaxRounds; ++r) {
    if (r < n_rounds && ((c_mask[r] >> lane) & 1)) {
      int pos = lanes_below(c_mask[r]);
      for (int q = 0; q < r * 2 + wave; ++q) pos += cnt_s[q];
      lst_a[pos] = c_where[r];
      lst_b[pos] = c_rows[r];
    }
  }
  __syncthreads();

  // ---- fixed fragments (B operands): fixed row 32 w + lane % 32, dims 16 ks + 8 (lane / 32) .. + 8 ----
  bf16x8 f1[KS], f2[KS];
  {
    const int row = min(32 * wave + qn, max(fixed_len, 1) - 1);
    const bf16_t *p1, *p2;
    const size_t base = kv_local ? ((size_t)h * a.n_loc_cap * a.B + (size_t)kv_slot_tile * kTile) * D
                                 : ((size_t)h * (a.C + 1) * a.B + (size_t)kv_slot_tile * kTile) * D;
    p1 = (kv_local ? a.Kl : a.Kp) + base + (size_t)row * D;
    p2 = (kv_local ? a.Vl : a.Vp) + base + (size_t)row * D;
  
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      f1[ks] = *reinterpret_cast<const bf16x8*>(p1 + 16 * ks + 8 * half);
      f2[ks] = *reinterpret_cast<const bf16x8*>(p2 + 16 * ks + 8 * half);
    }
  }
  // they have arrived before the walk starts: no wait for them inside it, where one would also wait for the tiles
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) asm volatile("" : "+v"(f1[ks]), "+v"(f2[ks]));

  f32x16 out1[DT], out2[DT];               // dK^T and dV^T   (32 dims x 32 keys each)
#pragma unroll
  for (int dt = 0; dt < DT; ++dt)
#pragma unroll
    for (int v = 0; v < 16; ++v) out1[dt][v] = out2[dt][v] = 0.0f;
  // The output accumulators are only ever touched by the second products: they live in the accumulator half of the
  // register file for the whole walk (the products are issued as instructions with an accumulator destination), which
  // leaves the architectural half to the fragments, the first products' results and the elementwise stage.
#pragma unroll
  for (int dt = 0; dt < DT; ++dt) {
    asm volatile("" : "+a"(out1[dt]));
    asm volatile("" : "+a"(out2[dt]));
  }

  // ---- LDS addresses of this lane's operand reads inside ring entry 0 -------------------------------
  const uint32_t smem_lds = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)smem;
  const uint32_t ring_s = __builtin_amdgcn_readfirstlane(smem_lds);
  const uint32_t rows_s = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)(__attribute__((address_space(3))) float*)rows_f);
  uint32_t ra[KS], ta[DT];
  {
    const int kb = qn * ROW + ((half ^ swz<CH>(qn)) << 4);              // row lane % 32, logical chunk 2 ks + half
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) ra[ks] = smem_lds + (uint32_t)(kb ^ (ks << 5));
    const int s16 = lane & 15, q16 = (lane >> 4) & 1;
    const int row0 = 4 * half + (s16 >> 2);                              // address row within 16 streamed rows
    const int sub = 2 * q16 + ((s16 & 3) >> 1), lo = (s16 & 1) * 8;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) ta[dt] = (uint32_t)(row0 * ROW + (((4 * dt + sub) ^ swz<CH>(row0)) << 4) + lo);
  }

  // ---- staging -------------------------------------------------------------------------------------
  // The unit that travels is a half tile: 32 streamed rows of T1 and of T2 (and, dkv, the lse and D of those
  // rows), one ring entry of four.  Wave w brings rows 16 w .. 16 w + 15 of the half.  Every wave issues the same
  // number of loads per half tile, so that one count serves the wait; past the end of the list the last half tile
  // is fetched again into an entry whose contents are never used.
  constexpr int HALF = TILE / 2, RING = 4, NH = NI / 2;    // NH: load instructions per wave, tensor and half tile
  constexpr int PER = 2 * NH + 2;               // loads per wave and half tile
  const int rl = lane / CH;
  const int n_half = 2 * n_tiles;
  long st1, st2;                           // row strides of the streamed tensors in bytes
  const unsigned char *b1l, *b2l, *b1p, *b2p;
  st1 = a.q_stride_t * 2;
  st2 = a.o_stride_t * 2;
  b1l = b1p = reinterpret_cast<const unsigned char*>(a.Q + (size_t)h * a.q_stride_h);
  b2l = b2p = reinterpret_cast<const unsigned char*>(a.dO + (size_t)h * a.o_stride_h);
  // per-lane source offsets of the wave's instructions within a half tile whose 32 rows all exist
  uint32_t so1[NH], so2[NH];
#pragma unroll
  for (int k = 0; k < NH; ++k) {
    const int r = 16 * wave + RPI * k + rl;
    const uint32_t chunk = (uint32_t)(((lane % CH) ^ swz<CH>(r)) << 4);
    so1[k] = (uint32_t)(r * st1) + chunk;
    so2[k] = (uint32_t)(r * st2) + chunk;
  }
  auto stage = [&](int u, int entry) {
    const int t = u >> 1, mg = u & 1;
    const int where = __builtin_amdgcn_readfirstlane(lst_a[t]);
    const int last = __builtin_amdgcn_readfirstlane(lst_b[t]) - 1;
    const size_t tile = (size_t)(where & 0x7FFFFFFF) * kTile;          // first row of the tile in its tensor
    const unsigned char* s1 = (where < 0 ? b1l : b1p) + tile * st1;
    const unsigned char* s2 = (where < 0 ? b2l : b2p) + tile * st2;
    const uint32_t dst = ring_s + (uint32_t)(entry * TILE + wave * (HALF / 2));
    if (last >= 32 * mg + 31) {
      s1 += (size_t)(32 * mg) * st1;
      s2 += (size_t)(32 * mg) * st2;
#pragma unroll
      for (int k = 0; k < NH; ++k) {
        dma16(s1, so1[k], dst + k * 1024);
        dma16(s2, so2[k], dst + HALF + k * 1024);
      }
    } else {                               // rows past the last one that exists are not touched: that row again
#pragma unroll
      for (int k = 0; k < NH; ++k) {
        const int r = 16 * wave + RPI * k + rl, src_row = min(32 * mg + r, last);
        const uint32_t chunk = (uint32_t)(((lane % CH) ^ swz<CH>(r)) << 4);
        dma16(s1, (uint32_t)(src_row * st1) + chunk, dst + k * 1024);
        dma16(s2, (uint32_t)(src_row * st2) + chunk, dst + HALF + k * 1024);
      }
    }
    // lse and D of the half's 32 rows, as they are (lanes 32..63 repeat lanes 0..31; both waves bring the same)
    const int tok = min(where * kTile + min(32 * mg + qn, last), a.Nq - 1);
    dma4(a.lse + (size_t)h * a.Nq, (uint32_t)tok * 4u, rows_s + (uint32_t)(entry * 512));
    dma4(a.Dr + (size_t)h * a.Nq, (uint32_t)tok * 4u, rows_s + (uint32_t)(entry * 512 + 256));
  
  };

  // ---- the walk: a software pipeline over half tiles ---------------------------------------------------
  // In turn u the wave runs the first products of half tile u+1 (A1, A2: 2 KS MFMAs) with the elementwise stage
  // of half tile u cut into as many slices, one behind each MFMA, so that the vector unit works while the
  // matrix pipe does; then the second products of half tile u.  Half tile u+1 must have landed when turn u
  // starts, u+2 is on its way, u+3 is asked for at the start of the turn (into the entry u-1 has left).
  constexpr int NS = 2 * KS, EPS = 16 / NS;                // slices, accumulator elements per slice
  static_assert(EPS * NS == 16 && (EPS == 1 || EPS == 2), "slices cover the 16 elements, pairs stay together");
  const f32x16 zero = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
  f32x16 c1 = zero, c2a = zero;            // A1, A2 of the half tile whose elementwise stage comes next
  if (n_half > 0) {
    for (int j = 0; j < RING - 1; ++j) stage(min(j, n_half - 1), j);
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"((RING - 2) * PER) : "memory");
    __syncthreads();
    bf16x8 x1[KS], x2[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      x1[ks] = lds_read_row(ra[ks]);
      x2[ks] = lds_read_row(ra[ks] + HALF);
    }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      c1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(x1[ks], f1[ks], c1, 0, 0, 0);
      c2a = __builtin_amdgcn_mfma_f32_32x32x16_bf16(x2[ks], f2[ks], c2a, 0, 0, 0);
    }
  }
  // Two turns per tile, so that the accumulator sets trade places by name (no copies) and the half is a constant.
  auto turn = [&](auto MG, int t, const f32x16& c1, const f32x16& c2a, f32x16& n1, f32x16& n2) {
    constexpr int mg = decltype(MG)::value;
    const int u = 2 * t + mg, e = 2 * (t & 1) + mg, en = (e + 1) % RING;
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"((RING - 3) * PER) : "memory");   // this wave's rows of half tile u+1 are in
    __syncthreads();                                        // everybody's are, and half tile u-1 has been used by all
    stage(min(u + RING - 1, n_half - 1), (u + RING - 1) % RING);
    const int rows = __builtin_amdgcn_readfirstlane(lst_b[t]);
    const uint32_t off1 = (uint32_t)(e * TILE), off2 = off1 + HALF, offn = (uint32_t)(en * TILE);
    // operand reads: the next half tile's rows for its first products, this one's transposed for its second ones
    bf16x8 x1[KS], x2[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      x1[ks] = lds_read_row(ra[ks] + offn);
      x2[ks] = lds_read_row(ra[ks] + offn + HALF);
    }
    // Row scalars and the transposed fragments are asked for inside the slices, shortly before they are
    // needed: the scalars of four streamed rows two slices ahead of their first use, the fragments two (one) per
    // slice over the second half of the slices, when the row fragments they replace in the register file are dead.
    float nlv[16], dv[16];
    auto fetch_scalars = [&](int g) {      // rows 8 g + 4 half .. + 3 of the half tile: elements 4 g .. 4 g + 3
      const float4 n4 = *reinterpret_cast<const float4*>(&rows_f[e * 128 + 8 * g + 4 * half]);
      const float4 d4 = *reinterpret_cast<const float4*>(&rows_f[e * 128 + 64 + 8 * g + 4 * half]);
      nlv[4 * g] = n4.x; nlv[4 * g + 1] = n4.y; nlv[4 * g + 2] = n4.z; nlv[4 * g + 3] = n4.w;
      dv[4 * g] = d4.x; dv[4 * g + 1] = d4.y; dv[4 * g + 2] = d4.z; dv[4 * g + 3] = d4.w;
    
    };
    constexpr int NTF = 2 * 2 * DT, TPS = NTF / (NS / 2);   // transposed fragments, per slice of the second half
    static_assert(TPS * (NS / 2) == NTF, "the transposed reads spread evenly");
    bf16x8 tf[NTF];                        // [tensor][j][dt]
    fetch_scalars(0);
    __builtin_amdgcn_sched_barrier(0);
    // accumulator element v: streamed row 32 mg + 8 (v / 4) + 4 half + v % 4, fixed row 32 w + lane % 32.  Streamed
    // rows past the tile's length hold a copy of its last row and take no part; a fixed row that does not exist
    // only fills its own column of the outputs, which is not written.
    const int lim = rows - 32 * mg - 4 * half;
    u32x4 eP[2], eZ[2];
    float pz[16], zz[16];
#pragma unroll
    for (int sl = 0; sl < NS; ++sl) {
      const int ks = sl / 2;
      if (sl % 2 == 0) n1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(x1[ks], f1[ks], ks == 0 ? zero : n1, 0, 0, 0);
      else n2 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(x2[ks], f2[ks], ks == 0 ? zero : n2, 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);   // the MFMA first, then the slice
      {
        // scalars of the group whose first element comes two slices from now
        const int v_ahead = (sl + 2) * EPS;
        if (v_ahead < 16 && v_ahead % 4 == 0 && (sl + 1) * EPS % 4 != 0) fetch_scalars(v_ahead / 4);
        else if (EPS == 2 && v_ahead < 16 && v_ahead % 4 == 0) fetch_scalars(v_ahead / 4);
      }
      if (sl >= NS / 2) {
#pragma unroll
        for (int q = 0; q < TPS; ++q) {
          const int i = (sl - NS / 2) * TPS + q, tensor = i / (2 * DT), j = (i / DT) % 2, dt = i % DT;
          tf[i] = lds_read_tr<ROW, HI_XOR>(smem_lds + (uint32_t)(16 * j * ROW) + (tensor ? off2 : off1), ta[dt]);
        }
      }
#pragma unroll
      for (int q = 0; q < EPS; ++q) {
        const int v = sl * EPS + q;
        const float nl = -nlv[v] * kLog2e, dd = dv[v];
        const float pe = __builtin_amdgcn_exp2f(__builtin_fmaf(c1[v], c2, nl));
        pz[v] = 8 * (v / 4) + (v % 4) < lim ? pe : 0.0f;
        zz[v] = pz[v] * (c2a[v] - dd);
        if (v % 2 == 1) {
          eP[v / 8][(v % 8) / 2] = pack2(pz[v - 1], pz[v]);
          eZ[v / 8][(v % 8) / 2] = pack2(zz[v - 1], zz[v]);
        }
      }
      __builtin_amdgcn_sched_barrier(0);
    }
    asm volatile("s_nop 4" ::: "memory");   // the last slice's operands are written before the products that read them issue
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int dt = 0; dt < DT; ++dt) {
        acc_mfma(out1[dt], tf[j * DT + dt], as_bf16x8(eZ[j]));
        acc_mfma(out2[dt], tf[(2 + j) * DT + dt], as_bf16x8(eP[j]));
      }
    __builtin_amdgcn_sched_barrier(0);
  };
  {
    f32x16 d1, d2;                         // the other accumulator set
    for (int t = 0; t < n_tiles; ++t) {
      turn(std::integral_constant<int, 0>{}, t, c1, c2a, d1, d2);
      turn(std::integral_constant<int, 1>{}, t, d1, d2, c1, c2a);
    }
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");         // the trailing loads land before the workgroup goes
  // the compiler does not see the matrix instructions that wrote the output accumulators: let the pipe drain
#pragma unroll
  for (int dt = 0; dt < DT; ++dt) {
    asm volatile("s_nop 15\n\ts_nop 15" : "+a"(out1[dt]));
    asm volatile("" : "+a"(out2[dt]));
  }

  // ---- outputs: element v of tile dt is dim 32 dt + 8 (v / 4) + 4 half + v % 4 of fixed row 32 w + lane % 32 ----
  const int frow = 32 * wave + qn;
  // every row of the tile's slot is written: zeros past the valid length and for a block nobody attends
  const size_t base = kv_local ? ((size_t)h * a.n_loc_cap * a.B + (size_t)kv_slot_tile * kTile) * D
                               : ((size_t)h * (a.C + 1) * a.B + (size_t)kv_slot_tile * kTile) * D;
  float* ok_ = (kv_local ? a.dKl : a.dKp) + base + (size_t)frow * D;
  float* ov_ = (kv_local ? a.dVl : a.dVp) + base + (size_t)frow * D;
  const float sc = frow < fixed_len ? a.scale : 0.0f, one = frow < fixed_len ? 1.0f : 0.0f;
#pragma unroll
  for (int dt = 0; dt < DT; ++dt)
#pragma unroll
    for (int v4 = 0; v4 < 4; ++v4) {
      *reinterpret_cast<float4*>(ok_ + 32 * dt + 8 * v4 + 4 * half) =
          make_float4(out1[dt][4 * v4] * sc, out1[dt][4 * v4 + 1] * sc, out1[dt][4 * v4 + 2] * sc, out1[dt][4 * v4 + 3] * sc);
      *reinterpret_cast<float4*>(ov_ + 32 * dt + 8 * v4 + 4 * half) =
          make_float4(out2[dt][4 * v4] * one, out2[dt][4 * v4 + 1] * one, out2[dt][4 * v4 + 2] * one, out2[dt][4 * v4 + 3] * one);
    }
}

// ------------------------------------------------------------------------------------------------
// dq with 64 query rows per wave.  One workgroup = one wave = 64 query rows (two MFMA column groups of 32), so
// that every K or V fragment read from LDS -- row-wise for the first products, transposed for the second --
// feeds two MFMAs: the kernel above, where a wave owns 32 rows, reads one fragment per MFMA and is bound by the
// LDS bandwidth.  The wave stages its own half tiles (32 keys of K and of V per ring entry, two entries) and is
// the only one to read them: no barrier anywhere.  Q and dO fragments and the dQ^T accumulators fill the
// accumulator half of the register file (128 + 128 registers at d = 128).  A turn, on one half tile:
//     first products of column group 0            (2 KS MFMAs)
//     first products of column group 1            (2 KS MFMAs)  with the elementwise stage of group 0 behind them
//     second products of group 0                  (2 DT MFMAs)  with the elementwise stage of group 1 behind them
//     second products of group 1                  (2 DT MFMAs)
// ------------------------------------------------------------------------------------------------
template <int LDS_IMM>
__device__ __forceinline__ void dma16x4(const void* base, uint32_t o0, uint32_t o1, uint32_t o2, uint32_t o3, uint32_t lds_base) {
  // four loads 1 KiB apart in LDS and in memory alike: the instruction's offset moves both addresses
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
__global__ void __launch_bounds__(64) __attribute__((amdgpu_waves_per_eu(1, 1))) bwd_dq_kernel(BwdArgs a) {
  constexpr int KS = D / 16, DT = D / 32, ROW = D * 2, TILE = kTile * ROW, HALF = TILE / 2;
  constexpr int CH = D / 8, RPI = 64 / CH;          // 16-byte chunks per row, rows per load instruction
  constexpr int NW = (32 / RPI) / 4;                // windows of four load instructions per tensor and half tile: 2 or 1
  constexpr int HI_XOR = CH == 16 ? 16 : 0;
  constexpr int NS = 2 * KS, EPS = 16 / NS;         // slices behind the first products, elements per slice
  extern __shared__ __align__(1024) unsigned char smem[];
  // ring: entry e holds 32 rows of K at e * TILE and 32 rows of V behind them
  int* lst_a = reinterpret_cast<int*>(smem + 2 * TILE);
  const int SUB = a.B / kTile;
  const int lane = threadIdx.x;
  const int qn = lane & 31, half = lane >> 5;
  const int h = blockIdx.y, r_tile = blockIdx.x;
  const float c2 = a.scale * kLog2e;
  const int i_blk = r_tile * kTile / a.B;
  const int n_pers = (a.C + 1) * SUB, n_cand = n_pers + a.k * SUB;
  int* lst_b = lst_a + n_cand;
  const int fixed_len = min(kTile, a.Nq - r_tile * kTile);

  // ---- the tiles these rows attend: persistent slots, then the blocks of their row of sel -----------------
  int n_tiles = 0;
  for (int i0 = 0; i0 < n_cand; i0 += 64) {
    const int i = i0 + lane;
    int where = 0, rows = 0;
    if (i < n_pers) {
      const int c = i / SUB, sub = i % SUB;
      rows = min(max(min(max(a.p_len[(size_t)h * (a.C + 1) + c], 0), a.B) - sub * kTile, 0), kTile);
      where = i;
    } else if (i < n_cand) {
      const int jj = (i - n_pers) / SUB, sub = (i - n_pers) % SUB;
      const int l = a.sel[((size_t)h * a.nqb + i_blk) * a.k + jj];
      if (l >= 0 && l < a.n_loc) {
        const int slot = a.l_map[l];
        if (slot >= 0 && slot < a.n_loc_cap) {
          rows = min(max(min(max(a.l_len[l], 0), a.B) - sub * kTile, 0), kTile);
          where = (int)(0x80000000u | (uint32_t)(slot * SUB + sub));
        }
      }
    }
    const unsigned long long m = __ballot(rows > 0);
    if (rows > 0) {
      const int pos = n_tiles + lanes_below(m);
      lst_a[pos] = where;
      lst_b[pos] = rows;
    }
    n_tiles += __popcll(m);
  }
  n_tiles = __builtin_amdgcn_readfirstlane(n_tiles);

  // ---- fixed fragments (B operands) of both column groups: row 32 n + lane % 32, dims 16 ks + 8 (lane / 32) .. + 8 ----
  bf16x8 f1[2][KS], f2[2][KS];
  float nl_fix[2], d_fix[2];
#pragma unroll
  for (int n = 0; n < 2; ++n) {
    const int row = min(32 * n + qn, fixed_len - 1), tok = r_tile * kTile + row;
    const bf16_t* p1 = a.Q + (size_t)h * a.q_stride_h + (size_t)tok * a.q_stride_t;
    const bf16_t* p2 = a.dO + (size_t)h * a.o_stride_h + (size_t)tok * a.o_stride_t;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      f1[n][ks] = *reinterpret_cast<const bf16x8*>(p1 + 16 * ks + 8 * half);
      f2[n][ks] = *reinterpret_cast<const bf16x8*>(p2 + 16 * ks + 8 * half);
    }
    const float l = a.lse[(size_t)h * a.Nq + tok];
    nl_fix[n] = 32 * n + qn < fixed_len && l > -INFINITY ? -l * kLog2e : -INFINITY;
    d_fix[n] = a.Dr[(size_t)h * a.Nq + tok];
  }
  // only ever MFMA operands: they live in the accumulator half of the register file (and have arrived: no wait
  // for them inside the walk, where one would also wait for the tiles)
#pragma unroll
  for (int n = 0; n < 2; ++n) {
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) asm volatile("" : "+a"(f1[n][ks]), "+a"(f2[n][ks]));
    asm volatile("" : "+v"(nl_fix[n]), "+v"(d_fix[n]));
  }
  f32x16 out[2][DT];                       // dQ^T: 32 dims x 32 rows per tile
#pragma unroll
  for (int n = 0; n < 2; ++n)
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) {
#pragma unroll
      for (int v = 0; v < 16; ++v) out[n][dt][v] = 0.0f;
      asm volatile("" : "+a"(out[n][dt]));
    }

  // ---- LDS addresses of this lane's operand reads inside ring entry 0 ----------------------------------
  const uint32_t smem_lds = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)smem;
  const uint32_t ring_s = __builtin_amdgcn_readfirstlane(smem_lds);
  uint32_t ra[KS], ta[DT];
  {
    const int kb = qn * ROW + ((half ^ swz<CH>(qn)) << 4);
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) ra[ks] = smem_lds + (uint32_t)(kb ^ (ks << 5));
    const int s16 = lane & 15, q16 = (lane >> 4) & 1;
    const int row0 = 4 * half + (s16 >> 2);
    const int sub = 2 * q16 + ((s16 & 3) >> 1), lo = (s16 & 1) * 8;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) ta[dt] = (uint32_t)(row0 * ROW + (((4 * dt + sub) ^ swz<CH>(row0)) << 4) + lo);
  }

  // ---- staging: the wave brings whole half tiles (32 rows of K and of V, dense rows) ---------------------
  const int rl = lane / CH;
  uint32_t so[4];                          // per-lane source offsets of the four instructions of a window
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    const int r = RPI * k + rl;            // the permutation repeats every 16 rows (8 when a row has 8 chunks)
    so[k] = (uint32_t)(r * ROW) + (uint32_t)(((lane % CH) ^ swz<CH>(r)) << 4) - (uint32_t)(k * 1024);
  }
  const size_t hl = (size_t)h * a.n_loc_cap * a.B * D * 2, hp = (size_t)h * (a.C + 1) * a.B * D * 2;
  const unsigned char* kl = reinterpret_cast<const unsigned char*>(a.Kl) + hl;
  const unsigned char* vl = reinterpret_cast<const unsigned char*>(a.Vl) + hl;
  const unsigned char* kp = reinterpret_cast<const unsigned char*>(a.Kp) + hp;
  const unsigned char* vp = reinterpret_cast<const unsigned char*>(a.Vp) + hp;
  auto stage = [&](int u, int entry) {
    const int t = u >> 1, mg = u & 1;
    const int where = __builtin_amdgcn_readfirstlane(lst_a[t]);
    const int last = __builtin_amdgcn_readfirstlane(lst_b[t]) - 1;
    const size_t off = (size_t)(where & 0x7FFFFFFF) * TILE;
    const unsigned char* s1 = (where < 0 ? kl : kp) + off;
    const unsigned char* s2 = (where < 0 ? vl : vp) + off;
    const uint32_t dst = ring_s + (uint32_t)(entry * TILE);
    if (last >= 32 * mg + 31) {
#pragma unroll
      for (int w = 0; w < NW; ++w) {
        dma16x4<0>(s1 + 32 * mg * ROW + w * 4096, so[0], so[1], so[2], so[3], dst + w * 4096);
        dma16x4<0>(s2 + 32 * mg * ROW + w * 4096, so[0], so[1], so[2], so[3], dst + HALF + w * 4096);
      }
    } else {                               // rows past the last one that exists are not touched: that row again
#pragma unroll
      for (int k = 0; k < 4 * NW; ++k) {
        const int r = RPI * k + rl, src_row = min(32 * mg + r, last);
        const uint32_t chunk = (uint32_t)(((lane % CH) ^ swz<CH>(r)) << 4);
        dma16(s1, (uint32_t)(src_row * ROW) + chunk, dst + k * 1024);
        dma16(s2, (uint32_t)(src_row * ROW) + chunk, dst + HALF + k * 1024);
      }
    }
  };

  const f32x16 zero = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
  const int n_half = 2 * n_tiles;
  if (n_half > 0) stage(0, 0);
  auto turn = [&](auto MG, int t) {
    constexpr int mg = decltype(MG)::value;
    const int u = 2 * t + mg, e = mg;      // two turns per tile: the entry is the half
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");        // half tile u is in (nobody else reads or writes the ring)
    if (u + 1 < n_half) stage(u + 1, e ^ 1);
    const int rows = __builtin_amdgcn_readfirstlane(lst_b[t]);
    const int lim = rows - 32 * mg - 4 * half;
    const uint32_t off1 = (uint32_t)(e * TILE), off2 = off1 + HALF;
    bf16x8 x1[KS], x2[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      x1[ks] = lds_read_row(ra[ks] + off1);
      x2[ks] = lds_read_row(ra[ks] + off2);
    }
    __builtin_amdgcn_sched_barrier(0);
    f32x16 a1[2], a2[2];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      a1[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(x1[ks], f1[0][ks], ks == 0 ? zero : a1[0], 0, 0, 0);
      a2[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(x2[ks], f2[0][ks], ks == 0 ? zero : a2[0], 0, 0, 0);
    }
    __builtin_amdgcn_sched_barrier(0);
    // accumulator element v: key 32 mg + 8 (v / 4) + 4 half + v % 4, query row 32 n + lane % 32.  Keys past the
    // tile's length hold a copy of its last row and take no part; a query row that does not exist has nl = -inf.
    u32x4 eZ[2][2];
    bf16x8 tf[2][DT];
    auto element = [&](int n, int v, float (&zz)[16]) {
      const float pe = __builtin_amdgcn_exp2f(__builtin_fmaf(a1[n][v], c2, nl_fix[n]));
      const float pm = 8 * (v / 4) + (v % 4) < lim ? pe : 0.0f;
      zz[v] = pm * (a2[n][v] - d_fix[n]);
      if (v % 2 == 1) eZ[n][v / 8][(v % 8) / 2] = pack2(zz[v - 1], zz[v]);
    };
    {
      float zz[16];
#pragma unroll
      for (int sl = 0; sl < NS; ++sl) {
        const int ks = sl / 2;
        if (sl % 2 == 0) a1[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(x1[ks], f1[1][ks], ks == 0 ? zero : a1[1], 0, 0, 0);
        else a2[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(x2[ks], f2[1][ks], ks == 0 ? zero : a2[1], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
        if (sl >= NS - 2 * DT) {           // the transposed fragments, asked for over the last slices
          const int i = sl - (NS - 2 * DT);
          tf[i / DT][i % DT] = lds_read_tr<ROW, HI_XOR>(smem_lds + (uint32_t)(16 * (i / DT) * ROW) + off1, ta[i % DT]);
        }
#pragma unroll
        for (int q = 0; q < EPS; ++q) element(0, sl * EPS + q, zz);
        __builtin_amdgcn_sched_barrier(0);
      }
    }
    asm volatile("s_nop 4" ::: "memory");
    {
      float zz[16];
      constexpr int EP2 = 16 / (2 * DT);   // elements of group 1 behind each second product of group 0
#pragma unroll
      for (int i = 0; i < 2 * DT; ++i) {
        acc_mfma(out[0][i % DT], tf[i / DT][i % DT], as_bf16x8(eZ[0][i / DT]));
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int q = 0; q < EP2; ++q) element(1, i * EP2 + q, zz);
        __builtin_amdgcn_sched_barrier(0);
      }
    }
    asm volatile("s_nop 4" ::: "memory");
#pragma unroll
    for (int i = 0; i < 2 * DT; ++i) acc_mfma(out[1][i % DT], tf[i / DT][i % DT], as_bf16x8(eZ[1][i / DT]));
    __builtin_amdgcn_sched_barrier(0);
  };
  for (int t = 0; t < n_tiles; ++t) {
    turn(std::integral_constant<int, 0>{}, t);
    turn(std::integral_constant<int, 1>{}, t);
  }
  // the compiler does not see the matrix instructions that wrote the output accumulators: let the pipe drain
#pragma unroll
  for (int n = 0; n < 2; ++n)
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) asm volatile("s_nop 15\n\ts_nop 15" : "+a"(out[n][dt]));
#pragma unroll
  for (int n = 0; n < 2; ++n) {
    const int frow = 32 * n + qn;
    if (frow < fixed_len) {
      float* o = a.dQ + ((size_t)h * a.Nq + (size_t)r_tile * kTile + frow) * D;
#pragma unroll
      for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int v4 = 0; v4 < 4; ++v4)
          *reinterpret_cast<float4*>(o + 32 * dt + 8 * v4 + 4 * half) =
              make_float4(out[n][dt][4 * v4] * a.scale, out[n][dt][4 * v4 + 1] * a.scale, out[n][dt][4 * v4 + 2] * a.scale,
                          out[n][dt][4 * v4 + 3] * a.scale);
    }
  }
}

template <typename K>
hipError_t launch_with_lds(K kernel, const BwdArgs& a, dim3 grid, int threads, size_t lds, hipStream_t stream) {
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(kernel, grid, dim3(threads), lds, stream, a);
  return hipGetLastError();
}

}  // namespace

size_t bwd_workspace_bytes(const pbsa_params& p) { return (((size_t)p.H * p.Nq * 4) + 255) & ~(size_t)255; }

hipError_t launch_attention_bwd(const pbsa_params& p, const bf16_t* Q, const bf16_t* Kp, const bf16_t* Vp,
                                const int32_t* p_len, const bf16_t* Kl, const bf16_t* Vl, const int32_t* l_len,
                                const int32_t* l_map, const int32_t* sel, const bf16_t* O, const bf16_t* dO,
                                const float* lse, float* dQ, float* dKp, float* dVp, float* dKl, float* dVl, float* Dr,
                                hipStream_t stream) {
  BwdArgs a{p.H, p.Nq, p.nqb, p.n_loc, p.n_loc_cap, p.C, p.k, p.B, p.scale, p.q_stride_h, p.q_stride_t, p.o_stride_h,
            p.o_stride_t, Q, Kp, Vp, p_len, Kl, Vl, l_len, l_map, sel, O, dO, lse, Dr, dQ, dKp, dVp, dKl, dVl};
  const int sub = p.B / kTile;
  const long n_lanes = (long)p.H * p.Nq * (p.d / 8);
  const dim3 pgrid((unsigned)((n_lanes + 255) / 256));
  if (p.d == 128) hipLaunchKernelGGL(bwd_prep_kernel<128>, pgrid, dim3(256), 0, stream, a);
  else hipLaunchKernelGGL(bwd_prep_kernel<64>, pgrid, dim3(256), 0, stream, a);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  const size_t ring = (size_t)4 * kTile * p.d * 2;
  {
    const size_t n_cand = (size_t)(p.C + 1 + p.k) * sub;
    const dim3 grid((p.Nq + kTile - 1) / kTile, p.H);
    const size_t lds = (size_t)2 * kTile * p.d * 2 + n_cand * 8 + 16;
    e = p.d == 128 ? launch_with_lds(bwd_dq_kernel<128>, a, grid, 64, lds, stream)
                   : launch_with_lds(bwd_dq_kernel<64>, a, grid, 64, lds, stream);
    if (e != hipSuccess) return e;
  }
  {
    const size_t n_cand = (size_t)p.nqb * sub;
    const dim3 grid((unsigned)((p.C + 1 + p.n_loc) * sub * p.H));
    const size_t lds = ring + n_cand * 8 + (size_t)p.nqb * 4 + 16;
    e = p.d == 128 ? launch_with_lds(bwd_dkv_kernel<128>, a, grid, kThreads, lds, stream)
                   : launch_with_lds(bwd_dkv_kernel<64>, a, grid, kThreads, lds, stream);
  }
  return e;
}

}  // namespace pbsa
