// PBSA fine stage (Eq. 3-5) for gfx950: block-sparse flash attention on bf16 MFMA.
//
// One workgroup = 4 waves = 128 consecutive query tokens of one head (one query block when B = 128,
// two when B = 64); a wave owns 32 query rows.  The workgroup walks a tile list: first every
// non-empty persistent slot (dense part of the mask, visible to all rows), then the union, in
// ascending order, of the local blocks selected by its query blocks; a wave skips a tile its own
// query block did not select.  K/V tiles of 64 keys are staged in LDS by all 256 threads.
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

constexpr int kThreads = 256;
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

// LDS layouts of a 64-key tile.
//  K: row pitch D+8 elements: the 16-byte reads of 16 consecutive rows at one column fall in 16
//     distinct 4-bank groups.
//  V: read with ds_read_b64_tr_b16, where within 16 lanes lane s supplies the address of row s/4,
//     columns 4(s%4)..+3 and lane j receives column j of those 4 rows.  D = 128: rows are unpadded
//     (256 bytes) and 16-byte chunk c of row r sits at chunk c ^ 4(r%4), so the 4 rows x 64 bytes a
//     half-wave reads cover all 64 banks.  D = 64: plain rows of pitch D+32.
template <int D>
__device__ __forceinline__ int v_byte_offset(int row, int chunk) {
  if constexpr (D == 128) return row * 256 + ((chunk ^ ((row & 3) << 2)) << 4);
  else return row * ((D + 32) * 2) + (chunk << 4);
}

template <int D, int B>
__global__ void __launch_bounds__(kThreads, 2) attention_kernel(AttnArgs a) {
  constexpr int G = kRowsPerWg / B;        // query blocks per workgroup
  constexpr int SUB = B / kTile;           // 64-key tiles per block
  constexpr int KPITCH = D + 8;            // K row pitch in elements
  constexpr int KS = D / 16;               // MFMA k-steps of Q K^T
  constexpr int DT = D / 32;               // 32-wide output tiles of O^T
  constexpr int K_BYTES = kTile * KPITCH * 2;
  constexpr int V_BYTES = D == 128 ? kTile * 256 : kTile * (D + 32) * 2;
  constexpr int CPT = kTile * (D / 8) / kThreads;   // 16-byte chunks per thread per tile (K or V)

  __shared__ __align__(16) unsigned char Ks[2][K_BYTES];
  __shared__ __align__(16) unsigned char Vs[2][V_BYTES];
  __shared__ int t_src[kMaxTiles];         // bit 31: local, bits 0..: (slot * SUB + sub)
  __shared__ int t_len[kMaxTiles];
  __shared__ int t_mask[kMaxTiles];        // which of the G query blocks attend the tile
  __shared__ int n_tiles_s;
  int* lflag = reinterpret_cast<int*>(&Ks[0][0]);   // setup scratch, dead before the first tile is staged
  static_assert(PBSA_MAX_N_LOC * 4 <= 2 * K_BYTES, "flag scratch must fit");

  // XCD-aware mapping: consecutive workgroup ids go round-robin to the 8 XCDs, so give XCD x the
  // contiguous range [x * per, (x+1) * per) of (head, query tile) pairs: neighbours share K/V in L2.
  const int n_qt = (a.Nq + kRowsPerWg - 1) / kRowsPerWg;
  const int n_wg = a.H * n_qt;
  const int per = (n_wg + 7) / 8;
  const int logical = (blockIdx.x % 8) * per + blockIdx.x / 8;
  if (logical >= n_wg) return;
  const int h = logical / n_qt;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int T0 = (logical % n_qt) * kRowsPerWg;
  const int i0 = T0 / B;
  const int my_g = (wave * 32) / B;

  // ---- tile list --------------------------------------------------------------------------------
  for (int l = tid; l < a.n_loc; l += kThreads) lflag[l] = 0;
  __syncthreads();
  for (int idx = tid; idx < G * a.k; idx += kThreads) {
    const int g = idx / a.k, j = idx % a.k;
    if (i0 + g < a.nqb) {
      const int l = a.sel[((size_t)h * a.nqb + i0 + g) * a.k + j];
      if (l >= 0 && l < a.n_loc) atomicOr(&lflag[l], 1 << g);
    }
  }
  if (tid == 0) {
    int n = 0;
    for (int c = 0; c <= a.C; ++c) {
      const int len = min(max(a.p_len[(size_t)h * (a.C + 1) + c], 0), B);
      for (int s = 0; s < SUB; ++s) {
        const int sl = min(kTile, len - s * kTile);
        if (sl > 0) { t_src[n] = c * SUB + s; t_len[n] = sl; t_mask[n] = (1 << G) - 1; ++n; }
      }
    }
    n_tiles_s = n;
  }
  __syncthreads();
  if (wave == 0) {
    int n = n_tiles_s;
    for (int l0 = 0; l0 < a.n_loc; l0 += 64) {
      const int l = l0 + lane;
      const int f = l < a.n_loc ? lflag[l] : 0;
      int len = 0, slot = 0;
      if (f) {
        len = min(max(a.l_len[l], 0), B);
        slot = a.l_map[l];
        if (slot < 0 || slot >= a.n_loc_cap) len = 0;
      }
      // a block yields ceil(len / 64) tiles (0, 1 or 2); positions by a wave prefix count
      const int nt = f ? (len + kTile - 1) / kTile : 0;
      const unsigned long long m1 = __ballot(nt >= 1), m2 = __ballot(nt >= 2);
      const int pos = n + lanes_below(m1) + lanes_below(m2);
      for (int s = 0; s < nt; ++s) {
        t_src[pos + s] = (int)(0x80000000u | (uint32_t)(slot * SUB + s));
        t_len[pos + s] = min(kTile, len - s * kTile);
        t_mask[pos + s] = f;
      }
      n += __popcll(m1) + __popcll(m2);
    }
    if (lane == 0) n_tiles_s = n;
  }
  __syncthreads();
  const int n_tiles = n_tiles_s;

  // ---- Q fragments (B operand of S^T = K Q^T): query row = lane % 32, dims 16*ks + 8*(lane/32) ..+8
  const int qn = lane & 31, half = lane >> 5;
  const int tok = T0 + wave * 32 + qn;
  const int tok_c = min(tok, a.Nq - 1);
  bf16x8 qf[KS];
  {
    const bf16_t* qrow = a.Q + (size_t)h * a.q_stride_h + (size_t)tok_c * a.q_stride_t + 8 * half;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) qf[ks] = *reinterpret_cast<const bf16x8*>(qrow + 16 * ks);
  }

  f32x16 o[DT];
#pragma unroll
  for (int dt = 0; dt < DT; ++dt)
#pragma unroll
    for (int v = 0; v < 16; ++v) o[dt][v] = 0.0f;
  float m_run = kNegBig, l_run = 0.0f;
  const float c2 = a.scale * 1.4426950408889634f;

  // staging: thread owns chunks c = tid + 256 n of the 64 x D tile: row c / (D/8), 16-byte chunk c % (D/8).
  // Named registers (not an array) so the prefetched tile stays in VGPRs across the compute phase.
  uint4 kr0, kr1, kr2, kr3, vr0, vr1, vr2, vr3;
  kr0 = kr1 = kr2 = kr3 = vr0 = vr1 = vr2 = vr3 = make_uint4(0u, 0u, 0u, 0u);
#define PBSA_LOAD_TILE(IT)                                                                              \
  {                                                                                                     \
    const int src_ = t_src[IT];                                                                         \
    const bool local_ = src_ < 0;                                                                       \
    const int idx_ = src_ & 0x7FFFFFFF;                                                                 \
    const size_t boff_ = (local_ ? ((size_t)h * a.n_loc_cap + idx_ / SUB) : ((size_t)h * (a.C + 1) + idx_ / SUB)) * \
                             B * D + (size_t)(idx_ % SUB) * kTile * D;                                  \
    const uint4* kb_ = reinterpret_cast<const uint4*>((local_ ? a.Kl : a.Kp) + boff_) + tid;            \
    const uint4* vb_ = reinterpret_cast<const uint4*>((local_ ? a.Vl : a.Vp) + boff_) + tid;            \
    kr0 = kb_[0]; vr0 = vb_[0];                                                                         \
    kr1 = kb_[kThreads]; vr1 = vb_[kThreads];                                                           \
    if constexpr (CPT > 2) {                                                                            \
      kr2 = kb_[2 * kThreads]; vr2 = vb_[2 * kThreads];                                                 \
      kr3 = kb_[3 * kThreads]; vr3 = vb_[3 * kThreads];                                                 \
    }                                                                                                   \
  }
  // V rows past the valid length become zeros: they meet p = 0, which must not see NaN / Inf bits
#define PBSA_STORE_ONE(N, KR, VR, BUF, TLEN)                                                            \
  {                                                                                                     \
    const int c_ = tid + kThreads * N;                                                                  \
    const int r_ = c_ / (D / 8), cc_ = c_ % (D / 8);                                                    \
    *reinterpret_cast<uint4*>(&Ks[BUF][(r_ * KPITCH + cc_ * 8) * 2]) = KR;                              \
    *reinterpret_cast<uint4*>(&Vs[BUF][v_byte_offset<D>(r_, cc_)]) = r_ < TLEN ? VR : make_uint4(0u, 0u, 0u, 0u); \
  }
#define PBSA_STORE_TILE(IT, BUF)                                                                        \
  {                                                                                                     \
    const int tlen_ = t_len[IT];                                                                        \
    PBSA_STORE_ONE(0, kr0, vr0, BUF, tlen_)                                                             \
    PBSA_STORE_ONE(1, kr1, vr1, BUF, tlen_)                                                             \
    if constexpr (CPT > 2) {                                                                            \
      PBSA_STORE_ONE(2, kr2, vr2, BUF, tlen_)                                                           \
      PBSA_STORE_ONE(3, kr3, vr3, BUF, tlen_)                                                           \
    }                                                                                                   \
  }
  static_assert(CPT == 2 || CPT == 4, "staging assumes 2 or 4 chunks per thread");

  if (n_tiles > 0) {
    PBSA_LOAD_TILE(0)
    __syncthreads();               // lflag (aliasing Ks) is dead
    PBSA_STORE_TILE(0, 0)
  }
  __syncthreads();

  // per-lane pieces of the V^T operand address: 16-lane group s -> row s/4, chunk pair 2q + (s%4)/2
  const int s16 = lane & 15, q16 = (lane >> 4) & 1;
  const int v_row0 = 4 * half + (s16 >> 2);
  const int v_sub = 2 * q16 + ((s16 & 3) >> 1);
  const int v_lo = (s16 & 1) * 8;

  for (int it = 0; it < n_tiles; ++it) {
    const int buf = it & 1;
    const int tlen = t_len[it], tmask = t_mask[it];
    if (it + 1 < n_tiles) PBSA_LOAD_TILE(it + 1)

    if ((tmask >> my_g) & 1) {
      // S^T for two 32-key sub-tiles
      f32x16 s[2];
#pragma unroll
      for (int st = 0; st < 2; ++st) {
#pragma unroll
        for (int v = 0; v < 16; ++v) s[st][v] = 0.0f;
        const unsigned char* krow = &Ks[buf][((32 * st + qn) * KPITCH + 8 * half) * 2];
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
          const bf16x8 kf = *reinterpret_cast<const bf16x8*>(krow + 32 * ks);
          s[st] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[ks], s[st], 0, 0, 0);
        }
      }
      // accumulator element v of sub-tile st is key 32 st + 8 (v/4) + 4 half + v%4
      if (tlen < kTile) {
#pragma unroll
        for (int st = 0; st < 2; ++st)
#pragma unroll
          for (int v = 0; v < 16; ++v)
            if (32 * st + 8 * (v / 4) + 4 * half + (v % 4) >= tlen) s[st][v] = kNegBig;
      }
      float tmax = s[0][0];
#pragma unroll
      for (int v = 1; v < 16; ++v) tmax = fmaxf(tmax, s[0][v]);
#pragma unroll
      for (int v = 0; v < 16; ++v) tmax = fmaxf(tmax, s[1][v]);
      tmax = fmaxf(tmax, __shfl_xor(tmax, 32, 64));
      const float m_new = fmaxf(m_run, tmax);
      const float mc = -m_new * c2;
      float psum = 0.0f;
#pragma unroll
      for (int st = 0; st < 2; ++st)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const float p = __builtin_amdgcn_exp2f(__builtin_fmaf(s[st][v], c2, mc));
          s[st][v] = p;
          psum += p;
        }
      if (__any(m_new != m_run)) {        // the running max moved for some row: rescale
        const float alpha = __builtin_amdgcn_exp2f((m_run - m_new) * c2);
        l_run *= alpha;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
          for (int v = 0; v < 16; ++v) o[dt][v] *= alpha;
        m_run = m_new;
      }
      l_run += psum;

      // O^T += V^T P^T, 4 k-steps of 16 keys; V^T fragments by transposing LDS reads
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        bf16x8 pf;
#pragma unroll
        for (int e = 0; e < 8; ++e) pf[e] = (__bf16)s[j / 2][8 * (j % 2) + e];
        const int r0 = 16 * j + v_row0;            // keys r0..r0+3 and r0+8..r0+11 of the tile
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) {
          const bf16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16(
              (bf16x4 __attribute__((address_space(3)))*)(&Vs[buf][v_byte_offset<D>(r0, 4 * dt + v_sub) + v_lo]));
          const bf16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16(
              (bf16x4 __attribute__((address_space(3)))*)(&Vs[buf][v_byte_offset<D>(r0 + 8, 4 * dt + v_sub) + v_lo]));
          const bf16x8 vf = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
          o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf, o[dt], 0, 0, 0);
        }
      }
    }
    if (it + 1 < n_tiles) PBSA_STORE_TILE(it + 1, buf ^ 1)
    __syncthreads();
  }

  // ---- epilogue ---------------------------------------------------------------------------------
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
