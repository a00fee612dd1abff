// Coarse stage and persistent-memory update kernels for gfx950 (HBM / latency bound, no MFMA).
//
//   pool_kernel         block representatives by average pooling            (Eq. 6)
//   select_kernel       coarse logits + row-wise top-k block selection      (Eq. 10-11)
//   score_rows_kernel   block-level softmax rows over persistent + local    (Eq. 7)
//   retain_kernel       column mean, Top-C retention, slot assignment       (Eq. 8-9)
//   fold_promote_kernel dropped blocks -> running-mean summary; kept newcomers -> slots
//
// This file is compiled with -ffp-contract=off: every fp32 operation below is exactly the one
// written (the arithmetic that decides block sets and slots is specified operation by operation
// in pbsa.h so that an independent implementation reproduces the integers bit for bit).
#include "pbsa_internal.h"
#include "pbsa_plan_device.h"

namespace pbsa {
namespace {

using namespace plan_dev;

constexpr int kThreads = 256;
constexpr int kXC = 32;   // pooled-key dimensions staged through LDS per step

__device__ __forceinline__ float bf_lo(uint32_t u) { return __uint_as_float(u << 16); }
__device__ __forceinline__ float bf_hi(uint32_t u) { return __uint_as_float(u & 0xFFFF0000u); }

__device__ __forceinline__ uint32_t f2bf_rne(float f) {
  uint32_t u = __float_as_uint(f);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return u >> 16;
}


// ------------------------------------------------------------------------------------------------
// Pooling.  One job = one block; D/2 threads per job, each owning 2 dimensions (one 4-byte load per
// token) and adding the tokens in ascending order.  The loads of 64 tokens are in flight together.
// ------------------------------------------------------------------------------------------------
struct PoolArgs {
  int mode;                 // 0: generic blocks, 1: select (local key blocks, then query blocks)
  int n_jobs;
  int H, B, Nq, nqb, n_loc, n_loc_cap, pool_from, n_kjobs_per_head;
  long q_stride_h, q_stride_t;
  const bf16_t* X;          // mode 0: [n][B][D]; mode 1: Kl
  const bf16_t* Q;
  const int32_t* len;       // mode 0: [n]; mode 1: l_len
  const int32_t* l_map;
  float* out;               // mode 0: [n][D]; mode 1: Kc_l
  float* Qc;
};

template <int D>
__device__ __forceinline__ void pool_body(const PoolArgs& a, const int bx) {
  constexpr int TPJ = D / 2;
  const int job = bx * (kThreads / TPJ) + threadIdx.x / TPJ;
  const int c = threadIdx.x % TPJ;
  if (job >= a.n_jobs) return;
  const bf16_t* src;
  long pitch = D;
  int len;
  float* dst;
  if (a.mode == 0) {
    src = a.X + (size_t)job * a.B * D;
    len = a.len[job];
    dst = a.out + (size_t)job * D;
  } else {
    // jobs [0, H*nk) pool local key blocks, the rest pool the chunk's query blocks
    const int nk = a.n_kjobs_per_head;
    if (job < a.H * nk) {
      const int h = job / nk, l = a.pool_from + job % nk;
      const int slot = a.l_map[l];
      if (slot < 0 || slot >= a.n_loc_cap) return;
      src = a.X + ((size_t)h * a.n_loc_cap + slot) * a.B * D;
      len = a.len[l];
      dst = a.out + ((size_t)h * a.n_loc_cap + slot) * D;
    } else {
      const int jq = job - a.H * nk;
      const int h = jq / a.nqb, i = jq % a.nqb;
      src = a.Q + (size_t)h * a.q_stride_h + (size_t)i * a.B * a.q_stride_t;
      pitch = a.q_stride_t;
      len = min(a.B, a.Nq - i * a.B);
      dst = a.Qc + ((size_t)h * a.nqb + i) * D;
    }
  }
  len = max(0, min(len, a.B));
  float acc0 = 0.0f, acc1 = 0.0f;
  const bf16_t* p = src + c * 2;
  for (int t0 = 0; t0 < len; t0 += 64) {
    uint32_t v[64];
#pragma unroll
    for (int u = 0; u < 64; ++u)
      v[u] = *reinterpret_cast<const uint32_t*>(p + (size_t)min(t0 + u, len - 1) * pitch);
#pragma unroll
    for (int u = 0; u < 64; ++u) {
      if (t0 + u < len) {
        acc0 = acc0 + bf_lo(v[u]);
        acc1 = acc1 + bf_hi(v[u]);
      }
    }
  }
  const float fl = (float)len;
  float2 o;
  o.x = len > 0 ? acc0 / fl : 0.0f;
  o.y = len > 0 ? acc1 / fl : 0.0f;
  *reinterpret_cast<float2*>(dst + c * 2) = o;
}

template <int D>
__global__ void __launch_bounds__(kThreads) pool_kernel(PoolArgs a) {
  pool_body<D>(a, blockIdx.x);
}

// ------------------------------------------------------------------------------------------------
// Coarse logits.  A workgroup of 4 waves handles 4 query blocks (one per wave) of one head; lane
// `lane` of a wave owns columns j = lane + 64 m.  The pooled keys of all columns are staged through
// LDS kXC dimensions at a time, transposed ([x][j], pitch NM*64+2 keeps both the transposing stores
// and the per-column loads free of bank conflicts), so each accumulator runs the fixed chain
// acc = fma(q[x], k[x], acc), x ascending.
// ------------------------------------------------------------------------------------------------
template <int D, int NM>
__device__ __forceinline__ void coarse_dots(const float* const* cols, int n_cols, const float* qrow, float* kct,
                                            float (&acc)[NM]) {
  constexpr int NPAD = NM * 64 + 2;
  constexpr int P = NM * 64 * (kXC / 4) / kThreads;     // float4 loads per thread per round
  const int lane = threadIdx.x & 63;
#pragma unroll
  for (int m = 0; m < NM; ++m) acc[m] = 0.0f;
  __syncthreads();                                       // cols[] and qrow are visible
  // the global loads of round r+1 are in flight while round r is multiplied
  float4 pre[P];
#pragma unroll
  for (int u = 0; u < P; ++u) {
    const int idx = threadIdx.x + u * kThreads;
    if (idx < n_cols * (kXC / 4)) pre[u] = *reinterpret_cast<const float4*>(cols[idx / (kXC / 4)] + 4 * (idx % (kXC / 4)));
  }
  for (int x0 = 0; x0 < D; x0 += kXC) {
    if (x0 > 0) __syncthreads();                         // previous round's reads of kct are done
#pragma unroll
    for (int u = 0; u < P; ++u) {
      const int idx = threadIdx.x + u * kThreads;
      if (idx < n_cols * (kXC / 4)) {
        const int j = idx / (kXC / 4), xq = idx % (kXC / 4);
        kct[(4 * xq + 0) * NPAD + j] = pre[u].x;
        kct[(4 * xq + 1) * NPAD + j] = pre[u].y;
        kct[(4 * xq + 2) * NPAD + j] = pre[u].z;
        kct[(4 * xq + 3) * NPAD + j] = pre[u].w;
      }
    }
    __syncthreads();
    if (x0 + kXC < D) {
#pragma unroll
      for (int u = 0; u < P; ++u) {
        const int idx = threadIdx.x + u * kThreads;
        if (idx < n_cols * (kXC / 4))
          pre[u] = *reinterpret_cast<const float4*>(cols[idx / (kXC / 4)] + x0 + kXC + 4 * (idx % (kXC / 4)));
      }
    }
#pragma unroll 4
    for (int xx = 0; xx < kXC; ++xx) {
      const float q = qrow[x0 + xx];
#pragma unroll
      for (int m = 0; m < NM; ++m) acc[m] = __builtin_fmaf(q, kct[xx * NPAD + lane + 64 * m], acc[m]);
    }
  }
}


struct SelectArgs {
  int H, nqb, n_loc, n_loc_cap, k, causal;
  float scale;
  const float* Kc_l;
  const float* Qc;
  const int32_t* l_map;
  int32_t* sel;
  float* Zl;                // optional out: scaled logits of every local block, [H][nqb][n_loc]
};

// One wave-wide global -> LDS load of 16 bytes per lane: LDS bytes [lds_off, lds_off + 1024) receive
// lane i's 16 bytes, fetched from base + voff, at lds_off + 16 i.  Completion is tracked by the issuing
// wave's vmcnt.  Earlier LDS reads of this wave are complete before the load is issued.
__device__ __forceinline__ void dma16(const void* base, uint32_t voff, uint32_t lds_off) {
  asm volatile("s_waitcnt lgkmcnt(0)\n\ts_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
               :
               : "s"(lds_off), "v"(voff), "s"(base)
               : "memory", "m0");
}

// Selection (Eq. 10-11).  A workgroup handles 4 query blocks of one head; its NM waves split the local
// blocks: lane `lane` of wave w owns column j = 64 w + lane and runs the four chains
// acc_r = fma(q_r[x], k_j[x], acc_r), x ascending.  The pooled keys reach LDS by direct global -> LDS
// loads, DX dimensions (4 DX bytes per column) per round, double buffered; a wave stages exactly the 64
// columns it consumes, so the rounds need no workgroup barrier.  Within a column's round the 16-byte
// chunks are permuted (logical chunk c of column j sits at c ^ ((j / 2) % (DX / 4))), which spreads the
// per-lane 16-byte reads of consecutive columns over the bank groups.  The logits then go to LDS and wave
// r ranks row r.  DX = 32 up to 8 waves; 16 beyond, where two rounds of 32 would not fit in LDS.
template <int D, int NM, int DX>
__device__ __forceinline__ void select_body(const SelectArgs& a, const int bx, const int h, unsigned char* smem) {
  constexpr int NCP = NM * 64;                        // padded columns
  constexpr int BUF = NCP * DX * 4;                   // one round of every column
  constexpr int NR = D / DX;
  constexpr int CPC = DX / 4;                         // 16-byte chunks per column and round
  constexpr int NI = 64 * CPC / 64;                   // load instructions per wave and round (64 columns)
  constexpr int CPI = 64 / CPC;                       // columns per instruction
  float* qs = reinterpret_cast<float*>(smem + 2 * BUF);                         // [4][D]
  float* zs = qs + 4 * D;                                                       // [4][NCP]
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int i0 = bx * 4;

  // this lane's share of the staging: instruction n fills columns 64 wave + CPI n + lane / CPC, physical chunk
  // lane % CPC
  uint32_t goff[NI];
#pragma unroll
  for (int n = 0; n < NI; ++n) {
    const int j = 64 * wave + CPI * n + lane / CPC;
    int slot = a.l_map[min(j, a.n_loc - 1)];
    slot = min(max(slot, 0), a.n_loc_cap - 1);
    const int chunk = (lane % CPC) ^ ((j >> 1) % CPC);
    goff[n] = (uint32_t)(((size_t)h * a.n_loc_cap + slot) * D * 4 + chunk * 16);
  }
  const uint32_t smem_lds = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)smem;
  const uint32_t wave_lds = __builtin_amdgcn_readfirstlane(smem_lds + wave * (64 * DX * 4));
  const unsigned char* kbase = reinterpret_cast<const unsigned char*>(a.Kc_l);
#define PBSA_STAGE(R_)                                                                                 \
  _Pragma("unroll") for (int n_ = 0; n_ < NI; ++n_)                                                     \
      dma16(kbase + (R_) * (DX * 4), goff[n_], wave_lds + ((R_) & 1) * BUF + n_ * 1024);
  PBSA_STAGE(0)
  if (NR > 1) PBSA_STAGE(1)

  for (int idx = threadIdx.x; idx < 4 * D; idx += 64 * NM) {
    const int r = idx / D, x = idx % D;
    qs[idx] = i0 + r < a.nqb ? a.Qc[((size_t)h * a.nqb + i0 + r) * D + x] : 0.0f;
  }
  __syncthreads();

  float acc[4] = {0.0f, 0.0f, 0.0f, 0.0f};
  const int jcol = 64 * wave + lane;
  const int sw = (jcol >> 1) % CPC;
#pragma unroll 1
  for (int r0 = 0; r0 < NR; ++r0) {
    if (r0 + 1 < NR) {
      if constexpr (NI == 8) asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
      else asm volatile("s_waitcnt vmcnt(4)" ::: "memory");
    } else {
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    }
    const unsigned char* kb = smem + (r0 & 1) * BUF + jcol * (DX * 4);
#pragma unroll
    for (int c = 0; c < CPC; ++c) {
      const float4 k4 = *reinterpret_cast<const float4*>(kb + ((c ^ sw) << 4));
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const float4 q4 = *reinterpret_cast<const float4*>(qs + r * D + r0 * DX + 4 * c);
        acc[r] = __builtin_fmaf(q4.x, k4.x, acc[r]);
        acc[r] = __builtin_fmaf(q4.y, k4.y, acc[r]);
        acc[r] = __builtin_fmaf(q4.z, k4.z, acc[r]);
        acc[r] = __builtin_fmaf(q4.w, k4.w, acc[r]);
      }
      if (c % 2 == 1) __builtin_amdgcn_sched_barrier(0);   // keep the operand reads close to their use
    }
    if (r0 + 2 < NR) PBSA_STAGE(r0 + 2)
  }
#undef PBSA_STAGE

#pragma unroll
  for (int r = 0; r < 4; ++r) {
    const float z = acc[r] * a.scale;
    zs[r * NCP + jcol] = z;
    if (a.Zl && i0 + r < a.nqb && jcol < a.n_loc) a.Zl[((size_t)h * a.nqb + i0 + r) * a.n_loc + jcol] = z;
  }
  __syncthreads();

  for (int r = wave; r < 4; r += NM) {
    const int i = i0 + r;
    if (i >= a.nqb) break;
    // order-preserving integer keys; invisible columns get 0, below every real value
    const int nvis = a.causal ? a.n_loc - a.nqb + i + 1 : a.n_loc;
    uint32_t key[NM];
#pragma unroll
    for (int m = 0; m < NM; ++m) {
      float z = zs[r * NCP + lane + 64 * m];
      if (z == 0.0f) z = 0.0f;                    // -0 and +0 compare equal: give them one key
      const uint32_t b = __float_as_uint(z);
      const uint32_t ordered = (b & 0x80000000u) ? ~b : (b | 0x80000000u);
      key[m] = (lane + 64 * m < nvis) ? ordered : 0u;
    }
    const int kk = min(a.k, nvis);
    int32_t* out = a.sel + ((size_t)h * a.nqb + i) * a.k;
    if (kk > 0) {
      // T = kk-th largest key, found bit by bit: the largest T with #{key >= T} >= kk
      uint32_t T = 0;
      for (int bit = 31; bit >= 0; --bit) {
        const uint32_t cand = T | (1u << bit);
        int cnt = 0;
#pragma unroll
        for (int m = 0; m < NM; ++m) cnt += __popcll(__ballot(key[m] >= cand));
        if (cnt >= kk) T = cand;
      }
      int n_gt = 0;
#pragma unroll
      for (int m = 0; m < NM; ++m) n_gt += __popcll(__ballot(key[m] > T));
      const int need_eq = kk - n_gt;              // ties at T taken in ascending block order
      int seen_eq = 0, pos = 0;
#pragma unroll
      for (int m = 0; m < NM; ++m) {
        const bool eq = key[m] == T;
        const uint64_t eq_mask = __ballot(eq);
        const bool take = key[m] > T || (eq && seen_eq + lanes_below(eq_mask) < need_eq);
        const uint64_t take_mask = __ballot(take);
        if (take) out[pos + lanes_below(take_mask)] = lane + 64 * m;
        seen_eq += __popcll(eq_mask);
        pos += __popcll(take_mask);
      }
    }
    for (int j = kk + lane; j < a.k; j += 64) out[j] = -1;
  }
}

template <int D, int NM, int DX>
__global__ void __launch_bounds__(64 * NM) select_kernel(SelectArgs a) {
  static_assert(DX == 32 || DX == 16, "a round is 8 or 4 load instructions per wave");
  extern __shared__ __align__(1024) unsigned char smem[];
  select_body<D, NM, DX>(a, blockIdx.x, blockIdx.y, smem);
}

// ------------------------------------------------------------------------------------------------
// Persistence scores, rows (Eq. 7): wave per query block; columns U = occupied persistent slots in
// slot order, then all local blocks.  Row softmax in the pinned order; the sum runs sequentially
// over the row in LDS.
// ------------------------------------------------------------------------------------------------

template <int D, int NM>
__global__ void __launch_bounds__(kThreads) score_rows_kernel(ScoreArgs a) {
  extern __shared__ __align__(16) unsigned char smem[];
  constexpr int NPAD = NM * 64 + 2;
  float* kct = reinterpret_cast<float*>(smem);
  float* qs = kct + kXC * NPAD;
  const float** cols = reinterpret_cast<const float**>(qs + 4 * D);
  float* erow = reinterpret_cast<float*>(cols + NM * 64);                       // [4][NM*64]
  __shared__ int nP_s;
  __shared__ float sum_s[4];
  const int h = blockIdx.y, wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int i = blockIdx.x * 4 + wave;
  const bool row_ok = i < a.nqb;
  if (threadIdx.x == 0) {
    int n = 0;
    for (int s = 0; s < a.C; ++s)
      if (a.p_len[(size_t)h * (a.C + 1) + s] > 0) cols[n++] = a.Kc_p + ((size_t)h * a.C + s) * D;
    nP_s = n;
  }
  __syncthreads();
  const int nP = nP_s, nU = nP + a.n_loc;
  for (int j = threadIdx.x; j < a.n_loc; j += kThreads) {
    int slot = a.l_map[j];
    slot = min(max(slot, 0), a.n_loc_cap - 1);
    cols[nP + j] = a.Kc_l + ((size_t)h * a.n_loc_cap + slot) * D;
  }
  for (int x = lane; x < D; x += 64) qs[wave * D + x] = row_ok ? a.Qc[((size_t)h * a.nqb + i) * D + x] : 0.0f;
  float acc[NM];
  coarse_dots<D, NM>(cols, nU, qs + wave * D, kct, acc);

  float mx = -INFINITY;
#pragma unroll
  for (int m = 0; m < NM; ++m) {
    acc[m] = acc[m] * a.scale;
    if (lane + 64 * m < nU) mx = fmaxf(mx, acc[m]);
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off, 64));
  float* er = erow + wave * (NM * 64);
#pragma unroll
  for (int m = 0; m < NM; ++m) {
    acc[m] = (lane + 64 * m < nU) ? pexp(acc[m] - mx) : 0.0f;
    er[lane + 64 * m] = acc[m];
  }
  __syncthreads();
  if (lane == 0) {
    float s = 0.0f;
#pragma unroll 16
    for (int j = 0; j < nU; ++j) s = s + er[j];
    sum_s[wave] = s;
  }
  __syncthreads();
  if (!row_ok) return;
  const float s = sum_s[wave];
  // stored column-major (A^T[h][j][i]) so the column means read contiguous rows
  // (only the columns that can be candidates are needed downstream: slots, then evicted blocks)
  float* acol = a.A + (size_t)h * a.nU_max * a.nqb_pad + i;
  const int n_need = nP + a.n_evict;
#pragma unroll
  for (int m = 0; m < NM; ++m)
    if (lane + 64 * m < n_need) acol[(size_t)(lane + 64 * m) * a.nqb_pad] = acc[m] / s;
}

// Same rows when the selection call has left the local logits in Zl: only the (at most 64) persistent
// columns are multiplied here; lane `lane` owns persistent column `lane` and local columns lane + 64 m.
template <int D, int NML>
__global__ void __launch_bounds__(kThreads) score_rows_z_kernel(ScoreArgs a) {
  extern __shared__ __align__(16) unsigned char smem[];
  float* kct = reinterpret_cast<float*>(smem);                                  // [64][D + 4]
  float* qs = kct + 64 * (D + 4);                                               // [4][D]
  const float** cols = reinterpret_cast<const float**>(qs + 4 * D);            // [64]
  float* erow = reinterpret_cast<float*>(cols + 64);                            // [4][64 + NML*64]
  __shared__ float sum_s[4];
  const int h = blockIdx.y, wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int i = blockIdx.x * 4 + wave;
  const bool row_ok = i < a.nqb;
  const bool occ = lane < a.C && a.p_len[(size_t)h * (a.C + 1) + lane] > 0;
  const uint64_t occ_mask = __ballot(occ);
  const int nP = __popcll(occ_mask), nU = nP + a.n_loc;
  if (wave == 0 && occ) cols[lanes_below(occ_mask)] = a.Kc_p + ((size_t)h * a.C + lane) * D;
  for (int x = lane; x < D; x += 64) qs[wave * D + x] = row_ok ? a.Qc[((size_t)h * a.nqb + i) * D + x] : 0.0f;
  float zl[NML];
  const float* zrow = a.Zl + ((size_t)h * a.nqb + min(i, a.nqb - 1)) * a.n_loc;
#pragma unroll
  for (int m = 0; m < NML; ++m) zl[m] = lane + 64 * m < a.n_loc ? zrow[lane + 64 * m] : 0.0f;
  // the occupied slots' pooled keys, whole, [nP][D + 4] (the pitch spreads the 16-byte reads of 16
  // lanes over all banks); then lane c runs the chain of column c
  __syncthreads();                                       // cols[] and qs are visible
  constexpr int KP = D + 4;
  for (int idx = threadIdx.x; idx < nP * (D / 4); idx += kThreads) {
    const int u = idx / (D / 4), x4 = idx % (D / 4);
    *reinterpret_cast<float4*>(kct + u * KP + 4 * x4) = reinterpret_cast<const float4*>(cols[u])[x4];
  }
  __syncthreads();
  float accp = 0.0f;
  if (lane < nP) {
    const float4* q4p = reinterpret_cast<const float4*>(qs + wave * D);
    const float4* k4p = reinterpret_cast<const float4*>(kct + lane * KP);
#pragma unroll 8
    for (int x4 = 0; x4 < D / 4; ++x4) {
      const float4 q = q4p[x4], k = k4p[x4];
      accp = __builtin_fmaf(q.x, k.x, accp);
      accp = __builtin_fmaf(q.y, k.y, accp);
      accp = __builtin_fmaf(q.z, k.z, accp);
      accp = __builtin_fmaf(q.w, k.w, accp);
    }
  }
  const float zp = accp * a.scale;

  float mx = lane < nP ? zp : -INFINITY;
#pragma unroll
  for (int m = 0; m < NML; ++m)
    if (lane + 64 * m < a.n_loc) mx = fmaxf(mx, zl[m]);
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off, 64));
  float* er = erow + wave * (64 + NML * 64);
  const float ep = lane < nP ? pexp(zp - mx) : 0.0f;
  if (lane < nP) er[lane] = ep;
#pragma unroll
  for (int m = 0; m < NML; ++m) {
    zl[m] = (lane + 64 * m < a.n_loc) ? pexp(zl[m] - mx) : 0.0f;
    if (lane + 64 * m < a.n_loc) er[nP + lane + 64 * m] = zl[m];
  }
  __syncthreads();
  if (lane == 0) {
    float s = 0.0f;
#pragma unroll 16
    for (int j = 0; j < nU; ++j) s = s + er[j];
    sum_s[wave] = s;
  }
  __syncthreads();
  if (!row_ok) return;
  const float s = sum_s[wave];
  float* acol = a.A + (size_t)h * a.nU_max * a.nqb_pad + i;
  if (lane < nP) acol[(size_t)lane * a.nqb_pad] = ep / s;
#pragma unroll
  for (int m = 0; m < NML; ++m)
    if (lane + 64 * m < a.n_evict) acol[(size_t)(nP + lane + 64 * m) * a.nqb_pad] = zl[m] / s;
}

// ------------------------------------------------------------------------------------------------
// Retention (Eq. 8-9): one workgroup per head (the body is shared with the attention launch that takes the
// decisions beside the attention: pbsa_plan_device.h).
// ------------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(kThreads) retain_kernel(RetainArgs a) {
  __shared__ RetainLds L;
  retain_body<kThreads>(a, blockIdx.x, L);
}

// ------------------------------------------------------------------------------------------------
// Fold + promote.  One thread owns 4 dimensions of one position t of K or V of one head: it adds
// the dropped blocks' rows to the running sum in candidate order, rewrites the summary row, then
// copies row t of every kept newcomer into its slot.  A slot that is both dropped and refilled is
// read and written by the same thread, in that order.
// ------------------------------------------------------------------------------------------------
struct FoldArgs {
  int H, B, d, C, n_loc_cap, n_evict, fold;
  bf16_t* Kp;
  bf16_t* Vp;
  const bf16_t* Kl;
  const bf16_t* Vl;
  float* S_sum;
  const int32_t* S_cnt;
  const int32_t* fold_n;
  const int32_t* fold_src;
  const int32_t* fold_len;
  const int32_t* promo_slot;
  const int32_t* plen_new;  // the slots' lengths after the update ...
  int32_t* p_len;           // ... which this kernel commits
};

constexpr int kFoldBatch = 40;
constexpr int kPromoBatch = 8;

template <int NT>
__device__ __forceinline__ void fold_promote_body(const FoldArgs& a, const int bx, const int h) {
  // per dropped candidate: its valid length and the address of its K and of its V block
  __shared__ const bf16_t* fptr_s[2][kMaxCand];
  __shared__ int flen_s[kMaxCand];
  __shared__ int promo_dst[PBSA_MAX_C], promo_src[PBSA_MAX_C], n_promo_s;   // refilled slots, compacted
  const int C = a.C, C1 = a.C + 1, ncand_max = a.C + a.n_evict;
  if (bx == 0)                             // nothing in this launch reads p_len: the lists carry the lengths they need
    for (int c = threadIdx.x; c < C1; c += NT) a.p_len[(size_t)h * C1 + c] = a.plen_new[(size_t)h * C1 + c];
  const int nf = a.fold && a.S_sum ? a.fold_n[h] : 0;
  const size_t blk = (size_t)a.B * a.d;
  for (int f = threadIdx.x; f < nf; f += NT) {
    const int src = a.fold_src[(size_t)h * ncand_max + f];
    flen_s[f] = a.fold_len[(size_t)h * ncand_max + f];
    fptr_s[0][f] = src < C ? a.Kp + ((size_t)h * C1 + src) * blk : a.Kl + ((size_t)h * a.n_loc_cap + (src - C)) * blk;
    fptr_s[1][f] = src < C ? a.Vp + ((size_t)h * C1 + src) * blk : a.Vl + ((size_t)h * a.n_loc_cap + (src - C)) * blk;
  }
  if (threadIdx.x < 64) {                  // wave 0 compacts the slots that are refilled (usually few or none)
    int n = 0;
    for (int c0 = 0; c0 < C; c0 += 64) {
      const int c = c0 + (int)threadIdx.x;
      const int ps = c < C ? a.promo_slot[(size_t)h * C + c] : -1;
      const uint64_t m = __ballot(ps >= 0);
      if (ps >= 0) {
        const int pos = n + lanes_below(m);
        promo_dst[pos] = c;
        promo_src[pos] = ps;
      }
      n += __popcll(m);
    }
    if (threadIdx.x == 0) n_promo_s = n;
  }
  __syncthreads();
  const int n_promo = n_promo_s;
  const int tpr = a.d / 4;                                     // threads per row: 4 dimensions each
  const int rows_per_wg = NT / tpr;
  const int row = bx * rows_per_wg + threadIdx.x / tpr;         // over [2][B]
  const int xc = (threadIdx.x % tpr) * 4;
  if (row >= 2 * a.B) return;
  const int kv = row / a.B, t = row % a.B;
  bf16_t* P = kv ? a.Vp : a.Kp;
  const bf16_t* L = kv ? a.Vl : a.Kl;
  const size_t rowoff = (size_t)t * a.d + xc;
  const bf16_t* Lh = L + (size_t)h * a.n_loc_cap * blk + rowoff;
  // promoted rows are independent of the fold: the first few are fetched before it starts
  uint2 pv[kPromoBatch];
#pragma unroll
  for (int u = 0; u < kPromoBatch; ++u)
    pv[u] = u < n_promo ? *reinterpret_cast<const uint2*>(Lh + (size_t)promo_src[u] * blk) : make_uint2(0u, 0u);
  if (nf > 0) {
    float* ssum = a.S_sum + ((size_t)h * 2 + kv) * blk + rowoff;
    float4 acc = *reinterpret_cast<float4*>(ssum);
    const int cnt = a.S_cnt[(size_t)h * a.B + t];     // already the new count (retain_kernel)
    // rows are loaded kFoldBatch at a time (row t exists in every block, valid or not) and added in
    // candidate order, the add predicated on t < len
    for (int f0 = 0; f0 < nf; f0 += kFoldBatch) {
      uint2 v[kFoldBatch];
#pragma unroll
      for (int u = 0; u < kFoldBatch; ++u)
        v[u] = *reinterpret_cast<const uint2*>(fptr_s[kv][min(f0 + u, nf - 1)] + rowoff);
#pragma unroll
      for (int u = 0; u < kFoldBatch; ++u) {
        if (f0 + u < nf && t < flen_s[f0 + u]) {
          acc.x = acc.x + bf_lo(v[u].x);
          acc.y = acc.y + bf_hi(v[u].x);
          acc.z = acc.z + bf_lo(v[u].y);
          acc.w = acc.w + bf_hi(v[u].y);
        }
      }
    }
    *reinterpret_cast<float4*>(ssum) = acc;
    if (cnt > 0) {
      const float fc = (float)cnt;
      uint2 w;
      w.x = f2bf_rne(acc.x / fc) | (f2bf_rne(acc.y / fc) << 16);
      w.y = f2bf_rne(acc.z / fc) | (f2bf_rne(acc.w / fc) << 16);
      *reinterpret_cast<uint2*>(P + ((size_t)h * C1 + C) * blk + rowoff) = w;
    }
  }
  // promoted rows: stores after the fold's loads (a refilled slot was read above by this thread)
#pragma unroll
  for (int u = 0; u < kPromoBatch; ++u)
    if (u < n_promo) *reinterpret_cast<uint2*>(P + ((size_t)h * C1 + promo_dst[u]) * blk + rowoff) = pv[u];
  for (int u0 = kPromoBatch; u0 < n_promo; u0 += kPromoBatch) {     // more than a few: the rest, batch by batch
#pragma unroll
    for (int u = 0; u < kPromoBatch; ++u)
      pv[u] = u0 + u < n_promo ? *reinterpret_cast<const uint2*>(Lh + (size_t)promo_src[u0 + u] * blk) : make_uint2(0u, 0u);
#pragma unroll
    for (int u = 0; u < kPromoBatch; ++u)
      if (u0 + u < n_promo) *reinterpret_cast<uint2*>(P + ((size_t)h * C1 + promo_dst[u0 + u]) * blk + rowoff) = pv[u];
  }
}

// The bf16 view of a summary given by its running sums and counts (slot C of every head): row t of K and of V is
// S_sum[t] / S_cnt[t], divided in fp32 and rounded to nearest even, where S_cnt[t] > 0; other rows stay as they are;
// the slot's length is the number of such rows.  One thread per 4 dimensions of a row, as in the fold.
__global__ void __launch_bounds__(kThreads) summary_view_kernel(int H, int B, int d, int C, const float* S_sum,
                                                                const int32_t* S_cnt, bf16_t* Kp, bf16_t* Vp,
                                                                int32_t* p_len) {
  const int h = blockIdx.y, C1 = C + 1;
  if (blockIdx.x == 0 && threadIdx.x < 64) {
    int n = 0;
    for (int t0 = 0; t0 < B; t0 += 64) {
      const int t = t0 + (int)threadIdx.x;
      n += __popcll(__ballot(t < B && S_cnt[(size_t)h * B + t] > 0));
    }
    if (threadIdx.x == 0) p_len[(size_t)h * C1 + C] = n;
  }
  const int tpr = d / 4, rows_per_wg = kThreads / tpr;
  const int row = blockIdx.x * rows_per_wg + threadIdx.x / tpr;
  if (row >= 2 * B) return;
  const int kv = row / B, t = row % B, xc = (threadIdx.x % tpr) * 4;
  const int cnt = S_cnt[(size_t)h * B + t];
  if (cnt <= 0) return;
  const size_t blk = (size_t)B * d, rowoff = (size_t)t * d + xc;
  const float4 acc = *reinterpret_cast<const float4*>(S_sum + ((size_t)h * 2 + kv) * blk + rowoff);
  const float fc = (float)cnt;
  uint2 w;
  w.x = f2bf_rne(acc.x / fc) | (f2bf_rne(acc.y / fc) << 16);
  w.y = f2bf_rne(acc.z / fc) | (f2bf_rne(acc.w / fc) << 16);
  *reinterpret_cast<uint2*>((kv ? Vp : Kp) + ((size_t)h * C1 + C) * blk + rowoff) = w;
}

__global__ void __launch_bounds__(kThreads) fold_promote_kernel(FoldArgs a) {
  fold_promote_body<kThreads>(a, blockIdx.x, blockIdx.y);
}

// The pooling of one chunk's selection call and the fold / promote of the update of the chunk before it, as one
// launch: the two touch disjoint data when the new chunk does not sit in the ring position whose blocks are being
// folded, and each is too short to fill the GPU for long.  The n_fold_x * H fold workgroups come first.
template <int D>
__global__ void __launch_bounds__(kThreads) pool_fold_kernel(PoolArgs pa, FoldArgs fa, int n_fold_x) {
  const int n_fold = n_fold_x * fa.H, b = (int)blockIdx.x;      // the fold's workgroups run longest: they start first
  if (b >= n_fold) pool_body<D>(pa, b - n_fold);
  else fold_promote_body<kThreads>(fa, b % n_fold_x, b / n_fold_x);
}

size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

template <typename K>
hipError_t allow_lds(K kernel, size_t bytes) {
  return hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                             (int)bytes);
}

template <int NM>
size_t coarse_lds_bytes(int d, bool with_rows) {
  size_t b = (size_t)kXC * (NM * 64 + 2) * 4 + (size_t)4 * d * 4 + (size_t)NM * 64 * 8;
  if (with_rows) b += (size_t)4 * NM * 64 * 4;
  return b;
}

}  // namespace

UpdateWs carve_update_ws(const pbsa_params& p, void* base) {
  UpdateWs w;
  char* b = static_cast<char*>(base);
  size_t off = 0;
  const size_t nU_max = (size_t)p.C + p.n_loc, ncand = (size_t)p.C + p.n_evict;
  const size_t nqb_pad = ((size_t)p.nqb + 3) & ~(size_t)3;
  w.A = reinterpret_cast<float*>(b + off);          off += align256((size_t)p.H * nU_max * nqb_pad * 4);
  w.fold_n = reinterpret_cast<int32_t*>(b + off);   off += align256((size_t)p.H * 4);
  w.fold_src = reinterpret_cast<int32_t*>(b + off); off += align256((size_t)p.H * ncand * 4);
  w.fold_len = reinterpret_cast<int32_t*>(b + off); off += align256((size_t)p.H * ncand * 4);
  w.promo_slot = reinterpret_cast<int32_t*>(b + off); off += align256((size_t)p.H * (p.C + 1) * 4);
  w.plen_new = reinterpret_cast<int32_t*>(b + off); off += align256((size_t)p.H * (p.C + 1) * 4);
  w.bytes = off;
  return w;
}

hipError_t launch_pool_blocks(const pbsa_params& p, const bf16_t* X, const int32_t* len, int32_t n_blocks,
                              float* out, hipStream_t stream) {
  if (n_blocks == 0) return hipSuccess;
  PoolArgs a{};
  a.mode = 0; a.n_jobs = n_blocks; a.B = p.B; a.X = X; a.len = len; a.out = out;
  const int jpw = kThreads / (p.d / 2);
  const dim3 grid((n_blocks + jpw - 1) / jpw);
  if (p.d == 128) hipLaunchKernelGGL(pool_kernel<128>, grid, dim3(kThreads), 0, stream, a);
  else hipLaunchKernelGGL(pool_kernel<64>, grid, dim3(kThreads), 0, stream, a);
  return hipGetLastError();
}

hipError_t launch_summary_view(const pbsa_params& p, const float* S_sum, const int32_t* S_cnt, bf16_t* Kp, bf16_t* Vp,
                               int32_t* p_len, hipStream_t stream) {
  const int rows_per_wg = kThreads / (p.d / 4);
  hipLaunchKernelGGL(summary_view_kernel, dim3((2 * p.B + rows_per_wg - 1) / rows_per_wg, p.H), dim3(kThreads), 0, stream,
                     p.H, p.B, p.d, p.C, S_sum, S_cnt, Kp, Vp, p_len);
  return hipGetLastError();
}

template <int D, int NM, int DX = 32>
static hipError_t launch_select_t(const SelectArgs& a, hipStream_t stream) {
  constexpr size_t lds = (size_t)2 * NM * 64 * DX * 4 + (size_t)4 * D * 4 + (size_t)4 * NM * 64 * 4;
  static_assert(lds <= 160 * 1024, "two rounds of every column, the queries and the logits must fit in LDS");
  hipError_t e = allow_lds(select_kernel<D, NM, DX>, lds);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL((select_kernel<D, NM, DX>), dim3((a.nqb + 3) / 4, a.H), dim3(64 * NM), lds, stream, a);
  return hipGetLastError();
}

static PoolArgs select_pool_args(const pbsa_params& p, const bf16_t* Q, const bf16_t* Kl, const int32_t* l_len,
                                 const int32_t* l_map, float* Kc_l, float* Qc) {
  PoolArgs pa{};
  pa.mode = 1; pa.H = p.H; pa.B = p.B; pa.Nq = p.Nq; pa.nqb = p.nqb; pa.n_loc = p.n_loc; pa.n_loc_cap = p.n_loc_cap;
  pa.pool_from = p.pool_from; pa.n_kjobs_per_head = p.n_loc - p.pool_from;
  pa.n_jobs = p.H * (pa.n_kjobs_per_head + p.nqb);
  pa.q_stride_h = p.q_stride_h; pa.q_stride_t = p.q_stride_t;
  pa.X = Kl; pa.Q = Q; pa.len = l_len; pa.l_map = l_map; pa.out = Kc_l; pa.Qc = Qc;
  return pa;
}

static FoldArgs fold_args(const pbsa_params& p, bf16_t* Kp, bf16_t* Vp, int32_t* p_len, float* S_sum,
                          const int32_t* S_cnt, const bf16_t* Kl, const bf16_t* Vl, const UpdateWs& ws) {
  return FoldArgs{p.H, p.B, p.d, p.C, p.n_loc_cap, p.n_evict, S_sum != nullptr, Kp, Vp, Kl, Vl, S_sum, S_cnt, ws.fold_n,
                  ws.fold_src, ws.fold_len, ws.promo_slot, ws.plen_new, p_len};
}

static hipError_t launch_select_logits(const pbsa_params& p, const int32_t* l_map, float* Kc_l, float* Qc, int32_t* sel,
                                       float* Zl, hipStream_t stream);

hipError_t launch_select(const pbsa_params& p, const bf16_t* Q, const bf16_t* Kl, const int32_t* l_len,
                         const int32_t* l_map, float* Kc_l, float* Qc, int32_t* sel, float* Zl,
                         hipStream_t stream) {
  const PoolArgs pa = select_pool_args(p, Q, Kl, l_len, l_map, Kc_l, Qc);
  const int jpw = kThreads / (p.d / 2);
  const dim3 grid((pa.n_jobs + jpw - 1) / jpw);
  if (p.d == 128) hipLaunchKernelGGL(pool_kernel<128>, grid, dim3(kThreads), 0, stream, pa);
  else hipLaunchKernelGGL(pool_kernel<64>, grid, dim3(kThreads), 0, stream, pa);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  return launch_select_logits(p, l_map, Kc_l, Qc, sel, Zl, stream);
}

hipError_t launch_select_apply(const pbsa_params& p, const bf16_t* Q, const bf16_t* Kl, const int32_t* l_len,
                               const int32_t* l_map, float* Kc_l, float* Qc, int32_t* sel, float* Zl,
                               const pbsa_params& pu, bf16_t* Kp, bf16_t* Vp, int32_t* p_len, float* S_sum,
                               const int32_t* S_cnt, const bf16_t* Vl, const UpdateWs& ws, hipStream_t stream) {
  const PoolArgs pa = select_pool_args(p, Q, Kl, l_len, l_map, Kc_l, Qc);
  const FoldArgs fa = fold_args(pu, Kp, Vp, p_len, S_sum, S_cnt, Kl, Vl, ws);
  // the fold / promote workgroups ride in the pooling launch: its workgroups have the same size and no LDS of their
  // own (in the logits launch, 80 KB of LDS per workgroup, they would wait for places: measured slower)
  const int jpw = kThreads / (p.d / 2), rows_per_wg = kThreads / (pu.d / 4);
  const int n_fold_x = (2 * pu.B + rows_per_wg - 1) / rows_per_wg;
  const dim3 grid(n_fold_x * pu.H + (pa.n_jobs + jpw - 1) / jpw);
  if (p.d == 128) hipLaunchKernelGGL(pool_fold_kernel<128>, grid, dim3(kThreads), 0, stream, pa, fa, n_fold_x);
  else hipLaunchKernelGGL(pool_fold_kernel<64>, grid, dim3(kThreads), 0, stream, pa, fa, n_fold_x);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  return launch_select_logits(p, l_map, Kc_l, Qc, sel, Zl, stream);
}

static hipError_t launch_select_logits(const pbsa_params& p, const int32_t* l_map, float* Kc_l, float* Qc, int32_t* sel,
                                       float* Zl, hipStream_t stream) {
  if (p.k == 0 && !Zl) return hipSuccess;

  SelectArgs a{p.H, p.nqb, p.n_loc, p.n_loc_cap, p.k, p.causal, p.scale, Kc_l, Qc, l_map, sel, Zl};
  const int nm = (p.n_loc + 63) / 64;
  if (p.d == 128) {
    if (nm <= 2) return launch_select_t<128, 2>(a, stream);
    if (nm <= 5) return launch_select_t<128, 5>(a, stream);
    if (nm <= 8) return launch_select_t<128, 8>(a, stream);
    return launch_select_t<128, 11, 16>(a, stream);
  }
  static_assert(PBSA_MAX_N_LOC <= 11 * 64, "one lane per local block");
  if (nm <= 2) return launch_select_t<64, 2>(a, stream);
  if (nm <= 5) return launch_select_t<64, 5>(a, stream);
  if (nm <= 8) return launch_select_t<64, 8>(a, stream);
  return launch_select_t<64, 11, 16>(a, stream);
}

template <int D, int NM>
static hipError_t launch_rows_t(const ScoreArgs& a, hipStream_t stream) {
  const size_t lds = coarse_lds_bytes<NM>(D, true);
  hipError_t e = allow_lds(score_rows_kernel<D, NM>, lds);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL((score_rows_kernel<D, NM>), dim3((a.nqb + 3) / 4, a.H), dim3(kThreads), lds, stream, a);
  return hipGetLastError();
}

template <int D, int NML>
static hipError_t launch_rows_z_t(const ScoreArgs& a, hipStream_t stream) {
  const size_t lds = (size_t)64 * (D + 4) * 4 + (size_t)4 * D * 4 + 64 * 8 + (size_t)4 * (64 + NML * 64) * 4;
  hipError_t e = allow_lds(score_rows_z_kernel<D, NML>, lds);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL((score_rows_z_kernel<D, NML>), dim3((a.nqb + 3) / 4, a.H), dim3(kThreads), lds, stream, a);
  return hipGetLastError();
}

static hipError_t launch_scores(const pbsa_params& p, const float* Qc, const float* Kc_l, const float* Zl,
                                const float* Kc_p, const int32_t* p_len, const int32_t* l_map, const UpdateWs& ws,
                                hipStream_t stream) {
  const int nU_max = p.C + p.n_loc;
  const ScoreArgs sa = make_score_args(p, Qc, Kc_l, Zl, Kc_p, p_len, l_map, ws);
  const int nm = (nU_max + 63) / 64;
  if (Zl) {
    const int nml = (p.n_loc + 63) / 64;
    if (p.d == 128)
      return nml <= 2 ? launch_rows_z_t<128, 2>(sa, stream) : nml <= 5 ? launch_rows_z_t<128, 5>(sa, stream)
                                                                      : launch_rows_z_t<128, 8>(sa, stream);
    return nml <= 2 ? launch_rows_z_t<64, 2>(sa, stream) : nml <= 5 ? launch_rows_z_t<64, 5>(sa, stream)
                                                                    : launch_rows_z_t<64, 8>(sa, stream);
  }
  if (p.d == 128)
    return nm <= 2 ? launch_rows_t<128, 2>(sa, stream) : nm <= 6 ? launch_rows_t<128, 6>(sa, stream)
                                                                : launch_rows_t<128, 9>(sa, stream);
  return nm <= 2 ? launch_rows_t<64, 2>(sa, stream) : nm <= 6 ? launch_rows_t<64, 6>(sa, stream)
                                                              : launch_rows_t<64, 9>(sa, stream);
}

// Retention given the matrix whose row sums are the scores (A: the coarse matrix in the workspace, or the mass matrix)
static hipError_t launch_retain(const pbsa_params& p, const float* A, int n_rows, int fine, const float* Kc_l,
                                float* Kc_p, const int32_t* p_len, int64_t* p_id, int32_t* S_cnt, int fold,
                                const int32_t* l_len, const int32_t* l_map, const int64_t* l_id, float* scores,
                                int32_t* slot_src, const UpdateWs& ws, hipStream_t stream) {
  const RetainArgs ra = make_retain_args(p, A, n_rows, fine, Kc_l, Kc_p, p_len, p_id, S_cnt, fold, l_len, l_map, l_id,
                                         scores, slot_src, ws);
  hipLaunchKernelGGL(retain_kernel, dim3(p.H), dim3(kThreads), 0, stream, ra);
  return hipGetLastError();
}

hipError_t launch_update_plan(const pbsa_params& p, const float* Qc, const float* Kc_l, const float* Zl, float* Kc_p,
                              const int32_t* p_len, int64_t* p_id, int32_t* S_cnt, int fold, const int32_t* l_len,
                              const int32_t* l_map, const int64_t* l_id, float* scores, int32_t* slot_src,
                              const UpdateWs& ws, hipStream_t stream) {
  hipError_t e = launch_scores(p, Qc, Kc_l, Zl, Kc_p, p_len, l_map, ws, stream);
  if (e != hipSuccess) return e;
  return launch_retain(p, ws.A, p.C + p.n_loc, 0, Kc_l, Kc_p, p_len, p_id, S_cnt, fold, l_len, l_map, l_id, scores,
                       slot_src, ws, stream);
}

hipError_t launch_update_apply(const pbsa_params& p, bf16_t* Kp, bf16_t* Vp, int32_t* p_len, float* S_sum,
                               const int32_t* S_cnt, const bf16_t* Kl, const bf16_t* Vl, const UpdateWs& ws,
                               hipStream_t stream) {
  const FoldArgs fa = fold_args(p, Kp, Vp, p_len, S_sum, S_cnt, Kl, Vl, ws);
  const int rows_per_wg = kThreads / (p.d / 4);
  hipLaunchKernelGGL(fold_promote_kernel, dim3((2 * p.B + rows_per_wg - 1) / rows_per_wg, p.H), dim3(kThreads), 0,
                     stream, fa);
  return hipGetLastError();
}

hipError_t launch_update(const pbsa_params& p, const float* Qc, const float* Kc_l, const float* Zl, bf16_t* Kp,
                         bf16_t* Vp, float* Kc_p, int32_t* p_len, int64_t* p_id, float* S_sum, int32_t* S_cnt,
                         const bf16_t* Kl, const bf16_t* Vl, const int32_t* l_len, const int32_t* l_map,
                         const int64_t* l_id, float* scores, int32_t* slot_src, const UpdateWs& ws,
                         hipStream_t stream) {
  hipError_t e = launch_update_plan(p, Qc, Kc_l, Zl, Kc_p, p_len, p_id, S_cnt, S_sum != nullptr, l_len, l_map, l_id, scores,
                                    slot_src, ws, stream);
  if (e != hipSuccess) return e;
  return launch_update_apply(p, Kp, Vp, p_len, S_sum, S_cnt, Kl, Vl, ws, stream);
}

hipError_t launch_update_fine(const pbsa_params& p, const float* Mt, const float* Kc_l, bf16_t* Kp, bf16_t* Vp,
                              float* Kc_p, int32_t* p_len, int64_t* p_id, float* S_sum, int32_t* S_cnt,
                              const bf16_t* Kl, const bf16_t* Vl, const int32_t* l_len, const int32_t* l_map,
                              const int64_t* l_id, float* scores, int32_t* slot_src, const UpdateWs& ws,
                              hipStream_t stream) {
  hipError_t e = launch_retain(p, Mt, p.C + 1 + p.n_loc, 1, Kc_l, Kc_p, p_len, p_id, S_cnt, S_sum != nullptr, l_len, l_map,
                               l_id, scores, slot_src, ws, stream);
  if (e != hipSuccess) return e;
  return launch_update_apply(p, Kp, Vp, p_len, S_sum, S_cnt, Kl, Vl, ws, stream);
}

}  // namespace pbsa
