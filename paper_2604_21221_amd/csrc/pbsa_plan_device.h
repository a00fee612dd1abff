// Device code of the update's decisions (Eq. 7-9) that more than one kernel runs: the retention of a head by one
// workgroup (retain_kernel; the extra workgroups of the attention launch that takes the decisions beside the
// attention), and the scoring of a whole head by one workgroup (those extra workgroups only).
//
// Every fp32 operation here is exactly the one written (the arithmetic that decides block sets and slots is
// specified operation by operation in pbsa.h): the functions switch contraction off for themselves, and every
// file that includes this one is compiled with correctly rounded fp32 division.
#pragma once

#include "pbsa_internal.h"

namespace pbsa {
namespace plan_dev {

__device__ __forceinline__ int lanes_below(uint64_t mask) {   // set bits of `mask` in lanes below this one
  return __builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0u));
}

// exp(x) for x <= 0 from fp32 mul / fma / rint only (steps fixed in pbsa.h).
__device__ __forceinline__ float pexp(float x) {
  if (x < -64.0f) return 0.0f;
  float n = __builtin_rintf(x * 0x1.715476p+0f);
  float r = __builtin_fmaf(n, -0x1.630000p-1f, x);
  r = __builtin_fmaf(n, 0x1.bd0106p-13f, r);
  float p = 0x1.6c16c2p-10f;
  p = __builtin_fmaf(p, r, 0x1.111112p-7f);
  p = __builtin_fmaf(p, r, 0x1.555556p-5f);
  p = __builtin_fmaf(p, r, 0x1.555556p-3f);
  p = __builtin_fmaf(p, r, 0.5f);
  p = __builtin_fmaf(p, r, 1.0f);
  p = __builtin_fmaf(p, r, 1.0f);
  return p * __uint_as_float((uint32_t)((int)n + 127) << 23);
}

struct ScoreArgs {
  int H, nqb, nqb_pad, n_loc, n_loc_cap, C, nU_max, n_evict;
  float scale;
  const float* Kc_l;
  const float* Kc_p;
  const float* Qc;
  const float* Zl;          // optional: scaled local logits [H][nqb][n_loc] from the selection call
  const int32_t* l_map;
  const int32_t* p_len;
  float* A;
};

constexpr int kMaxCand = PBSA_MAX_C + PBSA_MAX_N_LOC_AUX;

struct RetainArgs {
  int H, nqb, nqb_pad, n_loc, n_loc_cap, C, n_sink, n_evict, nU_max, d, B, fold;
  int fine, Nq;             // fine: A is the attention-mass matrix [H][C+1+n_loc][nqb_pad], one row per key block
                            // (slots 0..C, then the local blocks), and a score is its row sum over Nq
  const float* A;           // A^T [H][nU_max][nqb_pad]
  const float* Kc_l;
  float* Kc_p;
  const int32_t* p_len;
  int32_t* p_len_out;       // [H][C + 1] lengths after the update (the fold kernel commits them)
  int64_t* p_id;
  int32_t* S_cnt;
  const int32_t* l_len;
  const int32_t* l_map;
  const int64_t* l_id;
  float* scores;
  int32_t* slot_src;
  int32_t* fold_n;
  int32_t* fold_src;        // dropped candidate: < C persistent slot, else C + PHYSICAL local slot
  int32_t* fold_len;
  int32_t* promo_slot;      // [H][C] physical local slot a persistent slot is refilled from, or -1
};

// position of the n-th (0-based) set bit of mask
__device__ __forceinline__ int nth_set_bit(uint64_t mask, int n) {
  for (int i = 0; i < n; ++i) mask &= mask - 1;
  return __ffsll((unsigned long long)mask) - 1;
}

// LDS of retain_body
struct RetainLds {
  alignas(16) float cs[kMaxCand + 4];   // candidate scores
  float s[kMaxCand];   // mean column score of slot / evicted-block columns, U order
  int cand[kMaxCand];   // < C: slot, else C + local block
  unsigned char win[kMaxCand];
  int rank_s[kMaxCand];
  unsigned char vac_s[PBSA_MAX_C];   // slot whose occupant is dropped
  int old_len[PBSA_MAX_C + 1];
  int src_s[PBSA_MAX_C];
  int flen[kMaxCand];   // valid tokens of each dropped candidate
  int e_len[PBSA_MAX_N_LOC_AUX];   // valid tokens / physical slot of the evicted blocks
  int e_map[PBSA_MAX_N_LOC_AUX];
  long long e_id[PBSA_MAX_N_LOC_AUX];   // global ids of the evicted blocks
  int nf_s, npos_s;
};

// Retention (Eq. 8-9) of head h by one workgroup of NT threads (a multiple of 64, at least 128).
template <int NT>
__device__ inline void retain_body(const RetainArgs& a, const int h, RetainLds& L) {
#pragma clang fp contract(off)
  auto& cs = L.cs;
  auto& s = L.s;
  auto& cand = L.cand;
  auto& win = L.win;
  auto& rank_s = L.rank_s;
  auto& vac_s = L.vac_s;
  auto& old_len = L.old_len;
  auto& src_s = L.src_s;
  auto& flen = L.flen;
  auto& e_len = L.e_len;
  auto& e_map = L.e_map;
  auto& e_id = L.e_id;
  int& nf_s = L.nf_s;
  int& npos_s = L.npos_s;
  const int C = a.C, C1 = a.C + 1;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int32_t* plen = a.p_len + (size_t)h * C1;
  for (int c = threadIdx.x; c < C1; c += NT) old_len[c] = plen[c];
  for (int e = threadIdx.x; e < a.n_evict; e += NT) {
    e_len[e] = max(0, min(a.l_len[e], a.B));
    e_map[e] = min(max(a.l_map[e], 0), a.n_loc_cap - 1);
    e_id[e] = a.l_id[e];
  }
  // the summary's counts are needed at the very end: ask for them now, not after everything else
  static_assert(NT >= 128, "one thread per position of a block");
  const int cnt_mine = a.fold && threadIdx.x < a.B ? a.S_cnt[(size_t)h * a.B + threadIdx.x] : 0;
  if (threadIdx.x == 0) npos_s = 0;
  __syncthreads();
  // occupied slots: U position of slot c = number of occupied slots below it (C <= 64: one ballot)
  const bool occ = lane < C && old_len[lane] > 0;
  const uint64_t occ_mask = __ballot(occ);
  const int nP = __popcll(occ_mask), u_pos = lanes_below(occ_mask);
  // Column means (Eq. 8) of the columns that can be candidates: the occupied slots and the evicted
  // blocks, i.e. the first nP + n_evict columns of U.
  const int n_need = nP + a.n_evict;
  // A column is contiguous in A^T: its rows are fetched 64 at a time and added in ascending order.
  for (int j = threadIdx.x; j < n_need; j += NT) {
    float acc = 0.0f;
    // where column j of U sits: the coarse matrix is in U order (occupied slots, then local blocks); the mass
    // matrix has a row for every slot, the summary included
    const int at = !a.fine ? j : j < nP ? nth_set_bit(occ_mask, j) : C + 1 + (j - nP);
    const float4* col = reinterpret_cast<const float4*>(a.A + ((size_t)h * a.nU_max + at) * a.nqb_pad);
    for (int i0 = 0; i0 < a.nqb; i0 += 64) {
      float4 v[16];
#pragma unroll
      for (int u = 0; u < 16; ++u) v[u] = i0 + 4 * u < a.nqb ? col[i0 / 4 + u] : make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
      for (int u = 0; u < 16; ++u) {
        const int i = i0 + 4 * u;
        if (i + 0 < a.nqb) acc = acc + v[u].x;
        if (i + 1 < a.nqb) acc = acc + v[u].y;
        if (i + 2 < a.nqb) acc = acc + v[u].z;
        if (i + 3 < a.nqb) acc = acc + v[u].w;
      }
    }
    s[j] = acc / (float)(a.fine ? a.Nq : a.nqb);
  }
  __syncthreads();
  // candidates: occupants of slots >= n_sink in slot order, then the evicted blocks
  const int ncand_max = C + a.n_evict;
  const bool is_cand = occ && lane >= a.n_sink;
  const uint64_t cand_mask = __ballot(is_cand);
  const int ncP = __popcll(cand_mask), nc = ncP + a.n_evict, places = C - a.n_sink;
  if (wave == 0) {
    if (lane < C && a.scores) a.scores[(size_t)h * ncand_max + lane] = occ ? s[u_pos] : 0.0f;
    if (is_cand) {
      const int x = lanes_below(cand_mask);
      cand[x] = lane;
      cs[x] = s[u_pos];
    }
  }
  for (int e = threadIdx.x; e < a.n_evict; e += NT) {
    if (a.scores) a.scores[(size_t)h * ncand_max + C + e] = s[nP + e];
    cand[ncP + e] = C + e;
    cs[ncP + e] = s[nP + e];
  }
  __syncthreads();
  // rank of a candidate = how many beat it (higher score, or equal score and lower index).  All threads
  // take part: with P = NT / nc threads per candidate each counts over its share of the others
  // (several 16-byte reads in flight), and the shares meet in an integer counter.
  for (int x = threadIdx.x; x < nc; x += NT) rank_s[x] = 0;
  __syncthreads();
  {
    const int P = max(1, NT / max(nc, 1)), n4 = (nc + 3) / 4, per = (n4 + P - 1) / P;
    const float4* c4 = reinterpret_cast<const float4*>(cs);
    for (int idx = threadIdx.x; idx < nc * P; idx += NT) {
      const int x = idx % nc, part = idx / nc;
      const float mine = cs[x];
      int rank = 0;
      const int q_end = min(n4, (part + 1) * per);
#pragma unroll 4
      for (int q = part * per; q < q_end; ++q) {
        const float4 v = c4[q];
        const int y = 4 * q;
        // without branches: (in range) and (higher, or equal and earlier)
        rank += (int)(y + 0 < nc) & ((int)(v.x > mine) | ((int)(v.x == mine) & (int)(y + 0 < x)));
        rank += (int)(y + 1 < nc) & ((int)(v.y > mine) | ((int)(v.y == mine) & (int)(y + 1 < x)));
        rank += (int)(y + 2 < nc) & ((int)(v.z > mine) | ((int)(v.z == mine) & (int)(y + 2 < x)));
        rank += (int)(y + 3 < nc) & ((int)(v.w > mine) | ((int)(v.w == mine) & (int)(y + 3 < x)));
      }
      if (rank) atomicAdd(&rank_s[x], rank);
    }
  }
  __syncthreads();
  for (int x = threadIdx.x; x < nc; x += NT) win[x] = rank_s[x] < places;
  for (int c = threadIdx.x; c < C; c += NT) vac_s[c] = 0;
  __syncthreads();
  // wave 0: dropped candidates, in candidate order, go to the fold list; then kept newcomers, in
  // ascending block order, take the vacated and empty slots in ascending slot order
  if (wave == 0) {
    int nf = 0;
    for (int x0 = 0; x0 < nc; x0 += 64) {
      const int x = x0 + lane;
      const bool lose = x < nc && !win[x];
      const uint64_t lm = __ballot(lose);
      if (lose) {
        const int f = nf + lanes_below(lm);
        const bool slot_cand = cand[x] < C;
        const int len = slot_cand ? old_len[cand[x]] : e_len[cand[x] - C];
        a.fold_src[(size_t)h * ncand_max + f] = slot_cand ? cand[x] : C + e_map[cand[x] - C];
        a.fold_len[(size_t)h * ncand_max + f] = len;
        flen[f] = len;
        if (slot_cand) vac_s[cand[x]] = 1;
      }
      nf += __popcll(lm);
    }
    if (lane == 0) { a.fold_n[h] = nf; nf_s = nf; }
    // free slots = (empty or vacated) and >= n_sink (vac_s: written above by this wave, LDS keeps a wave's order)
    const bool vacated = lane < C && vac_s[lane];
    const bool is_free = lane < C && lane >= a.n_sink && (old_len[lane] <= 0 || vacated);
    const uint64_t free_mask = __ballot(is_free);
    if (lane < C) {
      src_s[lane] = -1;
      if (vacated) old_len[lane] = 0;
    }
    int taken = 0;
    for (int x0 = ncP; x0 < nc; x0 += 64) {
      const int x = x0 + lane;
      const bool keep = x < nc && win[x];
      const uint64_t km = __ballot(keep);
      if (keep) {
        const int r = taken + lanes_below(km);       // r-th kept newcomer takes the r-th free slot
        if (r < __popcll(free_mask)) {
          const int slot = nth_set_bit(free_mask, r);
          const int e = cand[x] - C;
          old_len[slot] = e_len[e];
          src_s[slot] = e;
        }
      }
      taken += __popcll(km);
    }
  }
  __syncthreads();
  // per-position counts of the summary: every dropped block adds one to each position it has
  if (a.fold && nf_s > 0) {
    if (threadIdx.x < a.B) {
      const int t = threadIdx.x;
      int cnt = cnt_mine;
#pragma unroll 8
      for (int f = 0; f < nf_s; ++f) cnt += (int)(t < flen[f]);
      a.S_cnt[(size_t)h * a.B + t] = cnt;
      if (cnt > 0) atomicAdd(&npos_s, 1);
    }
    __syncthreads();
    if (threadIdx.x == 0) old_len[C] = npos_s;
    __syncthreads();
  }
  for (int c = threadIdx.x; c < C1; c += NT) a.p_len_out[(size_t)h * C1 + c] = old_len[c];
  for (int c = threadIdx.x; c < C; c += NT) {
    const int e = src_s[c];
    a.slot_src[(size_t)h * C + c] = e;
    a.promo_slot[(size_t)h * C + c] = e >= 0 ? e_map[e] : -1;
    if (e >= 0) a.p_id[(size_t)h * C + c] = e_id[e];
    else if (c >= a.n_sink && old_len[c] == 0) a.p_id[(size_t)h * C + c] = -1;
  }
  // pooled keys move with the promoted blocks: independent float4 copies
  const int d4 = a.d / 4;
  for (int idx = threadIdx.x; idx < C * d4; idx += NT) {
    const int c = idx / d4, x = idx % d4;
    const int e = src_s[c];
    if (e >= 0)
      reinterpret_cast<float4*>(a.Kc_p + ((size_t)h * C + c) * a.d)[x] =
          reinterpret_cast<const float4*>(a.Kc_l + ((size_t)h * a.n_loc_cap + e_map[e]) * a.d)[x];
  }
}

// Rows of the block-level softmax (Eq. 7) of a whole head by one workgroup of NT threads, given the scaled local
// logits Zl the selection call left: the same operations in the same order as score_rows_z_kernel (pooled keys of
// the occupied slots staged once; per row the chain of each persistent column, the row maximum, the exponentials,
// their sum in column order, the quotients stored column-major), with each wave working on R rows at a time: lane c
// runs the chains of persistent column c for the R rows, lane r adds up row r.  No workgroup barrier in the row
// loop: a wave reads only what it wrote itself.  lds: score_head_lds_bytes<D, NT>(n_loc) bytes.
template <int D>
constexpr int score_head_rows() { return D >= 128 ? 4 : 2; }
template <int D, int NT>
constexpr int score_head_lds_bytes(int n_loc) {
  return 4 * (64 * (D + 4) + (NT / 64) * score_head_rows<D>() * (D + 64 + 64 * ((n_loc + 63) / 64)));
}

template <int D, int NT>
__device__ inline void score_head_body(const ScoreArgs& a, const int h, unsigned char* lds) {
#pragma clang fp contract(off)
  constexpr int R = score_head_rows<D>(), NW = NT / 64, KP = D + 4, D4 = D / 4;
  constexpr int NML_MAX = (PBSA_MAX_N_LOC_AUX + 63) / 64;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int nml = (a.n_loc + 63) / 64, EP = 64 + 64 * nml;
  float* kct = reinterpret_cast<float*>(lds);            // [64][KP]
  float* q_w = kct + 64 * KP + wave * R * D;             // [NW][R][D]
  float* er_w = kct + 64 * KP + NW * R * D + wave * R * EP;   // [NW][R][EP]
  const bool occ = lane < a.C && a.p_len[(size_t)h * (a.C + 1) + lane] > 0;
  const uint64_t occ_mask = __ballot(occ);
  const int nP = __popcll(occ_mask), nU = nP + a.n_loc;
  for (int idx = threadIdx.x; idx < nP * D4; idx += NT) {
    const int u = idx / D4, x4 = idx % D4;
    const int slot = nth_set_bit(occ_mask, u);
    *reinterpret_cast<float4*>(kct + u * KP + 4 * x4) =
        reinterpret_cast<const float4*>(a.Kc_p + ((size_t)h * a.C + slot) * D)[x4];
  }
  __syncthreads();
  for (int i0 = R * wave; i0 < a.nqb; i0 += R * NW) {
    for (int idx = lane; idx < R * D4; idx += 64) {
      const int i = min(i0 + idx / D4, a.nqb - 1);
      reinterpret_cast<float4*>(q_w)[idx] = reinterpret_cast<const float4*>(a.Qc + ((size_t)h * a.nqb + i) * D)[idx % D4];
    }
    float zl[R][NML_MAX];
#pragma unroll
    for (int r = 0; r < R; ++r) {
      const float* zrow = a.Zl + ((size_t)h * a.nqb + min(i0 + r, a.nqb - 1)) * a.n_loc;
#pragma unroll
      for (int m = 0; m < NML_MAX; ++m) zl[r][m] = m < nml && lane + 64 * m < a.n_loc ? zrow[lane + 64 * m] : 0.0f;
    }
    __builtin_amdgcn_wave_barrier();
    float accp[R];
#pragma unroll
    for (int r = 0; r < R; ++r) accp[r] = 0.0f;
    if (lane < nP) {
      const float4* k4p = reinterpret_cast<const float4*>(kct + lane * KP);
      const float4* q4p = reinterpret_cast<const float4*>(q_w);
#pragma unroll 4
      for (int x4 = 0; x4 < D4; ++x4) {
        const float4 k = k4p[x4];
#pragma unroll
        for (int r = 0; r < R; ++r) {
          const float4 q = q4p[r * D4 + x4];
          accp[r] = __builtin_fmaf(q.x, k.x, accp[r]);
          accp[r] = __builtin_fmaf(q.y, k.y, accp[r]);
          accp[r] = __builtin_fmaf(q.z, k.z, accp[r]);
          accp[r] = __builtin_fmaf(q.w, k.w, accp[r]);
        }
      }
    }
    float ep[R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
      const float zp = accp[r] * a.scale;
      float mx = lane < nP ? zp : -INFINITY;
#pragma unroll
      for (int m = 0; m < NML_MAX; ++m)
        if (m < nml && lane + 64 * m < a.n_loc) mx = fmaxf(mx, zl[r][m]);
#pragma unroll
      for (int off = 32; off > 0; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off, 64));
      float* er = er_w + r * EP;
      ep[r] = lane < nP ? pexp(zp - mx) : 0.0f;
      if (lane < nP) er[lane] = ep[r];
#pragma unroll
      for (int m = 0; m < NML_MAX; ++m)
        if (m < nml) {
          zl[r][m] = lane + 64 * m < a.n_loc ? pexp(zl[r][m] - mx) : 0.0f;
          if (lane + 64 * m < a.n_loc) er[nP + lane + 64 * m] = zl[r][m];
        }
    }
    __builtin_amdgcn_wave_barrier();
    float s = 0.0f;
    if (lane < R) {
      const float* er = er_w + lane * EP;
#pragma unroll 16
      for (int j = 0; j < nU; ++j) s = s + er[j];
    }
#pragma unroll
    for (int r = 0; r < R; ++r) {
      const float sr = __shfl(s, r, 64);
      if (i0 + r < a.nqb) {
        float* acol = a.A + (size_t)h * a.nU_max * a.nqb_pad + i0 + r;
        if (lane < nP) acol[(size_t)lane * a.nqb_pad] = ep[r] / sr;
#pragma unroll
        for (int m = 0; m < NML_MAX; ++m)
          if (m < nml && lane + 64 * m < a.n_evict) acol[(size_t)(nP + lane + 64 * m) * a.nqb_pad] = zl[r][m] / sr;
      }
    }
    __builtin_amdgcn_wave_barrier();
  }
}

// The two argument blocks of the update's decisions, from the caller's pointers and the workspace
inline ScoreArgs make_score_args(const pbsa_params& p, const float* Qc, const float* Kc_l, const float* Zl,
                                 const float* Kc_p, const int32_t* p_len, const int32_t* l_map, const UpdateWs& ws) {
  return ScoreArgs{p.H, p.nqb, (p.nqb + 3) & ~3, p.n_loc, p.n_loc_cap, p.C, p.C + p.n_loc, p.n_evict, p.scale,
                   Kc_l, Kc_p, Qc, Zl, l_map, p_len, ws.A};
}
// A: the matrix whose row sums are the scores (the coarse matrix in the workspace, or the mass matrix), n_rows of it per head
inline RetainArgs make_retain_args(const pbsa_params& p, const float* A, int n_rows, int fine, const float* Kc_l,
                                   float* Kc_p, const int32_t* p_len, int64_t* p_id, int32_t* S_cnt, int fold,
                                   const int32_t* l_len, const int32_t* l_map, const int64_t* l_id, float* scores,
                                   int32_t* slot_src, const UpdateWs& ws) {
  return RetainArgs{p.H, p.nqb, (p.nqb + 3) & ~3, p.n_loc, p.n_loc_cap, p.C, p.n_sink, p.n_evict, n_rows, p.d, p.B,
                    fold, fine, p.Nq, A, Kc_l, Kc_p, p_len, ws.plen_new, p_id, S_cnt, l_len, l_map, l_id, scores,
                    slot_src, ws.fold_n, ws.fold_src, ws.fold_len, ws.promo_slot};
}

}  // namespace plan_dev
}  // namespace pbsa
