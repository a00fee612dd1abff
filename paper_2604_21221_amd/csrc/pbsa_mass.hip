// Fine attention mass for gfx950: how much of the fine stage's attention (Eq. 3-5) each key block receives
// from each query block -- the token-level counterpart of the block-level matrix of Eq. 7, accumulated the
// way Eq. 8 accumulates it.  A second, light pass over the keys after the attention kernel: with the
// row normalisers known (the attention call's log-sum-exp output) a probability is exp(s - lse) and needs
// no running maximum, no values and no output accumulators, only S^T = K Q^T and a sum.
//
// One workgroup = 4 waves = 128 consecutive query tokens of one head (one query block when B = 128, two when
// B = 64), the same row tiling as the attention kernel.  The workgroup walks the 64-key tiles of every
// non-empty persistent slot and of the union of the local blocks its query blocks selected; wave w takes
// keys 32 (w % 2) .. +31 of a tile against rows 64 (w / 2) .. +63, so with B = 64 the two waves of a row
// half are one query block and skip the tiles only the other one attends.  Tiles go from global memory
// straight into a ring in LDS (global_load_lds, the 16-byte chunks of a row permuted so that the operand
// reads are free of bank conflicts), one barrier per tile, the loads of the next tiles in flight meanwhile.
//
// MFMA arrangement (v_mfma_f32_32x32x16_bf16): A = K rows (32 keys x 16 dims), B = Q^T (16 dims x 32 rows):
// a lane then holds 16 keys of one query row.  Each wave sums exp2(s c2 - lse log2 e) over its 32 x 64
// scores of a tile (in-lane, then across the wave in a fixed order) and leaves one number per tile in LDS;
// at the end the workgroup adds, per key block and query block, the numbers of the waves and tiles that
// belong together, always in the same order, and writes Mt.  No atomics: the result is deterministic.
#include "pbsa_internal.h"

namespace pbsa {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

constexpr int kThreads = 256;
constexpr int kRowsPerWg = 128;
constexpr int kTile = 64;
constexpr int kRingBytes = 48 * 1024;
constexpr int kMaxCand = 2 * (PBSA_MAX_C_AUX + 1) + 2 * PBSA_MAX_N_LOC_AUX;
constexpr int kMaxRounds = (kMaxCand + kThreads - 1) / kThreads;

struct MassArgs {
  int H, Nq, nqb, nqb_pad, n_loc, n_loc_cap, C, k;
  float scale;
  long q_stride_h, q_stride_t;
  const bf16_t* Q;
  const bf16_t* Kp;
  const int32_t* p_len;
  const bf16_t* Kl;
  const int32_t* l_len;
  const int32_t* l_map;
  const int32_t* sel;
  const float* lse;
  float* Mt;
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

typedef __attribute__((address_space(3))) const bf16x8* lds_b128_t;
__device__ __forceinline__ bf16x8 lds_read_k(uint32_t addr) { return *(lds_b128_t)(uintptr_t)addr; }

// x of lane i plus x of the lane a data-parallel-primitive pattern pairs it with
template <int CTRL>
__device__ __forceinline__ float add_dpp(float x) {
  const int y = __builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, 0xF, 0xF, false);
  return x + __int_as_float(y);
}
// Sum over the 64 lanes, the same association every time: within quads, the two quads of a half row, the
// two halves of a row of 16, then the four rows.
__device__ __forceinline__ float wave_sum(float x) {
  x = add_dpp<0xB1>(x);      // quad_perm [1, 0, 3, 2]
  x = add_dpp<0x4E>(x);      // quad_perm [2, 3, 0, 1]
  x = add_dpp<0x141>(x);     // row_half_mirror
  x = add_dpp<0x140>(x);     // row_mirror
  const float r0 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(x), 0));
  const float r1 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(x), 16));
  const float r2 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(x), 32));
  const float r3 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(x), 48));
  return (r0 + r1) + (r2 + r3);
}

template <int D, int B>
__global__ void __launch_bounds__(kThreads) mass_kernel(MassArgs a) {
  constexpr int G = kRowsPerWg / B;        // query blocks per workgroup
  constexpr int SUB = B / kTile;           // 64-key tiles per block
  constexpr int KS = D / 16, ROW = D * 2, TILE = kTile * ROW;
  constexpr int RING = kRingBytes / TILE;  // tiles in the ring: 3 (D = 128) or 6 (D = 64)
  constexpr int CH = D / 8, RPI = 64 / CH; // 16-byte chunks per row, rows per wave instruction
  constexpr int NI = (kTile / RPI) / 4;    // load instructions per wave per tile: 4 or 2
  static_assert(RING >= 3, "two tiles on their way while one is read");
  static_assert((3 * PBSA_MAX_N_LOC_AUX + PBSA_MAX_C_AUX + 1) * 4 <= kRingBytes, "setup scratch must fit");

  extern __shared__ __align__(1024) unsigned char smem[];
  __shared__ int cnt_s[kMaxRounds * 4];
  const int n_u = a.C + 1 + a.n_loc;                       // key blocks: slots 0..C, then the local blocks
  const int n_pers = (a.C + 1) * SUB, n_cand = n_pers + a.n_loc * SUB;
  float* part = reinterpret_cast<float*>(smem + kRingBytes);   // [tile][wave]
  int* t_src = reinterpret_cast<int*>(part + 4 * n_cand);  // bit 31: local; bits 0..: slot * SUB + sub
  int* t_meta = t_src + n_cand;                            // valid keys | row halves that attend << 8 | key block << 10
  int* pos_s = t_meta + n_cand;                            // [n_u] first tile of a key block in the list, or -1
  int* lflag = reinterpret_cast<int*>(smem);               // setup scratch, dead before the first tile is staged
  int* llen_s = lflag + PBSA_MAX_N_LOC_AUX;
  int* lmap_s = llen_s + PBSA_MAX_N_LOC_AUX;
  int* plen_s = lmap_s + PBSA_MAX_N_LOC_AUX;

  // consecutive workgroup ids go round-robin to the 8 XCDs: XCD x gets a contiguous range of (head, row tile)
  const int n_qt = (a.Nq + kRowsPerWg - 1) / kRowsPerWg;
  const int n_wg = a.H * n_qt;
  const int per = (n_wg + 7) / 8;
  const int logical = (blockIdx.x % 8) * per + blockIdx.x / 8;
  if (logical >= n_wg) return;
  const int h = logical / n_qt;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int kh = wave & 1, rh = wave >> 1;
  const int T0 = (logical % n_qt) * kRowsPerWg;
  const int i0 = T0 / B;
  const int qn = lane & 31, half = lane >> 5;

  for (int l = tid; l < a.n_loc; l += kThreads) {
    lflag[l] = 0;
    llen_s[l] = a.l_len[l];
    lmap_s[l] = a.l_map[l];
  }
  for (int c = tid; c <= a.C; c += kThreads) plen_s[c] = a.p_len[(size_t)h * (a.C + 1) + c];
  for (int u = tid; u < n_u; u += kThreads) pos_s[u] = -1;
  constexpr int kSelPer = (2 * PBSA_MAX_K_AUX + kThreads - 1) / kThreads;
  int selv[kSelPer];
#pragma unroll
  for (int u = 0; u < kSelPer; ++u) {
    const int idx = tid + u * kThreads;
    const int g = idx / max(a.k, 1), j = idx % max(a.k, 1);
    selv[u] = idx < G * a.k && i0 + g < a.nqb ? a.sel[((size_t)h * a.nqb + i0 + g) * a.k + j] : -1;
  }

  // Q fragments (B operand): row group g, query row lane % 32, dims 16 ks + 8 (lane / 32) .. +8; and minus the
  // log-sum-exp of that row in base-2 units (-inf for a row that does not exist or attends nothing)
  const int tok0 = T0 + rh * 64 + qn;
  bf16x8 qf[2][KS];
  float nl[2];
#pragma unroll
  for (int g = 0; g < 2; ++g) {
    const int tok = tok0 + 32 * g, tok_c = min(tok, a.Nq - 1);
    const bf16_t* qrow = a.Q + (size_t)h * a.q_stride_h + (size_t)tok_c * a.q_stride_t + 8 * half;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) qf[g][ks] = *reinterpret_cast<const bf16x8*>(qrow + 16 * ks);
    const float l = a.lse[(size_t)h * a.Nq + tok_c];
    nl[g] = tok < a.Nq && l > -INFINITY ? -l * 1.4426950408889634f : -INFINITY;
  }
  // B = 64: a tile that only the other query block of the workgroup attends is shared out among all four waves,
  // this wave taking that block's row group rh: its fragments and normaliser
  bf16x8 qo[KS];
  float nlo = -INFINITY;
  if constexpr (G == 2) {
    const int tok = T0 + (1 - rh) * 64 + rh * 32 + qn, tok_c = min(tok, a.Nq - 1);
    const bf16_t* qrow = a.Q + (size_t)h * a.q_stride_h + (size_t)tok_c * a.q_stride_t + 8 * half;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) qo[ks] = *reinterpret_cast<const bf16x8*>(qrow + 16 * ks);
    const float l = a.lse[(size_t)h * a.Nq + tok_c];
    nlo = tok < a.Nq && l > -INFINITY ? -l * 1.4426950408889634f : -INFINITY;
  }
  __syncthreads();
#pragma unroll
  for (int u = 0; u < kSelPer; ++u) {
    const int l = selv[u], g = (tid + u * kThreads) / max(a.k, 1);
    if (l >= 0 && l < a.n_loc) atomicOr(&lflag[l], G == 1 ? 3 : 1 << g);
  }
  __syncthreads();

  // ---- tile list: persistent tiles, then the flagged local tiles, in ascending order ------------------
  auto classify = [&](int i, int& src, int& meta) -> bool {
    if (i >= n_cand) return false;
    if (i < n_pers) {
      const int c = i / SUB, sub = i % SUB;
      const int tl = min(max(min(max(plen_s[c], 0), B) - sub * kTile, 0), kTile);
      src = i;
      meta = tl | (3 << 8) | (c << 10);
      return tl > 0;
    }
    const int l = (i - n_pers) / SUB, sub = (i - n_pers) % SUB;
    const int f = lflag[l], slot = lmap_s[l];
    if (f == 0 || slot < 0 || slot >= a.n_loc_cap) return false;
    const int tl = min(max(min(max(llen_s[l], 0), B) - sub * kTile, 0), kTile);
    src = (int)(0x80000000u | (uint32_t)(slot * SUB + sub));
    meta = tl | (f << 8) | ((a.C + 1 + l) << 10);
    return tl > 0;
  };
  const int n_rounds = (n_cand + kThreads - 1) / kThreads;
  for (int r = 0; r < n_rounds; ++r) {
    int src, meta;
    const unsigned long long m = __ballot(classify(r * kThreads + tid, src, meta));
    if (lane == 0) cnt_s[r * 4 + wave] = __popcll(m);
  }
  __syncthreads();
  int n_tiles = 0;
  for (int q = 0; q < 4 * n_rounds; ++q) n_tiles += cnt_s[q];
  for (int r = 0; r < n_rounds; ++r) {
    int src = 0, meta = 0;
    const bool on = classify(r * kThreads + tid, src, meta);
    const unsigned long long m = __ballot(on);
    if (on) {
      int pos = lanes_below(m);
      for (int q = 0; q < r * 4 + wave; ++q) pos += cnt_s[q];
      t_src[pos] = src;
      t_meta[pos] = meta;
      const int i = r * kThreads + tid;
      if ((i < n_pers ? i : i - n_pers) % SUB == 0) pos_s[meta >> 10] = pos;
    }
  }
  __syncthreads();                         // the list is complete and the setup scratch (in the ring) is dead

  // ---- the walk ------------------------------------------------------------------------------------------
  // The query fragments and normalisers have arrived by now.  Saying so here keeps the compiler from waiting for
  // them inside the walk, where a wait on the vector-memory counter would also wait for the tiles in flight.
#pragma unroll
  for (int g = 0; g < 2; ++g) {
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) asm volatile("" : "+v"(qf[g][ks]));
    asm volatile("" : "+v"(nl[g]));
  }
  if constexpr (G == 2) {
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) asm volatile("" : "+v"(qo[ks]));
    asm volatile("" : "+v"(nlo));
  }
  const uint32_t smem_lds = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)smem;
  const uint32_t ring_s = __builtin_amdgcn_readfirstlane(smem_lds);
  // K fragment of this lane inside a ring entry: key row 32 kh + lane % 32, logical chunk 2 ks + lane / 32 at
  // physical chunk (2 ks + half) ^ (row mod (D / 8))
  uint32_t ka[KS];
  {
    const int f = qn & (CH - 1);
    const int kb = (32 * kh + qn) * ROW + ((half ^ f) << 4);
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) ka[ks] = smem_lds + (uint32_t)(kb ^ (ks << 5));
  }
  // staging: wave w brings rows 16 w .. 16 w + 15 of a tile, NI instructions of RPI rows; lane i of an
  // instruction fills physical chunk i % CH of row i / CH with the logical chunk (i % CH) ^ (row mod CH)
  const int rl = lane / CH;
  uint32_t kpat[NI];
#pragma unroll
  for (int k = 0; k < NI; ++k) kpat[k] = (uint32_t)((RPI * k + rl) * ROW + (((lane % CH) ^ ((RPI * k + rl) & (CH - 1))) << 4));
  const size_t head_l = (size_t)h * a.n_loc_cap * B * D * 2, head_p = (size_t)h * (a.C + 1) * B * D * 2;
  auto stage = [&](int t, int entry) {
    const int src = __builtin_amdgcn_readfirstlane(t_src[t]);
    const unsigned char* tile =
        src < 0 ? reinterpret_cast<const unsigned char*>(a.Kl) + head_l + (size_t)(src & 0x7FFFFFFF) * TILE
                : reinterpret_cast<const unsigned char*>(a.Kp) + head_p + (size_t)src * TILE;
    const uint32_t dst = ring_s + (uint32_t)(entry * TILE + wave * (TILE / 4));
#pragma unroll
    for (int k = 0; k < NI; ++k) dma16(tile + wave * (TILE / 4), kpat[k], dst + k * 1024);
  };
  const float c2 = a.scale * 1.4426950408889634f;
  if (n_tiles > 0) {
    // past the end of the list the last tile is fetched again, into an entry that is never read, so that the
    // number of loads in flight is the same at every turn
    for (int j = 0; j < RING - 1; ++j) stage(min(j, n_tiles - 1), j);
    for (int t = 0; t < n_tiles; ++t) {
      asm volatile("s_waitcnt vmcnt(%0)" ::"n"((RING - 2) * NI) : "memory");   // this wave's rows of tile t are in
      __syncthreads();                                     // everybody's are, and tile t-1 has been read by all
      stage(min(t + RING - 1, n_tiles - 1), (t + RING - 1) % RING);
      const int meta = __builtin_amdgcn_readfirstlane(t_meta[t]);
      const int len = meta & 0xFF;
      float total = 0.0f;
      const uint32_t off = (uint32_t)((t % RING) * TILE);
      const int att = (meta >> 8) & 3;     // row halves that attend: both, or (B = 64) one query block alone
      // accumulator element v is key 8 (v / 4) + 4 half + v % 4 of the wave's 32; keys past the valid length hold
      // anything at all and are left out by selection, not by a product
      const int lim = len - 32 * kh - 4 * half;
      if (att == 3) {
        f32x16 s[2];
        bf16x8 kf[KS];                     // all operand reads first: their latency is paid once, not per k-step
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) kf[ks] = lds_read_k(ka[ks] + off);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
          const f32x16 zero = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
          for (int g = 0; g < 2; ++g)
            s[g] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[ks], qf[g][ks], ks == 0 ? zero : s[g], 0, 0, 0);
        }
        float acc[2] = {0.0f, 0.0f};
        if (len == kTile) {
#pragma unroll
          for (int g = 0; g < 2; ++g)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[g] += __builtin_amdgcn_exp2f(__builtin_fmaf(s[g][v], c2, nl[g]));
        } else {
#pragma unroll
          for (int g = 0; g < 2; ++g)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
              const float e = __builtin_amdgcn_exp2f(__builtin_fmaf(s[g][v], c2, nl[g]));
              acc[g] += 8 * (v / 4) + (v % 4) < lim ? e : 0.0f;
            }
        }
        total = wave_sum(acc[0] + acc[1]);
      } else if (G == 2) {
        // one query block alone: its 64 rows x 64 keys are four 32 x 32 products, one per wave
        const bool mine = att == 1 << rh;  // the block is this wave's own: row group rh of it is qf[rh]
        f32x16 s1;
        bf16x8 kf[KS];
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) kf[ks] = lds_read_k(ka[ks] + off);
        __builtin_amdgcn_sched_barrier(0);
        const f32x16 zero = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
        auto product = [&](const bf16x8 (&q)[KS]) {
#pragma unroll
          for (int ks = 0; ks < KS; ++ks)
            s1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[ks], q[ks], ks == 0 ? zero : s1, 0, 0, 0);
        };
        // three uniform branches rather than a choice of operands, which would copy the fragments
        if (!mine) product(qo);
        else if (rh == 0) product(qf[0]);
        else product(qf[1]);
        const float nsel = !mine ? nlo : rh == 0 ? nl[0] : nl[1];
        float acc = 0.0f;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const float e = __builtin_amdgcn_exp2f(__builtin_fmaf(s1[v], c2, nsel));
          acc += 8 * (v / 4) + (v % 4) < lim ? e : 0.0f;
        }
        total = wave_sum(acc);
      }
      if (lane == 0) part[4 * t + wave] = total;
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");       // the trailing loads land before the workgroup goes
  }
  __syncthreads();

  // ---- per key block and query block: the numbers that belong together, in a fixed order ----------------
  for (int idx = tid; idx < n_u * G; idx += kThreads) {
    const int u = idx / G, g = idx % G;
    if (i0 + g >= a.nqb) continue;
    float v = 0.0f;
    const int p0 = pos_s[u];
    if (p0 >= 0) {
#pragma unroll
      for (int sub = 0; sub < SUB; ++sub) {
        const int p = p0 + sub;
        if (p < n_tiles && (t_meta[p] >> 10) == u) {
          if constexpr (G == 2) {
            const int att = (t_meta[p] >> 8) & 3;
            if (att == 3) {                // each row half's two waves hold the two key halves of its query block
              v = v + part[4 * p + 2 * g];
              v = v + part[4 * p + 2 * g + 1];
            } else if (att == 1 << g) {    // this query block alone: all four waves worked for it
#pragma unroll
              for (int w = 0; w < 4; ++w) v = v + part[4 * p + w];
            }
          } else {
#pragma unroll
            for (int w = 0; w < 4; ++w) v = v + part[4 * p + w];
          }
        }
      }
    }
    a.Mt[((size_t)h * n_u + u) * a.nqb_pad + i0 + g] = v;
  }
}

// ------------------------------------------------------------------------------------------------
// The pass behind the mass variant of the attention kernel.  That kernel has left, per workgroup, its tile list
// and, per wave and tile, log2 of every row's unnormalised probability sum over the tile; with the rows'
// log-sum-exp the share of a row is 2^(that - log2 normaliser).  One workgroup here per workgroup there: every
// (tile, wave) pair is summed over the wave's 64 rows by one wave (lane = row), then the
// numbers of a key block and query block are added in a fixed order.
// ------------------------------------------------------------------------------------------------
struct ReduceArgs {
  int H, Nq, nqb, nqb_pad, n_u, r_slots, list_cap;
  const float* R;
  const int32_t* list;
  const float* lse;
  float* Mt;
};

// 16 waves: a workgroup's hundred or two (tile, wave) pairs are a batch or two per wave, so the loads of the whole
// workgroup are in flight together
constexpr int kReduceThreads = 1024;

template <int B>
__global__ void __launch_bounds__(kReduceThreads) mass_reduce_kernel(ReduceArgs a) {
  constexpr int G = kRowsPerWg / B, SUB = B / kTile;
  extern __shared__ __align__(16) unsigned char smem[];
  float* part = reinterpret_cast<float*>(smem);            // [tile][wave of the attention kernel]
  int* meta_s = reinterpret_cast<int*>(part + 2 * a.list_cap);
  int* pos_s = meta_s + a.list_cap;                        // [key block][tile of the block] -> list position or -1
  __shared__ int ends[4];
  const int n_qt = (a.Nq + kRowsPerWg - 1) / kRowsPerWg;
  const int logical = blockIdx.x, h = logical / n_qt, T0 = (logical % n_qt) * kRowsPerWg, i0 = T0 / B;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int32_t* list = a.list + (size_t)logical * a.list_cap;
  if (tid < 4) ends[tid] = list[tid];
  for (int i = tid; i < a.n_u * SUB; i += kReduceThreads) pos_s[i] = -1;
  __syncthreads();
  const int n_shared = min(ends[1], a.list_cap - 4), n_list = min(ends[3], a.list_cap - 4);
  const int solo1 = min(ends[2], n_list);                  // wave 0 alone: [n_shared, solo1), wave 1: [solo1, n_list)
  for (int i = tid; i < n_list; i += kReduceThreads) {
    const int m = list[4 + i];
    meta_s[i] = m;
    const int u = (m >> 10) & 1023, sub = (m >> 20) & 1;
    if (u < a.n_u && sub < SUB) pos_s[u * SUB + sub] = i;
  }
  // minus log2 of the normaliser of the rows this lane stands for, one per wave of the attention kernel; a row
  // that does not exist or attended nothing takes no part
  float nl[2];
  bool live[2];
#pragma unroll
  for (int aw = 0; aw < 2; ++aw) {
    const int tok = T0 + 64 * aw + lane;
    const float l = a.lse[(size_t)h * a.Nq + min(tok, a.Nq - 1)];
    live[aw] = tok < a.Nq && l > -INFINITY;
    nl[aw] = live[aw] ? -l * 1.4426950408889634f : 0.0f;
  }
  // (tile, wave) pairs in batches: all the records of a batch are asked for before any is used, and the cross-lane
  // sums of a batch interleave -- one pair at a time the loop is a chain of memory and reduction latencies
  constexpr int kBatch = 8;
  for (int q0 = wave * kBatch; q0 < 2 * n_list; q0 += (kReduceThreads / 64) * kBatch) {
    float x[kBatch];
#pragma unroll
    for (int j = 0; j < kBatch; ++j) {
      const int q = q0 + j, p = q >> 1, aw = q & 1;
      // the wave's record of the tile: shared tiles come first, then its own
      int slot = -1;
      if (q < 2 * n_list) {
        if (p < n_shared) slot = p;
        else if (aw == 0 && p < solo1) slot = p;
        else if (aw == 1 && p >= solo1) slot = n_shared + (p - solo1);
      }
      x[j] = slot >= 0 && slot < a.r_slots ? a.R[(((size_t)logical * 2 + aw) * a.r_slots + slot) * 64 + lane] : -INFINITY;
    }
    float tot[kBatch];
#pragma unroll
    for (int j = 0; j < kBatch; ++j) {
      const int aw = (q0 + j) & 1;
      const float e = __builtin_amdgcn_exp2f(x[j] + (aw ? nl[1] : nl[0]));
      tot[j] = wave_sum((aw ? live[1] : live[0]) ? e : 0.0f);
    }
#pragma unroll
    for (int j = 0; j < kBatch; ++j)
      if (lane == 0 && q0 + j < 2 * n_list) part[q0 + j] = tot[j];
  }
  __syncthreads();
  for (int idx = tid; idx < a.n_u * G; idx += kReduceThreads) {
    const int u = idx / G, g = idx % G;
    if (i0 + g >= a.nqb) continue;
    float v = 0.0f;
#pragma unroll
    for (int sub = 0; sub < SUB; ++sub) {
      const int p = pos_s[u * SUB + sub];
      if (p >= 0) {
        if constexpr (G == 2) {
          v = v + part[2 * p + g];           // wave g of the attention kernel is query block g
        } else {
          v = v + part[2 * p];
          v = v + part[2 * p + 1];
        }
      }
    }
    a.Mt[((size_t)h * a.n_u + u) * a.nqb_pad + i0 + g] = v;
  }
}

size_t mass_lds_bytes(const pbsa_params& p) {
  const size_t sub = p.B / kTile, n_cand = ((size_t)p.C + 1 + p.n_loc) * sub;
  return kRingBytes + n_cand * 16 + n_cand * 8 + ((size_t)p.C + 1 + p.n_loc) * 4;
}

template <int D, int B>
hipError_t launch_mass_t(const MassArgs& a, size_t lds, dim3 grid, hipStream_t stream) {
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(mass_kernel<D, B>),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL((mass_kernel<D, B>), grid, dim3(kThreads), lds, stream, a);
  return hipGetLastError();
}

}  // namespace

MassRows carve_mass_ws(const pbsa_params& p, void* base) {
  MassRows m;
  const int sub = p.B / kTile, g = kRowsPerWg / p.B;
  const int tiles = (p.C + 1) * sub + (g * p.k < p.n_loc ? g * p.k : p.n_loc) * sub;    // most a workgroup can list
  const size_t n_wg = (size_t)p.H * ((p.Nq + kRowsPerWg - 1) / kRowsPerWg);
  m.r_slots = tiles;
  m.list_cap = 4 + tiles;
  char* b = static_cast<char*>(base);
  const size_t r_bytes = (n_wg * 2 * m.r_slots * 64 * 4 + 255) & ~(size_t)255;
  m.R = reinterpret_cast<float*>(b);
  m.list = reinterpret_cast<int32_t*>(b + r_bytes);
  m.bytes = r_bytes + ((n_wg * m.list_cap * 4 + 255) & ~(size_t)255);
  return m;
}

hipError_t launch_mass_reduce(const pbsa_params& p, const MassRows& rows, const float* lse, float* Mt,
                              hipStream_t stream) {
  const int n_u = p.C + 1 + p.n_loc, sub = p.B / kTile;
  ReduceArgs a{p.H, p.Nq, p.nqb, (p.nqb + 3) & ~3, n_u, rows.r_slots, rows.list_cap, rows.R, rows.list, lse, Mt};
  const int n_wg = p.H * ((p.Nq + kRowsPerWg - 1) / kRowsPerWg);
  const size_t lds = (size_t)rows.list_cap * 12 + (size_t)n_u * sub * 4;
  if (p.B == 128) hipLaunchKernelGGL(mass_reduce_kernel<128>, dim3(n_wg), dim3(kReduceThreads), lds, stream, a);
  else hipLaunchKernelGGL(mass_reduce_kernel<64>, dim3(n_wg), dim3(kReduceThreads), lds, stream, a);
  return hipGetLastError();
}

hipError_t launch_attention_mass(const pbsa_params& p, const bf16_t* Q, const bf16_t* Kp, const int32_t* p_len,
                                 const bf16_t* Kl, const int32_t* l_len, const int32_t* l_map, const int32_t* sel,
                                 const float* lse, float* Mt, hipStream_t stream) {
  const int nqb_pad = (p.nqb + 3) & ~3;
  MassArgs a{p.H, p.Nq, p.nqb, nqb_pad, p.n_loc, p.n_loc_cap, p.C, p.k, p.scale, p.q_stride_h, p.q_stride_t,
             Q, Kp, p_len, Kl, l_len, l_map, sel, lse, Mt};
  const int n_wg = p.H * ((p.Nq + kRowsPerWg - 1) / kRowsPerWg);
  const dim3 grid(8 * ((n_wg + 7) / 8));
  const size_t lds = mass_lds_bytes(p);
  if (p.d == 128 && p.B == 128) return launch_mass_t<128, 128>(a, lds, grid, stream);
  if (p.d == 128 && p.B == 64) return launch_mass_t<128, 64>(a, lds, grid, stream);
  if (p.d == 64 && p.B == 128) return launch_mass_t<64, 128>(a, lds, grid, stream);
  return launch_mass_t<64, 64>(a, lds, grid, stream);
}

}  // namespace pbsa
