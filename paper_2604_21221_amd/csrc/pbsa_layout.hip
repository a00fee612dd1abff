// Locality-preserving block rearrange (App. "Rearrange for Locality Preserving", Alg. 3) for gfx950.
//
// A pure permutation of token rows (one head's d values of one token: 128 or 256 contiguous bytes on
// both sides), so the kernel is bound by HBM: every byte is read once and written once.  A thread moves
// 16 bytes; consecutive threads walk the block-major side in memory order (chunk of a row, row of a
// block, block), so that side is one contiguous stream per head and the token-major side is touched in
// whole rows.  blockIdx.y = tensor * H + head.
#include "pbsa_internal.h"

namespace pbsa {
namespace {

constexpr int kThreads = 256;

struct LayoutArgs {
  LayoutTensors t;
  int T, Hs, Ws, Bt, Bh, Bw, H, d, B;
  int Nh, Nw, n_blocks, rows;   // blocks along Hs and Ws, blocks per head, token rows per block
};

constexpr int kPerThread = 1;   // 16-byte pieces per thread (more, a quarter of the tensor apart, were slower: 33 us against 25)

template <bool TO_BLOCKS>
__global__ void __launch_bounds__(kThreads) blockify_kernel(LayoutArgs a) {
  const int cpr = a.d / 8;                                   // 16-byte chunks per row
  const long per_head = (long)a.n_blocks * a.rows * cpr;
  const long quarter = (per_head + kPerThread - 1) / kPerThread;   // pieces u of all threads form one contiguous part
  const long idx0 = (long)blockIdx.x * kThreads + threadIdx.x;
  if (idx0 >= quarter) return;
  const int ti = blockIdx.y / a.H, h = blockIdx.y % a.H;
  const bf16_t* src = TO_BLOCKS ? a.t.tok[ti] : a.t.blk[ti];
  bf16_t* dst = TO_BLOCKS ? a.t.blk[ti] : const_cast<bf16_t*>(a.t.tok[ti]);
  long from[kPerThread], to[kPerThread];
  uint4 v[kPerThread];
#pragma unroll
  for (int u = 0; u < kPerThread; ++u) {
    const long idx = idx0 + u * quarter;                     // the pieces of a thread are far apart, those of a wave adjacent
    const bool on = idx < per_head;
    const long id = on ? idx : 0;
    const int c = (int)(id % cpr);
    const long row = id / cpr;
    const int r = (int)(row % a.rows), b = (int)(row / a.rows);
    // block b = (t_b, h_b, w_b), row r = (dt, dh, dw), both row-major
    const int wb = b % a.Nw, hb = (b / a.Nw) % a.Nh, tb = b / (a.Nw * a.Nh);
    const int dw = r % a.Bw, dh = (r / a.Bw) % a.Bh, dt = r / (a.Bw * a.Bh);
    const long token = ((long)(tb * a.Bt + dt) * a.Hs + (hb * a.Bh + dh)) * a.Ws + (wb * a.Bw + dw);
    const long tok_off = (token * a.H + h) * a.d + 8 * c;
    const long blk_off = (long)h * a.t.blk_stride_h[ti] + ((long)b * a.B + r) * a.d + 8 * c;
    from[u] = TO_BLOCKS ? tok_off : blk_off;
    to[u] = on ? (TO_BLOCKS ? blk_off : tok_off) : -1;
    v[u] = *reinterpret_cast<const uint4*>(src + from[u]);
  }
#pragma unroll
  for (int u = 0; u < kPerThread; ++u)
    if (to[u] >= 0) *reinterpret_cast<uint4*>(dst + to[u]) = v[u];
}

}  // namespace

hipError_t launch_blockify(const pbsa_grid& g, const LayoutTensors& t, bool to_blocks, hipStream_t stream) {
  LayoutArgs a{t, g.T, g.Hs, g.Ws, g.Bt, g.Bh, g.Bw, g.H, g.d, g.B, g.Hs / g.Bh, g.Ws / g.Bw, 0, g.Bt * g.Bh * g.Bw};
  a.n_blocks = (g.T / g.Bt) * a.Nh * a.Nw;
  const long per_head = (long)a.n_blocks * a.rows * (g.d / 8);
  if (per_head == 0 || t.n == 0) return hipSuccess;
  const long quarter = (per_head + kPerThread - 1) / kPerThread;
  const dim3 grid((unsigned)((quarter + kThreads - 1) / kThreads), (unsigned)(t.n * g.H)), block(kThreads);
  if (to_blocks) hipLaunchKernelGGL(blockify_kernel<true>, grid, block, 0, stream, a);
  else hipLaunchKernelGGL(blockify_kernel<false>, grid, block, 0, stream, a);
  return hipGetLastError();
}

}  // namespace pbsa
