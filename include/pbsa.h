/*
 * pbsa.h -- C ABI of the MI355X (gfx950) Persistent Block-Sparse Attention decode path.
 *
 * The path is the per-chunk attention of a causal video DiT over a bounded KV memory
 * M = P u L (Sec. 3.3, Eq. 2): a persistent set P of at most C blocks that every query attends
 * densely, and a sliding local region L (window + the chunk being generated) in which each query
 * block attends only its top-k key blocks.  One layer-chunk step is
 *
 *     pbsa_select_blocks  ->  pbsa_attention_fwd  ->  pbsa_memory_update
 *
 * (or, ranking the persistent set by the attention actually paid:
 *     pbsa_select_blocks  ->  pbsa_attention_fwd_mass  ->  pbsa_memory_update_fine).
 *
 * Conventions
 *  - Every tensor pointer is a DEVICE pointer owned by the caller; `const pbsa_params*` and the
 *    `size_t*` result of pbsa_workspace_bytes are HOST pointers.  The library never allocates,
 *    frees or synchronises: a call validates its arguments on the host, enqueues kernels on
 *    `hip_stream` (a hipStream_t, NULL = the default stream) and returns.
 *  - bf16 tensors are raw 16-bit patterns.  bf16 and fp32 tensor base pointers and the workspace must be
 *    16-byte (workspace: 256-byte) aligned; integer arrays need only their natural alignment.
 *  - Block-major cache layout (App. "Rearrange for Locality Preserving", Alg. 3): the B tokens of a
 *    block are contiguous, [B][d] row-major.  Rows at or beyond a block's valid length are never
 *    trusted (pooling divides by the valid length, attention masks them).
 *  - Everything is per head: each head has its own block sets, persistent slots and summary.
 *  - Return value: PBSA_OK or a negative PBSA_E* code; pbsa_strerror() gives the text.  Validation
 *    happens before any HIP call, so argument errors are reported even on a machine with no GPU.
 *  - Results are deterministic: no floating-point atomics, fixed reduction orders.
 *
 * Shapes
 *   Q, O         [H][Nq][d] bf16, element strides (q_stride_h, q_stride_t) / (o_stride_h, o_stride_t),
 *                last dimension contiguous; query block i = chunk tokens iB .. min((i+1)B, Nq)-1
 *   Kl, Vl       [H][n_loc_cap][B][d] bf16   physical local slots (ring storage)
 *   l_map        [n_loc] int32               logical local block (oldest first, the chunk's nqb blocks
 *                                            last) -> physical slot
 *   l_len, l_id  [n_loc] int32 / int64       valid tokens (1..B) and global id of each logical block
 *   Kc_l         [H][n_loc_cap][d] fp32      pooled keys, indexed by physical slot
 *   Qc           [H][nqb][d] fp32            pooled queries of the chunk
 *   sel          [H][nqb][k] int32           selected logical local blocks per query block,
 *                                            ascending, padded with -1
 *   Zl           [H][nqb][n_loc] fp32        coarse logits dot(Qc_i, Kc_l) * scale of every local block
 *                                            (no visibility mask); optional hand-over from the
 *                                            selection call to the update call of the same chunk
 *   Kp, Vp       [H][C+1][B][d] bf16         persistent slots; slot C holds the compressed-history
 *                                            ("summary") block
 *   p_len        [H][C+1] int32              valid tokens per slot, 0 = empty (skipped)
 *   Kc_p, p_id   [H][C][d] fp32, [H][C] int64
 *   S_sum, S_cnt [H][2][B][d] fp32 (K then V), [H][B] int32   running sums / counts of the summary
 *
 * Arithmetic that decides an integer (block sets, slot assignment) is specified exactly, in IEEE
 * binary32 without contraction, so that an independent implementation reproduces it bit for bit:
 *   pool(X, len)[x]  = ( ...((0 + X[0][x]) + X[1][x]) ... + X[len-1][x]) / (float)len
 *   dot(q, k)        = fma(q[d-1], k[d-1], ... fma(q[1], k[1], fma(q[0], k[0], 0)) ...) * scale
 *   pexp(x), x <= 0  = 0 if x < -64, else with n = rint(x * 0x1.715476p+0f),
 *                      r = fma(n, 0x1.bd0106p-13f, fma(n, -0x1.63p-1f, x)),
 *                      p = Horner in r by fma of (1/720, 1/120, 1/24, 1/6, 1/2, 1, 1) rounded to
 *                      binary32, the value p * 2^n
 *   row softmax      m = max_j z_j; e_j = pexp(z_j - m); s = (...(0 + e_0) + e_1 ...); a_j = e_j / s
 *   column mean      (...((0 + a_0j) + a_1j) ... + a_(nqb-1)j) / (float)nqb
 *   summary fold     S_sum = S_sum + x, dropped blocks taken in candidate order
 * Ties in a ranking go to the lower index.
 */
#ifndef PBSA_H
#define PBSA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define PBSA_OK      0
#define PBSA_EINVAL (-1) /* NULL pointer, wrong .size, inconsistent counts                      */
#define PBSA_ESHAPE (-2) /* d, B, k, C, n_loc ... outside what the kernels support              */
#define PBSA_EALIGN (-3) /* pointer not 16-byte aligned, or a stride not a multiple of 8 elems  */
#define PBSA_EWS    (-4) /* workspace missing or smaller than pbsa_workspace_bytes()            */
#define PBSA_EHIP   (-5) /* a HIP call or kernel launch failed                                   */

/* Limits of pbsa_select_blocks and pbsa_attention_fwd (the largest shape of the paper's kernel benchmark,
 * N_C = 21504 queries against N_L = 4 N_C local and N_P = N_L / 2 persistent tokens in blocks of 128, fits). */
#define PBSA_MAX_N_LOC 672 /* logical local blocks          */
#define PBSA_MAX_K     672 /* selected blocks per query block */
#define PBSA_MAX_C_ATTEND 336 /* persistent slots that pbsa_attention_fwd can attend (pbsa_select_blocks does not
                               * look at them); above PBSA_MAX_C the caller maintains the set itself */
/* Limits of every other entry point (the memory update in all its forms, pbsa_select_blocks_apply,
 * pbsa_attention_fwd_plan, pbsa_attention_fwd_mass, pbsa_attention_mass, pbsa_attention_bwd): */
#define PBSA_MAX_N_LOC_AUX 512
#define PBSA_MAX_K_AUX     512
#define PBSA_MAX_C_AUX     192 /* slots attended, where the call attends                      */
#define PBSA_MAX_C          64 /* persistent slots that pbsa_memory_update can maintain       */

typedef struct pbsa_params {
  uint32_t size;            /* sizeof(pbsa_params); guards against ABI drift                        */
  int32_t H;                /* heads                                                                */
  int32_t d;                /* head dim: 64 or 128                                                  */
  int32_t B;                /* tokens per block: 64 or 128                                          */
  int32_t Nq;               /* chunk (query) tokens                                                 */
  int32_t nqb;              /* ceil(Nq / B): query blocks = key blocks the chunk contributes        */
  int32_t n_loc;            /* logical local blocks, the chunk's nqb included (nqb <= n_loc)        */
  int32_t n_loc_cap;        /* physical local slots per head (n_loc <= n_loc_cap)                   */
  int32_t C;                /* persistent slots, excluding the summary slot                         */
  int32_t n_sink;           /* leading slots that are never evicted (footnote to Eq. 9)             */
  int32_t k;                /* local blocks selected per query block (Eq. 11, as a count)           */
  int32_t causal;           /* 1: query block i sees local blocks 0 .. n_loc-nqb+i; 0: all n_loc    */
  int32_t n_evict;          /* |E_t|: leading local blocks leaving the window at this update        */
  int32_t pool_from;        /* select: pooled keys of logical blocks >= pool_from are recomputed,   */
                            /* earlier ones are trusted from Kc_l (normally n_loc - nqb)            */
  float scale;              /* softmax scale, 1/sqrt(d)                                             */
  int64_t q_stride_h, q_stride_t;
  int64_t o_stride_h, o_stride_t;
} pbsa_params;

/* Bytes of scratch that any call with these parameters may need (device memory, 256-byte aligned,
 * passed as `ws`).  Contents need not be preserved between calls.  Only pbsa_memory_update needs any, so
 * C is held to PBSA_MAX_C here as there. */
int pbsa_workspace_bytes(const pbsa_params* p, size_t* out);

/* Block representatives by average pooling (Eq. 6; pooling operator of Sec. 4.1):
 * out[n][:] = mean over the first len[n] rows of X[n].  X [n_blocks][B][d] bf16, len [n_blocks]
 * int32 (0 gives a zero vector), out [n_blocks][d] fp32.  Uses p->B and p->d only.  For seeding the
 * pooled keys of persistent blocks the caller installs by hand. */
int pbsa_pool_blocks(const pbsa_params* p, const void* X, const int32_t* len, int32_t n_blocks, float* out,
                     void* hip_stream);

/* The bf16 view of a compressed-history block from its running sums and counts (the pooling of the evicted blocks,
 * Sec. 3.3 "compressed global memory"; the same arithmetic as the fold of pbsa_memory_update): for every head, row t
 * of slot C of Kp and of Vp becomes S_sum[h][0 / 1][t][:] / S_cnt[h][t] (fp32 division, rounded to nearest even) where
 * S_cnt[h][t] > 0, other rows are left as they are, and p_len[h][C] becomes the number of such rows.  For a caller
 * that installs a summary by hand (a resumed roll-out).  S_sum [H][2][B][d] fp32 and S_cnt [H][B] int32 are read,
 * Kp, Vp [H][C+1][B][d] bf16 and p_len [H][C+1] int32 are written; all device memory.  Uses p->H, B, d, C only. */
int pbsa_summary_view(const pbsa_params* p, const float* S_sum, const int32_t* S_cnt, void* Kp, void* Vp,
                      int32_t* p_len, void* hip_stream);

/* Coarse routing inside the local region (Eq. 10-11).  Pools the chunk's queries into Qc, refreshes
 * the pooled keys Kc_l of logical blocks >= pool_from, scores every visible local block of every
 * query block with dot(Qc_i, Kc_l) (the argument of Eq. 10's softmax, which is monotone per row)
 * and writes the min(k, visible) best blocks of each row to `sel` (ascending, -1 padded; ties to
 * the lower block).  Kc_l is in/out, Qc and sel are out.  Zl (optional out) receives the logits of
 * all n_loc local blocks of every row, for pbsa_memory_update.  ws may be NULL. */
int pbsa_select_blocks(const pbsa_params* p, const void* Q, const void* Kl, const int32_t* l_len,
                       const int32_t* l_map, float* Kc_l, float* Qc, int32_t* sel, float* Zl, void* ws,
                       size_t ws_bytes, void* hip_stream);

/* PBSA fine stage (Eq. 3-5): for each query token one softmax, scaled by p->scale, over every
 * valid token of every non-empty persistent slot 0..C (summary included) and every valid token of
 * the local blocks listed in its query block's row of `sel`; O = P V.  bf16 MFMA with fp32
 * accumulation and fp32 online softmax; the probabilities are rounded to bf16 for the second product and
 * the normaliser is their sum after rounding; O is rounded to bf16 (nearest even).  `lse` (optional,
 * [H][Nq] fp32) receives the natural log of that normaliser (within 4e-3 of the exact one).  A row that sees no key gets O = 0,
 * lse = -inf.  Entries of sel must be -1 or in [0, n_loc).  ws may be NULL. */
int pbsa_attention_fwd(const pbsa_params* p, const void* Q, const void* Kp, const void* Vp, const int32_t* p_len,
                       const void* Kl, const void* Vl, const int32_t* l_len, const int32_t* l_map,
                       const int32_t* sel, void* O, float* lse, void* ws, size_t ws_bytes, void* hip_stream);

/* Persistent-memory update (Eq. 7-9).  Scores: block-level softmax of each pooled query over
 * U = occupied slots 0..C-1 followed by all n_loc local blocks, averaged over query blocks
 * (Eq. 7-8).  Candidates: occupants of slots n_sink..C-1 in slot order, then the n_evict leading
 * local blocks; the best C-n_sink by (score, then lower candidate index) stay (Eq. 9).  A kept
 * occupant keeps its slot; kept newcomers, in ascending block order, fill vacated and empty slots in
 * ascending slot order, and K, V, Kc_p, p_len, p_id move with them.  Every dropped candidate is
 * added position by position to S_sum/S_cnt and slot C is rewritten with their running mean
 * (bf16), p_len[C] = number of positions with a count; pass S_sum = S_cnt = NULL to drop without
 * compressing.  Qc and Kc_l are those pbsa_select_blocks produced for this chunk; Zl (optional) is
 * the logits array it produced with the same n_loc: given, the local columns of Eq. 7 are taken from
 * it (they are the same numbers) and only the persistent columns are multiplied again.
 * Outputs: scores (optional, [H][C+n_evict] fp32: slots 0..C-1, 0 if empty, then evicted blocks),
 * slot_src [H][C] int32: -1 = slot unchanged, e >= 0 = filled from local block e.
 * ws is required (pbsa_workspace_bytes). */
int pbsa_memory_update(const pbsa_params* p, const float* Qc, const float* Kc_l, const float* Zl, void* Kp,
                       void* Vp, float* Kc_p, int32_t* p_len, int64_t* p_id, float* S_sum, int32_t* S_cnt,
                       const void* Kl, const void* Vl, const int32_t* l_len, const int32_t* l_map,
                       const int64_t* l_id, float* scores, int32_t* slot_src, void* ws, size_t ws_bytes,
                       void* hip_stream);

/* pbsa_memory_update for callers that cannot allocate device memory or hand over a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments without ws / ws_bytes, same
 * results bit for bit (the same kernels run); the scratch is a fixed array of PBSA_STATIC_WS_BYTES inside the
 * library's code object, of which every GPU the library runs on holds its own copy until the process ends.  The
 * call allocates and frees nothing (the first call on a device looks the array's address up once).  Parameters
 * whose pbsa_workspace_bytes() exceeds PBSA_STATIC_WS_BYTES are refused with PBSA_EWS before anything is enqueued.
 * All calls on one GPU share that GPU's array: two of them that overlap in time (different streams, or different
 * threads) race -- serialise them.  Nothing in the array has to survive between calls or start at zero (the
 * kernels write every word before reading it). */
#define PBSA_STATIC_WS_BYTES (4u << 20)
int pbsa_memory_update_static(const pbsa_params* p, const float* Qc, const float* Kc_l, const float* Zl, void* Kp,
                              void* Vp, float* Kc_p, int32_t* p_len, int64_t* p_id, float* S_sum, int32_t* S_cnt,
                              const void* Kl, const void* Vl, const int32_t* l_len, const int32_t* l_map,
                              const int64_t* l_id, float* scores, int32_t* slot_src, void* hip_stream);

/* pbsa_memory_update in two calls, for a caller that overlaps the update's decisions with the attention of the same
 * chunk.  _plan scores and ranks (Eq. 7-9): it reads Qc, Kc_l, Zl, Kc_p, p_len and the local region's metadata and
 * writes scores, slot_src, p_id, Kc_p, S_cnt (pass S_cnt = NULL to drop without compressing) and, into ws, what
 * _apply needs; it touches neither K/V nor p_len, so it may run on another stream while pbsa_attention_fwd of the
 * chunk runs (after the chunk's pbsa_select_blocks; the arrays it writes are not read by the attention call).
 * _apply folds the dropped blocks into the summary, moves the promoted blocks into their slots and commits the
 * new p_len; it must follow both the attention call and _plan, with the same p and ws (whose contents must have
 * been left alone in between).  pbsa_memory_update is exactly the two in a row. */
int pbsa_memory_update_plan(const pbsa_params* p, const float* Qc, const float* Kc_l, const float* Zl, float* Kc_p,
                            const int32_t* p_len, int64_t* p_id, int32_t* S_cnt, const int32_t* l_len,
                            const int32_t* l_map, const int64_t* l_id, float* scores, int32_t* slot_src, void* ws,
                            size_t ws_bytes, void* hip_stream);
int pbsa_memory_update_apply(const pbsa_params* p, void* Kp, void* Vp, int32_t* p_len, float* S_sum, const int32_t* S_cnt,
                             const void* Kl, const void* Vl, void* ws, size_t ws_bytes, void* hip_stream);

/* pbsa_select_blocks of a chunk and pbsa_memory_update_apply of the update of the chunk BEFORE it, with the fold /
 * promote workgroups riding in the selection's pooling launch (Alg. 1 over consecutive chunks: the data movement that
 * ends one iteration and the coarse stage that starts the next touch disjoint data, and each alone is too short to
 * fill the GPU).  p and the arguments up to Zl are those of pbsa_select_blocks for the new chunk; p_upd and the
 * arguments after it are those of the pending pbsa_memory_update_apply (same Kl; same H, d, B, C, n_loc_cap, else
 * PBSA_EINVAL).  Results are those of the two calls, bit for bit.  The CALLER guarantees what makes the two
 * independent: the new chunk's K / V are not in the ring position whose blocks the pending update evicts (a ring of
 * window + 2 chunks gives that), and nothing between the attention launch that took the decisions and this call has
 * touched ws. */
int pbsa_select_blocks_apply(const pbsa_params* p, const void* Q, const void* Kl, const int32_t* l_len,
                             const int32_t* l_map, float* Kc_l, float* Qc, int32_t* sel, float* Zl,
                             const pbsa_params* p_upd, void* Kp, void* Vp, int32_t* p_len, float* S_sum,
                             const int32_t* S_cnt, const void* Vl, void* ws, size_t ws_bytes, void* hip_stream);

/* pbsa_attention_fwd and pbsa_memory_update_plan of the same chunk as ONE launch (Alg. 1 with the update's
 * decisions, Eq. 7-9, taken while the fine stage of Eq. 3-5 runs): the attention's grid gets H more workgroups, one
 * per head, that do the plan call's work.  Nothing they read is written by the attention part and the other way
 * round, so the results are those of the two calls, bit for bit; a launch whose attention workgroups do not fill
 * the GPU (two workgroups of 128 query rows per compute unit) has the plan's work for free.  Arguments: those of
 * pbsa_attention_fwd (p->C <= PBSA_MAX_C here), then those of pbsa_memory_update_plan that it does not have yet;
 * Zl is required (PBSA_EINVAL without), ws as for pbsa_memory_update.  pbsa_memory_update_apply completes the
 * update. */
int pbsa_attention_fwd_plan(const pbsa_params* p, const void* Q, const void* Kp, const void* Vp, const int32_t* p_len,
                            const void* Kl, const void* Vl, const int32_t* l_len, const int32_t* l_map,
                            const int32_t* sel, void* O, float* lse, const float* Qc, const float* Kc_l,
                            const float* Zl, float* Kc_p, int64_t* p_id, int32_t* S_cnt, const int64_t* l_id,
                            float* scores, int32_t* slot_src, void* ws, size_t ws_bytes, void* hip_stream);

/* Attention mass per key block (the fine-grained counterpart of Eq. 7: the attention of Eq. 3-5 as it was
 * actually paid, mask included, summed block by block).  Key blocks are numbered u = slot for the persistent
 * slots 0..C (the summary is u = C) and u = C + 1 + l for local block l.
 *   Mt[h][u][i] = sum over the tokens q of query block i and the valid tokens j of key block u of
 *                 exp(scale * dot(Q[q], K[j]) - lse[h][q]),
 * 0 where query block i does not attend block u (an empty slot, a local block outside its row of sel).
 * lse [H][Nq] fp32 is the output of pbsa_attention_fwd for the same arguments, so the masses of a query
 * block add up to its number of tokens (within 5e-3 relative: lse carries the rounding of the bf16
 * probabilities).  Mt [H][C+1+n_loc][nqb_pad] fp32 out, nqb_pad = nqb rounded up to a multiple of 4; the
 * padding columns are not written.  bf16 MFMA for the scores, fp32 sums in a fixed order. */
int pbsa_attention_mass(const pbsa_params* p, const void* Q, const void* Kp, const int32_t* p_len, const void* Kl,
                        const int32_t* l_len, const int32_t* l_map, const int32_t* sel, const float* lse, float* Mt,
                        void* hip_stream);

/* pbsa_attention_fwd and the attention mass in one call: the attention kernel also records, per sub-tile of
 * keys and per query row, the logarithm of the row's probability sum over that sub-tile (numbers its softmax
 * has anyway), and a short second kernel turns the records into Mt, laid out as above.  Costs a few per cent
 * over pbsa_attention_fwd where pbsa_attention_mass repeats the whole first product.  O, lse (required here)
 * and every argument before them are those of pbsa_attention_fwd; the masses are those of the bf16-rounded
 * probabilities the second product used, so a query block's masses add up to its number of tokens to fp32
 * rounding.  ws: pbsa_mass_workspace_bytes(p) bytes of device scratch, 256-byte aligned, contents not kept. */
int pbsa_mass_workspace_bytes(const pbsa_params* p, size_t* out);
int pbsa_attention_fwd_mass(const pbsa_params* p, const void* Q, const void* Kp, const void* Vp, const int32_t* p_len,
                            const void* Kl, const void* Vl, const int32_t* l_len, const int32_t* l_map,
                            const int32_t* sel, void* O, float* lse, float* Mt, void* ws, size_t ws_bytes,
                            void* hip_stream);

/* pbsa_memory_update with the persistence score taken from the attention mass instead of Eq. 7-8's
 * block-level softmax: the score of key block u is its mass per query token,
 *   (...((0 + Mt[h][u][0]) + Mt[h][u][1]) ... + Mt[h][u][nqb-1]) / (float)Nq      (binary32, this order),
 * 0 for an empty slot.  Candidates, ranking (Eq. 9), slot assignment, fold and every output are those of
 * pbsa_memory_update; Kc_l is only read to move the pooled keys of promoted blocks.  Mt is laid out as
 * pbsa_attention_mass writes it (any matrix of that shape is ranked the same way). */
int pbsa_memory_update_fine(const pbsa_params* p, const float* Mt, const float* Kc_l, void* Kp, void* Vp, float* Kc_p,
                            int32_t* p_len, int64_t* p_id, float* S_sum, int32_t* S_cnt, const void* Kl,
                            const void* Vl, const int32_t* l_len, const int32_t* l_map, const int64_t* l_id,
                            float* scores, int32_t* slot_src, void* ws, size_t ws_bytes, void* hip_stream);

/* Backward of pbsa_attention_fwd (the paper's training kernel: gradients through the block-sparse attention).
 * With P the masked row softmax of Eq. 3-5 and dO the gradient of a scalar loss with respect to O = P V:
 *   dV = P^T dO,  dZ = P o (dO V^T - D) with D[q] = dO[q] . O[q],  dQ = scale dZ K,  dK = scale dZ^T Q.
 * Inputs: everything pbsa_attention_fwd took, its outputs O (bf16) and lse (fp32, required), and dO, bf16 with
 * O's strides.  P is recomputed as exp(scale q.k - lse) on bf16 MFMA; P and dZ are rounded to bf16 for the second
 * products, sums are fp32.  Outputs, fp32, every element written exactly once (deterministic, no atomics):
 *   dQ [H][Nq][d] dense;  dKp, dVp [H][C+1][B][d] (the summary slot C included);  dKl, dVl [H][n_loc_cap][B][d] by
 *   physical slot: the slots of the n_loc logical blocks are written in full -- zeros for rows past a block's
 *   length and for blocks no query block selected -- other slots are left alone.
 * ws: pbsa_bwd_workspace_bytes(p) bytes of device scratch (the D vector), 256-byte aligned. */
int pbsa_bwd_workspace_bytes(const pbsa_params* p, size_t* out);
int pbsa_attention_bwd(const pbsa_params* p, const void* Q, const void* Kp, const void* Vp, const int32_t* p_len,
                       const void* Kl, const void* Vl, const int32_t* l_len, const int32_t* l_map, const int32_t* sel,
                       const void* O, const void* dO, const float* lse, float* dQ, float* dKp, float* dVp, float* dKl,
                       float* dVl, void* ws, size_t ws_bytes, void* hip_stream);

/* Locality-preserving block rearrange (App. "Rearrange for Locality Preserving", Alg. 3): the tokens of a
 * chunk come from the model in (frame, patch row, patch column) order, T x Hs x Ws of them, each a row of
 * H heads x d; a block is a Bt x Bh x Bw box of the grid, blocks are numbered (t_b, h_b, w_b) row-major and
 * the tokens of a block (dt, dh, dw) row-major, which is the block-major layout every other call here works
 * on.  Alg. 3 assumes that the block shape divides the grid; so does this call (PBSA_ESHAPE otherwise). */
typedef struct pbsa_grid {
  uint32_t size;            /* sizeof(pbsa_grid)                                                    */
  int32_t T, Hs, Ws;        /* latent grid of the chunk: frames, patch rows, patch columns          */
  int32_t Bt, Bh, Bw;       /* block shape                                                          */
  int32_t H, d;             /* heads, head dim (a multiple of 8)                                    */
  int32_t B;                /* token rows per block slot on the block-major side, >= Bt * Bh * Bw   */
} pbsa_grid;

/* Rearranges n tensors (1 <= n <= 4: say Q, K and V of a chunk) in one launch.  X[i] is token-major,
 * [T][Hs][Ws][H][d] bf16.  On the block-major side head h of tensor i starts blk_stride_h[i] * h elements
 * after Xblk[i], block b of it b * B * d elements further, token row r of the block r * d further; rows
 * Bt*Bh*Bw .. B-1 of a slot are left as they are (their block's valid length is Bt*Bh*Bw).  With Xblk[i]
 * pointing at the first slot of a ring position of Kl / Vl and blk_stride_h[i] = n_loc_cap * B * d this is
 * the cache append.  X, Xblk and blk_stride_h are HOST arrays of n entries; the pointers in X and Xblk are
 * device pointers, 16-byte aligned; strides are multiples of 8 elements. */
int pbsa_blockify(const pbsa_grid* g, int32_t n, const void* const* X, void* const* Xblk, const int64_t* blk_stride_h,
                  void* hip_stream);
/* The inverse for one tensor (the attention output): block-major Xblk -> token-major X. */
int pbsa_unblockify(const pbsa_grid* g, const void* Xblk, int64_t blk_stride_h, void* X, void* hip_stream);

const char* pbsa_strerror(int code);
int pbsa_version(void);

#ifdef __cplusplus
}
#endif
#endif /* PBSA_H */
