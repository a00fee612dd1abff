// Internal launcher interface between the C-ABI shim (pbsa_api.hip) and the kernel files.
// Every launcher only enqueues on `stream` and returns the hipError_t of the launch.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "pbsa.h"

namespace pbsa {

typedef uint16_t bf16_t;   // raw bf16 bit pattern

// Scratch layout of pbsa_memory_update inside the caller's workspace (all offsets 256-byte aligned).
struct UpdateWs {
  float* A;           // [H][nU_max][nqb_pad] row-softmax of the coarse logits, column-major; nU_max = C + n_loc
  int32_t* fold_n;    // [H] number of dropped candidates
  int32_t* fold_src;  // [H][C + n_evict] dropped candidate: < C persistent slot, else C + physical local slot
  int32_t* promo_slot;  // [H][C] physical local slot a persistent slot is refilled from, or -1
  int32_t* fold_len;  // [H][C + n_evict] its valid tokens (read before p_len is rewritten)
  int32_t* plen_new;  // [H][C + 1] the slots' lengths after the update, committed to p_len by the fold kernel
  size_t bytes;
};
UpdateWs carve_update_ws(const pbsa_params& p, void* base);

hipError_t launch_pool_blocks(const pbsa_params& p, const bf16_t* X, const int32_t* len, int32_t n_blocks,
                              float* out, hipStream_t stream);
hipError_t launch_summary_view(const pbsa_params& p, const float* S_sum, const int32_t* S_cnt, bf16_t* Kp, bf16_t* Vp,
                               int32_t* p_len, hipStream_t stream);
hipError_t launch_select(const pbsa_params& p, const bf16_t* Q, const bf16_t* Kl, const int32_t* l_len,
                         const int32_t* l_map, float* Kc_l, float* Qc, int32_t* sel, float* Zl,
                         hipStream_t stream);
// launch_select of a chunk with launch_update_apply of the update of the chunk before it (parameters pu, same Kl) riding
// in its pooling launch.  The caller guarantees that the new chunk's ring position is not the one being folded.
hipError_t launch_select_apply(const pbsa_params& p, const bf16_t* Q, const bf16_t* Kl, const int32_t* l_len,
                               const int32_t* l_map, float* Kc_l, float* Qc, int32_t* sel, float* Zl,
                               const pbsa_params& pu, bf16_t* Kp, bf16_t* Vp, int32_t* p_len, float* S_sum,
                               const int32_t* S_cnt, const bf16_t* Vl, const UpdateWs& ws, hipStream_t stream);
// Scratch of the attention call that also produces the attention mass: what the attention kernel leaves for
// the pass that follows it.  Per workgroup (128 query rows of a head) a tile list of list_cap ints: the ends of
// the list's four parts, then a descriptor per tile; per wave r_slots records of 64 floats, one per tile in
// the order the wave walks them (log2 of each row's share of its normaliser, absolute).
struct MassRows {
  float* R;
  int32_t* list;
  int r_slots, list_cap;
  size_t bytes;
};
MassRows carve_mass_ws(const pbsa_params& p, void* base);

// rows == nullptr: the plain attention kernel
hipError_t launch_attention(const pbsa_params& p, const bf16_t* Q, const bf16_t* Kp, const bf16_t* Vp,
                            const int32_t* p_len, const bf16_t* Kl, const bf16_t* Vl, const int32_t* l_len,
                            const int32_t* l_map, const int32_t* sel, bf16_t* O, float* lse, const MassRows* rows,
                            hipStream_t stream);
// The same launch with H more workgroups that take the decisions of the memory update (launch_update_plan's work)
// while the attention runs; Zl is required.  launch_update_apply completes the update.
hipError_t launch_attention_plan(const pbsa_params& p, const bf16_t* Q, const bf16_t* Kp, const bf16_t* Vp,
                                 const int32_t* p_len, const bf16_t* Kl, const bf16_t* Vl, const int32_t* l_len,
                                 const int32_t* l_map, const int32_t* sel, bf16_t* O, float* lse, const float* Qc,
                                 const float* Kc_l, const float* Zl, float* Kc_p, int64_t* p_id, int32_t* S_cnt, int fold,
                                 const int64_t* l_id, float* scores, int32_t* slot_src, const UpdateWs& ws,
                                 hipStream_t stream);
hipError_t launch_mass_reduce(const pbsa_params& p, const MassRows& rows, const float* lse, float* Mt,
                              hipStream_t stream);
// The update in two parts.  plan: scoring and retention -- reads the cache's metadata and pooled keys, writes the
// decisions (scores, slot_src, p_id, Kc_p, S_cnt, and into the workspace the fold list, the promotions and the new
// slot lengths); touches neither K/V nor p_len, so it may run while the attention kernel of the same chunk does.
// apply: fold, promote and the commit of p_len.  launch_update is the two in a row.
hipError_t launch_update_plan(const pbsa_params& p, const float* Qc, const float* Kc_l, const float* Zl, float* Kc_p,
                              const int32_t* p_len, int64_t* p_id, int32_t* S_cnt, int fold, const int32_t* l_len,
                              const int32_t* l_map, const int64_t* l_id, float* scores, int32_t* slot_src,
                              const UpdateWs& ws, hipStream_t stream);
hipError_t launch_update_apply(const pbsa_params& p, bf16_t* Kp, bf16_t* Vp, int32_t* p_len, float* S_sum,
                               const int32_t* S_cnt, const bf16_t* Kl, const bf16_t* Vl, const UpdateWs& ws,
                               hipStream_t stream);
hipError_t launch_update(const pbsa_params& p, const float* Qc, const float* Kc_l, const float* Zl, bf16_t* Kp,
                         bf16_t* Vp,
                         float* Kc_p, int32_t* p_len, int64_t* p_id, float* S_sum, int32_t* S_cnt,
                         const bf16_t* Kl, const bf16_t* Vl, const int32_t* l_len, const int32_t* l_map,
                         const int64_t* l_id, float* scores, int32_t* slot_src, const UpdateWs& ws,
                         hipStream_t stream);

// fine attention mass Mt [H][C+1+n_loc][nqb rounded up to 4] and the update ranked by it (Mt given: Qc / Zl unused)
hipError_t launch_attention_mass(const pbsa_params& p, const bf16_t* Q, const bf16_t* Kp, const int32_t* p_len,
                                 const bf16_t* Kl, const int32_t* l_len, const int32_t* l_map, const int32_t* sel,
                                 const float* lse, float* Mt, hipStream_t stream);
hipError_t launch_update_fine(const pbsa_params& p, const float* Mt, const float* Kc_l, bf16_t* Kp, bf16_t* Vp,
                              float* Kc_p, int32_t* p_len, int64_t* p_id, float* S_sum, int32_t* S_cnt,
                              const bf16_t* Kl, const bf16_t* Vl, const int32_t* l_len, const int32_t* l_map,
                              const int64_t* l_id, float* scores, int32_t* slot_src, const UpdateWs& ws,
                              hipStream_t stream);

// backward of the fine stage; Dr: [H][Nq] floats of scratch (bwd_workspace_bytes)
size_t bwd_workspace_bytes(const pbsa_params& p);
hipError_t launch_attention_bwd(const pbsa_params& p, const bf16_t* Q, const bf16_t* Kp, const bf16_t* Vp,
                                const int32_t* p_len, const bf16_t* Kl, const bf16_t* Vl, const int32_t* l_len,
                                const int32_t* l_map, const int32_t* sel, const bf16_t* O, const bf16_t* dO,
                                const float* lse, float* dQ, float* dKp, float* dVp, float* dKl, float* dVl, float* Dr,
                                hipStream_t stream);

// blockify: to_blocks = true moves token-major -> block-major, false the other way
struct LayoutTensors {
  int n;
  const bf16_t* tok[4];     // token-major side (read when to_blocks, written otherwise)
  bf16_t* blk[4];           // block-major side
  long blk_stride_h[4];
};
hipError_t launch_blockify(const pbsa_grid& g, const LayoutTensors& t, bool to_blocks, hipStream_t stream);

}  // namespace pbsa
