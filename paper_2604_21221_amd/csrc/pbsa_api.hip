// C-ABI shim of libpbsa: host-side argument validation, then kernel launches.  Validation makes no
// HIP call, so every argument error is reported on a machine without a GPU as well.
#include <string.h>

#include "pbsa_internal.h"

namespace {

thread_local char g_hip_msg[256] = "";

int hip_fail(hipError_t e) {
  snprintf(g_hip_msg, sizeof g_hip_msg, "HIP error %d: %s", (int)e, hipGetErrorString(e));
  return PBSA_EHIP;
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Checks that do not depend on which call is made, but for the number of persistent slots it can handle.
int check_common(const pbsa_params* p, int max_c = PBSA_MAX_C, int max_n_loc = PBSA_MAX_N_LOC_AUX,
                 int max_k = PBSA_MAX_K_AUX) {
  if (!p) return PBSA_EINVAL;
  if (p->size != sizeof(pbsa_params)) return PBSA_EINVAL;
  if (p->H < 1 || p->Nq < 1 || p->n_loc < 0 || p->C < 0 || p->k < 0 || p->n_sink < 0 || p->n_evict < 0 ||
      p->pool_from < 0)
    return PBSA_EINVAL;
  if (p->d != 64 && p->d != 128) return PBSA_ESHAPE;
  if (p->B != 64 && p->B != 128) return PBSA_ESHAPE;
  if (p->nqb != (p->Nq + p->B - 1) / p->B) return PBSA_EINVAL;
  if (p->n_loc < p->nqb || p->n_loc > p->n_loc_cap) return PBSA_EINVAL;
  if (p->n_sink > p->C || p->n_evict > p->n_loc || p->pool_from > p->n_loc) return PBSA_EINVAL;
  if (p->causal != 0 && p->causal != 1) return PBSA_EINVAL;
  if (!(p->scale > 0.0f) || !(p->scale < 1e30f)) return PBSA_EINVAL;
  if (p->n_loc > max_n_loc || p->C > max_c || p->k > max_k) return PBSA_ESHAPE;
  if ((int64_t)p->H * p->n_loc_cap * p->B * p->d >= ((int64_t)1 << 40)) return PBSA_ESHAPE;
  // heads are a grid dimension of the selection, scoring and fold launches, and the selection forms 32-bit byte
  // offsets into the pooled keys
  if (p->H > 65535) return PBSA_ESHAPE;
  if ((int64_t)p->H * p->n_loc_cap * p->d * 4 >= ((int64_t)1 << 32)) return PBSA_ESHAPE;
  return PBSA_OK;
}

int check_strides(int64_t sh, int64_t st, const pbsa_params* p) {
  if (st < p->d || sh < 0) return PBSA_EINVAL;
  if (st % 8 != 0 || sh % 8 != 0) return PBSA_EALIGN;
  return PBSA_OK;
}

size_t workspace_bytes(const pbsa_params& p) { return pbsa::carve_update_ws(p, nullptr).bytes; }

}  // namespace

// Scratch of pbsa_memory_update_static: device memory that belongs to the library, one copy per GPU, for callers
// that cannot allocate.  Host code never uses the array's name as an address; it asks the runtime once per
// device where that device's copy lives (static_scratch) and passes that pointer on.
static __device__ __align__(256) unsigned char scratch[PBSA_STATIC_WS_BYTES];

namespace {

constexpr int kMaxDevices = 64;
void* g_scratch_ptr[kMaxDevices] = {};      // per device: address of its copy of `scratch`, once resolved

// Address of the current device's copy of `scratch` (resolved on the first call on that device; no allocation).
hipError_t static_scratch(void** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  void* ptr = __atomic_load_n(&g_scratch_ptr[dev], __ATOMIC_ACQUIRE);
  if (!ptr) {
    e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!ptr) return hipErrorInvalidSymbol;
    __atomic_store_n(&g_scratch_ptr[dev], ptr, __ATOMIC_RELEASE);   // every thread resolves the same address
  }
  *out = ptr;
  return hipSuccess;
}

}  // namespace

extern "C" {
#pragma GCC visibility push(default)

int pbsa_version(void) { return 1; }

const char* pbsa_strerror(int code) {
  switch (code) {
    case PBSA_OK: return "ok";
    case PBSA_EINVAL: return "invalid argument (NULL pointer, wrong params.size, or inconsistent counts)";
    case PBSA_ESHAPE: return "unsupported shape (d and B must be 64 or 128; n_loc, C, k within PBSA_MAX_*; a block shape must divide its grid)";
    case PBSA_EALIGN: return "misaligned pointer (16 bytes) or stride (multiple of 8 elements)";
    case PBSA_EWS: return "workspace missing or too small (see pbsa_workspace_bytes), or the call needs more than PBSA_STATIC_WS_BYTES of built-in scratch";
    case PBSA_EHIP: return g_hip_msg[0] ? g_hip_msg : "HIP call failed";
    default: return "unknown pbsa error code";
  }
}

int pbsa_workspace_bytes(const pbsa_params* p, size_t* out) {
  if (!out) return PBSA_EINVAL;
  int rc = check_common(p);
  if (rc) return rc;
  *out = workspace_bytes(*p);
  return PBSA_OK;
}

int pbsa_pool_blocks(const pbsa_params* p, const void* X, const int32_t* len, int32_t n_blocks, float* out,
                     void* hip_stream) {
  if (!p || p->size != sizeof(pbsa_params)) return PBSA_EINVAL;
  if (p->d != 64 && p->d != 128) return PBSA_ESHAPE;
  if (p->B != 64 && p->B != 128) return PBSA_ESHAPE;
  if (n_blocks < 0) return PBSA_EINVAL;
  if (n_blocks > 0 && (!X || !len || !out)) return PBSA_EINVAL;
  if (!aligned16(X) || !aligned16(out)) return PBSA_EALIGN;
  hipError_t e = pbsa::launch_pool_blocks(*p, static_cast<const pbsa::bf16_t*>(X), len, n_blocks, out,
                                          static_cast<hipStream_t>(hip_stream));
  return e == hipSuccess ? PBSA_OK : hip_fail(e);
}

int pbsa_summary_view(const pbsa_params* p, const float* S_sum, const int32_t* S_cnt, void* Kp, void* Vp, int32_t* p_len,
                      void* hip_stream) {
  if (!p || p->size != sizeof(pbsa_params)) return PBSA_EINVAL;
  if (p->H < 1 || p->C < 0) return PBSA_EINVAL;
  if (p->d != 64 && p->d != 128) return PBSA_ESHAPE;
  if (p->B != 64 && p->B != 128) return PBSA_ESHAPE;
  if (p->H > 65535 || p->C > PBSA_MAX_C_ATTEND) return PBSA_ESHAPE;
  if (!S_sum || !S_cnt || !Kp || !Vp || !p_len) return PBSA_EINVAL;
  if (!aligned16(S_sum) || !aligned16(Kp) || !aligned16(Vp)) return PBSA_EALIGN;
  hipError_t e = pbsa::launch_summary_view(*p, S_sum, S_cnt, static_cast<pbsa::bf16_t*>(Kp),
                                           static_cast<pbsa::bf16_t*>(Vp), p_len, static_cast<hipStream_t>(hip_stream));
  return e == hipSuccess ? PBSA_OK : hip_fail(e);
}

int pbsa_select_blocks(const pbsa_params* p, const void* Q, const void* Kl, const int32_t* l_len,
                       const int32_t* l_map, float* Kc_l, float* Qc, int32_t* sel, float* Zl, void* ws,
                       size_t ws_bytes, void* hip_stream) {
  (void)ws; (void)ws_bytes;
  int rc = check_common(p, PBSA_MAX_C_ATTEND, PBSA_MAX_N_LOC, PBSA_MAX_K);
  if (rc) return rc;
  if (!Q || !Kl || !l_len || !l_map || !Kc_l || !Qc) return PBSA_EINVAL;
  if (p->k > 0 && !sel) return PBSA_EINVAL;
  rc = check_strides(p->q_stride_h, p->q_stride_t, p);
  if (rc) return rc;
  if (!aligned16(Q) || !aligned16(Kl) || !aligned16(Kc_l) || !aligned16(Qc)) return PBSA_EALIGN;
  hipError_t e = pbsa::launch_select(*p, static_cast<const pbsa::bf16_t*>(Q), static_cast<const pbsa::bf16_t*>(Kl),
                                     l_len, l_map, Kc_l, Qc, sel, Zl, static_cast<hipStream_t>(hip_stream));
  return e == hipSuccess ? PBSA_OK : hip_fail(e);
}

int pbsa_select_blocks_apply(const pbsa_params* p, const void* Q, const void* Kl, const int32_t* l_len,
                             const int32_t* l_map, float* Kc_l, float* Qc, int32_t* sel, float* Zl,
                             const pbsa_params* p_upd, void* Kp, void* Vp, int32_t* p_len, float* S_sum,
                             const int32_t* S_cnt, const void* Vl, void* ws, size_t ws_bytes, void* hip_stream) {
  int rc = check_common(p, PBSA_MAX_C_AUX);
  if (rc) return rc;
  rc = check_common(p_upd);
  if (rc) return rc;
  if (p->H != p_upd->H || p->d != p_upd->d || p->B != p_upd->B || p->C != p_upd->C || p->n_loc_cap != p_upd->n_loc_cap)
    return PBSA_EINVAL;
  if (!Q || !Kl || !l_len || !l_map || !Kc_l || !Qc) return PBSA_EINVAL;
  if (p->k > 0 && !sel) return PBSA_EINVAL;
  if (!Kp || !Vp || !p_len || !Vl) return PBSA_EINVAL;
  if ((S_sum == nullptr) != (S_cnt == nullptr)) return PBSA_EINVAL;
  rc = check_strides(p->q_stride_h, p->q_stride_t, p);
  if (rc) return rc;
  if (!aligned16(Q) || !aligned16(Kl) || !aligned16(Kc_l) || !aligned16(Qc) || !aligned16(Kp) || !aligned16(Vp) ||
      !aligned16(Vl) || !aligned16(S_sum))
    return PBSA_EALIGN;
  if (!ws || ws_bytes < workspace_bytes(*p_upd)) return PBSA_EWS;
  if (reinterpret_cast<uintptr_t>(ws) & 255u) return PBSA_EALIGN;
  const pbsa::UpdateWs w = pbsa::carve_update_ws(*p_upd, ws);
  hipError_t e = pbsa::launch_select_apply(
      *p, static_cast<const pbsa::bf16_t*>(Q), static_cast<const pbsa::bf16_t*>(Kl), l_len, l_map, Kc_l, Qc, sel, Zl,
      *p_upd, static_cast<pbsa::bf16_t*>(Kp), static_cast<pbsa::bf16_t*>(Vp), p_len, S_sum, S_cnt,
      static_cast<const pbsa::bf16_t*>(Vl), w, static_cast<hipStream_t>(hip_stream));
  return e == hipSuccess ? PBSA_OK : hip_fail(e);
}

int pbsa_attention_fwd(const pbsa_params* p, const void* Q, const void* Kp, const void* Vp, const int32_t* p_len,
                       const void* Kl, const void* Vl, const int32_t* l_len, const int32_t* l_map,
                       const int32_t* sel, void* O, float* lse, void* ws, size_t ws_bytes, void* hip_stream) {
  (void)ws; (void)ws_bytes;
  int rc = check_common(p, PBSA_MAX_C_ATTEND, PBSA_MAX_N_LOC, PBSA_MAX_K);
  if (rc) return rc;
  if (!Q || !Kp || !Vp || !p_len || !Kl || !Vl || !l_len || !l_map || !O) return PBSA_EINVAL;
  if (p->k > 0 && !sel) return PBSA_EINVAL;
  rc = check_strides(p->q_stride_h, p->q_stride_t, p);
  if (rc) return rc;
  rc = check_strides(p->o_stride_h, p->o_stride_t, p);
  if (rc) return rc;
  if (!aligned16(Q) || !aligned16(Kp) || !aligned16(Vp) || !aligned16(Kl) || !aligned16(Vl) || !aligned16(O))
    return PBSA_EALIGN;
  hipError_t e = pbsa::launch_attention(
      *p, static_cast<const pbsa::bf16_t*>(Q), static_cast<const pbsa::bf16_t*>(Kp),
      static_cast<const pbsa::bf16_t*>(Vp), p_len, static_cast<const pbsa::bf16_t*>(Kl),
      static_cast<const pbsa::bf16_t*>(Vl), l_len, l_map, sel, static_cast<pbsa::bf16_t*>(O), lse, nullptr,
      static_cast<hipStream_t>(hip_stream));
  return e == hipSuccess ? PBSA_OK : hip_fail(e);
}

int pbsa_mass_workspace_bytes(const pbsa_params* p, size_t* out) {
  if (!out) return PBSA_EINVAL;
  int rc = check_common(p, PBSA_MAX_C_AUX);
  if (rc) return rc;
  *out = pbsa::carve_mass_ws(*p, nullptr).bytes;
  return PBSA_OK;
}

int pbsa_attention_fwd_mass(const pbsa_params* p, const void* Q, const void* Kp, const void* Vp, const int32_t* p_len,
                            const void* Kl, const void* Vl, const int32_t* l_len, const int32_t* l_map,
                            const int32_t* sel, void* O, float* lse, float* Mt, void* ws, size_t ws_bytes,
                            void* hip_stream) {
  int rc = check_common(p, PBSA_MAX_C_AUX);
  if (rc) return rc;
  if (!Q || !Kp || !Vp || !p_len || !Kl || !Vl || !l_len || !l_map || !O || !lse || !Mt) return PBSA_EINVAL;
  if (p->k > 0 && !sel) return PBSA_EINVAL;
  rc = check_strides(p->q_stride_h, p->q_stride_t, p);
  if (rc) return rc;
  rc = check_strides(p->o_stride_h, p->o_stride_t, p);
  if (rc) return rc;
  if (!aligned16(Q) || !aligned16(Kp) || !aligned16(Vp) || !aligned16(Kl) || !aligned16(Vl) || !aligned16(O) ||
      !aligned16(Mt))
    return PBSA_EALIGN;
  if (!ws || ws_bytes < pbsa::carve_mass_ws(*p, nullptr).bytes) return PBSA_EWS;
  if (reinterpret_cast<uintptr_t>(ws) & 255u) return PBSA_EALIGN;
  const pbsa::MassRows rows = pbsa::carve_mass_ws(*p, ws);
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  hipError_t e = pbsa::launch_attention(
      *p, static_cast<const pbsa::bf16_t*>(Q), static_cast<const pbsa::bf16_t*>(Kp),
      static_cast<const pbsa::bf16_t*>(Vp), p_len, static_cast<const pbsa::bf16_t*>(Kl),
      static_cast<const pbsa::bf16_t*>(Vl), l_len, l_map, sel, static_cast<pbsa::bf16_t*>(O), lse, &rows, stream);
  if (e != hipSuccess) return hip_fail(e);
  e = pbsa::launch_mass_reduce(*p, rows, lse, Mt, stream);
  return e == hipSuccess ? PBSA_OK : hip_fail(e);
}

int pbsa_memory_update(const pbsa_params* p, const float* Qc, const float* Kc_l, const float* Zl, void* Kp,
                       void* Vp, float* Kc_p, int32_t* p_len, int64_t* p_id, float* S_sum, int32_t* S_cnt,
                       const void* Kl, const void* Vl, const int32_t* l_len, const int32_t* l_map,
                       const int64_t* l_id, float* scores, int32_t* slot_src, void* ws, size_t ws_bytes,
                       void* hip_stream) {
  int rc = check_common(p);
  if (rc) return rc;
  if (!Qc || !Kc_l || !Kp || !Vp || !p_len || !Kl || !Vl || !l_len || !l_map || !l_id) return PBSA_EINVAL;
  if (p->C > 0 && (!Kc_p || !p_id || !slot_src)) return PBSA_EINVAL;
  if ((S_sum == nullptr) != (S_cnt == nullptr)) return PBSA_EINVAL;
  if (!aligned16(Kp) || !aligned16(Vp) || !aligned16(Kl) || !aligned16(Vl) || !aligned16(Kc_l) ||
      !aligned16(Kc_p) || !aligned16(Qc) || !aligned16(S_sum))
    return PBSA_EALIGN;
  if (!ws || ws_bytes < workspace_bytes(*p)) return PBSA_EWS;
  if (reinterpret_cast<uintptr_t>(ws) & 255u) return PBSA_EALIGN;
  const pbsa::UpdateWs w = pbsa::carve_update_ws(*p, ws);
  hipError_t e = pbsa::launch_update(*p, Qc, Kc_l, Zl, static_cast<pbsa::bf16_t*>(Kp), static_cast<pbsa::bf16_t*>(Vp),
                                     Kc_p, p_len, p_id, S_sum, S_cnt, static_cast<const pbsa::bf16_t*>(Kl),
                                     static_cast<const pbsa::bf16_t*>(Vl), l_len, l_map, l_id, scores, slot_src, w,
                                     static_cast<hipStream_t>(hip_stream));
  return e == hipSuccess ? PBSA_OK : hip_fail(e);
}

int pbsa_memory_update_static(const pbsa_params* p, const float* Qc, const float* Kc_l, const float* Zl, void* Kp,
                              void* Vp, float* Kc_p, int32_t* p_len, int64_t* p_id, float* S_sum, int32_t* S_cnt,
                              const void* Kl, const void* Vl, const int32_t* l_len, const int32_t* l_map,
                              const int64_t* l_id, float* scores, int32_t* slot_src, void* hip_stream) {
  int rc = check_common(p);
  if (rc) return rc;
  if (!Qc || !Kc_l || !Kp || !Vp || !p_len || !Kl || !Vl || !l_len || !l_map || !l_id) return PBSA_EINVAL;
  if (p->C > 0 && (!Kc_p || !p_id || !slot_src)) return PBSA_EINVAL;
  if ((S_sum == nullptr) != (S_cnt == nullptr)) return PBSA_EINVAL;
  if (!aligned16(Kp) || !aligned16(Vp) || !aligned16(Kl) || !aligned16(Vl) || !aligned16(Kc_l) ||
      !aligned16(Kc_p) || !aligned16(Qc) || !aligned16(S_sum))
    return PBSA_EALIGN;
  if (workspace_bytes(*p) > (size_t)PBSA_STATIC_WS_BYTES) return PBSA_EWS;   // before any HIP call
  void* ws = nullptr;
  hipError_t e = static_scratch(&ws);
  if (e != hipSuccess) return hip_fail(e);
  const pbsa::UpdateWs w = pbsa::carve_update_ws(*p, ws);
  e = pbsa::launch_update(*p, Qc, Kc_l, Zl, static_cast<pbsa::bf16_t*>(Kp), static_cast<pbsa::bf16_t*>(Vp), Kc_p, p_len,
                          p_id, S_sum, S_cnt, static_cast<const pbsa::bf16_t*>(Kl), static_cast<const pbsa::bf16_t*>(Vl),
                          l_len, l_map, l_id, scores, slot_src, w, static_cast<hipStream_t>(hip_stream));
  return e == hipSuccess ? PBSA_OK : hip_fail(e);
}

int pbsa_memory_update_plan(const pbsa_params* p, const float* Qc, const float* Kc_l, const float* Zl, float* Kc_p,
                            const int32_t* p_len, int64_t* p_id, int32_t* S_cnt, const int32_t* l_len,
                            const int32_t* l_map, const int64_t* l_id, float* scores, int32_t* slot_src, void* ws,
                            size_t ws_bytes, void* hip_stream) {
  int rc = check_common(p);
  if (rc) return rc;
  if (!Qc || !Kc_l || !p_len || !l_len || !l_map || !l_id) return PBSA_EINVAL;
  if (p->C > 0 && (!Kc_p || !p_id || !slot_src)) return PBSA_EINVAL;
  if (!aligned16(Kc_l) || !aligned16(Kc_p) || !aligned16(Qc)) return PBSA_EALIGN;
  if (!ws || ws_bytes < workspace_bytes(*p)) return PBSA_EWS;
  if (reinterpret_cast<uintptr_t>(ws) & 255u) return PBSA_EALIGN;
  const pbsa::UpdateWs w = pbsa::carve_update_ws(*p, ws);
  hipError_t e = pbsa::launch_update_plan(*p, Qc, Kc_l, Zl, Kc_p, p_len, p_id, S_cnt, S_cnt != nullptr, l_len, l_map, l_id,
                                          scores, slot_src, w, static_cast<hipStream_t>(hip_stream));
  return e == hipSuccess ? PBSA_OK : hip_fail(e);
}

int pbsa_attention_fwd_plan(const pbsa_params* p, const void* Q, const void* Kp, const void* Vp, const int32_t* p_len,
                            const void* Kl, const void* Vl, const int32_t* l_len, const int32_t* l_map,
                            const int32_t* sel, void* O, float* lse, const float* Qc, const float* Kc_l,
                            const float* Zl, float* Kc_p, int64_t* p_id, int32_t* S_cnt, const int64_t* l_id,
                            float* scores, int32_t* slot_src, void* ws, size_t ws_bytes, void* hip_stream) {
  int rc = check_common(p);
  if (rc) return rc;
  if (!Q || !Kp || !Vp || !p_len || !Kl || !Vl || !l_len || !l_map || !O) return PBSA_EINVAL;
  if (p->k > 0 && !sel) return PBSA_EINVAL;
  if (!Qc || !Kc_l || !Zl || !l_id) return PBSA_EINVAL;
  if (p->C > 0 && (!Kc_p || !p_id || !slot_src)) return PBSA_EINVAL;
  rc = check_strides(p->q_stride_h, p->q_stride_t, p);
  if (rc) return rc;
  rc = check_strides(p->o_stride_h, p->o_stride_t, p);
  if (rc) return rc;
  if (!aligned16(Q) || !aligned16(Kp) || !aligned16(Vp) || !aligned16(Kl) || !aligned16(Vl) || !aligned16(O) ||
      !aligned16(Kc_l) || !aligned16(Kc_p) || !aligned16(Qc))
    return PBSA_EALIGN;
  if (!ws || ws_bytes < workspace_bytes(*p)) return PBSA_EWS;
  if (reinterpret_cast<uintptr_t>(ws) & 255u) return PBSA_EALIGN;
  const pbsa::UpdateWs w = pbsa::carve_update_ws(*p, ws);
  hipError_t e = pbsa::launch_attention_plan(
      *p, static_cast<const pbsa::bf16_t*>(Q), static_cast<const pbsa::bf16_t*>(Kp),
      static_cast<const pbsa::bf16_t*>(Vp), p_len, static_cast<const pbsa::bf16_t*>(Kl),
      static_cast<const pbsa::bf16_t*>(Vl), l_len, l_map, sel, static_cast<pbsa::bf16_t*>(O), lse, Qc, Kc_l, Zl, Kc_p,
      p_id, S_cnt, S_cnt != nullptr, l_id, scores, slot_src, w, static_cast<hipStream_t>(hip_stream));
  return e == hipSuccess ? PBSA_OK : hip_fail(e);
}

int pbsa_memory_update_apply(const pbsa_params* p, void* Kp, void* Vp, int32_t* p_len, float* S_sum, const int32_t* S_cnt,
                             const void* Kl, const void* Vl, void* ws, size_t ws_bytes, void* hip_stream) {
  int rc = check_common(p);
  if (rc) return rc;
  if (!Kp || !Vp || !p_len || !Kl || !Vl) return PBSA_EINVAL;
  if ((S_sum == nullptr) != (S_cnt == nullptr)) return PBSA_EINVAL;
  if (!aligned16(Kp) || !aligned16(Vp) || !aligned16(Kl) || !aligned16(Vl) || !aligned16(S_sum)) return PBSA_EALIGN;
  if (!ws || ws_bytes < workspace_bytes(*p)) return PBSA_EWS;
  if (reinterpret_cast<uintptr_t>(ws) & 255u) return PBSA_EALIGN;
  const pbsa::UpdateWs w = pbsa::carve_update_ws(*p, ws);
  hipError_t e = pbsa::launch_update_apply(*p, static_cast<pbsa::bf16_t*>(Kp), static_cast<pbsa::bf16_t*>(Vp), p_len, S_sum,
                                           S_cnt, static_cast<const pbsa::bf16_t*>(Kl), static_cast<const pbsa::bf16_t*>(Vl),
                                           w, static_cast<hipStream_t>(hip_stream));
  return e == hipSuccess ? PBSA_OK : hip_fail(e);
}

int pbsa_attention_mass(const pbsa_params* p, const void* Q, const void* Kp, const int32_t* p_len, const void* Kl,
                        const int32_t* l_len, const int32_t* l_map, const int32_t* sel, const float* lse, float* Mt,
                        void* hip_stream) {
  int rc = check_common(p, PBSA_MAX_C_AUX);
  if (rc) return rc;
  if (!Q || !Kp || !p_len || !Kl || !l_len || !l_map || !lse || !Mt) return PBSA_EINVAL;
  if (p->k > 0 && !sel) return PBSA_EINVAL;
  rc = check_strides(p->q_stride_h, p->q_stride_t, p);
  if (rc) return rc;
  if (!aligned16(Q) || !aligned16(Kp) || !aligned16(Kl) || !aligned16(Mt)) return PBSA_EALIGN;
  hipError_t e = pbsa::launch_attention_mass(*p, static_cast<const pbsa::bf16_t*>(Q), static_cast<const pbsa::bf16_t*>(Kp),
                                             p_len, static_cast<const pbsa::bf16_t*>(Kl), l_len, l_map, sel, lse, Mt,
                                             static_cast<hipStream_t>(hip_stream));
  return e == hipSuccess ? PBSA_OK : hip_fail(e);
}

int pbsa_memory_update_fine(const pbsa_params* p, const float* Mt, const float* Kc_l, void* Kp, void* Vp, float* Kc_p,
                            int32_t* p_len, int64_t* p_id, float* S_sum, int32_t* S_cnt, const void* Kl,
                            const void* Vl, const int32_t* l_len, const int32_t* l_map, const int64_t* l_id,
                            float* scores, int32_t* slot_src, void* ws, size_t ws_bytes, void* hip_stream) {
  int rc = check_common(p);
  if (rc) return rc;
  if (!Mt || !Kc_l || !Kp || !Vp || !p_len || !Kl || !Vl || !l_len || !l_map || !l_id) return PBSA_EINVAL;
  if (p->C > 0 && (!Kc_p || !p_id || !slot_src)) return PBSA_EINVAL;
  if ((S_sum == nullptr) != (S_cnt == nullptr)) return PBSA_EINVAL;
  if (!aligned16(Kp) || !aligned16(Vp) || !aligned16(Kl) || !aligned16(Vl) || !aligned16(Kc_l) ||
      !aligned16(Kc_p) || !aligned16(Mt) || !aligned16(S_sum))
    return PBSA_EALIGN;
  if (!ws || ws_bytes < workspace_bytes(*p)) return PBSA_EWS;
  if (reinterpret_cast<uintptr_t>(ws) & 255u) return PBSA_EALIGN;
  const pbsa::UpdateWs w = pbsa::carve_update_ws(*p, ws);
  hipError_t e = pbsa::launch_update_fine(*p, Mt, Kc_l, static_cast<pbsa::bf16_t*>(Kp), static_cast<pbsa::bf16_t*>(Vp),
                                          Kc_p, p_len, p_id, S_sum, S_cnt, static_cast<const pbsa::bf16_t*>(Kl),
                                          static_cast<const pbsa::bf16_t*>(Vl), l_len, l_map, l_id, scores, slot_src, w,
                                          static_cast<hipStream_t>(hip_stream));
  return e == hipSuccess ? PBSA_OK : hip_fail(e);
}

int pbsa_bwd_workspace_bytes(const pbsa_params* p, size_t* out) {
  if (!out) return PBSA_EINVAL;
  int rc = check_common(p, PBSA_MAX_C_AUX);
  if (rc) return rc;
  *out = pbsa::bwd_workspace_bytes(*p);
  return PBSA_OK;
}

int pbsa_attention_bwd(const pbsa_params* p, const void* Q, const void* Kp, const void* Vp, const int32_t* p_len,
                       const void* Kl, const void* Vl, const int32_t* l_len, const int32_t* l_map, const int32_t* sel,
                       const void* O, const void* dO, const float* lse, float* dQ, float* dKp, float* dVp, float* dKl,
                       float* dVl, void* ws, size_t ws_bytes, void* hip_stream) {
  int rc = check_common(p, PBSA_MAX_C_AUX);
  if (rc) return rc;
  if (!Q || !Kp || !Vp || !p_len || !Kl || !Vl || !l_len || !l_map || !O || !dO || !lse || !dQ || !dKp || !dVp ||
      !dKl || !dVl)
    return PBSA_EINVAL;
  if (p->k > 0 && !sel) return PBSA_EINVAL;
  rc = check_strides(p->q_stride_h, p->q_stride_t, p);
  if (rc) return rc;
  rc = check_strides(p->o_stride_h, p->o_stride_t, p);
  if (rc) return rc;
  // a tile's lane offsets are 32-bit: 64 rows of the widest stride must fit
  if (p->q_stride_t >= ((int64_t)1 << 24) || p->o_stride_t >= ((int64_t)1 << 24)) return PBSA_ESHAPE;
  if (!aligned16(Q) || !aligned16(Kp) || !aligned16(Vp) || !aligned16(Kl) || !aligned16(Vl) || !aligned16(O) ||
      !aligned16(dO) || !aligned16(dQ) || !aligned16(dKp) || !aligned16(dVp) || !aligned16(dKl) || !aligned16(dVl))
    return PBSA_EALIGN;
  if (!ws || ws_bytes < pbsa::bwd_workspace_bytes(*p)) return PBSA_EWS;
  if (reinterpret_cast<uintptr_t>(ws) & 255u) return PBSA_EALIGN;
  hipError_t e = pbsa::launch_attention_bwd(
      *p, static_cast<const pbsa::bf16_t*>(Q), static_cast<const pbsa::bf16_t*>(Kp),
      static_cast<const pbsa::bf16_t*>(Vp), p_len, static_cast<const pbsa::bf16_t*>(Kl),
      static_cast<const pbsa::bf16_t*>(Vl), l_len, l_map, sel, static_cast<const pbsa::bf16_t*>(O),
      static_cast<const pbsa::bf16_t*>(dO), lse, dQ, dKp, dVp, dKl, dVl, static_cast<float*>(ws),
      static_cast<hipStream_t>(hip_stream));
  return e == hipSuccess ? PBSA_OK : hip_fail(e);
}

namespace {
int check_grid(const pbsa_grid* g) {
  if (!g || g->size != sizeof(pbsa_grid)) return PBSA_EINVAL;
  if (g->T < 1 || g->Hs < 1 || g->Ws < 1 || g->Bt < 1 || g->Bh < 1 || g->Bw < 1 || g->H < 1 || g->d < 8 || g->B < 1)
    return PBSA_EINVAL;
  if (g->d % 8 != 0) return PBSA_ESHAPE;
  if (g->T % g->Bt != 0 || g->Hs % g->Bh != 0 || g->Ws % g->Bw != 0) return PBSA_ESHAPE;
  if ((int64_t)g->Bt * g->Bh * g->Bw > g->B) return PBSA_ESHAPE;
  if ((int64_t)g->T * g->Hs * g->Ws * g->H * g->d >= ((int64_t)1 << 40)) return PBSA_ESHAPE;
  if ((int64_t)g->H * 4 > 65535) return PBSA_ESHAPE;
  return PBSA_OK;
}
}  // namespace

int pbsa_blockify(const pbsa_grid* g, int32_t n, const void* const* X, void* const* Xblk, const int64_t* blk_stride_h,
                  void* hip_stream) {
  int rc = check_grid(g);
  if (rc) return rc;
  if (n < 1 || n > 4 || !X || !Xblk || !blk_stride_h) return PBSA_EINVAL;
  pbsa::LayoutTensors t{};
  t.n = n;
  for (int i = 0; i < n; ++i) {
    if (!X[i] || !Xblk[i] || blk_stride_h[i] < 0) return PBSA_EINVAL;
    if (!aligned16(X[i]) || !aligned16(Xblk[i]) || blk_stride_h[i] % 8 != 0) return PBSA_EALIGN;
    t.tok[i] = static_cast<const pbsa::bf16_t*>(X[i]);
    t.blk[i] = static_cast<pbsa::bf16_t*>(Xblk[i]);
    t.blk_stride_h[i] = blk_stride_h[i];
  }
  hipError_t e = pbsa::launch_blockify(*g, t, true, static_cast<hipStream_t>(hip_stream));
  return e == hipSuccess ? PBSA_OK : hip_fail(e);
}

int pbsa_unblockify(const pbsa_grid* g, const void* Xblk, int64_t blk_stride_h, void* X, void* hip_stream) {
  int rc = check_grid(g);
  if (rc) return rc;
  if (!X || !Xblk || blk_stride_h < 0) return PBSA_EINVAL;
  if (!aligned16(X) || !aligned16(Xblk) || blk_stride_h % 8 != 0) return PBSA_EALIGN;
  pbsa::LayoutTensors t{};
  t.n = 1;
  t.tok[0] = static_cast<const pbsa::bf16_t*>(X);
  t.blk[0] = static_cast<pbsa::bf16_t*>(const_cast<void*>(Xblk));
  t.blk_stride_h[0] = blk_stride_h;
  hipError_t e = pbsa::launch_blockify(*g, t, false, static_cast<hipStream_t>(hip_stream));
  return e == hipSuccess ? PBSA_OK : hip_fail(e);
}

#pragma GCC visibility pop
}  // extern "C"
