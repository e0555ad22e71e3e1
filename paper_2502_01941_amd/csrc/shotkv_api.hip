// C ABI of the ShotKV library: argument checks, workspace carving and kernel sequencing.
// Every entry point only enqueues work on the caller's stream.
#include "common.hpp"

#include <atomic>

// Scratch memory of shotkv_decode_step_static: one copy per GPU the library runs on, held until the
// process ends.  In host code this name is only a handle for hipGetSymbolAddress, never an address.
static __device__ __align__(256) unsigned char scratch[SHOTKV_STATIC_SCRATCH_BYTES];

namespace shotkv {

namespace {
constexpr int kMaxDevices = 64;
std::atomic<void*> g_scratch_ptr[kMaxDevices];  // device address of `scratch` on each GPU, once known

// Device address of the scratch array on the current GPU; looked up once per device.
int static_scratch(void** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return SHOTKV_E_LAUNCH;
  void* ptr = g_scratch_ptr[dev].load(std::memory_order_acquire);
  if (!ptr) {
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return SHOTKV_E_LAUNCH;
    g_scratch_ptr[dev].store(ptr, std::memory_order_release);  // a racing thread stores the same value
  }
  *out = ptr;
  return SHOTKV_OK;
}
}  // namespace

hipError_t launch_score_partials_generic(const PrefillDims& d, const void* q_obs, const void* k,
                                         const PrefillWorkspace& w, hipStream_t s);
hipError_t launch_score_partials_mfma(const PrefillDims& d, const void* q_obs, const void* k,
                                      const PrefillWorkspace& w, hipStream_t s);

hipError_t launch_score_partials(const PrefillDims& d, const void* q_obs, const void* k,
                                 const PrefillWorkspace& w, hipStream_t s) {
  return score_uses_mfma(d) ? launch_score_partials_mfma(d, q_obs, k, w, s)
                            : launch_score_partials_generic(d, q_obs, k, w, s);
}

namespace {

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

int check_config(const shotkv_config* cfg) {
  if (!cfg) return SHOTKV_E_NULL;
  if (cfg->dtype != SHOTKV_BF16 && cfg->dtype != SHOTKV_F32) return SHOTKV_E_SHAPE;
  if (cfg->head_dim != 64 && cfg->head_dim != 128) return SHOTKV_E_SHAPE;
  if (cfg->n_kv_heads < 1 || cfg->n_q_heads < 1 || cfg->n_q_heads % cfg->n_kv_heads) return SHOTKV_E_SHAPE;
  const int G = cfg->n_q_heads / cfg->n_kv_heads;
  if (G > 8) return SHOTKV_E_SHAPE;
  if (cfg->n_q_heads > 64) return SHOTKV_E_SHAPE;
  if (cfg->select_mode != SHOTKV_SELECT_PREFIX && cfg->select_mode != SHOTKV_SELECT_FIRST_FIT)
    return SHOTKV_E_SHAPE;
  if (cfg->head_mode != SHOTKV_HEADS_PER_LAYER && cfg->head_mode != SHOTKV_HEADS_PER_KV_HEAD)
    return SHOTKV_E_SHAPE;
  if (!(cfg->sm_scale > 0.f)) return SHOTKV_E_SHAPE;
  return SHOTKV_OK;
}

int make_prefill_dims(const shotkv_config* cfg, int P, int n_tokens, int n_shots, PrefillDims* d) {
  const int rc = check_config(cfg);
  if (rc != SHOTKV_OK) return rc;
  if (cfg->window < 1 || cfg->window > 64) return SHOTKV_E_SHAPE;
  const int G = cfg->n_q_heads / cfg->n_kv_heads;
  if (G * cfg->window > 256) return SHOTKV_E_SHAPE;
  if (P < 1 || n_tokens < cfg->window || n_shots < 0 || n_shots > SHOTKV_MAX_SHOTS) return SHOTKV_E_SHAPE;
  d->P = P; d->n_tokens = n_tokens; d->n_shots = n_shots;
  d->H = cfg->n_q_heads; d->H_kv = cfg->n_kv_heads; d->G = G; d->D = cfg->head_dim;
  d->W = cfg->window; d->R_rows = G * cfg->window; d->R = d->R_rows; d->dtype = cfg->dtype;
  d->sm_scale = cfg->sm_scale;
  if (score_uses_mfma(*d)) {  // the matrix-core kernel works on 1, 2, 4, 6 or 8 blocks of 32 query rows
    const int need = ceil_div(d->R_rows, 32);
    const int blocks = need <= 2 ? need : need <= 4 ? 4 : need <= 6 ? 6 : 8;
    d->R = blocks * 32;
  }
  d->select_mode = cfg->select_mode;
  d->timing = cfg->timing_events;
  d->share = 1;
  if (cfg->head_mode == SHOTKV_HEADS_PER_KV_HEAD) {
    // A KV head with its G query heads is a problem of its own: [P][H_kv][...] tensors are
    // [P * H_kv][1][...] tensors, and only the shot boundaries and the budget are shared by the
    // H_kv consecutive problems that came from one (batch, layer) pair.
    d->share = d->H_kv;
    d->P = P * d->H_kv;
    d->H = G;
    d->H_kv = 1;
  }
  if (d->P > 32767) return SHOTKV_E_SHAPE;
  return SHOTKV_OK;
}

PrefillWorkspace carve(const PrefillDims& d, void* base) {
  return carve_prefill(base, d.P, d.H_kv, d.R, d.n_tokens, d.n_shots, score_uses_mfma(d));
}

int from_hip(hipError_t e) { return e == hipSuccess ? SHOTKV_OK : SHOTKV_E_LAUNCH; }

}  // namespace
}  // namespace shotkv

using namespace shotkv;

extern "C" {

const char* shotkv_strerror(int code) {
  switch (code) {
    case SHOTKV_OK: return "ok";
    case SHOTKV_E_NULL: return "required pointer is NULL";
    case SHOTKV_E_SHAPE: return "unsupported or inconsistent shape, dtype or mode";
    case SHOTKV_E_WORKSPACE: return "workspace too small";
    case SHOTKV_E_ALIGN: return "tensor pointer not 16-byte aligned";
    case SHOTKV_E_LAUNCH: return "HIP launch failed";
    case SHOTKV_E_SCRATCH: return "problem needs more scratch than the static buffer holds";
    default: return "unknown shotkv error";
  }
}

int32_t shotkv_abi_version(void) { return 3; }

size_t shotkv_prefill_workspace_bytes(const shotkv_config* cfg, int32_t P, int32_t n_tokens,
                                      int32_t n_shots) {
  PrefillDims d;
  if (make_prefill_dims(cfg, P, n_tokens, n_shots, &d) != SHOTKV_OK) return 0;
  return carve(d, nullptr).bytes;
}

int shotkv_prefill_scores(const shotkv_config* cfg, int32_t P, int32_t n_tokens, int32_t n_shots,
                          const void* q_obs, const void* k, const int32_t* shot_offsets,
                          float* shot_scores, int32_t* status, void* workspace,
                          size_t workspace_bytes, void* stream) {
  PrefillDims d;
  const int rc = make_prefill_dims(cfg, P, n_tokens, n_shots, &d);
  if (rc != SHOTKV_OK) return rc;
  if (!q_obs || !k || !shot_offsets || !shot_scores || !status || !workspace) return SHOTKV_E_NULL;
  if (!aligned16(q_obs) || !aligned16(k) || !aligned16(workspace)) return SHOTKV_E_ALIGN;
  const PrefillWorkspace w = carve(d, workspace);
  if (workspace_bytes < w.bytes) return SHOTKV_E_WORKSPACE;
  hipStream_t s = static_cast<hipStream_t>(stream);
  hipError_t e = launch_plan_chunks(d, shot_offsets, status, w, s);
  if (e == hipSuccess) e = launch_score_partials(d, q_obs, k, w, s);
  if (e == hipSuccess) e = launch_row_stats(d, w, s);
  if (e == hipSuccess) e = launch_chunk_mass(d, w, s);
  if (e == hipSuccess)
    e = launch_reduce_select(d, true, false, shot_scores, shot_offsets, nullptr, 0, nullptr, nullptr, status,
                             nullptr, w, s);
  return from_hip(e);
}

int shotkv_select_and_compact(const shotkv_config* cfg, int32_t P, int32_t n_tokens, int32_t n_shots,
                              const float* shot_scores, const void* k, const void* v,
                              const int32_t* shot_offsets, const int32_t* budget_tokens, void* k_out,
                              void* v_out, int32_t cap, int32_t* kept_positions, int32_t* kept_count,
                              uint8_t* shot_selected, int32_t* status, void* workspace,
                              size_t workspace_bytes, void* stream) {
  PrefillDims d;
  const int rc = make_prefill_dims(cfg, P, n_tokens, n_shots, &d);
  if (rc != SHOTKV_OK) return rc;
  if (cap < 1) return SHOTKV_E_SHAPE;
  if (!k || !v || !shot_offsets || !budget_tokens || !k_out || !v_out || !kept_positions ||
      !kept_count || !status || !workspace || (n_shots > 0 && !shot_scores))
    return SHOTKV_E_NULL;
  if (!aligned16(k) || !aligned16(v) || !aligned16(k_out) || !aligned16(v_out) || !aligned16(workspace))
    return SHOTKV_E_ALIGN;
  const PrefillWorkspace w = carve(d, workspace);
  if (workspace_bytes < w.bytes) return SHOTKV_E_WORKSPACE;
  hipStream_t s = static_cast<hipStream_t>(stream);
  hipError_t e = launch_reduce_select(d, false, true, const_cast<float*>(shot_scores), shot_offsets,
                                      budget_tokens, cap, kept_count, shot_selected, status, kept_positions,
                                      w, s);
  if (e == hipSuccess) e = launch_compact(d, k, v, k_out, v_out, cap, kept_positions, kept_count, s);
  return from_hip(e);
}

int shotkv_prefill_compress(const shotkv_config* cfg, int32_t P, int32_t n_tokens, int32_t n_shots,
                            const void* q_obs, const void* k, const void* v,
                            const int32_t* shot_offsets, const int32_t* budget_tokens, void* k_out,
                            void* v_out, int32_t cap, int32_t* kept_positions, int32_t* kept_count,
                            float* shot_scores, uint8_t* shot_selected, int32_t* status,
                            void* workspace, size_t workspace_bytes, void* stream) {
  PrefillDims d;
  const int rc = make_prefill_dims(cfg, P, n_tokens, n_shots, &d);
  if (rc != SHOTKV_OK) return rc;
  if (cap < 1) return SHOTKV_E_SHAPE;
  if (!q_obs || !k || !v || !shot_offsets || !budget_tokens || !k_out || !v_out || !kept_positions ||
      !kept_count || !status || !workspace)
    return SHOTKV_E_NULL;
  if (!aligned16(q_obs) || !aligned16(k) || !aligned16(v) || !aligned16(k_out) || !aligned16(v_out) ||
      !aligned16(workspace))
    return SHOTKV_E_ALIGN;
  const PrefillWorkspace w = carve(d, workspace);
  if (workspace_bytes < w.bytes) return SHOTKV_E_WORKSPACE;
  float* scores = shot_scores ? shot_scores : w.scores;
  hipStream_t s = static_cast<hipStream_t>(stream);
  hipError_t e = launch_plan_chunks(d, shot_offsets, status, w, s);
  if (e == hipSuccess) e = launch_score_partials(d, q_obs, k, w, s);
  if (e == hipSuccess) e = launch_row_stats(d, w, s);
  if (e == hipSuccess) e = launch_chunk_mass(d, w, s);
  if (e == hipSuccess)
    e = launch_reduce_select(d, true, true, scores, shot_offsets, budget_tokens, cap, kept_count,
                             shot_selected, status, kept_positions, w, s);
  if (e == hipSuccess) e = launch_compact(d, k, v, k_out, v_out, cap, kept_positions, kept_count, s);
  return from_hip(e);
}

// dims and workspace of the fused attention entry point: the row stride is exactly G * W (no matrix-core
// row padding: the attention kernel writes every row that exists), chunks as on the matrix-core path
static int make_attention_dims(const shotkv_config* cfg, int P, int n_tokens, int n_shots, PrefillDims* d) {
  const int rc = make_prefill_dims(cfg, P, n_tokens, n_shots, d);
  if (rc != SHOTKV_OK) return rc;
  if (!attention_supported(*d)) return SHOTKV_E_SHAPE;
  d->R = d->R_rows;
  return SHOTKV_OK;
}

static PrefillWorkspace carve_attention(const PrefillDims& d, void* base) {
  const size_t vt_bytes = static_cast<size_t>(d.P) * d.H_kv * attention_key_blocks(d.n_tokens) * 32 * d.D * 2;
  return carve_prefill(base, d.P, d.H_kv, d.R, d.n_tokens, d.n_shots, true, vt_bytes);
}

size_t shotkv_prefill_attention_workspace_bytes(const shotkv_config* cfg, int32_t P, int32_t n_tokens,
                                                int32_t n_shots) {
  PrefillDims d;
  if (make_attention_dims(cfg, P, n_tokens, n_shots, &d) != SHOTKV_OK) return 0;
  return carve_attention(d, nullptr).bytes;
}

int shotkv_prefill_attention_compress(const shotkv_config* cfg, int32_t P, int32_t n_tokens, int32_t n_shots,
                                      const void* q, const void* k, const void* v,
                                      const int32_t* shot_offsets, const int32_t* budget_tokens,
                                      float* attn_out, void* k_out, void* v_out, int32_t cap,
                                      int32_t* kept_positions, int32_t* kept_count, float* shot_scores,
                                      uint8_t* shot_selected, int32_t* status, void* workspace,
                                      size_t workspace_bytes, void* stream) {
  PrefillDims d;
  const int rc = make_attention_dims(cfg, P, n_tokens, n_shots, &d);
  if (rc != SHOTKV_OK) return rc;
  if (cap < 1) return SHOTKV_E_SHAPE;
  if (!q || !k || !v || !shot_offsets || !budget_tokens || !attn_out || !k_out || !v_out || !kept_positions ||
      !kept_count || !status || !workspace)
    return SHOTKV_E_NULL;
  if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(attn_out) || !aligned16(k_out) ||
      !aligned16(v_out) || !aligned16(workspace))
    return SHOTKV_E_ALIGN;
  const PrefillWorkspace w = carve_attention(d, workspace);
  if (workspace_bytes < w.bytes) return SHOTKV_E_WORKSPACE;
  float* scores = shot_scores ? shot_scores : w.scores;
  hipStream_t s = static_cast<hipStream_t>(stream);
  hipError_t e = launch_plan_chunks(d, shot_offsets, status, w, s);
  if (e == hipSuccess) e = launch_pack_vt(d, v, w, s);
  if (e == hipSuccess) e = launch_attention_scores(d, q, k, w.vt, attn_out, w, s);
  if (e == hipSuccess) e = launch_chunk_mass(d, w, s);
  if (e == hipSuccess)
    e = launch_reduce_select(d, true, true, scores, shot_offsets, budget_tokens, cap, kept_count,
                             shot_selected, status, kept_positions, w, s);
  if (e == hipSuccess) e = launch_compact(d, k, v, k_out, v_out, cap, kept_positions, kept_count, s);
  return from_hip(e);
}

static int make_decode_dims(const shotkv_config* cfg, int S, int cap, int n_slots, DecodeDims* d) {
  const int rc = check_config(cfg);
  if (rc != SHOTKV_OK) return rc;
  if (S < 1 || cap < 0 || n_slots < 1) return SHOTKV_E_SHAPE;
  d->S = S; d->H = cfg->n_q_heads; d->H_kv = cfg->n_kv_heads; d->G = d->H / d->H_kv;
  if (cfg->head_mode == SHOTKV_HEADS_PER_KV_HEAD) {
    // every (sequence, KV head) pair is a sequence of its own with G query heads and one KV head
    d->S = S * d->H_kv;
    d->H = d->G;
    d->H_kv = 1;
  }
  if (d->S > 65535) return SHOTKV_E_SHAPE;
  d->D = cfg->head_dim; d->dtype = cfg->dtype; d->cap = cap; d->n_slots = n_slots;
  d->sm_scale = cfg->sm_scale;
  d->timing = cfg->timing_events;
  const int total = cap + n_slots;
  d->n_splits = decode_splits(d->S, d->H_kv, total);  // pairs after the per-KV-head rewrite
  d->split_tokens = ceil_div(total, d->n_splits);
  return SHOTKV_OK;
}

size_t shotkv_decode_workspace_bytes(const shotkv_config* cfg, int32_t S, int32_t cap, int32_t n_slots) {
  DecodeDims d;
  if (make_decode_dims(cfg, S, cap, n_slots, &d) != SHOTKV_OK) return 0;
  return carve_decode(nullptr, d.S, d.H, d.H_kv, d.D, d.n_slots, d.n_splits).bytes;
}

int shotkv_decode_step(const shotkv_config* cfg, int32_t S, const shotkv_decode_state* st,
                       int32_t step_index, const void* q_new, const void* k_new, const void* v_new,
                       float* out, float* token_scores, int32_t* evicted_pos, int32_t* status,
                       void* workspace, size_t workspace_bytes, void* stream) {
  if (!st) return SHOTKV_E_NULL;
  DecodeDims d;
  const int rc = make_decode_dims(cfg, S, st->cap, st->n_slots, &d);
  if (rc != SHOTKV_OK) return rc;
  if (st->decode_budget < 1 || step_index < 0) return SHOTKV_E_SHAPE;
  if (!st->prefill_count || !st->k_dec || !st->v_dec || !st->slot_pos || !q_new || !k_new || !v_new ||
      !out || !status || !workspace || (st->cap > 0 && (!st->k_prefill || !st->v_prefill)))
    return SHOTKV_E_NULL;
  if (!aligned16(st->k_prefill) || !aligned16(st->v_prefill) || !aligned16(st->k_dec) ||
      !aligned16(st->v_dec) || !aligned16(q_new) || !aligned16(k_new) || !aligned16(v_new) ||
      !aligned16(workspace))
    return SHOTKV_E_ALIGN;
  const DecodeWorkspace w = carve_decode(workspace, d.S, d.H, d.H_kv, d.D, d.n_slots, d.n_splits);
  if (workspace_bytes < w.bytes) return SHOTKV_E_WORKSPACE;
  d.budget = st->decode_budget;
  d.step = step_index;
  hipStream_t s = static_cast<hipStream_t>(stream);
  hipError_t e = launch_decode_partial(d, *st, q_new, k_new, v_new, w, s);
  if (e == hipSuccess) e = launch_decode_finish(d, *st, out, token_scores, evicted_pos, status, w, s);
  return from_hip(e);
}

int shotkv_decode_step_static(const shotkv_config* cfg, int32_t S, const shotkv_decode_state* st,
                              int32_t step_index, const void* q_new, const void* k_new, const void* v_new,
                              float* out, float* token_scores, int32_t* evicted_pos, int32_t* status,
                              void* stream) {
  if (!st) return SHOTKV_E_NULL;
  DecodeDims d;
  const int rc = make_decode_dims(cfg, S, st->cap, st->n_slots, &d);
  if (rc != SHOTKV_OK) return rc;
  const size_t need = carve_decode(nullptr, d.S, d.H, d.H_kv, d.D, d.n_slots, d.n_splits).bytes;
  if (need > static_cast<size_t>(SHOTKV_STATIC_SCRATCH_BYTES)) return SHOTKV_E_SCRATCH;
  void* ptr = nullptr;
  const int rs = static_scratch(&ptr);
  if (rs != SHOTKV_OK) return rs;
  // nothing in the decode workspace has to start at zero: every word a step reads it has written itself
  return shotkv_decode_step(cfg, S, st, step_index, q_new, k_new, v_new, out, token_scores, evicted_pos,
                            status, ptr, need, stream);
}

}  // extern "C"
