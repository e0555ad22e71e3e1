/*
 * shotkv.h - C ABI of the MI355X (gfx950) ShotKV KV-cache compression library.
 *
 * ShotKV (arXiv 2502.01941, Section 5 "ShotKV", Eq. 2-9, Algorithm 1) compresses a transformer's KV
 * cache in two phases.  Prefill: every few-shot example ("shot") of the prompt is scored by the
 * attention mass its tokens receive, whole shots are kept in descending score order under a token
 * budget, and the kept K/V rows are compacted into a dense cache that then stays fixed.  Decoding:
 * generated tokens are retained at token level by the attention the current query gives them, and
 * attention runs over the union of the two caches.
 *
 * Conventions for every entry point
 *   - All data pointers are DEVICE pointers owned by the caller.  The library never allocates, frees
 *     or synchronises; it enqueues kernels on `stream` (a hipStream_t passed as void*, NULL = the
 *     default stream) and returns.  Inputs are never written.
 *   - Return value: SHOTKV_OK or a negative SHOTKV_E_* for errors the host can see (null pointer,
 *     unsupported shape, workspace too small, misaligned pointer).  Nothing is enqueued on error.
 *   - Data-dependent errors are reported per problem in a device-side `status` word (SHOTKV_ST_*);
 *     a failed problem keeps nothing (kept_count = 0).
 *   - Tensors are dense, row-major, innermost dimension head_dim; every tensor pointer must be
 *     16-byte aligned.  "dtype" below is cfg->dtype: bf16 (2 bytes) or fp32 (4 bytes).
 *   - Supported shapes: head_dim 64 or 128; n_q_heads = G * n_kv_heads with 1 <= G <= 8, n_q_heads <= 64;
 *     1 <= window <= 64 and G * window <= 256; n_shots <= SHOTKV_MAX_SHOTS.
 *   - Two calls that share a workspace or outputs must be ordered on one stream.
 */
#ifndef SHOTKV_H
#define SHOTKV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SHOTKV_MAX_SHOTS 4096

#if defined(__GNUC__)
#define SHOTKV_API __attribute__((visibility("default")))
#else
#define SHOTKV_API
#endif

enum { SHOTKV_BF16 = 0, SHOTKV_F32 = 1 };

/* How the ranked walk treats a shot that does not fit (Section 5.1, the paragraph after Eq. 3: shots
 * are taken in descending score order up to the budget).  PREFIX stops at the first misfit (the literal
 * reading, default); FIRST_FIT skips it and continues with lower-ranked shots. */
enum { SHOTKV_SELECT_PREFIX = 0, SHOTKV_SELECT_FIRST_FIT = 1 };

/* Which heads a shot's score sums over.  PER_LAYER is Eq. 3 as printed: all H query heads, one
 * selection per (batch, layer) problem shared by its KV heads.  PER_KV_HEAD restricts the head sum to
 * the G query heads that read a KV head, so every KV head ranks the shots, keeps its own subset under
 * the same budget and owns its own cache ("ragged" caches); in decoding each KV head then also
 * retains its own generated tokens by the attention of its own query group.  In this mode every
 * per-problem output and per-sequence state array gains an H_kv dimension, as noted at each entry
 * point; inputs are unchanged. */
enum { SHOTKV_HEADS_PER_LAYER = 0, SHOTKV_HEADS_PER_KV_HEAD = 1 };

enum {
  SHOTKV_OK = 0,
  SHOTKV_E_NULL = -1,      /* a required pointer is NULL                         */
  SHOTKV_E_SHAPE = -2,     /* unsupported or inconsistent shape / dtype / mode   */
  SHOTKV_E_WORKSPACE = -3, /* workspace_bytes smaller than *_workspace_bytes()   */
  SHOTKV_E_ALIGN = -4,     /* a tensor pointer is not 16-byte aligned            */
  SHOTKV_E_LAUNCH = -5,    /* the HIP runtime refused a launch                   */
  SHOTKV_E_SCRATCH = -6    /* shotkv_decode_step_static: needs more than SHOTKV_STATIC_SCRATCH_BYTES */
};

/* Per-problem device-side status words. */
enum {
  SHOTKV_ST_OK = 0,
  SHOTKV_ST_BAD_OFFSETS = -1,      /* shot offsets not strictly increasing or outside [0, n_tokens] */
  SHOTKV_ST_BUDGET_TOO_SMALL = -2, /* tokens outside every shot already exceed the budget            */
  SHOTKV_ST_NO_FREE_SLOT = -3      /* decode: the slot pool is full                                  */
};

typedef struct {
  int32_t n_q_heads;   /* H                                                       */
  int32_t n_kv_heads;  /* H_kv; query head h reads KV head h / (H / H_kv)         */
  int32_t head_dim;    /* D                                                       */
  int32_t window;      /* W: observation-window queries = last W prefill positions */
  int32_t dtype;       /* SHOTKV_BF16 or SHOTKV_F32: element type of Q, K, V      */
  float   sm_scale;    /* logits = sm_scale * <q, k>                              */
  int32_t select_mode; /* SHOTKV_SELECT_*                                          */
  int32_t head_mode;   /* SHOTKV_HEADS_*                                           */
  /* Optional per-kernel timing for benchmarks (not part of the method): NULL, or a host array of
   * 2 * SHOTKV_KERNEL_KINDS hipEvent_t handles created and owned by the caller.  A call records
   * events [2 * kind] and [2 * kind + 1] on its stream around each kernel of that kind it enqueues;
   * the caller synchronises and reads elapsed times.  The library creates no objects and keeps no
   * state between calls.  Kinds, in order: chunk plan, score, row statistics, chunk mass, shot scores
   * and selection, compaction, decode partial, decode finish, V packing, fused attention. */
  void* const* timing_events;
} shotkv_config;

SHOTKV_API const char* shotkv_strerror(int code);
SHOTKV_API int32_t shotkv_abi_version(void);

#define SHOTKV_KERNEL_KINDS 10

/* Bytes of device workspace shotkv_prefill_compress / _scores / _select_and_compact need for P
 * problems of n_tokens tokens and n_shots shots.  0 if the shape is unsupported. */
SHOTKV_API size_t shotkv_prefill_workspace_bytes(const shotkv_config* cfg, int32_t P, int32_t n_tokens,
                                      int32_t n_shots);

/*
 * Prefill compression (Section 5.1, Eq. 3-6; Algorithm 1, phase 1) of P independent (batch, layer)
 * problems that share one shape.
 *
 * Per problem: (1) softmax attention of the W window queries of every query head over the n_tokens
 * keys of its KV head, causal inside the window (query j sits at position n_tokens-W+j); (2) the
 * weights are summed over all H heads and W queries per key and averaged over each shot's tokens,
 * Score(s_i) of Eq. 3; (3) shots are ranked by score descending, ties to the lower index, and whole
 * shots are kept while they fit (Eq. 5-6); tokens outside every shot - before shot_offsets[0] and
 * from shot_offsets[n_shots] on - are always kept and are charged to the budget first; (4) the kept
 * rows of K and V are copied, in ascending position, into the dense output (Eq. 4).
 *
 *   q_obs          [P][H][W][D] dtype          window queries, unscaled
 *   k, v           [P][H_kv][n_tokens][D] dtype
 *   shot_offsets   [P][n_shots+1] int32        shot i = [off[i], off[i+1]); strictly increasing
 *   budget_tokens  [P] int32                   N_budget: most tokens a problem may retain
 *   k_out, v_out   [P][H_kv][cap][D] dtype     rows [0, kept_count) written, the rest untouched
 *   cap            rows per head in k_out/v_out; must be >= every budget (larger budgets are clamped)
 *   kept_positions [P][cap] int32              original position of each output row, ascending
 *   kept_count     [P] int32
 *   shot_scores    [P][n_shots] float          Score(s_i)                       (may be NULL)
 *   shot_selected  [P][n_shots] uint8          1 = kept                          (may be NULL)
 *   status         [P] int32                   SHOTKV_ST_*
 *
 * With cfg->head_mode = SHOTKV_HEADS_PER_KV_HEAD steps (2)-(4) run once per KV head over that head's
 * G query heads, and kept_positions is [P][H_kv][cap], kept_count [P][H_kv], shot_scores
 * [P][H_kv][n_shots], shot_selected [P][H_kv][n_shots], status [P][H_kv]; head g of k_out/v_out holds
 * kept_count[p][g] rows.
 */
SHOTKV_API int shotkv_prefill_compress(const shotkv_config* cfg, int32_t P, int32_t n_tokens, int32_t n_shots,
                            const void* q_obs, const void* k, const void* v,
                            const int32_t* shot_offsets, const int32_t* budget_tokens,
                            void* k_out, void* v_out, int32_t cap,
                            int32_t* kept_positions, int32_t* kept_count,
                            float* shot_scores, uint8_t* shot_selected, int32_t* status,
                            void* workspace, size_t workspace_bytes, void* stream);

/* The scoring half alone (steps 1-2 above; Eq. 3): writes shot_scores [P][n_shots] and status
 * ([P][H_kv][n_shots] and [P][H_kv] in per-KV-head mode). */
SHOTKV_API int shotkv_prefill_scores(const shotkv_config* cfg, int32_t P, int32_t n_tokens, int32_t n_shots,
                          const void* q_obs, const void* k, const int32_t* shot_offsets,
                          float* shot_scores, int32_t* status,
                          void* workspace, size_t workspace_bytes, void* stream);

/* The selection and compaction half alone (steps 3-4 above; Eq. 4-6) from caller-supplied scores.
 * Arguments as in shotkv_prefill_compress; shot_scores is an input here.  -0 ranks with +0; a NaN has no
 * rank and is placed by its bit pattern (deterministic, otherwise unspecified). */
SHOTKV_API int shotkv_select_and_compact(const shotkv_config* cfg, int32_t P, int32_t n_tokens, int32_t n_shots,
                              const float* shot_scores, const void* k, const void* v,
                              const int32_t* shot_offsets, const int32_t* budget_tokens,
                              void* k_out, void* v_out, int32_t cap,
                              int32_t* kept_positions, int32_t* kept_count,
                              uint8_t* shot_selected, int32_t* status,
                              void* workspace, size_t workspace_bytes, void* stream);

/*
 * Prefill compression fused into the prompt's own attention pass (Section 5.1, Eq. 3-6; the appendix on
 * limitations names kernel-level optimisation of the scoring step as open).  The prefill phase of a
 * decoder computes causal attention for every prompt position anyway, and the last W query rows of that
 * pass are the observation-window rows whose weights Eq. 3 pools.  This entry point computes
 *
 *   attn_out [P][H][n_tokens][D] float   softmax(sm_scale * Q K^T) V, causal, query head h on KV head h / G
 *
 * for the whole prompt and takes the window rows' weights from the same pass, so K is not read a second
 * time for scoring; steps (2)-(4) of shotkv_prefill_compress then run unchanged.
 *
 *   q   [P][H][n_tokens][D] dtype   all query rows of the layer (the last W are the window queries)
 *
 * Every other argument is as in shotkv_prefill_compress, and so is every result: shot_scores agree with
 * that entry point's to rounding (both head modes).  Shapes: bf16, head_dim 128; anything else returns
 * SHOTKV_E_SHAPE.  The workspace (shotkv_prefill_attention_workspace_bytes) also holds a packed copy of V.
 * Accuracy of attn_out: Q K^T in bf16 with fp32 accumulation, the weighted sum of V rows in fp16 (weights
 * with 11 significant bits, V scaled per KV-head plane by an exact power of two so that any finite bf16
 * values are representable) with fp32 accumulation and fp32 weight sums: each output row is within 1e-3 of
 * its largest magnitude of the exact result.
 */
SHOTKV_API size_t shotkv_prefill_attention_workspace_bytes(const shotkv_config* cfg, int32_t P, int32_t n_tokens,
                                                int32_t n_shots);
SHOTKV_API int shotkv_prefill_attention_compress(const shotkv_config* cfg, int32_t P, int32_t n_tokens, int32_t n_shots,
                                      const void* q, const void* k, const void* v,
                                      const int32_t* shot_offsets, const int32_t* budget_tokens,
                                      float* attn_out, void* k_out, void* v_out, int32_t cap,
                                      int32_t* kept_positions, int32_t* kept_count, float* shot_scores,
                                      uint8_t* shot_selected, int32_t* status, void* workspace,
                                      size_t workspace_bytes, void* stream);

/*
 * Decode state of one layer for S sequences: caller-owned device buffers.
 * The prefill cache is what shotkv_prefill_compress produced and is never written here (Section 5.1,
 * Eq. 2: the prefill part is compressed one time only and kept as it is while decoding).  Generated
 * tokens live in a pool of n_slots slots per
 * sequence; slot_pos holds the generated-token index in each slot, -1 when free (initialise to -1).
 * n_slots must be >= decode_budget + 1 unless the caller guarantees fewer steps than n_slots.
 * Rows of the prefill cache past prefill_count may hold anything: they may be fetched but never
 * influence a result.  decode_budget may stay or grow from step to step, e.g. ceil(r_d * (step_index +
 * 1)) for the ratio form of Eq. 8; a step evicts at most one token, so a budget that shrinks is not
 * honoured (the cache keeps the size it has).
 * In per-KV-head mode prefill_count is [S][H_kv] and slot_pos [S][H_kv][n_slots]: every KV head has
 * its own live row count and its own slot map.
 */
typedef struct {
  const void*    k_prefill;      /* [S][H_kv][cap][D] dtype                                   */
  const void*    v_prefill;      /* [S][H_kv][cap][D] dtype                                   */
  const int32_t* prefill_count;  /* [S] live rows in the prefill cache, <= cap                */
  void*          k_dec;          /* [S][H_kv][n_slots][D] dtype                               */
  void*          v_dec;          /* [S][H_kv][n_slots][D] dtype                               */
  int32_t*       slot_pos;       /* [S][n_slots]                                              */
  int32_t        cap;
  int32_t        n_slots;
  int32_t        decode_budget;  /* B_d; INT32_MAX = never evict (prefill-only ablation)      */
} shotkv_decode_state;

SHOTKV_API size_t shotkv_decode_workspace_bytes(const shotkv_config* cfg, int32_t S, int32_t cap, int32_t n_slots);

/*
 * One decoding step (Section 5.1, Eq. 7-9; Algorithm 1, phase 2) for S sequences.
 *
 * Per sequence: the new token's k_new/v_new go into the lowest-numbered free slot (slot_pos becomes
 * step_index); every query head attends over the live prefill rows plus the occupied slots (Eq. 9);
 * Score(t) = sum over heads of the weight given to decode token t at this step (Eq. 7); if the
 * decode cache now holds more than decode_budget tokens, the lowest-scored earlier token is evicted
 * (the token just appended is exempt; among equal scores the newest goes) and its slot freed (Eq. 8
 * with a fixed capacity).
 *
 *   q_new        [S][H][D] dtype       k_new, v_new [S][H_kv][D] dtype
 *   out          [S][H][D] float       attention output                          (required)
 *   token_scores [S][n_slots] float    Score(t) per slot, 0 on free slots         (may be NULL)
 *   evicted_pos  [S] int32             token index evicted this step, else -1     (may be NULL)
 *   status       [S] int32             SHOTKV_ST_*                                (required)
 *
 * In per-KV-head mode Eq. 7 sums over the G query heads of a KV head, Eq. 8 runs per KV head, and
 * token_scores is [S][H_kv][n_slots], evicted_pos and status [S][H_kv].
 */
SHOTKV_API int shotkv_decode_step(const shotkv_config* cfg, int32_t S, const shotkv_decode_state* st,
                       int32_t step_index, const void* q_new, const void* k_new, const void* v_new,
                       float* out, float* token_scores, int32_t* evicted_pos, int32_t* status,
                       void* workspace, size_t workspace_bytes, void* stream);

/*
 * shotkv_decode_step without a workspace argument, for callers that cannot allocate device memory:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same kernels,
 * same arguments, same results as shotkv_decode_step; the workspace is a buffer of
 * SHOTKV_STATIC_SCRATCH_BYTES that is part of the library's device image (one copy per GPU, held until
 * the process ends).  The call allocates and frees nothing and creates no objects.  The first call on
 * a GPU looks up the buffer's address (make that call outside a graph capture).
 *
 * Limit: returns SHOTKV_E_SCRATCH, and enqueues nothing, when shotkv_decode_workspace_bytes(cfg, S,
 * st->cap, st->n_slots) exceeds SHOTKV_STATIC_SCRATCH_BYTES (8 MiB holds e.g. 16 sequences with 32
 * query heads, head_dim 128, a 4096-row prefill cache and 1025 slots).
 * All calls on one GPU share the buffer, whatever their stream: calls that may overlap in time race
 * with each other; order them on one stream or with events.  The buffer keeps the last call's
 * contents; a step reads nothing from it that it has not written itself.
 */
#define SHOTKV_STATIC_SCRATCH_BYTES (8u << 20)
SHOTKV_API int shotkv_decode_step_static(const shotkv_config* cfg, int32_t S, const shotkv_decode_state* st,
                              int32_t step_index, const void* q_new, const void* k_new, const void* v_new,
                              float* out, float* token_scores, int32_t* evicted_pos, int32_t* status,
                              void* stream);

#ifdef __cplusplus
}
#endif
#endif /* SHOTKV_H */
