/*
 * zsm.h - C ABI of the ZSMerge budgeted KV-cache step for MI355X (gfx950).
 *
 * One "unit" is one (layer, sequence, KV head).  A unit owns B = B_r + B_c + B_p cache
 * slots (budget split of Sec. 3.2, Eq. 2): slots [0, B_r) are residual slots that hold
 * incremental means of evicted tokens, slots [B_r, B) hold single tokens.  All units are
 * independent; every entry point works on many units per launch.
 *
 * Conventions
 *   - Every pointer named "device" is HIP device memory owned by the caller (the Python
 *     binding passes torch tensors' data pointers).  Host pointers are read during the
 *     call only.  The library owns nothing but the small host descriptor zsm_cache_t.
 *   - Device tensors are contiguous, row-major in the index order written next to them,
 *     and 16-byte aligned.  Q/K/V inputs and token slots use the cache's kv_dtype;
 *     residual slots, scores and attention outputs are fp32; counts and positions int32.
 *   - `stream` is a hipStream_t (NULL = the default stream).  Calls only enqueue work;
 *     they never synchronise (unless zsm_set_debug_checks is on), allocate or free device
 *     memory.
 *   - Return value: ZSM_OK or a negative zsm_status.  Arguments are validated on the
 *     host before anything is enqueued, so a failed call leaves the cache untouched.
 *   - One stream per cache at a time; calls on one cache must not overlap.
 */
#ifndef ZSM_H
#define ZSM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct zsm_cache zsm_cache_t;

enum zsm_dtype { ZSM_F32 = 0, ZSM_F16 = 1, ZSM_BF16 = 2 };

enum zsm_status {
    ZSM_OK = 0,
    ZSM_E_NULL = -1,   /* a required pointer is NULL                                  */
    ZSM_E_SHAPE = -2,  /* unsupported or inconsistent sizes                            */
    ZSM_E_DTYPE = -3,  /* unknown kv_dtype                                             */
    ZSM_E_ALIGN = -4,  /* a device pointer is not 16-byte aligned                      */
    ZSM_E_NOMEM = -5,  /* caller's buffer or workspace is too small                    */
    ZSM_E_RANGE = -6,  /* layer index / range outside the cache                        */
    ZSM_E_HIP = -7,    /* the HIP runtime refused a launch (text via zsm_strerror)     */
    ZSM_E_STATE = -8,  /* the cache state breaks the call's precondition (only reported
                          while zsm_set_debug_checks is on)                            */
    ZSM_E_SCRATCH = -9 /* zsm_decode_step_static: the launch needs more scratch than
                          the library holds                                            */
};

/* Sticky per-unit condition bits, read with zsm_cache_flags. */
enum zsm_flag {
    ZSM_FLAG_DECODE_SPREAD = 1,   /* zsm_decode_step met a logit beyond its range (see there)      */
    ZSM_FLAG_PREFILL_SPREAD = 2   /* zsm_prefill_compress met a logit beyond its range (see there) */
};

#define ZSM_MAX_Q_PER_KV 128

typedef struct {
    int32_t n_layers;       /* L                                                        */
    int32_t n_seqs;         /* S: sequences in the batch                                */
    int32_t n_kv_heads;     /* H: KV heads per layer                                    */
    int32_t q_per_kv;       /* G: query heads sharing one KV head, 1 to                 */
                            /* ZSM_MAX_Q_PER_KV (3 runs the kernels of 4, 5 to 7 those  */
                            /* of 8, at their cost; more than 8, multi-query models:    */
                            /* the decode step sweeps the unit once per 8 heads)        */
    int32_t head_dim;       /* d: 64 or 128                                             */
    int32_t slot_capacity;  /* slot stride: max over sequences of B_r + B_c + B_p       */
    int32_t n_residual;     /* B_r (0 = pure eviction, Sec. 3.2)                        */
    int32_t kv_dtype;       /* enum zsm_dtype                                           */
    float lambda;           /* score decay of Eq. 3 (paper: 0.98)                       */
    float alpha;            /* weight of log w in Eq. 4, in [0, 1] (paper: 1)           */
    float scale;            /* logit scale; 0 selects 1/sqrt(d) (Eq. 1)                 */
} zsm_config_t;

/* Bytes of device memory a cache of this shape needs, the decode step's scratch area
 * included (0 if the config is invalid). */
size_t zsm_cache_bytes(const zsm_config_t* cfg);

/*
 * zsm_cache_alloc - lay a cache out in the caller's device buffer and empty it
 * (Alg. 1 "Init": all three regions empty, no token seen).
 *   B_p, B_c   host arrays [n_seqs]: proximity and context budgets of each sequence
 *              (Eq. 2); B_p >= 1, B_c >= 0, B_r + B_c + B_p <= slot_capacity.
 *   dev_buf    device, 256-byte aligned, dev_bytes >= zsm_cache_bytes(cfg).
 *   out        receives the descriptor; release it with zsm_cache_free (the device
 *              buffer stays the caller's).
 */
int zsm_cache_alloc(const zsm_config_t* cfg, const int32_t* B_p, const int32_t* B_c,
                    void* dev_buf, size_t dev_bytes, void* stream, zsm_cache_t** out);
int zsm_cache_free(zsm_cache_t* cache);

/* Bytes of device workspace a zsm_prefill_compress call over n_layers layers needs for
 * prompts of up to T_max tokens scored from W query rows (0 on invalid arguments).  Scores,
 * masks and partial sums grow with the units of the call (about 5 bytes per unit and prompt
 * token, plus 16 * d bytes per unit and 1024 tokens); besides them it holds up to 1 GiB of
 * softmax numerators (8 bytes per window row and key) when one unit's fit: K is then swept
 * once for the scores instead of twice. */
size_t zsm_prefill_workspace_bytes(const zsm_cache_t* cache, int32_t n_layers, int32_t T_max,
                                   int32_t W);

/*
 * zsm_prefill_compress - one-shot compression of the prompts of layers [layer_begin,
 * layer_end) into the (empty) cache of those layers.  Layers are independent; passing several
 * at once only puts more units into each launch (which is what the sequential absorption for
 * B_r >= 2 needs to fill the chip: one wave per unit).
 *   Scores: Eq. 3 unrolled over the last n_b = min(W, T_b) prompt queries, each query a
 *   causal softmax row (Eq. 1), grouped query heads pooled by their mean (appendix, GQA
 *   adaptation); W >= T_max is the full-history initialisation, a smaller W the
 *   windowed one (appendix "Implementation Details").
 *   Selection: the latest B_p tokens plus the top-B_c of the others by score (Sec. 3.2);
 *   equal scores keep the earlier position.  A prompt with T_b <= B_p + B_c is kept whole.
 *   Residual: every token not kept is absorbed in position order as in Alg. 1's
 *   residual branch (Eq. 5, Eq. 6).
 *   Slot order afterwards: residual slots, context tokens by position, proximity tokens
 *   by position.
 *   Q          device [Ln, S, H, G, W, d], Ln = layer_end - layer_begin; row r of sequence b
 *              is the query at position T_b - n_b + r; rows r >= n_b are ignored.
 *   K, V       device [Ln, S, H, T_max, d]; rows >= T_b are ignored.
 *   seq_lens   device int32 [S]: T_b, 0 <= T_b <= T_max (the same for every layer).
 *   workspace  device, 256-byte aligned, ws_bytes >= zsm_prefill_workspace_bytes(Ln, ..).
 * The layers' caches must be empty (freshly allocated or re-imported empty); this is only
 * verified while zsm_set_debug_checks is on (ZSM_E_STATE).  S * H <= 32768 (ZSM_E_SHAPE).
 * Logit range: each softmax row (Eq. 1) is evaluated in fp64 as exp(z_t - z_self) / sum, with
 * z_self the query's logit against the key at its own position, so no running maximum is
 * kept.  This is exact as long as no counted key's logit exceeds z_self by more than 690
 * (e^690 is near the top of the fp64 range; a softmax over 16- or 32-bit inputs whose
 * logits spread that far has a single non-zero entry).  Beyond that the difference is clamped at
 * 690, the keys beyond it get equal weight and the scores of that unit are not the method's.
 * The clamp never acts unseen: a row whose sum of exponentials reaches e^680 raises the unit's
 * ZSM_FLAG_PREFILL_SPREAD bit (so the bit may already be up, with exact results, when the
 * spread is within ln(T) of 680).  The call still returns ZSM_OK (nothing is read back from the
 * device here); a caller that feeds unnormalised activations checks zsm_cache_flags afterwards.
 * With B_r = 1 the residual slot is the mean of all absorbed tokens (parallel sums); with
 * B_r >= 2 the tokens are absorbed one after the other as Alg. 1 prescribes (sequential per
 * unit: about a microsecond per absorbed token).  B_r <= 64 here (the decode step takes any
 * B_r); ZSM_E_SHAPE otherwise.
 */
int zsm_prefill_compress(zsm_cache_t* cache, int32_t layer_begin, int32_t layer_end,
                         const void* Q, int32_t W, const void* K, const void* V,
                         const int32_t* seq_lens, int32_t T_max, void* workspace,
                         size_t ws_bytes, void* stream);

/*
 * zsm_decode_step - one fused decode step (the loop body of Alg. 1 with the attention
 * of Eq. 4) for every unit of layers [layer_begin, layer_end).  Per unit, with T tokens
 * seen so far:
 *   1. logits q.k/sqrt(d) + alpha*log(w) over the occupied slots and the incoming token
 *      itself, softmax, output (Eq. 4); one softmax per query head;
 *   2. scores s <- lambda*s + mean over the group of the probabilities; the incoming
 *      token starts at its own probability (Eq. 3);
 *   3. if a token slot is free the incoming token takes the lowest free one; otherwise
 *      the token with the lowest (score, position) among those outside the latest B_p
 *      positions (incoming token counted) is evicted (Alg. 1, context overflow);
 *   4. the evicted key/value opens the lowest unused residual slot, or is merged into
 *      the residual slot with the largest key dot product (lowest index on ties) by the
 *      incremental mean, whose count grows by one (Eq. 5, Eq. 6); B_r = 0 drops it;
 *   5. the incoming token is written to the freed slot with position T.
 *   q            device [Ln, S, H, G, d], Ln = layer_end - layer_begin
 *   k_new,v_new  device [Ln, S, H, d]
 *   out          device fp32 [Ln, S, H, G, d]
 *   write_slot   device int32 [Ln, S, H] or NULL: slot that received the token
 *   evicted_pos  device int32 [Ln, S, H] or NULL: position of the evicted token, -1 if none
 *   merged_slot  device int32 [Ln, S, H] or NULL: residual slot that absorbed it, -1 if none
 * Logit range: the softmax of Eq. 4 is evaluated in fp64 as exp(z_j - z_new) / sum, z_new being
 * the incoming token's own logit, so no running maximum is kept.  This is exact as long as no
 * slot's logit (log-count term included) exceeds z_new by more than 690.  Beyond that the
 * difference is clamped at 690: the slots beyond it tie, and that unit's output, scores and
 * eviction choice are not the method's.  The clamp never acts unseen: a softmax denominator
 * that reaches e^680 raises the unit's ZSM_FLAG_DECODE_SPREAD bit (sticky, read with
 * zsm_cache_flags; it may already be up, with exact results, when the spread is within ln(B)
 * of 680).  The call still returns ZSM_OK.
 * Launch shape: one workgroup per unit when the launch has many units; a launch of few
 * units (one layer of a single sequence, say) is cut into several workgroups per unit,
 * each sweeping a share of the slots, so that it still fills the chip.  The share's
 * partial softmax sums and outputs meet in a scratch area inside the cache buffer; the
 * result does not depend on the cut beyond fp32 rounding of the output (scores, choices
 * and merged rows are formed in fp64 from the same per-slot values either way).
 * More than 8 query heads per KV head: the step runs as ceil(G / 8) sweeps of the unit's slots, 8
 * heads each, whose per-slot probabilities are pooled in the cache buffer's scratch section, and a
 * finishing launch; such a step is never cut over workgroups (zsm_cache_set_decode_parts has no
 * effect), so the limit below applies whatever the launch, with G' = 4 (the sweeps then take 4
 * heads each where 8 do not fit).
 * Positions are kept as int32: a unit may see at most 2^31 - 1 tokens in all.
 * Limit: the per-slot values of one workgroup, (slots + 1) * G' * 8 bytes (G' = G rounded up
 * to 1, 2, 4 or 8), must fit the 160 KB LDS together with ~24 KB of staging; a capacity too large for one workgroup is
 * split automatically where the launch is small enough to be split (at most 1024 units),
 * else ZSM_E_SHAPE.
 */
int zsm_decode_step(zsm_cache_t* cache, int32_t layer_begin, int32_t layer_end,
                    const void* q, const void* k_new, const void* v_new, float* out,
                    int32_t* write_slot, int32_t* evicted_pos, int32_t* merged_slot,
                    void* stream);

/*
 * zsm_decode_step_static - zsm_decode_step for callers that cannot allocate device memory
 * (code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc) and
 * do not want the split launch's scratch inside their cache buffer to be what is used: the
 * partial softmax sums, output shares and per-slot exponentials of a launch that is cut over
 * several workgroups per unit go to an array of ZSM_STATIC_SCRATCH_BYTES that the library
 * itself holds on every GPU it runs on, from the first call on that GPU until the process ends.
 * Same arguments, results and launch shapes as zsm_decode_step (to fp32 rounding: identical).
 * The call allocates and frees nothing and calls no allocating routine.
 *   Limit: a split launch of n units in p parts needs about
 *   n*p*G*(8 + 4*d) + n*G*(slot_capacity + 1)*8 bytes (each of the three sections rounded up to
 *   256); beyond ZSM_STATIC_SCRATCH_BYTES the call enqueues nothing and returns ZSM_E_SCRATCH.
 *   One layer of 32 units with 2700 slots (16 parts) needs 0.9 MB, one layer of 128 units of four
 *   query heads with 1024 slots (4 parts) 5 MB.  A launch that is not split needs none.
 *   Sharing: all calls on one GPU use that GPU's one array, whatever the cache or stream.  It
 *   keeps the previous call's contents; nothing in it has to start at zero (every value a
 *   launch reads was written by the same launch).  Calls that overlap in time on one GPU (two
 *   streams, two host threads) race on it: serialise them, or use zsm_decode_step, whose
 *   scratch is per cache.
 *   The first call on a GPU resolves the array's address there; make it outside a capture.
 */
#define ZSM_STATIC_SCRATCH_BYTES (8u << 20)
int zsm_decode_step_static(zsm_cache_t* cache, int32_t layer_begin, int32_t layer_end,
                           const void* q, const void* k_new, const void* v_new, float* out,
                           int32_t* write_slot, int32_t* evicted_pos, int32_t* merged_slot,
                           void* stream);

/*
 * zsm_cache_set_decode_parts - how many workgroups share one unit in zsm_decode_step (a
 * launch-shape knob of this library, not something the paper defines): 0 = chosen per launch
 * from the number of units (the default), 1 = never split, 2..64 = this many where the launch
 * allows it (at most 1024 units and 8192 workgroups; fewer parts are used beyond that).
 * ZSM_E_RANGE for other values.
 */
int zsm_cache_set_decode_parts(zsm_cache_t* cache, int32_t parts);

/* Workgroups per unit that zsm_decode_step would use for layers [layer_begin, layer_end)
 * with the current setting (>= 1), or a negative zsm_status (ZSM_E_SHAPE: no permitted
 * cut fits the LDS).  Host-only, launches nothing. */
int zsm_decode_parts(const zsm_cache_t* cache, int32_t layer_begin, int32_t layer_end);

/*
 * zsm_cache_export / zsm_cache_import - copy one layer's state out of / into the cache
 * (checkpointing and test hook).  All arrays are device memory; any may be NULL to skip.
 *   K, V    kv_dtype [S, H, slot_capacity - B_r, d]   token slots
 *   Kr, Vr  fp32     [S, H, B_r, d]                    residual slots
 *   s       fp32     [S, H, slot_capacity]             scores, slot order (residual first)
 *   pos     int32    [S, H, slot_capacity]             original position, -1 = empty
 *   w       int32    [S, H, slot_capacity]             fusion count, 0 = empty
 *   n_seen  int64    [S, H]                            tokens seen (T)
 * Import trusts the caller: every slot must have w = 0 exactly where pos = -1, token slots
 * w in {0,1}, positions below n_seen, and slots past the sequence's B_r + B_c + B_p empty.
 * While zsm_set_debug_checks is on, import verifies this on the arrays it is given (a NULL one
 * is taken from the cache) before it copies anything, and returns ZSM_E_STATE otherwise.
 */
int zsm_cache_export(const zsm_cache_t* cache, int32_t layer, void* K, void* V, float* Kr,
                     float* Vr, float* s, int32_t* pos, int32_t* w, int64_t* n_seen,
                     void* stream);
int zsm_cache_import(zsm_cache_t* cache, int32_t layer, const void* K, const void* V,
                     const float* Kr, const float* Vr, const float* s, const int32_t* pos,
                     const int32_t* w, const int64_t* n_seen, void* stream);

/*
 * zsm_cache_flags - the sticky condition bits (enum zsm_flag) of one layer's units.
 *   flags   device int32 [S, H] or NULL: receives the bits
 *   clear   non-zero: the layer's bits are reset after they have been copied
 * The bits are also reset by zsm_cache_alloc.  Only kernels set them; nothing is read back on
 * the host here, the call enqueues one small kernel.
 */
int zsm_cache_flags(zsm_cache_t* cache, int32_t layer, int32_t* flags, int32_t clear, void* stream);

/*
 * zsm_set_debug_checks - process-wide switch (default off) for checks of device-side state
 * that the normal path cannot afford: while on, zsm_prefill_compress verifies that the layer
 * is empty and zsm_cache_import that the state it is given is well formed.  Each check runs
 * a small kernel, WAITS for the stream and reads one counter back, so it is for development
 * and tests; a violation is reported as ZSM_E_STATE before the call changes anything.
 * Returns the previous setting.
 */
int zsm_set_debug_checks(int32_t on);

/*
 * zsm_stream_read / zsm_stream_copy - plain streaming kernels of known size, used to
 * calibrate hardware counters and to measure the achievable HBM rate next to the decode
 * step.  `src`/`dst` device, 16-byte aligned, `bytes` a multiple of 16.  zsm_stream_read
 * sums the buffer into sink[0] (fp32, device) so the reads cannot be elided.
 */
int zsm_stream_read(const void* src, size_t bytes, float* sink, void* stream);
int zsm_stream_copy(void* dst, const void* src, size_t bytes, void* stream);

/* Text for a status code; for ZSM_E_HIP the last HIP error text of this thread. */
const char* zsm_strerror(int status);

#ifdef __cplusplus
}
#endif
#endif /* ZSM_H */
