/*
 * keydiff.h -- C ABI of the MI355X (gfx950) KeyDiff block-prefill library.
 *
 * One call processes one prompt block of one transformer layer:
 *   append the block's keys/values to a fixed-budget KV cache        (Eq. 5)
 *   attention of the block over cache || block, causal in the block  (Eq. 1-2)
 *   KeyDiff score of every one of the n = len + Bt keys per KV head:
 *   cosine similarity to the anchor (the mean key)   (Method, "Efficient Variant";
 *                                          appendix "FLOP count of KeyDiff")
 *   keep the N keys with the lowest similarity, evict the rest       (Eq. 6-7, Fig. 3)
 *   move the surviving K/V rows so the cache again occupies rows [0, N)  (Eq. 6, gather)
 * in that order (Background, Fig. 1: attention precedes scoring and eviction).
 *
 * Conventions
 *   - All tensor pointers are DEVICE pointers unless a comment says "host".
 *     The library never allocates or frees device memory: the caller owns the
 *     cache, metadata and scratch buffers for the lifetime of the handle.
 *   - Tensors are bf16, innermost dimension head_dim contiguous, 16-byte aligned:
 *       q, out        [batch][n_q_heads ][Bt][head_dim]
 *       k_new, v_new  [batch][n_kv_heads][Bt][head_dim]
 *       k/v cache     [batch][n_kv_heads][cap][head_dim], cap = budget_N + block_B
 *                     rounded up to a multiple of four rows
 *     q and k arrive as the model produced them (rotary embedding already
 *     applied by the caller); keys are scored exactly as they sit in the cache.
 *   - Query head h reads KV head h / (n_q_heads / n_kv_heads).
 *   - Every call enqueues its kernels on `stream` (a hipStream_t passed as
 *     void*, NULL = default stream) and returns without synchronising.  Calls on
 *     one handle must be issued in order on one stream.
 *   - Every call reads and updates host-side state of the handle (the row count, which half of
 *     the key-sum double buffer is current, a pending eviction) and bakes it into the launches:
 *     replaying such launches from a captured HIP graph would run them with stale parameters and
 *     is not supported.
 *   - Return value: KEYDIFF_OK (0) or a negative error.  Argument, shape and
 *     state errors are found before anything is enqueued and leave the cache
 *     unchanged; KEYDIFF_EHIP (a failed launch) may leave part of the step
 *     enqueued and the handle must then be discarded.  keydiff_last_error()
 *     gives a thread-local message.  No exception crosses this boundary.
 *   - Inputs must be finite, and values (v_new, and what keydiff_cache_load brings in) must not exceed
 *     65504 in magnitude: where the keys of a step are cut into several ranges, the attention output
 *     of each range travels as fp16, normalised by its own weight sum (so it is bounded by the largest
 *     |v| it covers), before the ranges are merged; a larger value would become infinite there.  The
 *     library does not check this.  Queries and keys have no such limit.
 *   - Scores are IEEE double arithmetic on the bf16
 *     data rounded once to float; the eviction decision is taken on that float
 *     and ties keep the lower token position.
 */
#ifndef KEYDIFF_H
#define KEYDIFF_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define KEYDIFF_VERSION 1
#define KEYDIFF_API __attribute__((visibility("default")))

enum {
    KEYDIFF_OK = 0,
    KEYDIFF_EINVAL = -1, /* null or misaligned pointer, bad enum value          */
    KEYDIFF_ESHAPE = -2, /* unsupported or inconsistent sizes                  */
    KEYDIFF_ESTATE = -3, /* call not valid in the handle's current state       */
    KEYDIFF_EHIP = -4    /* a HIP runtime call or kernel launch failed         */
};

/* Which mean is the anchor (Method, "Efficient Variant of KeyDiff"). */
enum {
    KEYDIFF_ANCHOR_MEAN_KEY = 0,     /* mu(K): mean of the raw keys -- the variant the paper evaluates */
    KEYDIFF_ANCHOR_MEAN_UNIT_KEY = 1 /* mu(K^): mean of the unit keys -- Eq. 7 as printed              */
};

/* Row order of the cache after an eviction (the paper's gather leaves it open;
 * attention and the score do not depend on it). */
enum {
    KEYDIFF_LAYOUT_ORDERED = 0, /* survivors in ascending token position (stable shift)               */
    KEYDIFF_LAYOUT_FILL = 1     /* survivors of rows [N, n) fill the evicted slots of rows [0, N), both
                                   in ascending slot order: at most block_B rows move per head          */
};

typedef struct keydiff_cache keydiff_cache_t; /* opaque host handle (metadata only) */

typedef struct {
    int32_t batch;         /* independent sequences                                           */
    int32_t n_q_heads;     /* multiple of n_kv_heads                                          */
    int32_t n_kv_heads;
    int32_t head_dim;      /* 64 or 128                                                       */
    int32_t budget_N;      /* cache budget N (Background, "KV Cache Eviction Methods")        */
    int32_t block_B;       /* largest block size B (Eq. 5); capacity is N + B rows per head
                              (rounded up to a multiple of four)                               */
    int32_t anchor_mode;   /* KEYDIFF_ANCHOR_*                                                */
    int32_t window_W;      /* most recent tokens exempt from eviction (Method, "KeyDiff with
                              Sliding Window"); 0 = plain KeyDiff; must be < budget_N          */
    int32_t layout;        /* KEYDIFF_LAYOUT_*                                                */
    float eps;             /* clamp of |mu||k| in the cosine; <= 0 selects 1e-8               */
    float softmax_scale;   /* <= 0 selects 1/sqrt(head_dim) (Eq. 1)                            */
} keydiff_config_t;

/* Sizes (bytes) of the four device buffers the caller must provide for `cfg`.
 * k_bytes == v_bytes: one K (or V) cache.  meta: persistent state (token
 * positions, the running key sum the anchor is derived from, a status word).
 * scratch: per-call temporaries (attention partials, scores, selection lists);
 * its contents carry nothing between calls.  Host call, nothing is enqueued.   */
KEYDIFF_API int keydiff_workspace_bytes(const keydiff_config_t *cfg, size_t *k_bytes, size_t *v_bytes,
                            size_t *meta_bytes, size_t *scratch_bytes);

/* Create a handle over caller-owned device buffers of at least the sizes
 * above (256-byte aligned).  The cache starts empty: C_0 = {} (Eq. 5).  Clears
 * `meta` on `stream`.  *out receives the handle.                               */
KEYDIFF_API int keydiff_init_cache(const keydiff_config_t *cfg, void *k_cache, void *v_cache, void *meta,
                       void *scratch, void *stream, keydiff_cache_t **out);

/* One block step (Fig. 1 steps 2-4 after the append of Eq. 5).
 *   Bt      rows in this block, 1 <= Bt <= block_B
 *   pos0    prompt position of the block's first token; row j gets pos0 + j
 *   out     attention output of the block, computed BEFORE eviction
 *   scores_out  nullable; float [batch][n_kv_heads][len + Bt]: the score of every
 *           row of the intermediate cache in row order before eviction
 *           (cached rows, then the block)
 * With len the rows cached before the call and n = len + Bt: if n <= N the block
 * is only appended; otherwise exactly n - N rows per (sequence, KV head) are
 * evicted and the cache length becomes N.                                      */
KEYDIFF_API int keydiff_prefill_block(keydiff_cache_t *cache, const void *q, const void *k_new,
                          const void *v_new, int32_t Bt, int64_t pos0, void *out,
                          float *scores_out, void *stream);

/* keydiff_prefill_block for callers that must not allocate device memory and hold no scratch
 * buffer of their own to lend (code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc): the step's temporaries (attention partials, scores, selection lists,
 * destination map) live in a static device array of KEYDIFF_STATIC_SCRATCH_BYTES inside the
 * library instead of the handle's scratch buffer, which this call does not touch.  Each GPU holds
 * its own copy of the array from library load until the process ends; its address on a GPU is
 * looked up once, in the keydiff_init_cache that creates the first handle on that GPU.  Same
 * arguments, results and errors as keydiff_prefill_block, plus KEYDIFF_ESHAPE when the handle's
 * configuration needs more scratch than the array holds (every shape with
 * keydiff_workspace_bytes' scratch_bytes <= KEYDIFF_STATIC_SCRATCH_BYTES fits).  The call makes no
 * hipMalloc / hipFree and calls no allocating routine.  Nothing in the array has to start at
 * zero: every word a step reads it has written before.  All handles on one GPU share the array,
 * and it keeps the last call's contents: calls that overlap on one GPU (different streams or
 * threads) race, so issue them in order on one stream.                                      */
#define KEYDIFF_STATIC_SCRATCH_BYTES (40u << 20)
KEYDIFF_API int keydiff_prefill_block_static(keydiff_cache_t *cache, const void *q, const void *k_new,
                                 const void *v_new, int32_t Bt, int64_t pos0, void *out,
                                 float *scores_out, void *stream);

/* The block step of one layer of a model whose layers run one after the other, with its
 * eviction left pending.  Attention of layer l + 1 does not depend on the eviction of layer l
 * (Fig. 1: the eviction follows the attention; only the same layer's next block reads the
 * compacted cache), and a selection keeps one compute unit per head busy with a chain of short
 * stages while the attention fills the others: so this call appends, attends and scores
 * `cache` as keydiff_prefill_block does, merges the attention partials so that `out` is complete
 * in stream order, and leaves the selection and compaction of `cache` to be done
 *   - inside the step_main launch of a later keydiff_prefill_block_deferred call that names
 *     this cache as `carry` (same stream, same head_dim), or
 *   - by keydiff_finish, or by any other call on `cache` (each finishes it first, on its own
 *     stream argument or, for keydiff_destroy_cache, on the stream of the deferred call).
 * `carry` is nullable and must differ from `cache`; if it has a pending eviction this call
 * enqueues it (in the same launch when the shapes allow it, otherwise as a launch of its own
 * before it), so after the call `carry` has none.  Until its eviction is enqueued the rows of
 * `cache` are the n = len + Bt rows before compaction and its scratch buffer is in use: a
 * cache used this way needs a scratch buffer of its own.  In the ORDERED layout only the
 * selection rides; the stable row shift of `carry` follows in the same call, inside this step's
 * merge launch (or in a launch of its own where the step has none).  The scores and the retained set are those
 * of keydiff_prefill_block bit for bit; `out` may differ in the last bf16 bit, because the
 * keys are cut into a different number of ranges when passengers take part of the chip.    */
KEYDIFF_API int keydiff_prefill_block_deferred(keydiff_cache_t *cache, const void *q, const void *k_new,
                                   const void *v_new, int32_t Bt, int64_t pos0, void *out,
                                   keydiff_cache_t *carry, void *stream);

/* One block through every layer of a model (Eq. 5 applied per layer, Fig. 1's four steps in each):
 * caches, q, k_new, v_new and out are host arrays of n_layers pointers, the tensors of layer l
 * shaped as for keydiff_prefill_block; Bt and pos0 are the block's, the same in every layer.
 * Equivalent to keydiff_prefill_block_deferred on layer 0, 1, ... in turn with the layer before it
 * as `carry` (for layer 0 the last layer, whose eviction from the previous block is still
 * pending): every layer's selection and compaction runs inside the next layer's attention
 * launch, and the last layer's stays pending until the next block (or keydiff_finish, or any
 * other call on that cache).  With n_layers == 1 nothing can be carried and the eviction is
 * enqueued at the start of the next call on the cache.  ORDERED layout with three layers or more:
 * the stable row shift of layer l, whose selection rode in the launch of layer l + 1, rides in the
 * attention launch of layer l + 2 where the shapes allow it (a block that evicts at most 128 rows,
 * 256-row query tiles that are full, the same head_dim), so after the call the shifts of the last
 * two layers may still be pending as well; like a pending eviction, a pending shift is enqueued
 * first by any other call on its cache, and the rows of such a cache are not in position order
 * until then.  All pointers are checked before
 * anything is enqueued; an error met later (a state error of one layer) leaves the layers
 * before it enqueued and returns that layer's code.  The caches must be distinct.          */
KEYDIFF_API int keydiff_prefill_block_layers(keydiff_cache_t *const *caches, int32_t n_layers,
                                 const void *const *q, const void *const *k_new, const void *const *v_new,
                                 int32_t Bt, int64_t pos0, void *const *out, void *stream);

/* The block step with the rotary position embedding applied inside the call (Background, Fig. 1:
 * step (1) of a layer forms the block's queries and keys, of which the rotation is the part that
 * can live behind this boundary; the paper's method takes the keys as the cache holds them, i.e.
 * rotated).  q and k_new arrive as the projections produced them; they are rotated at the positions
 * pos0 + j (row j of the block) into buffers inside the scratch buffer, by one more launch ahead of
 * the step's own, and everything after that is keydiff_prefill_block / _layers on the rotated block.
 *   cos_table, sin_table  device, float [table_rows][head_dim / 2], 16-byte aligned: cosine and sine of
 *                         the angle of position p (row p) and frequency i (column i)
 *   pairing               element i of a row is rotated with element i + head_dim / 2:
 *                         y_i = x_i cos - x_(i+h) sin,  y_(i+h) = x_(i+h) cos + x_i sin,  every product and
 *                         sum rounded to float on its own, the result rounded once to bf16
 * KEYDIFF_ESHAPE if pos0 + Bt exceeds table_rows.  The inputs are not modified.                      */
KEYDIFF_API int keydiff_prefill_block_rope(keydiff_cache_t *cache, const void *q, const void *k_new,
                               const void *v_new, int32_t Bt, int64_t pos0, const float *cos_table,
                               const float *sin_table, int64_t table_rows, void *out, float *scores_out,
                               void *stream);
KEYDIFF_API int keydiff_prefill_block_layers_rope(keydiff_cache_t *const *caches, int32_t n_layers,
                                      const void *const *q, const void *const *k_new,
                                      const void *const *v_new, int32_t Bt, int64_t pos0,
                                      const float *cos_table, const float *sin_table, int64_t table_rows,
                                      void *const *out, void *stream);

/* Enqueue the pending eviction of `cache` on `stream`, if it has one (else a no-op). */
KEYDIFF_API int keydiff_finish(keydiff_cache_t *cache, void *stream);

/* Generation phase: the block step with B = 1 (Background, block prompt
 * processing).  q [batch][n_q_heads][1][head_dim] and so on.                   */
KEYDIFF_API int keydiff_decode_step(keydiff_cache_t *cache, const void *q, const void *k_new,
                        const void *v_new, int64_t pos, void *out, void *stream);

/* KeyDiff scores of the rows currently cached, no mutation (a pending eviction is finished first):
 * scores_out float [batch][n_kv_heads][len], row order of the cache.
 * ESTATE if the cache is empty.                                                */
KEYDIFF_API int keydiff_scores(const keydiff_cache_t *cache, float *scores_out, void *stream);

/* Rows currently cached per (sequence, KV head); host value, no sync. */
KEYDIFF_API int keydiff_cache_len(const keydiff_cache_t *cache, int32_t *len);

/* How the last block step on `cache` was cut up for the chip (host values, no sync): plan_out[0] the
 * number of key ranges (split-KV partials per output row the merge adds up; 1 = no merge launch),
 * [1] workgroups of 256 query rows per KV head, [2] 64-key tiles of the step, [3] bit 0: the step's
 * launch carried another cache's pending eviction, bit 1: it carried another cache's pending row
 * shift (ORDERED layout).  For byte and launch accounting by a benchmark.  */
KEYDIFF_API int keydiff_cache_plan(const keydiff_cache_t *cache, int32_t plan_out[4]);

/* Token position of every cached row: pos_out int32 [batch][n_kv_heads][len] (device). */
KEYDIFF_API int keydiff_cache_positions(const keydiff_cache_t *cache, int32_t *pos_out, void *stream);

/* Replace the cache contents (resume / teacher forcing): k, v device
 * [batch][n_kv_heads][len][head_dim] bf16, pos device int32 [batch][n_kv_heads][len],
 * 0 <= len <= budget_N.  Positions must be unique per head (ascending if the
 * layout is ORDERED).                                                           */
KEYDIFF_API int keydiff_cache_load(keydiff_cache_t *cache, const void *k, const void *v, const int32_t *pos,
                       int32_t len, void *stream);

/* Device-side consistency word: synchronises `stream`, then *status_out (host)
 * is 0 unless a kernel met an impossible state (for instance a selection whose
 * evicted count differs from n - N, or an expired bounded wait).               */
KEYDIFF_API int keydiff_cache_status(const keydiff_cache_t *cache, int32_t *status_out, void *stream);

/* Per-kernel timing with HIP events recorded on the stream the kernels run on.
 * enable != 0 starts recording around every kernel this handle launches;
 * keydiff_profile_read synchronises, writes the summed milliseconds and launch
 * counts of each kernel class (arrays of KEYDIFF_NKERNELS, host) and resets.    */
enum {
    KEYDIFF_K_MAIN = 0,    /* step_main: append + attention partials + key sum + cosine scores
                              (+ the carried selection of another cache, if any)               */
    KEYDIFF_K_SCORE = 1,   /* step_score: cosine scores outside a block step (keydiff_scores)  */
    KEYDIFF_K_POST = 2,    /* step_post: partial merge || selection and compaction of the step (the
                              merge alone when the eviction is deferred)                       */
    KEYDIFF_K_COMPACT = 3, /* stable in-place row shift (ORDERED layout only)                  */
    KEYDIFF_K_AUX = 4,     /* cache load helpers                                               */
    KEYDIFF_K_EVENT_PAIR = 5, /* no kernel: an empty event pair recorded once per profiled block
                              step; its time is what the two records themselves add to every
                              class above, to be subtracted by the reader                      */
    KEYDIFF_K_SELECT = 6,  /* step_post as the selection and compaction alone: a deferred eviction
                              that no attention launch carried                                 */
    KEYDIFF_NKERNELS = 7
};
KEYDIFF_API int keydiff_profile_enable(keydiff_cache_t *cache, int32_t enable);
KEYDIFF_API int keydiff_profile_read(keydiff_cache_t *cache, float *ms_out, int32_t *launches_out);

KEYDIFF_API void keydiff_destroy_cache(keydiff_cache_t *cache);

/* Message of the calling thread's last failed call ("" if none). */
KEYDIFF_API const char *keydiff_last_error(void);

KEYDIFF_API int keydiff_version(void);

#ifdef __cplusplus
}
#endif
#endif /* KEYDIFF_H */
