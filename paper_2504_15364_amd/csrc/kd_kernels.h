// Internal launcher interface between the C-ABI host layer and the gfx950 kernels.
//
// One block step is two launches:
//   step_main  append (Eq. 5) + split-KV flash attention partials (Eq. 1-2)
//              + running key sum S' = S + sum of the block's keys (the anchor is S' / n)
//              + cosine score of every row, taken from the K tiles while they sit in LDS
//   step_post  merge of the attention partials  ||  selection of the rows to evict
//              and compaction, one workgroup per head (Eq. 6-7)
// plus, for the ORDERED layout only, one more launch that shifts rows in place.
// With the eviction deferred the second launch is the merge alone, and the selection and
// compaction ride in the step_main launch of the next cache (launch_step_main_carry).
// step_score scores a cache outside a block step (keydiff_scores).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace kd {

constexpr int TILE_KEYS = 64;       // keys per attention K/V tile
constexpr int POST_THREADS = 1024;  // workgroup size of step_post
constexpr int SCORE_THREADS = 256;  // workgroup size of step_score
constexpr int SCORE_ROWS = 128;     // rows per step_score workgroup: 32 per wave
constexpr int HIST_BINS = 4096;     // score histogram resolution in step_post (bins over [-1, 1])
constexpr int CHUNK_ROWS = 128;     // rows per workgroup in the from-scratch key-sum pass
constexpr int ORD_ROWS = 128;       // rows per workgroup of the ordered compaction
constexpr int ORD_THREADS = 1024;   // ... and its threads: 4 16-byte units each
constexpr int ORD_SPIN_LIMIT = 1 << 20;  // polls of a predecessor's flag before giving up
constexpr int MAX_CAP = 32768;      // budget_N + block_B limit (selection bitmaps, ownership)

// status bits kernels may raise (device word in the metadata buffer)
constexpr int STATUS_SELECT_COUNT = 1;  // selection evicted a number of rows other than n - N
constexpr int STATUS_ORDER_TIMEOUT = 2; // ordered compaction: a workgroup gave up waiting for its predecessors

struct StepParams {
    // tensors of the call
    const uint16_t *q;               // [batch][hq][Bt][D]
    const uint16_t *k_new, *v_new;   // [batch][hkv][Bt][D]
    uint16_t *out;                   // [batch][hq][Bt][D]
    float *scores_out;               // nullable [BH][n]
    // caller-owned state
    uint16_t *k, *v;                 // caches [BH][cap][D]
    int32_t *pos;                    // [BH][cap] token position of every row
    const double *ksum;              // [BH][D] running sum of the (raw or unit) keys in the cache before this step
    double *ksum_next;               // [BH][D] ... after it (the other half of a double buffer): written by
                                     // step_main (+ the block's keys), then by step_post (- the evicted keys)
    int32_t *status;
    // scratch
    _Float16 *part_o;                // [psplits][BH][blocks of 32 rows][D/8 slabs][64 lanes][4] partial outputs in the
                                     // MFMA accumulator layout, each normalised by its row sum
    float2 *part_ml;                 // [psplits][BH * G * Bt]    (reference max in log2 units, row sum)
    float *scores;                   // [BH][cap]
    int32_t *dstmap;                 // [BH][cap] ORDERED layout: destination row or -1
    int32_t *lists;                  // [BH][4 * B] evicted rows | holes | movers | mover rank of each tail row
    unsigned long long *argmax_rec;  // nullable [BH][splits][2]: the generation phase (one row to evict, no window):
                                     // per step_main workgroup the largest (orderable score bits << 32 | row) among the
                                     // rows it scored, and whether another of its rows has the same score bits
    // sizes
    int batch, hq, hkv, G, D, Bt, len, n, N, B, cap;
    int splits, mtiles, ntiles, NW;      // NW: waves (of 32 query rows) per step_main workgroup
    int psplits;                     // partials per output row the merge adds up: splits, or 2 * splits when two
                                     // waves of a workgroup take alternate tiles of its key range (decode)
    int edge_cost;                   // weight (in plain tiles: 1 or 2) of a tile holding rows of the block when
                                     // the key tiles are divided over the splits
    int score_chunks;                // step_score workgroups per head
    int lists_in_lds;                // selection lists live in LDS (else in `lists`)
    int merge_wgs;                   // merge workgroups in step_post (0 when psplits == 1)
    int do_score, do_evict;
    int anchor_mode, layout, window_W;
    int32_t pos0, window_pos_min;
    float scale_log2e;
    double eps;
#ifdef KD_TIMELINE
    unsigned long long *timeline;    // [workgroup][32] wall-clock stamps of this launch (profiling build only)
#endif
};

hipError_t configure_kernels();      // one-time function attributes (dynamic LDS sizes)
hipError_t launch_step_main(const StepParams &p, hipStream_t s);
// step_main of `p` whose first workgroups run the selection and compaction `cy` describes (the
// parameters of an earlier step of another cache; for the ORDERED layout the caller still launches
// the row shift afterwards); can_carry says whether the pair fits
bool can_carry(const StepParams &p, const StepParams &cy);
hipError_t launch_step_main_carry(const StepParams &p, const StepParams &cy, hipStream_t s);
// An ORDERED cache's row shift riding in an attention launch: `p` is the step whose selection wrote the
// destination map, `parts` workgroups per head share the head's chunks (flags, epoch: as for
// launch_compact_ordered).  can_host_shift says whether the attention step `p` can take it along.
struct ShiftRide {
    StepParams p;
    int32_t *flags;
    int nchunks, parts, nshift;
    int32_t epoch;
};
bool can_host_shift(const StepParams &p, const StepParams &shifted);
// step_main of `p` with passengers: the selection `cy` (or none: nullptr) and the shift `ride`
hipError_t launch_step_main_ride(const StepParams &p, const StepParams *cy, const ShiftRide &ride, hipStream_t s);
hipError_t launch_step_score(const StepParams &p, hipStream_t s);
hipError_t launch_step_post(const StepParams &p, hipStream_t s);
// flags: [BH][ceil(cap / ORD_ROWS)] int32 in zero-initialised device memory; epoch: a value no earlier launch used
hipError_t launch_compact_ordered(const StepParams &p, int32_t *flags, int32_t epoch, hipStream_t s);
// the merge of pm's partials and the ordered shift of ps's cache in one launch (same head_dim)
hipError_t launch_merge_shift(const StepParams &pm, const StepParams &ps, int32_t *flags, int32_t epoch, hipStream_t s);
hipError_t launch_ksum_rebuild(const StepParams &p, double *partials, hipStream_t s);
// rotary embedding of the block's queries (q_rows rows) and keys (k_rows rows), Bt tokens per (sequence,
// head) at positions pos0 + j, by the caller's float tables [position][D / 2]
hipError_t launch_rope(const uint16_t *q, const uint16_t *k, uint16_t *q_rot, uint16_t *k_rot, const float *cos_t,
                       const float *sin_t, int q_rows, int k_rows, int Bt, int D, int32_t pos0, hipStream_t s);
hipError_t launch_zero_words(int32_t *p, size_t nwords, hipStream_t s);
hipError_t launch_load_rows(const uint16_t *src, uint16_t *dst, int BH, int cap, int D, int len,
                            hipStream_t s);
hipError_t launch_load_pos(const int32_t *src, int32_t *dst, int BH, int cap, int len, int to_cache,
                           hipStream_t s);

bool lists_fit_lds(int n, int N);

}  // namespace kd
