// Internal launcher interface between the C-ABI host layer and the gfx950 kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace kd {

constexpr int TILE_KEYS = 64;      // keys per attention K/V tile
constexpr int CHUNK_ROWS = 128;    // rows per workgroup in the anchor / score passes
constexpr int SELECT_THREADS = 1024;

// status bits kernels may raise (device word in the metadata buffer)
constexpr int STATUS_SELECT_COUNT = 1;   // selection evicted a number of rows other than n - N
constexpr int STATUS_WAIT_EXPIRED = 2;   // a bounded wait ran out

struct AttnParams {
    const uint16_t *q;        // [batch][hq][Bt][D]
    const uint16_t *k, *v;    // caches [batch][hkv][cap][D], block already appended
    uint16_t *out;            // [batch][hq][Bt][D]
    float *part_o;            // [splits][BH * G * Bt][D]   unnormalised partial outputs
    float2 *part_ml;          // [splits][BH * G * Bt]      (running max in log2 units, row sum)
    int batch, hq, hkv, G, Bt, len, n, cap;
    int splits, mtiles, ntiles;
    float scale_log2e;        // softmax scale * log2(e)
};

struct EvictParams {
    uint16_t *k, *v;          // caches
    int32_t *pos;             // [BH][cap]
    double *anchor_part;      // [BH][nchunks][D]
    float *scores;            // [BH][cap]
    int32_t *dstmap;          // [BH][cap]   ORDERED layout: destination row or -1
    int32_t *status;          // device status word
    int BH, cap, D, n, N, nchunks;
    int anchor_mode, layout, window_W;
    int32_t window_pos_min;   // rows with pos >= this are exempt when window_W > 0
    double eps;
};

hipError_t launch_append(const uint16_t *k_new, const uint16_t *v_new, uint16_t *k, uint16_t *v,
                         int32_t *pos, int BH, int cap, int D, int len, int Bt, int32_t pos0,
                         hipStream_t s);
hipError_t launch_attention(const AttnParams &p, int D, int NQ, hipStream_t s);
hipError_t launch_merge(const AttnParams &p, int D, hipStream_t s);
hipError_t launch_anchor(const EvictParams &p, hipStream_t s);
hipError_t launch_score(const EvictParams &p, hipStream_t s);
hipError_t launch_select(const EvictParams &p, hipStream_t s);
hipError_t launch_compact_ordered(const EvictParams &p, hipStream_t s);
hipError_t launch_zero_words(int32_t *p, size_t nwords, hipStream_t s);
hipError_t launch_load_rows(const uint16_t *src, uint16_t *dst, int BH, int cap, int D, int len,
                            hipStream_t s);
hipError_t launch_load_pos(const int32_t *src, int32_t *dst, int BH, int cap, int len, int to_cache,
                           hipStream_t s);
hipError_t launch_copy_scores(const float *src, float *dst, int BH, int cap, int n, hipStream_t s);

size_t select_lds_bytes(int n, int N);
size_t compact_lds_bytes(int D);

}  // namespace kd
