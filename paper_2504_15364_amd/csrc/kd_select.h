// Selection of the rows to evict and compaction of one head (Eq. 6-7), as device code shared by
// the kernels that can run it: step_post (one workgroup of 1024 threads per head) and the variant of
// step_main that carries another cache's pending eviction (workgroups of 512 threads).
//
// One workgroup copies the head's scores and positions into LDS once (asynchronously, no registers),
// bins the scores into a 4096-bin LDS histogram (a monotone map of the float), scans it for the bin
// that holds the E-th largest score, evicts everything above that bin and ranks the few rows inside
// it exactly by (score bits, position): equal scores keep the lower position.  It then compacts the
// cache and takes the evicted keys out of ksum.
//
// The passes over the rows are short rolled loops over the LDS copy.  As a passenger the selection
// runs on one compute unit per head, whose instruction cache nothing has warmed, while the
// attention saturates the memory system: with the rows in registers and every pass unrolled
// (25 KB of straight-line code) it spent most of its time waiting for its own instructions.
#pragma once
#include "kd_kernels.h"
#include "kd_device.h"

namespace kd {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef int32_t i32x4 __attribute__((ext_vector_type(4)));

constexpr int CAND_MAX = 1024;  // rows of the threshold bin ranked in LDS; more fall back to a radix select
constexpr int MAX_SELECT_WAVES = POST_THREADS / 64;   // PostShared is laid out for the largest workgroup
constexpr int TAIL_WORDS = 72;                      // bitmap words the tail rows [N, n) may span on the fast path
constexpr int CARRY_THREADS = 512;                  // workgroup size of the step_main variant that carries a selection
constexpr int SELECT_TAILU = 8;                     // 16-byte units of the tail rows [N, n) a thread keeps in registers

// float -> unsigned key with the same order
__device__ __forceinline__ uint32_t orderable(float s)
{
    const uint32_t b = __float_as_uint(s);
    return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}

// monotone non-decreasing map of a score onto [0, HIST_BINS)
__device__ __forceinline__ int score_bin(float s)
{
    const float f = floorf((s + 1.0f) * (float)(HIST_BINS / 2));
    return (int)fminf(fmaxf(f, 0.f), (float)(HIST_BINS - 1));
}

struct PostShared {
    uint32_t hist[HIST_BINS];  // score histogram of the head (a monotone map of the float)
    uint32_t wave_tot[MAX_SELECT_WAVES];
    uint64_t wave_tot64[MAX_SELECT_WAVES];
    uint32_t radix_hist[256];
    uint32_t sel_bin, sel_rank, sel_cnt;
    int tb;           // threshold bin
    uint32_t need;    // rows to evict from the threshold bin
    uint32_t ncand, nev;
    uint32_t cand_slot[CAND_MAX];
    uint32_t cand_key[CAND_MAX];
    int32_t cand_pos[CAND_MAX];
    double colsum[MAX_SELECT_WAVES][128];
    uint32_t tail_word[TAIL_WORDS], tail_base[TAIL_WORDS];  // mover bitmap words of rows >= N and movers before each
};

// bytes of dynamic LDS a carried selection places PostShared in, ahead of its bitmap and lists
__host__ __device__ constexpr size_t carry_shared_bytes() { return (sizeof(PostShared) + 255) & ~(size_t)255; }

// value of the lane `ctrl` names (DPP), 0 where that lane lies outside the row or the row is masked out
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ uint32_t dpp_fetch(uint32_t x)
{
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, CTRL, ROW_MASK, 0xF, true);
}

// inclusive prefix sum over the 64 lanes of a wave, on the vector ALU alone: Hillis-Steele inside
// each row of 16 lanes (row_shr 1, 2, 4, 8), then lane 15 of rows 0 and 2 into rows 1 and 3
// (row_bcast:15), then lane 31 into rows 2 and 3 (row_bcast:31)
__device__ __forceinline__ uint32_t wave_inclusive_scan(uint32_t x)
{
    x += dpp_fetch<0x111, 0xF>(x);
    x += dpp_fetch<0x112, 0xF>(x);
    x += dpp_fetch<0x114, 0xF>(x);
    x += dpp_fetch<0x118, 0xF>(x);
    x += dpp_fetch<0x142, 0xA>(x);
    x += dpp_fetch<0x143, 0xC>(x);
    return x;
}
__device__ __forceinline__ uint64_t wave_inclusive_scan(uint64_t x)
{
#define KD_STEP64(CTRL, MASK)                                                                   \
    x += ((uint64_t)dpp_fetch<CTRL, MASK>((uint32_t)(x >> 32)) << 32) | dpp_fetch<CTRL, MASK>((uint32_t)x);
    KD_STEP64(0x111, 0xF)
    KD_STEP64(0x112, 0xF)
    KD_STEP64(0x114, 0xF)
    KD_STEP64(0x118, 0xF)
    KD_STEP64(0x142, 0xA)
    KD_STEP64(0x143, 0xC)
#undef KD_STEP64
    return x;
}

// exclusive prefix sum over the workgroup (32-bit, or three packed 21-bit counters in 64 bits)
template <int THREADS, typename T>
__device__ __forceinline__ T block_exclusive_scan_t(T v, T *wave_tot, T *total)
{
    constexpr int NWAVES = THREADS / 64;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const T inc = wave_inclusive_scan(v);
    __syncthreads();  // wave_tot free for reuse
    if (lane == 63) wave_tot[wave] = inc;
    __syncthreads();
    T base = 0, tot = 0;
#pragma unroll
    for (int w = 0; w < NWAVES; ++w) {
        const T t = wave_tot[w];
        if (w < wave) base += t;
        tot += t;
    }
    *total = tot;
    return base + inc - v;
}

// ---------------------------------------------------- slow path: radix select in a bin
// More than CAND_MAX rows share the threshold bin (near-identical keys).  MSB-first
// 8-bit radix select over the 64-bit key (orderable score : position) restricted to
// that bin; reads scores and positions again on every pass.  Marks the
// `need` largest in the evict bitmap.
template <int THREADS>
__device__ void radix_select_in_bin(const StepParams &p, PostShared &sh, const float *sc, const int32_t *pos,
                                    uint32_t *evbits, int tb, uint32_t need)
{
    const int tid = threadIdx.x, lane = tid & 63;
    uint64_t prefix = 0;
    uint32_t rank = need;
    int resolved = 0;
    for (int pass = 0; pass < 8; ++pass) {
        const int shift = 56 - 8 * pass;
        for (int i = tid; i < 256; i += THREADS) sh.radix_hist[i] = 0;
        __syncthreads();
        for (int i0 = 0; i0 < p.n; i0 += THREADS) {
            const int i = i0 + tid;
            bool part = false;
            uint32_t digit = 0;
            if (i < p.n) {
                const float s = sc[i];
                const bool exempt = p.window_W > 0 && pos[i] >= p.window_pos_min;
                if (!exempt && score_bin(s) == tb) {
                    const uint64_t key = ((uint64_t)orderable(s) << 32) | (uint32_t)pos[i];
                    part = pass == 0 || (key >> (shift + 8)) == prefix;
                    digit = (uint32_t)(key >> shift) & 255u;
                }
            }
            const uint64_t active = __ballot(part);
            if (active) {
                const int leader = __ffsll((unsigned long long)active) - 1;
                const uint32_t ld = __shfl(digit, leader);
                const uint64_t same = __ballot(part && digit == ld);
                if (lane == leader) atomicAdd(&sh.radix_hist[ld], (uint32_t)__popcll(same));
                else if (part && digit != ld) atomicAdd(&sh.radix_hist[digit], 1u);
            }
        }
        __syncthreads();
        if (tid < 64) {
            const uint32_t c0 = sh.radix_hist[4 * lane], c1 = sh.radix_hist[4 * lane + 1],
                           c2 = sh.radix_hist[4 * lane + 2], c3 = sh.radix_hist[4 * lane + 3];
            const uint32_t mine = c0 + c1 + c2 + c3;
            uint32_t suf = mine;
#pragma unroll
            for (int off = 1; off < 64; off <<= 1) {
                const uint32_t t = __shfl_down(suf, off);
                if (lane + off < 64) suf += t;
            }
            const uint64_t reach = __ballot(suf >= rank);
            const int owner = reach ? 63 - __clzll((unsigned long long)reach) : 0;
            if (lane == owner) {
                uint32_t above = suf - mine, bin, cnt;
                if (above + c3 >= rank) { bin = 3; cnt = c3; }
                else if ((above += c3) + c2 >= rank) { bin = 2; cnt = c2; }
                else if ((above += c2) + c1 >= rank) { bin = 1; cnt = c1; }
                else { above += c1; bin = 0; cnt = c0; }
                sh.sel_bin = 4 * lane + bin;
                sh.sel_rank = rank - above;
                sh.sel_cnt = cnt;
            }
        }
        __syncthreads();
        prefix = (prefix << 8) | sh.sel_bin;
        rank = sh.sel_rank;
        resolved = 8 * (pass + 1);
        const bool done = sh.sel_cnt == rank;
        __syncthreads();
        if (done) break;
    }
    for (int i = tid; i < p.n; i += THREADS) {
        const float s = sc[i];
        const bool exempt = p.window_W > 0 && pos[i] >= p.window_pos_min;
        if (!exempt && score_bin(s) == tb) {
            const uint64_t key = ((uint64_t)orderable(s) << 32) | (uint32_t)pos[i];
            if ((key >> (64 - resolved)) >= prefix) atomicOr(&evbits[i >> 5], 1u << (i & 31));
        }
    }
    __syncthreads();
}

// bytes of dynamic LDS the selection of a step uses behind PostShared: the eviction bitmap, the
// lists (when they fit) and, for the resident variant, the copies of the scores and positions
__host__ __device__ inline size_t select_dyn_bytes(int n, int N, int cap, bool lists_in_lds, bool resident)
{
    size_t b = ((size_t)((n + 31) / 32) * 4 + 15) & ~(size_t)15;
    if (lists_in_lds) b += (size_t)(n - N) * 16;
    if (resident) b += (size_t)cap * 8;
    return b;
}

// ------------------------------------------------------------- select + compaction
// `dyn`: dynamic LDS of select_dyn_bytes(...) bytes, 16-byte aligned.  The lists are three arrays of
// E row indices (evicted | holes | movers) and the mover rank of every tail row: in LDS when they
// fit, else in the scratch buffer.
// RES: the head's scores and positions are copied into LDS once and every pass reads the copy;
// otherwise (caches too large for that) the passes read them from memory.
// The caller keeps n <= 32 * THREADS (a thread owns one word of the eviction bitmap).
template <int D, bool RES, int THREADS>
__device__ void select_and_compact(const StepParams &p, PostShared &sh, unsigned char *dyn, int bh)
{
    constexpr int UPR = D / 8;
    constexpr int TAILU = SELECT_TAILU;
    constexpr int NWAVES = THREADS / 64;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int E = p.n - p.N;
    const float *sc_g = p.scores + (size_t)bh * p.cap;
    int32_t *pos = p.pos + (size_t)bh * p.cap;
    uint16_t *kb = p.k + (size_t)bh * p.cap * D;
    uint16_t *vb = p.v + (size_t)bh * p.cap * D;
    const int nwords = (p.n + 31) / 32;
    uint32_t *evbits = reinterpret_cast<uint32_t *>(dyn);
    size_t dyn_off = ((size_t)nwords * 4 + 15) & ~(size_t)15;
    int32_t *lists = p.lists + (size_t)bh * 4 * p.B;
    if (p.lists_in_lds) {
        lists = reinterpret_cast<int32_t *>(dyn + dyn_off);
        dyn_off += (size_t)E * 16;
    }
    float *sc_l = reinterpret_cast<float *>(dyn + dyn_off);
    int32_t *pos_l = reinterpret_cast<int32_t *>(dyn + dyn_off + (size_t)p.cap * 4);
    // what the passes read: the LDS copies (as LDS pointers, so that the loops use ds_read) or memory
    typedef __attribute__((address_space(3))) const float lds_cf32;
    typedef __attribute__((address_space(3))) const int32_t lds_ci32;
    lds_cf32 *sc_s = (lds_cf32 *)sc_l;
    lds_ci32 *pos_s = (lds_ci32 *)pos_l;
    auto SC = [&](int i) -> float {
        if constexpr (RES) return sc_s[i];
        else return sc_g[i];
    };
    auto PS = [&](int i) -> int32_t {
        if constexpr (RES) return pos_s[i];
        else return pos[i];
    };
    KD_TL_DECL
    KD_TL(0);
#ifdef KD_TIMELINE
    if (threadIdx.x == 0) kd_tl[31] = 2;   // record kind: selection workgroup
#define KD_SEL_RETURN do { KD_TL(12); KD_TL_DUMP(p.timeline, blockIdx.x); return; } while (0)
#else
#define KD_SEL_RETURN return
#endif

    // ---- 0. every load that does not depend on the selection is issued here, so that the chain
    // below costs one memory round trip now and one for the evicted rows later: the scores and
    // positions of all rows (asynchronous copies into LDS, 1 KB per wave and instruction; the buffers
    // hold a multiple of four rows), the running key sum, and (FILL layout) the K/V rows [N, n), the
    // only ones that can move, into registers.
    if (RES) {
        const int nchunks = (p.cap * 4 + 1023) / 1024;
        for (int c = wave; c < 2 * nchunks; c += NWAVES) {      // wave uniform
            const bool second = c >= nchunks;
            const int w0 = (second ? c - nchunks : c) * 256 + 4 * lane;   // first of this lane's four words
            const uint32_t dst = (uint32_t)(uintptr_t)(second ? (void *)pos_l : (void *)sc_l) + (uint32_t)(w0 - 4 * lane) * 4u;
            if (w0 < p.cap) lds_copy16(dst, second ? (const void *)(pos + w0) : (const void *)(sc_g + w0));
        }
    }
    const double ksum_old = tid < D ? p.ksum_next[(size_t)bh * D + tid] : 0.0;  // the sum step_main just wrote
    const bool tail_regs = p.layout == 1 && 2 * E * UPR <= TAILU * THREADS;
    u32x4 tailv[TAILU];
    if (tail_regs) {
#pragma unroll
        for (int q = 0; q < TAILU; ++q) {
            const int w = q * THREADS + tid;
            tailv[q] = u32x4{0u, 0u, 0u, 0u};
            if (q * THREADS < 2 * E * UPR && w < 2 * E * UPR) {
                const int which = w >= E * UPR, rem = w - which * E * UPR;
                tailv[q] = *reinterpret_cast<const u32x4 *>((which ? vb : kb) + (size_t)(p.N + rem / UPR) * D + (rem % UPR) * 8);
            }
        }
    }
    for (int i = tid; i < nwords; i += THREADS) evbits[i] = 0;
    const bool use_rec = E == 1 && p.argmax_rec != nullptr && p.window_W == 0 && 4 * p.splits <= HIST_BINS;   // uniform
    if (use_rec) {
        // the arg-max records of the attention launch travel with the loads above (the histogram's space
        // holds them: a single eviction builds no histogram)
        uint64_t *recs = reinterpret_cast<uint64_t *>(sh.hist);
        for (int s_ = tid; s_ < 2 * p.splits; s_ += THREADS) recs[s_] = p.argmax_rec[(size_t)bh * p.splits * 2 + s_];
    } else {
        for (int i = tid; i < HIST_BINS; i += THREADS) sh.hist[i] = 0;
    }
    if (tid == 0) {
        sh.ncand = 0;
        sh.nev = 0;
        sh.tb = 0;
        sh.need = 0;
    }
    KD_TL(1);   // loads issued
    if (RES) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // this wave's copies have landed
    __syncthreads();   // every wave's part of the copies; the cleared histogram and bitmap
    KD_TL(2);   // scores and positions in LDS

    if (E == 1) {
        // ---- 1'. a single row to evict (the generation phase): the arg-max by (score bits, position)
        // replaces histogram, threshold and ranking
        // The attention launch may have left the arg-max by (score bits, row) of every workgroup's rows
        // (p.argmax_rec): unless two rows share the largest score bits -- then the lower position has to
        // win, and positions are not row numbers -- the row to evict is read off those few records.
        uint64_t gbest = 0;
        bool known = false;
        if (use_rec) {
            if (tid == 0) {
                const uint64_t *recs = reinterpret_cast<const uint64_t *>(sh.hist);
                uint64_t b0 = 0;
                bool tie = false;
                for (int s_ = 0; s_ < p.splits; ++s_) {
                    const uint64_t ob = recs[2 * s_];
                    const bool ot = recs[2 * s_ + 1] != 0;
                    const uint32_t hb = (uint32_t)(b0 >> 32), ho = (uint32_t)(ob >> 32);
                    if (ho > hb) {
                        b0 = ob;
                        tie = ot;
                    } else if (ho == hb && ob != 0) {
                        tie = true;
                        b0 = ob > b0 ? ob : b0;
                    }
                }
                sh.sel_cnt = (b0 != 0 && !tie) ? 1u : 0u;
                sh.tb = (int)(uint32_t)b0;
                if (b0 != 0 && !tie) evbits[(uint32_t)b0 >> 5] |= 1u << ((uint32_t)b0 & 31);
            }
            __syncthreads();
            known = sh.sel_cnt != 0;   // uniform
            gbest = known ? 1 : 0;
        }
        if (!known) {
        uint64_t best = 0;   // 0: no row (every real key is larger: orderable() of a finite score is > 0)
        int besti = -1;
#pragma unroll 2
        for (int i = tid; i < p.n; i += THREADS) {
            const int32_t pi = PS(i);
            if (!(p.window_W > 0 && pi >= p.window_pos_min)) {
                const uint64_t key = ((uint64_t)orderable(SC(i)) << 32) | (uint32_t)pi;
                if (key > best) {
                    best = key;
                    besti = i;
                }
            }
        }
        uint64_t wbest = best;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const uint32_t lo = __shfl_xor((uint32_t)wbest, off), hi = __shfl_xor((uint32_t)(wbest >> 32), off);
            const uint64_t o = ((uint64_t)hi << 32) | lo;
            wbest = o > wbest ? o : wbest;
        }
        if (lane == 0) sh.wave_tot64[wave] = wbest;
        __syncthreads();
#pragma unroll
        for (int w = 0; w < NWAVES; ++w) gbest = sh.wave_tot64[w] > gbest ? sh.wave_tot64[w] : gbest;
        // positions are unique within a head, so exactly one thread holds the winning key
        if (besti >= 0 && best == gbest) {
            atomicOr(&evbits[besti >> 5], 1u << (besti & 31));
            sh.tb = besti;
        }
        __syncthreads();
        }   // !known
        if (p.layout == 1 && tail_regs && gbest != 0) {
            // FILL with the one tail row (row N, this step's token) in registers: the rest of the work
            // is one row read and at most one row moved, done here without lists
            const int e = sh.tb;
            double x[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) x[i] = 0.0;
            if (tid < UPR) {
                const u32x4 w = *reinterpret_cast<const u32x4 *>(kb + (size_t)e * D + tid * 8);
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    x[2 * i] = bf16_lo(w[i]);
                    x[2 * i + 1] = bf16_hi(w[i]);
                }
            }
            if (p.anchor_mode == 1 && tid < 64) {  // unit key: x / |k|; the row's UPR lanes are the first of wave 0
                double k2 = 0.0;
#pragma unroll
                for (int i = 0; i < 8; ++i) k2 += x[i] * x[i];
                k2 = row_allreduce_f64<UPR>(k2);
                const double nk = sqrt(k2);
                const double inv = nk > 0.0 ? 1.0 / nk : 0.0;
#pragma unroll
                for (int i = 0; i < 8; ++i) x[i] *= inv;
            }
            if (tid < UPR) {
#pragma unroll
                for (int i = 0; i < 8; ++i) sh.colsum[0][tid * 8 + i] = x[i];
            }
            // the evicted key has been read: its slot may take the tail row (the thread that read
            // unit u of K is the one that writes unit u of K)
            if (e != p.N && tid < 2 * UPR) {
                const int which = tid >= UPR, unit = tid - which * UPR;
                *reinterpret_cast<u32x4 *>((which ? vb : kb) + (size_t)e * D + unit * 8) = tailv[0];
                if (tid == 0) pos[e] = p.pos0 + (p.N - p.len);
            }
            __syncthreads();
            if (tid < D) p.ksum_next[(size_t)bh * D + tid] = ksum_old - sh.colsum[0][tid];
            KD_SEL_RETURN;
        }
    } else {
    // ---- 1. histogram of the non-exempt scores in LDS
#pragma unroll 2
    for (int i = tid; i < p.n; i += THREADS)
        if (!(p.window_W > 0 && PS(i) >= p.window_pos_min)) atomicAdd(&sh.hist[score_bin(SC(i))], 1u);
    __syncthreads();
    KD_TL(3);   // scores binned

    // ---- 2. threshold bin: thread t owns the HIST_BINS / THREADS bins below its top one, highest first
    uint32_t cnt[HIST_BINS / THREADS];
    uint32_t mine = 0;
    const int top = HIST_BINS - 1 - (HIST_BINS / THREADS) * tid;
#pragma unroll
    for (int j = 0; j < HIST_BINS / THREADS; ++j) {
        cnt[j] = sh.hist[top - j];
        mine += cnt[j];
    }
    uint32_t total;
    uint32_t above = block_exclusive_scan_t<THREADS, uint32_t>(mine, sh.wave_tot, &total);
    if (above < (uint32_t)E && above + mine >= (uint32_t)E) {
#pragma unroll
        for (int j = 0; j < HIST_BINS / THREADS; ++j) {
            if (above + cnt[j] >= (uint32_t)E) {
                sh.tb = top - j;
                sh.need = (uint32_t)E - above;
                break;
            }
            above += cnt[j];
        }
    }
    if (tid == 0 && total < (uint32_t)E) atomicOr(p.status, STATUS_SELECT_COUNT);  // cannot happen: E <= candidates
    __syncthreads();
    const int tb = sh.tb;
    const uint32_t need = sh.need;
    KD_TL(4);   // threshold bin known

    // above the bin -> evicted, inside it -> candidate for the exact ranking
#pragma unroll 2
    for (int i = tid; i < p.n; i += THREADS) {
        const int32_t pi = PS(i);
        const float s = SC(i);
        // bin of the row, -1 if it cannot be evicted (exempt)
        const int sb = !(p.window_W > 0 && pi >= p.window_pos_min) ? score_bin(s) : -1;
        if (sb > tb) atomicOr(&evbits[i >> 5], 1u << (i & 31));
        else if (sb == tb) {
            const uint32_t c = atomicAdd(&sh.ncand, 1u);
            if (c < CAND_MAX) {
                sh.cand_slot[c] = (uint32_t)i;
                sh.cand_key[c] = orderable(s);
                sh.cand_pos[c] = pi;
            }
        }
    }
    __syncthreads();
    const uint32_t ncand = sh.ncand;
    KD_TL(5);   // candidates collected

    // ---- 3. exact ranking inside the bin by (score bits, position), largest first: a wave takes a
    // candidate, its lanes compare it with 64 others at a time and count by ballot
    if (ncand <= CAND_MAX) {
        for (uint32_t c = wave; c < ncand; c += NWAVES) {   // uniform per wave
            const uint32_t key = sh.cand_key[c];
            const int32_t cp = sh.cand_pos[c];
            uint32_t rank = 0;
            for (uint32_t o0 = 0; o0 < ncand; o0 += 64) {
                const uint32_t o = o0 + lane;
                bool gt = false;
                if (o < ncand) {
                    const uint32_t ok = sh.cand_key[o];
                    gt = (ok > key) || (ok == key && sh.cand_pos[o] > cp);
                }
                rank += (uint32_t)__popcll(__ballot(gt));
            }
            if (lane == 0 && rank < need) {
                const uint32_t i = sh.cand_slot[c];
                atomicOr(&evbits[i >> 5], 1u << (i & 31));
            }
        }
        __syncthreads();
    } else {
        radix_select_in_bin<THREADS>(p, sh, RES ? sc_l : sc_g, RES ? pos_l : pos, evbits, tb, need);
    }
    }   // E > 1
    KD_TL(6);   // ranking done: the eviction bitmap is final

    // ---- 4. ordered lists: thread t owns bitmap word t = rows [32 t, 32 t + 32)
    const int own0 = min(p.n, 32 * tid), own1 = min(p.n, own0 + 32);
    const uint32_t valid = own1 - own0 == 32 ? 0xFFFFFFFFu : ((1u << (own1 - own0)) - 1u);
    const uint32_t low = own0 + 32 <= p.N ? 0xFFFFFFFFu : (own0 >= p.N ? 0u : ((1u << (p.N - own0)) - 1u));  // rows < N
    const uint32_t evw = tid < nwords ? (evbits[tid] & valid) : 0u;
    const uint32_t holew = evw & low, movew = ~evw & ~low & valid;
    uint64_t tot3;
    const uint64_t ex3 = block_exclusive_scan_t<THREADS, uint64_t>((uint64_t)__popc(evw) | ((uint64_t)__popc(holew) << 21) |
                                                    ((uint64_t)__popc(movew) << 42),
                                                sh.wave_tot64, &tot3);
    constexpr uint64_t M21 = (1ull << 21) - 1;
    uint32_t eb = (uint32_t)(ex3 & M21);
    const uint32_t hm_h = (uint32_t)((ex3 >> 21) & M21), hm_m = (uint32_t)((ex3 >> 42) & M21);
    const uint32_t tot_ev = (uint32_t)(tot3 & M21), nholes = (uint32_t)((tot3 >> 21) & M21),
                   nmov = (uint32_t)((tot3 >> 42) & M21);
    // an impossible count is reported and nothing is moved (keeps every index in range)
    const bool sane = tot_ev == (uint32_t)E && nholes == nmov;
    if (!sane) {
        if (tid == 0) atomicOr(p.status, STATUS_SELECT_COUNT);
        KD_SEL_RETURN;
    }
    // evicted rows | holes (evicted rows below N) | movers (kept rows from N on) | rank of tail row N + r
    // among the movers (-1: evicted)
    int32_t *evlist = lists, *holes = lists + E, *movers = lists + 2 * E, *mrank = lists + 3 * E;
    const bool tail_par = E <= THREADS && (nwords - (p.N >> 5)) <= TAIL_WORDS;
    {
        uint32_t hb = hm_h, mb = hm_m, e2 = eb;
        for (uint32_t w = evw; w; w &= w - 1) {
            const int i = own0 + __ffs(w) - 1;
            evlist[e2++] = i;
            if (i < p.N) holes[hb++] = i;
            else mrank[i - p.N] = -1;
        }
        // The tail rows [N, n) sit in a few words that are mostly movers: those words and their
        // mover counts before them go to LDS, and one thread per tail row finishes below.
        const int tw = tid - (p.N >> 5);
        if (tail_par) {
            if (tw >= 0 && tid < nwords) {
                sh.tail_word[tw] = movew;
                sh.tail_base[tw] = mb;
            }
        } else {
            for (uint32_t w = movew; w; w &= w - 1) {
                const int i = own0 + __ffs(w) - 1;
                mrank[i - p.N] = (int32_t)mb;
                movers[mb++] = i;
            }
        }
    }
    __syncthreads();
    if (tail_par && tid < E) {
        const int row = p.N + tid, tw = (row >> 5) - (p.N >> 5), bit = row & 31;
        const uint32_t mw = sh.tail_word[tw];
        if ((mw >> bit) & 1u) {
            const uint32_t r = sh.tail_base[tw] + (uint32_t)__popc(mw & ((1u << bit) - 1u));
            mrank[tid] = (int32_t)r;
            movers[r] = row;
        }   // an evicted tail row got its -1 above
    }
    // (the ranks are first read after the barrier inside step 5)
    KD_TL(7);   // lists written

    // ---- 5. take the evicted keys out of the running key sum (before rows are overwritten).
    // UPR lanes share an evicted row (16 bytes each); a wave holds 64/UPR rows at a time.
    {
        constexpr int RPW = 64 / UPR;
        const int u = lane % UPR, rl = lane / UPR;
        double acc[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[i] = 0.0;
        // the rows of up to EV_BATCH rounds are requested together: one memory round trip, not one per round
        constexpr int EV_BATCH = 4;
        for (int rb0 = wave * RPW; rb0 < E; rb0 += EV_BATCH * NWAVES * RPW) {  // uniform per wave
            u32x4 wv[EV_BATCH];
#pragma unroll
            for (int b = 0; b < EV_BATCH; ++b) {
                const int r = rb0 + b * NWAVES * RPW + rl;
                wv[b] = u32x4{0u, 0u, 0u, 0u};
                if (r < E) wv[b] = *reinterpret_cast<const u32x4 *>(kb + (size_t)evlist[r] * D + u * 8);
            }
#pragma unroll
            for (int b = 0; b < EV_BATCH; ++b) {
                if (rb0 + b * NWAVES * RPW >= E) break;   // uniform
                double x[8];
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    x[2 * i] = bf16_lo(wv[b][i]);
                    x[2 * i + 1] = bf16_hi(wv[b][i]);
                }
                double inv = 1.0;
                if (p.anchor_mode == 1) {  // unit key: x / |k|
                    double k2 = 0.0;
#pragma unroll
                    for (int i = 0; i < 8; ++i) k2 += x[i] * x[i];
                    k2 = row_allreduce_f64<UPR>(k2);
                    const double nk = sqrt(k2);
                    inv = nk > 0.0 ? 1.0 / nk : 0.0;
                }
#pragma unroll
                for (int i = 0; i < 8; ++i) acc[i] += (p.anchor_mode == 1) ? x[i] * inv : x[i];
            }
        }
        // fold the rows of the wave (lanes with equal u), then the waves
#pragma unroll
        for (int i = 0; i < 8; ++i) {
#pragma unroll
            for (int off = UPR; off < 64; off <<= 1) acc[i] += shfl_xor_f64(acc[i], off);
        }
        if (rl == 0) {
#pragma unroll
            for (int i = 0; i < 8; ++i) sh.colsum[wave][u * 8 + i] = acc[i];
        }
        __syncthreads();   // also: every evicted row has been read before the compaction overwrites it
        if (tid < D) {
            double s = 0.0;
#pragma unroll
            for (int w = 0; w < NWAVES; ++w) s += sh.colsum[w][tid];
            p.ksum_next[(size_t)bh * D + tid] = ksum_old - s;
        }
    }
    KD_TL(8);   // evicted rows read, key sum stored

    // ---- 6. compaction
    if (p.layout == 1) {
        // FILL: k-th surviving row of [N, n) moves into the k-th evicted slot of [0, N).  Rows from N
        // on belong to this step's block: row i holds token pos0 + (i - len).
        if (tail_regs) {
#pragma unroll
            for (int q = 0; q < TAILU; ++q) {
                const int w = q * THREADS + tid;
                if (q * THREADS < 2 * E * UPR && w < 2 * E * UPR) {
                    const int which = w >= E * UPR, rem = w - which * E * UPR;
                    const int mr = mrank[rem / UPR];
                    if (mr >= 0)
                        *reinterpret_cast<u32x4 *>((which ? vb : kb) + (size_t)holes[mr] * D + (rem % UPR) * 8) = tailv[q];
                }
            }
        } else {
            const int nmove = (int)nholes;
            for (int w = tid; w < nmove * UPR * 2; w += THREADS) {
                const int r = w / (UPR * 2), rem = w % (UPR * 2);
                const int u = rem % UPR;
                uint16_t *base_ptr = rem < UPR ? kb : vb;
                const u32x4 val = *reinterpret_cast<const u32x4 *>(base_ptr + (size_t)movers[r] * D + u * 8);
                *reinterpret_cast<u32x4 *>(base_ptr + (size_t)holes[r] * D + u * 8) = val;
            }
        }
        for (int r = tid; r < (int)nholes; r += THREADS) pos[holes[r]] = p.pos0 + (movers[r] - p.len);
    } else {
        // ORDERED: kept row i moves to i - (evicted rows before i); positions are compacted here, the
        // K/V rows by compact_ordered_kernel.  The evicted count before a row comes from the bitmap
        // and the per-word counts of the scan.  A position lands at or below the row it came from,
        // and the rows are taken in ascending chunks: reading from the LDS copy nothing can be
        // overwritten before it is read; reading from memory, a chunk is read, then (barrier) written.
        uint32_t *word_base = sh.cand_slot;   // the candidate arrays are free by now
        static_assert(MAX_CAP / 32 <= CAND_MAX, "one count per bitmap word");
        if (tid < nwords) word_base[tid] = eb;
        __syncthreads();
        int32_t *dst = p.dstmap + (size_t)bh * p.cap;
        for (int i0 = 0; i0 < p.n; i0 += THREADS) {   // uniform
            const int i = i0 + tid;
            const int32_t pi = i < p.n ? PS(i) : 0;
            if (!RES) __syncthreads();
            if (i < p.n) {
                const uint32_t word = evbits[i >> 5], bit = (uint32_t)i & 31u;
                if ((word >> bit) & 1u) dst[i] = -1;
                else {
                    const int to = i - (int)(word_base[i >> 5] + (uint32_t)__popc(word & ((1u << bit) - 1u)));
                    dst[i] = to;
                    pos[to] = pi;
                }
            }
        }
    }
    KD_TL(9);   // moves issued
#ifdef KD_TIMELINE
    __builtin_amdgcn_s_waitcnt(0x0F70);
    KD_SEL_RETURN;
#endif
#undef KD_SEL_RETURN
}

}  // namespace kd
