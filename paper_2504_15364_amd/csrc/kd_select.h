// Selection of the rows to evict and compaction of one head (Eq. 6-7), as device code shared by
// the kernels that can run it: step_post (one workgroup of 1024 threads per head) and the variant of
// step_main that carries another cache's pending eviction (workgroups of 512 threads).
//
// One workgroup loads the head's scores once, bins them into a 4096-bin LDS histogram (a monotone
// map of the float), scans it for the bin that holds the E-th largest score, evicts everything
// above that bin and ranks the few rows inside it exactly by (score bits, position): equal scores
// keep the lower position.  It then compacts the cache and takes the evicted keys out of ksum.
#pragma once
#include "kd_kernels.h"
#include "kd_device.h"

namespace kd {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef int32_t i32x4 __attribute__((ext_vector_type(4)));

constexpr int CAND_MAX = 2048;  // rows of the threshold bin ranked in LDS; more fall back to a radix select
constexpr int MAX_SELECT_WAVES = POST_THREADS / 64;   // PostShared is laid out for the largest workgroup
constexpr int TAIL_WORDS = 72;                      // bitmap words the tail rows [N, n) may span on the fast path
constexpr int SPT_SMALL = 12;                       // scores per thread: caches of up to 12288 rows
constexpr int SPT_LARGE = MAX_CAP / POST_THREADS;   // ... and up to the limit
constexpr int CARRY_THREADS = 512;                  // workgroup size of the step_main variant that carries a selection
constexpr int SPT_CARRY = 24;                       // ... which covers caches of up to 12288 rows as well

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
// that bin; reads scores and positions from memory on every pass.  Marks the
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

// ------------------------------------------------------------- select + compaction
// `lists` holds three arrays of E row indices (evicted | holes | movers): in LDS when
// they fit, else in the scratch buffer.
// SPT: scores per thread the instantiation can hold (n <= SPT * THREADS); the caller also keeps
// n <= 32 * THREADS (a thread owns one word of the eviction bitmap)
template <int D, int SPT, int THREADS>
__device__ void select_and_compact(const StepParams &p, PostShared &sh, uint32_t *evbits, int32_t *lists, int bh)
{
    constexpr int UPR = D / 8;
    // 16-byte units of the tail rows a thread keeps in registers (the large instantiation has none to spare)
    constexpr int TAILU = SPT * THREADS < MAX_CAP ? 8 : 0;
    constexpr int NWAVES = THREADS / 64;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int E = p.n - p.N;
    const float *sc = p.scores + (size_t)bh * p.cap;
    int32_t *pos = p.pos + (size_t)bh * p.cap;
    uint16_t *kb = p.k + (size_t)bh * p.cap * D;
    uint16_t *vb = p.v + (size_t)bh * p.cap * D;
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
    // positions of all rows, the running key sum, and (FILL layout) the K/V rows [N, n), the only
    // ones that can move.
    // A thread takes groups of four consecutive rows (one 16-byte load each for scores and positions:
    // the memory pipeline spends the same time on a wave's load whatever its width): slot k of a
    // thread is row 4 ((k / 4) THREADS + tid) + k % 4.  The buffers hold a multiple of four rows.
    static_assert(SPT % 4 == 0, "slots come in groups of four");
    auto row_of = [&](int k) { return 4 * ((k >> 2) * THREADS + tid) + (k & 3); };
    auto group_live = [&](int k) { return 4 * (k >> 2) * THREADS < p.n; };   // uniform: some thread has rows there
    float sv[SPT];
    int32_t sp[SPT];
#pragma unroll
    for (int g = 0; g < SPT / 4; ++g) {
        const int r0 = 4 * (g * THREADS + tid);
        f32x4 s4 = {0.f, 0.f, 0.f, 0.f};
        i32x4 p4 = {0, 0, 0, 0};
        if (4 * g * THREADS < p.n && r0 < p.n) {
            s4 = *reinterpret_cast<const f32x4 *>(sc + r0);
            p4 = *reinterpret_cast<const i32x4 *>(pos + r0);
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            sv[4 * g + j] = s4[j];
            sp[4 * g + j] = p4[j];
        }
    }
    const double ksum_old = tid < D ? p.ksum_next[(size_t)bh * D + tid] : 0.0;  // the sum step_main just wrote
    const bool tail_regs = TAILU > 0 && p.layout == 1 && 2 * E * UPR <= TAILU * THREADS;
    u32x4 tailv[TAILU > 0 ? TAILU : 1];
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

    KD_TL(1);   // loads issued
    const int nwords = (p.n + 31) / 32;
    if (E == 1) {
        // ---- 1'. a single row to evict (the generation phase): the arg-max by (score bits, position)
        // replaces histogram, threshold and ranking
        for (int i = tid; i < nwords; i += THREADS) evbits[i] = 0;
        uint64_t best = 0;   // 0: no row (every real key is larger: orderable() of a finite score is > 0)
        int besti = -1;
#pragma unroll
        for (int k = 0; k < SPT; ++k) {
            const int i = row_of(k);
            if (!group_live(k)) break;
            if (i < p.n && !(p.window_W > 0 && sp[k] >= p.window_pos_min)) {
                const uint64_t key = ((uint64_t)orderable(sv[k]) << 32) | (uint32_t)sp[k];
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
        __syncthreads();   // also: the bitmap is clear
        uint64_t gbest = 0;
#pragma unroll
        for (int w = 0; w < NWAVES; ++w) gbest = sh.wave_tot64[w] > gbest ? sh.wave_tot64[w] : gbest;
        // positions are unique within a head, so exactly one thread holds the winning key
        if (besti >= 0 && best == gbest) {
            atomicOr(&evbits[besti >> 5], 1u << (besti & 31));
            sh.tb = besti;
        }
        __syncthreads();
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
    KD_TL(2);
    for (int i = tid; i < nwords; i += THREADS) evbits[i] = 0;
    for (int i = tid; i < HIST_BINS; i += THREADS) sh.hist[i] = 0;
    if (tid == 0) {
        sh.ncand = 0;
        sh.nev = 0;
        sh.tb = 0;
        sh.need = 0;
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < SPT; ++k) {
        const int i = row_of(k);
        if (!group_live(k)) break;
        if (i < p.n && !(p.window_W > 0 && sp[k] >= p.window_pos_min)) atomicAdd(&sh.hist[score_bin(sv[k])], 1u);
    }
    __syncthreads();

    KD_TL(3);   // scores arrived and binned
    // ---- 2. threshold bin: thread t owns the 4 bins below 4*(1023-t)+3, highest first
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
#pragma unroll
    for (int k = 0; k < SPT; ++k) {
        const int i = row_of(k);
        if (!group_live(k)) break;
        // bin of the row, -1 if it cannot be evicted (exempt or past the end)
        const int sb = (i < p.n && !(p.window_W > 0 && sp[k] >= p.window_pos_min)) ? score_bin(sv[k]) : -1;
        if (sb > tb) atomicOr(&evbits[i >> 5], 1u << (i & 31));
        else if (sb == tb) {
            const uint32_t c = atomicAdd(&sh.ncand, 1u);
            if (c < CAND_MAX) {
                sh.cand_slot[c] = (uint32_t)i;
                sh.cand_key[c] = orderable(sv[k]);
                sh.cand_pos[c] = sp[k];
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
            const int32_t ps = sh.cand_pos[c];
            uint32_t rank = 0;
            for (uint32_t o0 = 0; o0 < ncand; o0 += 64) {
                const uint32_t o = o0 + lane;
                bool gt = false;
                if (o < ncand) {
                    const uint32_t ok = sh.cand_key[o];
                    gt = (ok > key) || (ok == key && sh.cand_pos[o] > ps);
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
        radix_select_in_bin<THREADS>(p, sh, sc, pos, evbits, tb, need);
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
        // ORDERED: kept row i moves to i - (evicted rows before i); positions are compacted here
        // (they were all read into registers at the start), the K/V rows by compact_ordered_kernel.
        // Every thread handles the rows it loaded (groups of four consecutive rows: coalesced), with
        // the evicted count before a row taken from the bitmap and the per-word counts of the scan.
        uint32_t *word_base = sh.cand_slot;   // the candidate arrays are free by now; nwords <= CAND_MAX
        static_assert(MAX_CAP / 32 <= CAND_MAX, "one count per bitmap word");
        if (tid < nwords) word_base[tid] = eb;
        __syncthreads();
        int32_t *dst = p.dstmap + (size_t)bh * p.cap;
#pragma unroll
        for (int k = 0; k < SPT; ++k) {
            const int i = row_of(k);
            if (!group_live(k)) break;
            if (i < p.n) {
                const uint32_t word = evbits[i >> 5], bit = (uint32_t)i & 31u;
                if ((word >> bit) & 1u) dst[i] = -1;
                else {
                    const int to = i - (int)(word_base[i >> 5] + (uint32_t)__popc(word & ((1u << bit) - 1u)));
                    dst[i] = to;
                    pos[to] = sp[k];
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
