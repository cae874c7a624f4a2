// step_post: selection and compaction (Eq. 6-7) running next to the log-sum-exp merge of the
// attention partials; step_score: the cosine score (appendix "FLOP count of KeyDiff") of a cache
// outside a block step (inside one, step_main scores the keys while it holds them in LDS).
//
// The score that decides an eviction is IEEE double arithmetic on the bf16 data,
// rounded once to float: s_i = mu.k_i / max(|mu||k_i|, eps) with mu = ksum / n, so
// the retained set does not depend on summation order beyond the last bit of a double.
//
// Selection.  One workgroup per head loads the head's scores once, bins them into a
// 4096-bin LDS histogram (a monotone map of the float), scans it for the bin that
// holds the E-th largest score, evicts everything above that bin and ranks the few
// rows inside it exactly by (score bits, position): equal scores keep the lower
// position.  It then compacts the cache and takes the evicted keys out of ksum.
#include "kd_kernels.h"
#include "kd_device.h"

namespace kd {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));

constexpr int CAND_MAX = 2048;  // rows of the threshold bin ranked in LDS; more fall back to a radix select
constexpr int NWAVES = POST_THREADS / 64;
constexpr int TAIL_WORDS = 72;                      // bitmap words the tail rows [N, n) may span on the fast path
constexpr int SPT_SMALL = 12;                       // scores per thread: caches of up to 12288 rows
constexpr int SPT_LARGE = MAX_CAP / POST_THREADS;   // ... and up to the limit
constexpr int SCORE_WAVES = SCORE_THREADS / 64;

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
    uint32_t wave_tot[NWAVES];
    uint64_t wave_tot64[NWAVES];
    uint32_t radix_hist[256];
    uint32_t sel_bin, sel_rank, sel_cnt;
    int tb;           // threshold bin
    uint32_t need;    // rows to evict from the threshold bin
    uint32_t ncand, nev;
    uint32_t cand_slot[CAND_MAX];
    uint32_t cand_key[CAND_MAX];
    int32_t cand_pos[CAND_MAX];
    double colsum[NWAVES][128];
    uint32_t tail_word[TAIL_WORDS], tail_base[TAIL_WORDS];  // mover bitmap words of rows >= N and movers before each
};

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
template <typename T>
__device__ __forceinline__ T block_exclusive_scan_t(T v, T *wave_tot, T *total)
{
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
__device__ __forceinline__ uint32_t block_exclusive_scan(uint32_t v, uint32_t *wave_tot, uint32_t *total)
{
    return block_exclusive_scan_t<uint32_t>(v, wave_tot, total);
}
__device__ __forceinline__ uint64_t block_exclusive_scan64(uint64_t v, uint64_t *wave_tot, uint64_t *total)
{
    return block_exclusive_scan_t<uint64_t>(v, wave_tot, total);
}

// ------------------------------------------------------------------------ scores
struct ScoreShared {
    double mu[128];
    double red[SCORE_WAVES];
    double dot[SCORE_WAVES][64];  // per-wave staging of (mu.k, |k|^2) so that sqrt and divide run on full waves
    double k2[SCORE_WAVES][64];
};

// Rows [row0, row1) of head bh.  D/8 lanes share a row (one 16-byte unit each); a wave takes 64
// consecutive rows per round, stages (mu.k, |k|^2) of each row in LDS and then lane i finishes
// row i of the round.
template <int D>
__device__ __forceinline__ void score_rows(const StepParams &p, ScoreShared &sh, int bh, int row0, int row1)
{
    constexpr int UPR = D / 8;
    constexpr int RPW = 64 / UPR;  // rows per wave per pass
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int u = lane % UPR, rl = lane / UPR;
    const uint16_t *kb = p.k + (size_t)bh * p.cap * D;
    // the rows of the first round are requested before the anchor is formed: the two memory
    // round trips (key sum, rows) then overlap
    auto load_round = [&](int base, u32x4 (&w)[UPR]) {
#pragma unroll
        for (int ps = 0; ps < UPR; ++ps) {
            const int row = base + ps * RPW + rl;
            u32x4 z = {0u, 0u, 0u, 0u};
            if (row < row1) z = *reinterpret_cast<const u32x4 *>(kb + (size_t)row * D + u * 8);
            w[ps] = z;
        }
    };
    const int base0 = row0 + wave * 64;
    u32x4 w[UPR];
    load_round(base0, w);
    // anchor = ksum / n (Method, "Efficient Variant"); |mu| by a fixed-shape reduction
    double m = 0.0;
    if (tid < D) {
        m = p.ksum[(size_t)bh * D + tid] / (double)p.n;
        sh.mu[tid] = m;
    }
    double sq = m * m;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) sq += shfl_xor_f64(sq, off);
    if (lane == 0) sh.red[wave] = sq;
    __syncthreads();
    double mu2 = 0.0;
#pragma unroll
    for (int w = 0; w < SCORE_WAVES; ++w) mu2 += sh.red[w];
    const double nmu = sqrt(mu2);

    double mreg[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) mreg[i] = sh.mu[u * 8 + i];
    // a round = 64 rows per wave; rounds are spread over the waves
    for (int base = base0; base < row1; base += SCORE_WAVES * 64) {
        if (base != base0) load_round(base, w);  // the round's loads are issued together
#pragma unroll
        for (int ps = 0; ps < UPR; ++ps) {
            double dot = 0.0, k2 = 0.0;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const double a = bf16_lo(w[ps][i]), b = bf16_hi(w[ps][i]);
                dot += mreg[2 * i] * a;
                k2 += a * a;
                dot += mreg[2 * i + 1] * b;
                k2 += b * b;
            }
            dot = row_allreduce_f64<UPR>(dot);
            k2 = row_allreduce_f64<UPR>(k2);
            if (u == 0) {
                sh.dot[wave][ps * RPW + rl] = dot;
                sh.k2[wave][ps * RPW + rl] = k2;
            }
        }
        // same wave wrote and reads: the LDS accesses of one wave complete in order; the fence only
        // keeps the compiler from moving the reads above the writes
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        const int row = base + lane;
        if (row < row1) {
            const double dot = sh.dot[wave][lane], k2 = sh.k2[wave][lane];
            const float s = finish_score(dot, k2, nmu, p.eps);
            p.scores[(size_t)bh * p.cap + row] = s;
            if (p.scores_out) p.scores_out[(size_t)bh * p.n + row] = s;
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    }
}

// ---------------------------------------------------- slow path: radix select in a bin
// More than CAND_MAX rows share the threshold bin (near-identical keys).  MSB-first
// 8-bit radix select over the 64-bit key (orderable score : position) restricted to
// that bin; reads scores and positions from memory on every pass.  Marks the
// `need` largest in the evict bitmap.
__device__ void radix_select_in_bin(const StepParams &p, PostShared &sh, const float *sc, const int32_t *pos,
                                    uint32_t *evbits, int tb, uint32_t need)
{
    const int tid = threadIdx.x, lane = tid & 63;
    uint64_t prefix = 0;
    uint32_t rank = need;
    int resolved = 0;
    for (int pass = 0; pass < 8; ++pass) {
        const int shift = 56 - 8 * pass;
        for (int i = tid; i < 256; i += POST_THREADS) sh.radix_hist[i] = 0;
        __syncthreads();
        for (int i0 = 0; i0 < p.n; i0 += POST_THREADS) {
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
    for (int i = tid; i < p.n; i += POST_THREADS) {
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
// SPT: scores per thread the instantiation can hold (n <= SPT * POST_THREADS)
template <int D, int SPT>
__device__ void select_and_compact(const StepParams &p, PostShared &sh, uint32_t *evbits, int32_t *lists, int bh)
{
    constexpr int UPR = D / 8;
    // 16-byte units of the tail rows a thread keeps in registers (the large instantiation has none to spare)
    constexpr int TAILU = SPT * POST_THREADS < MAX_CAP ? 8 : 0;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int E = p.n - p.N;
    const float *sc = p.scores + (size_t)bh * p.cap;
    int32_t *pos = p.pos + (size_t)bh * p.cap;
    uint16_t *kb = p.k + (size_t)bh * p.cap * D;
    uint16_t *vb = p.v + (size_t)bh * p.cap * D;

    // ---- 0. every load that does not depend on the selection is issued here, so that the chain
    // below costs one memory round trip now and one for the evicted rows later: the scores and
    // positions of all rows, the running key sum, and (FILL layout) the K/V rows [N, n), the only
    // ones that can move.
    float sv[SPT];
    int32_t sp[SPT];
#pragma unroll
    for (int k = 0; k < SPT; ++k) {
        const int i = k * POST_THREADS + tid;
        sv[k] = 0.f;
        sp[k] = 0;
        if (k * POST_THREADS < p.n && i < p.n) {
            sv[k] = sc[i];
            sp[k] = pos[i];
        }
    }
    const double ksum_old = tid < D ? p.ksum_next[(size_t)bh * D + tid] : 0.0;  // the sum step_main just wrote
    const bool tail_regs = TAILU > 0 && p.layout == 1 && 2 * E * UPR <= TAILU * POST_THREADS;
    u32x4 tailv[TAILU > 0 ? TAILU : 1];
    if (tail_regs) {
#pragma unroll
        for (int q = 0; q < TAILU; ++q) {
            const int w = q * POST_THREADS + tid;
            tailv[q] = u32x4{0u, 0u, 0u, 0u};
            if (q * POST_THREADS < 2 * E * UPR && w < 2 * E * UPR) {
                const int which = w >= E * UPR, rem = w - which * E * UPR;
                tailv[q] = *reinterpret_cast<const u32x4 *>((which ? vb : kb) + (size_t)(p.N + rem / UPR) * D + (rem % UPR) * 8);
            }
        }
    }

    // ---- 1. histogram of the non-exempt scores in LDS
    const int nwords = (p.n + 31) / 32;
    for (int i = tid; i < nwords; i += POST_THREADS) evbits[i] = 0;
    for (int i = tid; i < HIST_BINS; i += POST_THREADS) sh.hist[i] = 0;
    if (tid == 0) {
        sh.ncand = 0;
        sh.nev = 0;
        sh.tb = 0;
        sh.need = 0;
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < SPT; ++k) {
        const int i = k * POST_THREADS + tid;
        if (k * POST_THREADS >= p.n) break;
        if (i < p.n && !(p.window_W > 0 && sp[k] >= p.window_pos_min)) atomicAdd(&sh.hist[score_bin(sv[k])], 1u);
    }
    __syncthreads();

    // ---- 2. threshold bin: thread t owns the 4 bins below 4*(1023-t)+3, highest first
    uint32_t cnt[HIST_BINS / POST_THREADS];
    uint32_t mine = 0;
    const int top = HIST_BINS - 1 - (HIST_BINS / POST_THREADS) * tid;
#pragma unroll
    for (int j = 0; j < HIST_BINS / POST_THREADS; ++j) {
        cnt[j] = sh.hist[top - j];
        mine += cnt[j];
    }
    uint32_t total;
    uint32_t above = block_exclusive_scan(mine, sh.wave_tot, &total);
    if (above < (uint32_t)E && above + mine >= (uint32_t)E) {
#pragma unroll
        for (int j = 0; j < HIST_BINS / POST_THREADS; ++j) {
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

    // above the bin -> evicted, inside it -> candidate for the exact ranking
#pragma unroll
    for (int k = 0; k < SPT; ++k) {
        const int i = k * POST_THREADS + tid;
        if (k * POST_THREADS >= p.n) break;
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
        radix_select_in_bin(p, sh, sc, pos, evbits, tb, need);
    }

    // ---- 4. ordered lists: thread t owns bitmap word t = rows [32 t, 32 t + 32)
    static_assert(MAX_CAP / 32 <= POST_THREADS, "one bitmap word per thread");
    const int own0 = min(p.n, 32 * tid), own1 = min(p.n, own0 + 32);
    const uint32_t valid = own1 - own0 == 32 ? 0xFFFFFFFFu : ((1u << (own1 - own0)) - 1u);
    const uint32_t low = own0 + 32 <= p.N ? 0xFFFFFFFFu : (own0 >= p.N ? 0u : ((1u << (p.N - own0)) - 1u));  // rows < N
    const uint32_t evw = tid < nwords ? (evbits[tid] & valid) : 0u;
    const uint32_t holew = evw & low, movew = ~evw & ~low & valid;
    uint64_t tot3;
    const uint64_t ex3 = block_exclusive_scan64((uint64_t)__popc(evw) | ((uint64_t)__popc(holew) << 21) |
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
        return;
    }
    // evicted rows | holes (evicted rows below N) | movers (kept rows from N on) | rank of tail row N + r
    // among the movers (-1: evicted)
    int32_t *evlist = lists, *holes = lists + E, *movers = lists + 2 * E, *mrank = lists + 3 * E;
    const bool tail_par = E <= POST_THREADS && (nwords - (p.N >> 5)) <= TAIL_WORDS;
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

    // ---- 5. take the evicted keys out of the running key sum (before rows are overwritten).
    // UPR lanes share an evicted row (16 bytes each); a wave holds 64/UPR rows at a time.
    {
        constexpr int RPW = 64 / UPR;
        const int u = lane % UPR, rl = lane / UPR;
        double acc[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[i] = 0.0;
        for (int rb = wave * RPW; rb < E; rb += NWAVES * RPW) {  // uniform per wave
            const int r = rb + rl;
            double x[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) x[i] = 0.0;
            if (r < E) {
                const u32x4 w = *reinterpret_cast<const u32x4 *>(kb + (size_t)evlist[r] * D + u * 8);
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    x[2 * i] = bf16_lo(w[i]);
                    x[2 * i + 1] = bf16_hi(w[i]);
                }
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

    // ---- 6. compaction
    if (p.layout == 1) {
        // FILL: k-th surviving row of [N, n) moves into the k-th evicted slot of [0, N).  Rows from N
        // on belong to this step's block: row i holds token pos0 + (i - len).
        if (tail_regs) {
#pragma unroll
            for (int q = 0; q < TAILU; ++q) {
                const int w = q * POST_THREADS + tid;
                if (q * POST_THREADS < 2 * E * UPR && w < 2 * E * UPR) {
                    const int which = w >= E * UPR, rem = w - which * E * UPR;
                    const int mr = mrank[rem / UPR];
                    if (mr >= 0)
                        *reinterpret_cast<u32x4 *>((which ? vb : kb) + (size_t)holes[mr] * D + (rem % UPR) * 8) = tailv[q];
                }
            }
        } else {
            const int nmove = (int)nholes;
            for (int w = tid; w < nmove * UPR * 2; w += POST_THREADS) {
                const int r = w / (UPR * 2), rem = w % (UPR * 2);
                const int u = rem % UPR;
                uint16_t *base_ptr = rem < UPR ? kb : vb;
                const u32x4 val = *reinterpret_cast<const u32x4 *>(base_ptr + (size_t)movers[r] * D + u * 8);
                *reinterpret_cast<u32x4 *>(base_ptr + (size_t)holes[r] * D + u * 8) = val;
            }
        }
        for (int r = tid; r < (int)nholes; r += POST_THREADS) pos[holes[r]] = p.pos0 + (movers[r] - p.len);
    } else {
        // ORDERED: kept row i moves to i - (evicted rows before i); positions are compacted here
        // (all reads precede all writes), the K/V rows by compact_ordered_kernel.
        int32_t mypos[32];
        int32_t *dst = p.dstmap + (size_t)bh * p.cap;
        for (int i = own0, j = 0; i < own1; ++i, ++j) mypos[j] = pos[i];
        __syncthreads();
        for (int i = own0, j = 0; i < own1; ++i, ++j) {
            const bool ev = (evw >> j) & 1u;
            if (ev) {
                dst[i] = -1;
                ++eb;
            } else {
                dst[i] = i - (int)eb;
                pos[i - (int)eb] = mypos[j];
            }
        }
    }
}

// ------------------------------------------------------------------------ merge
template <int D>
__device__ __forceinline__ void merge_rows(const StepParams &p, size_t gid)
{
    const int BH = p.batch * p.hkv;
    const int Mtot = p.G * p.Bt;
    const size_t rows = (size_t)BH * Mtot;
    const int d4 = (int)(gid % (D / 4));
    const size_t row = gid / (D / 4);
    if (row >= rows) return;
    // the loads of a batch of splits are issued together: a serial chain would cost a memory
    // round trip per split
    constexpr int MB = 8;
    float mx = -INFINITY;
    for (int s0 = 0; s0 < p.splits; s0 += MB) {
        float2 ml[MB];
#pragma unroll
        for (int i = 0; i < MB; ++i)
            ml[i] = s0 + i < p.splits ? p.part_ml[(size_t)(s0 + i) * rows + row] : make_float2(-INFINITY, 0.f);
#pragma unroll
        for (int i = 0; i < MB; ++i) mx = fmaxf(mx, ml[i].x);
    }
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    float L = 0.f;
    for (int s0 = 0; s0 < p.splits; s0 += MB) {
        float2 ml[MB];
        f16x4 o[MB];
#pragma unroll
        for (int i = 0; i < MB; ++i) {
            const bool live = s0 + i < p.splits;
            const f16x4 zero = {(_Float16)0.f, (_Float16)0.f, (_Float16)0.f, (_Float16)0.f};
            ml[i] = live ? p.part_ml[(size_t)(s0 + i) * rows + row] : make_float2(-INFINITY, 0.f);
            o[i] = live ? *reinterpret_cast<const f16x4 *>(p.part_o + ((size_t)(s0 + i) * rows + row) * D + 4 * d4) : zero;
        }
#pragma unroll
        for (int i = 0; i < MB; ++i) {
            // a partial is its split's output normalised by its own row sum: weight it by that sum
            const float w = ml[i].x == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(ml[i].x - mx) * ml[i].y;
            acc.x += w * (float)o[i][0];
            acc.y += w * (float)o[i][1];
            acc.z += w * (float)o[i][2];
            acc.w += w * (float)o[i][3];
            L += w;
        }
    }
    const float inv = 1.f / L;
    const int bh = (int)(row / Mtot), m = (int)(row % Mtot);
    const int b = bh / p.hkv, kvh = bh % p.hkv;
    const int g = m / p.Bt, j = m % p.Bt;
    bf16x4 o;
    o[0] = (__bf16)(acc.x * inv);
    o[1] = (__bf16)(acc.y * inv);
    o[2] = (__bf16)(acc.z * inv);
    o[3] = (__bf16)(acc.w * inv);
    *reinterpret_cast<bf16x4 *>(p.out + ((size_t)(b * p.hq + kvh * p.G + g) * p.Bt + j) * D + 4 * d4) = o;
}

// step_score: every workgroup scores SCORE_ROWS rows of one head.  The launch boundary after it
// makes the scores visible to step_post.
template <int D>
__global__ __launch_bounds__(SCORE_THREADS) void step_score_kernel(StepParams p)
{
    __shared__ ScoreShared sh;
    const int BH = p.batch * p.hkv;
    const int bh = blockIdx.x % BH, chunk = blockIdx.x / BH;
    const int row0 = chunk * SCORE_ROWS, row1 = min(p.n, row0 + SCORE_ROWS);
    score_rows<D>(p, sh, bh, row0, row1);
}

// step_post: workgroups [0, BH) select and compact one head each (when this step evicts); the
// rest merge the attention partials.
template <int D, int SPT>
__global__ __launch_bounds__(POST_THREADS) void step_post_kernel(StepParams p)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    __shared__ PostShared sh;
    const int n_select = p.do_evict ? p.batch * p.hkv : 0;
    if ((int)blockIdx.x >= n_select) {
        merge_rows<D>(p, (size_t)(blockIdx.x - n_select) * POST_THREADS + threadIdx.x);
        return;
    }
    const int bh = blockIdx.x;
    uint32_t *evbits = reinterpret_cast<uint32_t *>(smem_raw);
    int32_t *lists = p.lists_in_lds ? reinterpret_cast<int32_t *>(evbits + (p.n + 31) / 32)
                                    : p.lists + (size_t)bh * 4 * p.B;
    select_and_compact<D, SPT>(p, sh, evbits, lists, bh);
}

// ------------------------------------------------------------- ordered compaction
// Stable in-place shift: kept row i moves to dst[i] = i - (evicted rows before i), so a row moves
// down by at most E = n - N rows.  One workgroup per ORD_ROWS rows reads its moving rows into
// registers, announces that (flag = epoch of this launch), waits until the workgroups whose rows
// it may overwrite -- the ceil(E / ORD_ROWS) chunks before it -- have announced the same, and
// stores.  Workgroups are numbered chunk-major, so a workgroup only ever waits for lower-numbered
// ones; the wait is bounded and reports a timeout in the status word instead of hanging.
template <int D>
__global__ __launch_bounds__(1024) void compact_ordered_kernel(StepParams p, int32_t *flags, int nchunks, int32_t epoch)
{
    constexpr int UPR = D / 8;
    constexpr int UPT = ORD_ROWS * UPR * 2 / 1024;   // 16-byte units (K and V) per thread
    static_assert(UPT * 1024 == ORD_ROWS * UPR * 2, "the chunk must divide over the threads");
    const int BH = p.batch * p.hkv;
    const int bh = blockIdx.x % BH, chunk = blockIdx.x / BH, tid = threadIdx.x;
    uint16_t *kb = p.k + (size_t)bh * p.cap * D;
    uint16_t *vb = p.v + (size_t)bh * p.cap * D;
    const int32_t *dst = p.dstmap + (size_t)bh * p.cap;
    const int r0 = chunk * ORD_ROWS;
    u32x4 val[UPT];
    int drow[UPT];
#pragma unroll
    for (int q = 0; q < UPT; ++q) {
        const int w = q * 1024 + tid;
        const int which = w >= ORD_ROWS * UPR, rem = w - which * ORD_ROWS * UPR;
        const int row = r0 + rem / UPR, u = rem % UPR;
        drow[q] = -1;
        val[q] = u32x4{0u, 0u, 0u, 0u};
        if (row < p.n) {
            const int d = dst[row];
            if (d >= 0 && d != row) {
                drow[q] = d;
                val[q] = *reinterpret_cast<const u32x4 *>((which ? vb : kb) + (size_t)row * D + u * 8);
            }
        }
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // every row of this chunk is in registers
    __syncthreads();
    int32_t *myflags = flags + (size_t)bh * nchunks;
    if (tid == 0) __hip_atomic_store(&myflags[chunk], epoch, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    const int reach = (p.n - p.N + ORD_ROWS - 1) / ORD_ROWS;   // chunks below this one its rows can land in
    if (tid < reach && chunk - 1 - tid >= 0) {
        int spins = 0;
        while (__hip_atomic_load(&myflags[chunk - 1 - tid], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != epoch) {
            if (++spins > ORD_SPIN_LIMIT) {
                atomicOr(p.status, STATUS_ORDER_TIMEOUT);
                break;
            }
            __builtin_amdgcn_s_sleep(8);
        }
    }
    __syncthreads();
#pragma unroll
    for (int q = 0; q < UPT; ++q) {
        const int w = q * 1024 + tid;
        const int which = w >= ORD_ROWS * UPR, rem = w - which * ORD_ROWS * UPR;
        if (drow[q] >= 0)
            *reinterpret_cast<u32x4 *>((which ? vb : kb) + (size_t)drow[q] * D + (rem % UPR) * 8) = val[q];
    }
}

// --------------------------------------------------- key sum from scratch (cache load)
// Column sums of CHUNK_ROWS rows in double; unit keys for anchor mode 1.
template <int D>
__global__ __launch_bounds__(256) void ksum_partial_kernel(StepParams p, double *partials, int nchunks)
{
    constexpr int UPR = D / 8;
    constexpr int RL = 256 / UPR;
    __shared__ double red[RL][D];
    const int bh = blockIdx.y, chunk = blockIdx.x;
    const int u = threadIdx.x % UPR, rl = threadIdx.x / UPR;
    const uint16_t *kb = p.k + (size_t)bh * p.cap * D;
    double acc[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) acc[i] = 0.0;
    const int r0 = chunk * CHUNK_ROWS;
    for (int r = rl; r < CHUNK_ROWS; r += RL) {
        const int row = r0 + r;
        double x[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) x[i] = 0.0;
        if (row < p.n) {
            const u32x4 w = *reinterpret_cast<const u32x4 *>(kb + (size_t)row * D + u * 8);
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                x[2 * i] = bf16_lo(w[i]);
                x[2 * i + 1] = bf16_hi(w[i]);
            }
        }
        double inv = 1.0;
        if (p.anchor_mode == 1) {
            double k2 = 0.0;
#pragma unroll
            for (int i = 0; i < 8; ++i) k2 += x[i] * x[i];
#pragma unroll
            for (int m = 1; m < UPR; m <<= 1) k2 += shfl_xor_f64(k2, m);
            const double nk = sqrt(k2);
            inv = nk > 0.0 ? 1.0 / nk : 0.0;
        }
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[i] += (p.anchor_mode == 1) ? x[i] * inv : x[i];
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) red[rl][u * 8 + i] = acc[i];
    __syncthreads();
    if (threadIdx.x < D) {
        double s = 0.0;
        for (int r = 0; r < RL; ++r) s += red[r][threadIdx.x];
        partials[((size_t)bh * nchunks + chunk) * D + threadIdx.x] = s;
    }
}

__global__ void ksum_final_kernel(const double *partials, double *ksum, int nchunks, int D)
{
    const int bh = blockIdx.x, c = threadIdx.x;
    if (c >= D) return;
    double s = 0.0;
    for (int k = 0; k < nchunks; ++k) s += partials[((size_t)bh * nchunks + k) * D + c];
    ksum[(size_t)bh * D + c] = s;
}

// ------------------------------------------------------------------ small helpers
__global__ void zero_words_kernel(int32_t *p, size_t n)
{
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n) p[i] = 0;
}

// rows [BH][len][D] (dense) -> cache rows [BH][cap][D]
__global__ void load_rows_kernel(const uint16_t *src, uint16_t *dst, int cap, int D, int len)
{
    const int bh = blockIdx.y;
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;  // 16-byte unit within the head
    const size_t units = (size_t)len * (D / 8);
    if (i < units)
        *reinterpret_cast<u32x4 *>(dst + (size_t)bh * cap * D + i * 8) =
            *reinterpret_cast<const u32x4 *>(src + (size_t)bh * len * D + i * 8);
}

// int32 [BH][len] dense <-> [BH][cap] strided
__global__ void load_pos_kernel(const int32_t *src, int32_t *dst, int cap, int len, int to_cache)
{
    const int bh = blockIdx.y;
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i < len) {
        if (to_cache) dst[(size_t)bh * cap + i] = src[(size_t)bh * len + i];
        else dst[(size_t)bh * len + i] = src[(size_t)bh * cap + i];
    }
}

// ---------------------------------------------------------------------- launchers
constexpr size_t LISTS_LDS_MAX = 48 * 1024;

bool lists_fit_lds(int n, int N) { return n > N && (size_t)(n - N) * 16 <= LISTS_LDS_MAX; }

size_t post_lds_bytes(int n, int N)
{
    size_t b = (size_t)((n + 31) / 32) * 4;
    if (lists_fit_lds(n, N)) b += (size_t)(n - N) * 16;
    return b + 16;
}


hipError_t configure_main_kernels();

hipError_t configure_kernels()
{
    hipError_t e = configure_main_kernels();
    if (e != hipSuccess) return e;
    const int post_max = (int)(MAX_CAP / 8 + LISTS_LDS_MAX + 16);
    const void *post_fns[] = {reinterpret_cast<const void *>(step_post_kernel<128, SPT_SMALL>),
                              reinterpret_cast<const void *>(step_post_kernel<128, SPT_LARGE>),
                              reinterpret_cast<const void *>(step_post_kernel<64, SPT_SMALL>),
                              reinterpret_cast<const void *>(step_post_kernel<64, SPT_LARGE>)};
    for (const void *fn : post_fns) {
        e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, post_max);
        if (e != hipSuccess) return e;
    }
    return e;
}

hipError_t launch_step_score(const StepParams &p, hipStream_t s)
{
    const int grid = p.batch * p.hkv * p.score_chunks;
    if (p.D == 128) hipLaunchKernelGGL((step_score_kernel<128>), dim3(grid), dim3(SCORE_THREADS), 0, s, p);
    else if (p.D == 64) hipLaunchKernelGGL((step_score_kernel<64>), dim3(grid), dim3(SCORE_THREADS), 0, s, p);
    else return hipErrorInvalidValue;
    return hipGetLastError();
}

hipError_t launch_step_post(const StepParams &p, hipStream_t s)
{
    const int grid = (p.do_evict ? p.batch * p.hkv : 0) + p.merge_wgs;
    if (grid == 0) return hipSuccess;
    const size_t lds = post_lds_bytes(p.n, p.N);
    const bool small = p.n <= SPT_SMALL * POST_THREADS;
    if (p.D == 128 && small) hipLaunchKernelGGL((step_post_kernel<128, SPT_SMALL>), dim3(grid), dim3(POST_THREADS), lds, s, p);
    else if (p.D == 128) hipLaunchKernelGGL((step_post_kernel<128, SPT_LARGE>), dim3(grid), dim3(POST_THREADS), lds, s, p);
    else if (p.D == 64 && small) hipLaunchKernelGGL((step_post_kernel<64, SPT_SMALL>), dim3(grid), dim3(POST_THREADS), lds, s, p);
    else if (p.D == 64) hipLaunchKernelGGL((step_post_kernel<64, SPT_LARGE>), dim3(grid), dim3(POST_THREADS), lds, s, p);
    else return hipErrorInvalidValue;
    return hipGetLastError();
}

hipError_t launch_compact_ordered(const StepParams &p, int32_t *flags, int32_t epoch, hipStream_t s)
{
    const int nchunks = (p.n + ORD_ROWS - 1) / ORD_ROWS;
    const int grid = p.batch * p.hkv * nchunks;
    if (p.n - p.N > 1024 * ORD_ROWS) return hipErrorInvalidValue;   // one waiting thread per chunk in reach
    if (p.D == 128) hipLaunchKernelGGL((compact_ordered_kernel<128>), dim3(grid), dim3(1024), 0, s, p, flags, nchunks, epoch);
    else if (p.D == 64) hipLaunchKernelGGL((compact_ordered_kernel<64>), dim3(grid), dim3(1024), 0, s, p, flags, nchunks, epoch);
    else return hipErrorInvalidValue;
    return hipGetLastError();
}

hipError_t launch_ksum_rebuild(const StepParams &p, double *partials, hipStream_t s)
{
    const int BH = p.batch * p.hkv;
    if (p.n == 0) return launch_zero_words(reinterpret_cast<int32_t *>(const_cast<double *>(p.ksum)), (size_t)BH * p.D * 2, s);
    const int nchunks = (p.n + CHUNK_ROWS - 1) / CHUNK_ROWS;
    dim3 grid(nchunks, BH);
    if (p.D == 128) hipLaunchKernelGGL((ksum_partial_kernel<128>), grid, dim3(256), 0, s, p, partials, nchunks);
    else if (p.D == 64) hipLaunchKernelGGL((ksum_partial_kernel<64>), grid, dim3(256), 0, s, p, partials, nchunks);
    else return hipErrorInvalidValue;
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(ksum_final_kernel, dim3(BH), dim3(128), 0, s, partials, const_cast<double *>(p.ksum), nchunks, p.D);
    return hipGetLastError();
}

hipError_t launch_zero_words(int32_t *ptr, size_t nwords, hipStream_t s)
{
    if (nwords == 0) return hipSuccess;
    hipLaunchKernelGGL(zero_words_kernel, dim3((unsigned)((nwords + 255) / 256)), dim3(256), 0, s, ptr, nwords);
    return hipGetLastError();
}

hipError_t launch_load_rows(const uint16_t *src, uint16_t *dst, int BH, int cap, int D, int len, hipStream_t s)
{
    if (len == 0) return hipSuccess;
    const size_t units = (size_t)len * (D / 8);
    hipLaunchKernelGGL(load_rows_kernel, dim3((unsigned)((units + 255) / 256), BH), dim3(256), 0, s, src, dst,
                       cap, D, len);
    return hipGetLastError();
}

hipError_t launch_load_pos(const int32_t *src, int32_t *dst, int BH, int cap, int len, int to_cache,
                           hipStream_t s)
{
    if (len == 0) return hipSuccess;
    hipLaunchKernelGGL(load_pos_kernel, dim3((len + 255) / 256, BH), dim3(256), 0, s, src, dst, cap, len,
                       to_cache);
    return hipGetLastError();
}

}  // namespace kd
