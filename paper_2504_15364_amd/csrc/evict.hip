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
#include "kd_select.h"

namespace kd {

constexpr int SCORE_WAVES = SCORE_THREADS / 64;
constexpr int MERGE_THREADS = 256;   // workgroup size of the stand-alone merge


// ------------------------------------------------------------------------ scores
struct ScoreShared {
    double mu[128];
    double red[SCORE_WAVES];
    double dot[SCORE_WAVES][64];  // per-wave staging of (mu.k, |k|^2) so that sqrt and divide run on full waves
    double k2[SCORE_WAVES][64];
};

// Rows [row0, row1) of head bh (at most SCORE_ROWS), scored against the anchor ksum / n.  D/8 lanes
// share a row (one 16-byte unit each); a wave takes SCORE_ROWS / SCORE_WAVES consecutive rows, stages
// (mu.k, |k|^2) of each row in LDS and then lane i finishes row i of them.  Small row counts per wave
// and two waves per SIMD: the pass is one memory round trip plus a chain of double-precision
// arithmetic, and what hides either is other waves.
template <int D>
__device__ __forceinline__ void score_rows(const StepParams &p, ScoreShared &sh, int bh, int row0, int row1)
{
    constexpr int UPR = D / 8;
    constexpr int RPW = 64 / UPR;                   // rows per wave per pass
    constexpr int WROWS = SCORE_ROWS / SCORE_WAVES; // rows per wave
    constexpr int NP = WROWS / RPW;                 // passes per wave
    static_assert(NP >= 2 && NP % 2 == 0 && WROWS <= 64, "a wave takes an even number of passes and at most 64 rows");
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int u = lane % UPR, rl = lane / UPR;
    const uint16_t *kb = p.k + (size_t)bh * p.cap * D;
    // the rows are requested before the anchor is formed: the two memory round trips (key sum, rows) overlap
    const int base = row0 + wave * WROWS;
    u32x4 w[NP];
#pragma unroll
    for (int ps = 0; ps < NP; ++ps) {
        const int row = base + ps * RPW + rl;
        u32x4 z = {0u, 0u, 0u, 0u};
        if (row < row1) z = *reinterpret_cast<const u32x4 *>(kb + (size_t)row * D + u * 8);
        w[ps] = z;
    }
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
    for (int wv = 0; wv < SCORE_WAVES; ++wv) mu2 += sh.red[wv];
    const double nmu = sqrt(mu2);

    double mreg[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) mreg[i] = sh.mu[u * 8 + i];
    // products of two bf16 values are exact in double, so fma(a, a, .) is the plain sum of squares;
    // mu.k takes one rounding per term either way
    auto partial = [&](const u32x4 &wv, double &dot, double &k2) {
        dot = 0.0;
        k2 = 0.0;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const double a = bf16_lo(wv[i]), b = bf16_hi(wv[i]);
            dot = __builtin_fma(mreg[2 * i], a, dot);
            k2 = __builtin_fma(a, a, k2);
            dot = __builtin_fma(mreg[2 * i + 1], b, dot);
            k2 = __builtin_fma(b, b, k2);
        }
    };
    if constexpr (UPR == 16) {
        // two passes at a time: the four quantities are summed over the 16 lanes of a row with 5
        // additions per lane; lanes 0-3 of a row end with mu.k of the first pass, 4-7 with its
        // |k|^2, 8-11 and 12-15 with those of the second
#pragma unroll
        for (int ps = 0; ps < NP; ps += 2) {
            double d0, q0, d1, q1;
            partial(w[ps], d0, q0);
            partial(w[ps + 1], d1, q1);
            const double v = row_reduce_scatter4_f64(d0, q0, d1, q1, u);
            if ((u & 3) == 0) {
                const int slot = (ps + (u >> 3)) * RPW + rl;
                if (u & 4) sh.k2[wave][slot] = v;
                else sh.dot[wave][slot] = v;
            }
        }
    } else {
#pragma unroll
        for (int ps = 0; ps < NP; ++ps) {
            double dot, k2;
            partial(w[ps], dot, k2);
            dot = row_allreduce_f64<UPR>(dot);
            k2 = row_allreduce_f64<UPR>(k2);
            if (u == 0) {
                sh.dot[wave][ps * RPW + rl] = dot;
                sh.k2[wave][ps * RPW + rl] = k2;
            }
        }
    }
    // same wave wrote and reads: the LDS accesses of one wave complete in order; the fence only
    // keeps the compiler from moving the reads above the writes
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    const int row = base + lane;
    if (lane < WROWS && row < row1) {
        const double dot = sh.dot[wave][lane], k2 = sh.k2[wave][lane];
        const float sc = finish_score(dot, k2, nmu, p.eps);
        p.scores[(size_t)bh * p.cap + row] = sc;
        if (p.scores_out) p.scores_out[(size_t)bh * p.n + row] = sc;
    }
}


// ------------------------------------------------------------------------ merge
// Thread gid takes four output values: step_main leaves a partial in its accumulator layout -- per
// 32-row block D/8 slabs of 512 bytes, slab 4 db + jj holding for lane (h, l32) the values
// d = 32 db + 8 jj + 4 h .. + 3 of row l32 -- and consecutive threads read consecutive lanes of a slab.
// MB: splits requested together
template <int D, int MB = 16>
__device__ __forceinline__ void merge_rows(const StepParams &p, size_t gid)
{
    constexpr int SLABS = D / 8;
    const int BH = p.batch * p.hkv;
    const int Mtot = p.G * p.Bt;
    const int nblk = (Mtot + 31) / 32;
    const size_t rows = (size_t)BH * Mtot;
    const int L = (int)(gid % 64), slab = (int)((gid / 64) % SLABS);
    const size_t blkid = gid / (64 * SLABS);   // (head, 32-row block)
    if (blkid >= (size_t)BH * nblk) return;
    const int bh = (int)(blkid / nblk), m = (int)(blkid % nblk) * 32 + (L & 31);
    if (m >= Mtot) return;
    const size_t row = (size_t)bh * Mtot + m;
    const size_t pstride = (size_t)BH * nblk * SLABS * 64 * 4;          // halfs per split
    const _Float16 *pbase = p.part_o + ((blkid * SLABS + slab) * 64 + L) * 4;
    // One memory round trip: the (max, sum) pairs and the partial rows of a batch of splits are
    // requested together; only with more splits than a batch holds does a second batch follow, and
    // the running result is then rescaled to the larger reference (as inside the attention).
    float mx = -INFINITY;
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    float Lsum = 0.f;
    for (int s0 = 0; s0 < p.psplits; s0 += MB) {
        float2 ml[MB];
        f16x4 o[MB];
#pragma unroll
        for (int i = 0; i < MB; ++i) {
            const bool live = s0 + i < p.psplits;
            const f16x4 zero = {(_Float16)0.f, (_Float16)0.f, (_Float16)0.f, (_Float16)0.f};
            ml[i] = live ? p.part_ml[(size_t)(s0 + i) * rows + row] : make_float2(-INFINITY, 0.f);
            o[i] = live ? *reinterpret_cast<const f16x4 *>(pbase + (size_t)(s0 + i) * pstride) : zero;
        }
        float bm = ml[0].x;
#pragma unroll
        for (int i = 1; i < MB; ++i) bm = fmaxf(bm, ml[i].x);
        if (bm > mx) {
            const float down = mx == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(mx - bm);
            acc.x *= down;
            acc.y *= down;
            acc.z *= down;
            acc.w *= down;
            Lsum *= down;
            mx = bm;
        }
#pragma unroll
        for (int i = 0; i < MB; ++i) {
            // a partial is its split's output normalised by its own row sum: weight it by that sum
            const float w = ml[i].x == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(ml[i].x - mx) * ml[i].y;
            acc.x += w * (float)o[i][0];
            acc.y += w * (float)o[i][1];
            acc.z += w * (float)o[i][2];
            acc.w += w * (float)o[i][3];
            Lsum += w;
        }
    }
    const float inv = 1.f / Lsum;
    const int b = bh / p.hkv, kvh = bh % p.hkv;
    const int g = m / p.Bt, j = m % p.Bt;
    const int d0 = 8 * slab + 4 * (L >> 5);
    bf16x4 o;
    o[0] = (__bf16)(acc.x * inv);
    o[1] = (__bf16)(acc.y * inv);
    o[2] = (__bf16)(acc.z * inv);
    o[3] = (__bf16)(acc.w * inv);
    *reinterpret_cast<bf16x4 *>(p.out + ((size_t)(b * p.hq + kvh * p.G + g) * p.Bt + j) * D + d0) = o;
}

// The merge as a kernel of its own (a step whose eviction is deferred has nothing else to run
// here): small workgroups, so that the rows spread over every compute unit.
// Workgroup i takes head i % BH, like the workgroups of step_main: on a chip whose workgroups go
// round-robin over the XCDs the partials of a head are then read on the XCD that wrote them.
template <int D>
__global__ __launch_bounds__(MERGE_THREADS) void merge_kernel(StepParams p)
{
    const int BH = p.batch * p.hkv;
    const size_t per_head = (size_t)((p.G * p.Bt + 31) / 32) * (D / 8) * 64;
    const int bh = blockIdx.x % BH;
    const size_t local = (size_t)(blockIdx.x / BH) * MERGE_THREADS + threadIdx.x;
    if (local < per_head) merge_rows<D>(p, (size_t)bh * per_head + local);
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
// rest merge the attention partials.  RES: the selection works on LDS copies of the head's scores
// and positions (they fit next to its other tables).
template <int D, bool RES>
__global__ __launch_bounds__(POST_THREADS) void step_post_kernel(StepParams p)
{
    warm_arguments<sizeof(StepParams)>();
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    __shared__ PostShared sh;
    const int n_select = p.do_evict ? p.batch * p.hkv : 0;
    if ((int)blockIdx.x >= n_select) {
#ifdef KD_TIMELINE
        unsigned long long *tl = reinterpret_cast<unsigned long long *>(&sh);   // (the selection's tables are not in use here)
        if (threadIdx.x < 32) tl[threadIdx.x] = 0;
        __syncthreads();
        if (threadIdx.x == 0) tl[0] = wall_clock64();
#endif
        merge_rows<D>(p, (size_t)(blockIdx.x - n_select) * POST_THREADS + threadIdx.x);
#ifdef KD_TIMELINE
        __builtin_amdgcn_s_waitcnt(0x0F70);
        __syncthreads();
        if (threadIdx.x == 0) {
            tl[12] = wall_clock64();
            tl[31] = 4;   // record kind: merging workgroup
        }
        __syncthreads();
        if (p.timeline && threadIdx.x < 32) p.timeline[(size_t)blockIdx.x * 32 + threadIdx.x] = tl[threadIdx.x];
#endif
        return;
    }
    select_and_compact<D, RES, POST_THREADS>(p, sh, smem_raw, (int)blockIdx.x);
}

// ------------------------------------------------------------- ordered compaction
// Stable in-place shift: kept row i moves to dst[i] = i - (evicted rows before i), so a row moves
// down by at most E = n - N rows.  One workgroup per ORD_ROWS rows reads its moving rows into
// registers, announces that (flag = epoch of this launch), waits until the workgroups whose rows
// it may overwrite -- the ceil(E / ORD_ROWS) chunks before it -- have announced the same, and
// stores.  Workgroups are numbered chunk-major, so a workgroup only ever waits for lower-numbered
// ones; the wait is bounded and reports a timeout in the status word instead of hanging.
template <int D>
__device__ __forceinline__ void shift_chunk(const StepParams &p, int32_t *flags, int nchunks, int32_t epoch, int block)
{
    constexpr int UPR = D / 8;
    constexpr int UPT = ORD_ROWS * UPR * 2 / ORD_THREADS;   // 16-byte units (K and V) per thread
    static_assert(UPT * ORD_THREADS == ORD_ROWS * UPR * 2, "the chunk must divide over the threads");
    const int BH = p.batch * p.hkv;
    const int bh = block % BH, chunk = block / BH, tid = threadIdx.x;
    uint16_t *kb = p.k + (size_t)bh * p.cap * D;
    uint16_t *vb = p.v + (size_t)bh * p.cap * D;
    const int32_t *dst = p.dstmap + (size_t)bh * p.cap;
    const int r0 = chunk * ORD_ROWS;
    u32x4 val[UPT];
    int drow[UPT];
#pragma unroll
    for (int q = 0; q < UPT; ++q) {
        const int w = q * ORD_THREADS + tid;
        const int which = w >= ORD_ROWS * UPR, rem = w - which * ORD_ROWS * UPR;
        const int row = r0 + rem / UPR, u = rem % UPR;
        // the row is requested together with its destination, not after it: one memory round trip
        // (rows that turn out to stay, or to be evicted, are the few ahead of the first eviction and
        // the evicted ones themselves)
        drow[q] = -1;
        val[q] = u32x4{0u, 0u, 0u, 0u};
        if (row < p.n) {
            val[q] = *reinterpret_cast<const u32x4 *>((which ? vb : kb) + (size_t)row * D + u * 8);
            const int d = dst[row];
            if (d >= 0 && d != row) drow[q] = d;
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
        const int w = q * ORD_THREADS + tid;
        const int which = w >= ORD_ROWS * UPR, rem = w - which * ORD_ROWS * UPR;
        if (drow[q] >= 0)
            *reinterpret_cast<u32x4 *>((which ? vb : kb) + (size_t)drow[q] * D + (rem % UPR) * 8) = val[q];
    }
}

template <int D>
__global__ __launch_bounds__(ORD_THREADS) __attribute__((amdgpu_waves_per_eu(8, 8))) void compact_ordered_kernel(StepParams p, int32_t *flags, int nchunks, int32_t epoch)
{
    shift_chunk<D>(p, flags, nchunks, epoch, (int)blockIdx.x);
}

// The merge of one cache's attention partials and the ordered shift of another cache in one launch
// (eviction deferred, ORDERED layout: the selection of the other cache rode in the attention launch
// just before, and its rows have no reader until that cache's next step).  The merge is a memory
// round trip on a chip it leaves mostly idle; the shift is bound by HBM traffic: together they take
// what the shift takes alone.  Workgroups [0, merge_wgs) merge -- they are dispatched first and
// the caller waits for their output -- the others shift one chunk each, numbered chunk-major
// behind them, so a shifting workgroup still only ever waits for lower-numbered ones.
template <int D>
__global__ __launch_bounds__(ORD_THREADS) __attribute__((amdgpu_waves_per_eu(8, 8))) void merge_shift_kernel(StepParams pm, StepParams ps, int32_t *flags, int nchunks,
                                                                  int32_t epoch, int merge_wgs)
{
    if ((int)blockIdx.x < merge_wgs) {
        // (few splits per round trip: the launch lasts as long as the shift does, and the registers
        // decide how many of its workgroups a compute unit holds)
        merge_rows<D, 4>(pm, (size_t)blockIdx.x * ORD_THREADS + threadIdx.x);
        return;
    }
    shift_chunk<D>(ps, flags, nchunks, epoch, (int)blockIdx.x - merge_wgs);
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

// ------------------------------------------------------------------ rotary embedding
// Fig. 1 step (1), the part of it that can live inside this boundary: the block's queries and keys
// arrive as the projections produced them and are rotated here, at the positions pos0 + j, into
// buffers the block step then reads.  Half-split pairing (i, i + D/2); cos and sin come from the
// caller's float tables [position][D/2]; x1 cos - x2 sin and x2 cos + x1 sin with every product and
// sum rounded to float on its own, then one rounding to bf16.
// rows: all (sequence, head) rows of q followed by those of k_new, Bt tokens each; a thread takes the
// 8 + 8 paired elements of one 16-byte unit of the first half.
template <int D>
__global__ __launch_bounds__(256) void rope_kernel(const uint16_t *q, const uint16_t *k, uint16_t *q_rot, uint16_t *k_rot,
                                                   const float *cos_t, const float *sin_t, int q_rows, int k_rows, int Bt,
                                                   int32_t pos0)
{
    constexpr int UPH = D / 16;   // 16-byte units per half row
    const size_t gid = (size_t)blockIdx.x * 256 + threadIdx.x;
    const size_t row = gid / UPH;
    const int unit = (int)(gid % UPH);
    if (row >= (size_t)q_rows + k_rows) return;
    const bool isk = row >= (size_t)q_rows;
    const size_t r = isk ? row - q_rows : row;
    const uint16_t *src = (isk ? k : q) + r * D;
    uint16_t *dst = (isk ? k_rot : q_rot) + r * D;
    const int j = (int)(r % Bt);
    const float *cs = cos_t + ((size_t)pos0 + j) * (D / 2) + unit * 8;
    const float *sn = sin_t + ((size_t)pos0 + j) * (D / 2) + unit * 8;
    const u32x4 a = *reinterpret_cast<const u32x4 *>(src + unit * 8);           // x1: elements 8 unit .. + 7
    const u32x4 b = *reinterpret_cast<const u32x4 *>(src + D / 2 + unit * 8);   // x2: the paired elements
    const f32x4 c0 = *reinterpret_cast<const f32x4 *>(cs), c1 = *reinterpret_cast<const f32x4 *>(cs + 4);
    const f32x4 s0 = *reinterpret_cast<const f32x4 *>(sn), s1 = *reinterpret_cast<const f32x4 *>(sn + 4);
    u32x4 o1, o2;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        float y1[2], y2[2];
#pragma unroll
        for (int hw = 0; hw < 2; ++hw) {
            const float x1 = __uint_as_float(hw ? (a[i] & 0xFFFF0000u) : (a[i] << 16));
            const float x2 = __uint_as_float(hw ? (b[i] & 0xFFFF0000u) : (b[i] << 16));
            const int e = 2 * i + hw;
            const float c = e < 4 ? c0[e] : c1[e - 4], sgn = e < 4 ? s0[e] : s1[e - 4];
            y1[hw] = __fsub_rn(__fmul_rn(x1, c), __fmul_rn(x2, sgn));
            y2[hw] = __fadd_rn(__fmul_rn(x2, c), __fmul_rn(x1, sgn));
        }
        const __bf16 l1 = (__bf16)y1[0], h1 = (__bf16)y1[1], l2 = (__bf16)y2[0], h2 = (__bf16)y2[1];
        o1[i] = (uint32_t)__builtin_bit_cast(uint16_t, l1) | ((uint32_t)__builtin_bit_cast(uint16_t, h1) << 16);
        o2[i] = (uint32_t)__builtin_bit_cast(uint16_t, l2) | ((uint32_t)__builtin_bit_cast(uint16_t, h2) << 16);
    }
    *reinterpret_cast<u32x4 *>(dst + unit * 8) = o1;
    *reinterpret_cast<u32x4 *>(dst + D / 2 + unit * 8) = o2;
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

// dynamic LDS a step_post launch may ask for next to its static tables (160 KB per compute unit)
constexpr size_t POST_DYN_MAX = 160 * 1024 - sizeof(PostShared) - 1024;

static bool post_resident(const StepParams &p)
{
    return select_dyn_bytes(p.n, p.N, p.cap, p.lists_in_lds != 0, true) <= POST_DYN_MAX;
}


hipError_t configure_main_kernels();

hipError_t configure_kernels()
{
    hipError_t e = configure_main_kernels();
    if (e != hipSuccess) return e;
    static_assert(MAX_CAP / 8 + LISTS_LDS_MAX + 16 <= POST_DYN_MAX, "the non-resident selection always fits");
    const void *post_fns[] = {reinterpret_cast<const void *>(step_post_kernel<128, true>),
                              reinterpret_cast<const void *>(step_post_kernel<128, false>),
                              reinterpret_cast<const void *>(step_post_kernel<64, true>),
                              reinterpret_cast<const void *>(step_post_kernel<64, false>)};
    for (const void *fn : post_fns) {
        e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)POST_DYN_MAX);
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
    if (!p.do_evict) {   // merge only
        const size_t per_head = (size_t)((p.G * p.Bt + 31) / 32) * (p.D / 8) * 64;
        const int mgrid = p.batch * p.hkv * (int)((per_head + MERGE_THREADS - 1) / MERGE_THREADS);
        if (p.D == 128) hipLaunchKernelGGL((merge_kernel<128>), dim3(mgrid), dim3(MERGE_THREADS), 0, s, p);
        else if (p.D == 64) hipLaunchKernelGGL((merge_kernel<64>), dim3(mgrid), dim3(MERGE_THREADS), 0, s, p);
        else return hipErrorInvalidValue;
        return hipGetLastError();
    }
    if (p.n > 32 * POST_THREADS) return hipErrorInvalidValue;   // a thread owns one word of the eviction bitmap
    const bool res = post_resident(p) && !p.argmax_rec;   // (the arg-max records make the copies of the scores unnecessary)
    const size_t lds = select_dyn_bytes(p.n, p.N, p.cap, p.lists_in_lds != 0, res);
    if (p.D == 128 && res) hipLaunchKernelGGL((step_post_kernel<128, true>), dim3(grid), dim3(POST_THREADS), lds, s, p);
    else if (p.D == 128) hipLaunchKernelGGL((step_post_kernel<128, false>), dim3(grid), dim3(POST_THREADS), lds, s, p);
    else if (p.D == 64 && res) hipLaunchKernelGGL((step_post_kernel<64, true>), dim3(grid), dim3(POST_THREADS), lds, s, p);
    else if (p.D == 64) hipLaunchKernelGGL((step_post_kernel<64, false>), dim3(grid), dim3(POST_THREADS), lds, s, p);
    else return hipErrorInvalidValue;
    return hipGetLastError();
}

hipError_t launch_compact_ordered(const StepParams &p, int32_t *flags, int32_t epoch, hipStream_t s)
{
    const int nchunks = (p.n + ORD_ROWS - 1) / ORD_ROWS;
    const int grid = p.batch * p.hkv * nchunks;
    if (p.n - p.N > ORD_THREADS * ORD_ROWS) return hipErrorInvalidValue;   // one waiting thread per chunk in reach
    if (p.D == 128) hipLaunchKernelGGL((compact_ordered_kernel<128>), dim3(grid), dim3(ORD_THREADS), 0, s, p, flags, nchunks, epoch);
    else if (p.D == 64) hipLaunchKernelGGL((compact_ordered_kernel<64>), dim3(grid), dim3(ORD_THREADS), 0, s, p, flags, nchunks, epoch);
    else return hipErrorInvalidValue;
    return hipGetLastError();
}

// pm: the step whose partials are merged; ps: the step of the other cache whose destination map is applied
hipError_t launch_merge_shift(const StepParams &pm, const StepParams &ps, int32_t *flags, int32_t epoch, hipStream_t s)
{
    const int nchunks = (ps.n + ORD_ROWS - 1) / ORD_ROWS;
    const size_t merge_threads = (size_t)pm.batch * pm.hkv * ((pm.G * pm.Bt + 31) / 32) * (pm.D / 8) * 64;
    const int mw = (int)((merge_threads + ORD_THREADS - 1) / ORD_THREADS);
    const int grid = mw + ps.batch * ps.hkv * nchunks;
    if (ps.n - ps.N > ORD_THREADS * ORD_ROWS || pm.D != ps.D || pm.psplits < 2) return hipErrorInvalidValue;
    if (pm.D == 128) hipLaunchKernelGGL((merge_shift_kernel<128>), dim3(grid), dim3(ORD_THREADS), 0, s, pm, ps, flags, nchunks, epoch, mw);
    else if (pm.D == 64) hipLaunchKernelGGL((merge_shift_kernel<64>), dim3(grid), dim3(ORD_THREADS), 0, s, pm, ps, flags, nchunks, epoch, mw);
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

hipError_t launch_rope(const uint16_t *q, const uint16_t *k, uint16_t *q_rot, uint16_t *k_rot, const float *cos_t,
                       const float *sin_t, int q_rows, int k_rows, int Bt, int D, int32_t pos0, hipStream_t s)
{
    const size_t threads = ((size_t)q_rows + k_rows) * (D / 16);
    const unsigned grid = (unsigned)((threads + 255) / 256);
    if (D == 128) hipLaunchKernelGGL((rope_kernel<128>), dim3(grid), dim3(256), 0, s, q, k, q_rot, k_rot, cos_t, sin_t, q_rows, k_rows, Bt, pos0);
    else if (D == 64) hipLaunchKernelGGL((rope_kernel<64>), dim3(grid), dim3(256), 0, s, q, k, q_rot, k_rot, cos_t, sin_t, q_rows, k_rows, Bt, pos0);
    else return hipErrorInvalidValue;
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
