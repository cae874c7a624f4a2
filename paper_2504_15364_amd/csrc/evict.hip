// Append, anchor, cosine score, selection and compaction kernels for gfx950.
//
// The score that decides an eviction is IEEE double arithmetic on the bf16 data,
// rounded once to float (appendix "FLOP count of KeyDiff":
// s_i = mu.k_i / max(|mu||k_i|, eps)).  These passes are bandwidth bound, so the
// double FMAs cost nothing; in exchange the retained set does not depend on
// summation order beyond the last bit of a double.
#include "kd_kernels.h"

namespace kd {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ double bf16_lo(uint32_t w) { return (double)__uint_as_float(w << 16); }
__device__ __forceinline__ double bf16_hi(uint32_t w) { return (double)__uint_as_float(w & 0xFFFF0000u); }

__device__ __forceinline__ double shfl_xor_f64(double x, int m)
{
    int lo = __double2loint(x), hi = __double2hiint(x);
    lo = __shfl_xor(lo, m);
    hi = __shfl_xor(hi, m);
    return __hiloint2double(hi, lo);
}

// ------------------------------------------------------------------- append (Eq. 5)
__global__ __launch_bounds__(256) void append_kernel(const uint16_t *k_new, const uint16_t *v_new,
                                                     uint16_t *k, uint16_t *v, int32_t *pos, int cap,
                                                     int D, int len, int Bt, int32_t pos0)
{
    const int bh = blockIdx.y;
    const int units = Bt * (D / 8);
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i < units) {
        const size_t src = (size_t)bh * Bt * D + (size_t)i * 8;
        const size_t dst = ((size_t)bh * cap + len) * D + (size_t)i * 8;
        *reinterpret_cast<u32x4 *>(k + dst) = *reinterpret_cast<const u32x4 *>(k_new + src);
        *reinterpret_cast<u32x4 *>(v + dst) = *reinterpret_cast<const u32x4 *>(v_new + src);
    }
    if (i < Bt) pos[(size_t)bh * cap + len + i] = pos0 + i;
}

// ------------------------------------------------------------------ anchor partial sums
// Column sums of CHUNK_ROWS rows in double.  mode 1 sums unit keys (Eq. 7): each
// row is scaled by 1/|k| first (a zero key contributes nothing).
template <int D>
__global__ __launch_bounds__(256) void anchor_kernel(EvictParams p)
{
    constexpr int UPR = D / 8;
    constexpr int RL = 256 / UPR;  // rows in flight per pass
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
        if (row < p.n) {
            const u32x4 w = *reinterpret_cast<const u32x4 *>(kb + (size_t)row * D + u * 8);
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                x[2 * i] = bf16_lo(w[i]);
                x[2 * i + 1] = bf16_hi(w[i]);
            }
        } else {
#pragma unroll
            for (int i = 0; i < 8; ++i) x[i] = 0.0;
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
        p.anchor_part[((size_t)bh * p.nchunks + chunk) * D + threadIdx.x] = s;
    }
}

// ------------------------------------------------------------------------- score
template <int D>
__global__ __launch_bounds__(256) void score_kernel(EvictParams p)
{
    constexpr int UPR = D / 8;
    constexpr int RL = 256 / UPR;
    __shared__ double mu[D];
    __shared__ double wsum[4];
    const int bh = blockIdx.y, chunk = blockIdx.x;
    const int tid = threadIdx.x;
    // anchor = (sum of the chunk partials, fixed order) / n
    double m = 0.0;
    if (tid < D) {
        const double *ap = p.anchor_part + (size_t)bh * p.nchunks * D + tid;
        for (int c = 0; c < p.nchunks; ++c) m += ap[(size_t)c * D];
        m /= (double)p.n;
        mu[tid] = m;
    }
    // |mu|^2: every thread with tid >= D contributes zero
    double sq = m * m;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) sq += shfl_xor_f64(sq, off);
    if ((tid & 63) == 0) wsum[tid >> 6] = sq;
    __syncthreads();
    const double nmu = sqrt(wsum[0] + wsum[1] + wsum[2] + wsum[3]);

    const int u = tid % UPR, rl = tid / UPR;
    const uint16_t *kb = p.k + (size_t)bh * p.cap * D;
    double mreg[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) mreg[i] = mu[u * 8 + i];
    const int r0 = chunk * CHUNK_ROWS;
    for (int r = rl; r < CHUNK_ROWS; r += RL) {
        const int row = r0 + r;
        double dot = 0.0, k2 = 0.0;
        if (row < p.n) {
            const u32x4 w = *reinterpret_cast<const u32x4 *>(kb + (size_t)row * D + u * 8);
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const double a = bf16_lo(w[i]), b = bf16_hi(w[i]);
                dot += mreg[2 * i] * a;
                k2 += a * a;
                dot += mreg[2 * i + 1] * b;
                k2 += b * b;
            }
        }
#pragma unroll
        for (int mk = 1; mk < UPR; mk <<= 1) {
            dot += shfl_xor_f64(dot, mk);
            k2 += shfl_xor_f64(k2, mk);
        }
        if (u == 0 && row < p.n) {
            double den = nmu * sqrt(k2);
            if (den < p.eps) den = p.eps;
            const float s = (float)(dot / den) + 0.0f;  // +0 folds -0 into +0
            p.scores[(size_t)bh * p.cap + row] = s;
        }
    }
}

// ------------------------------------------------------------------------ select
// One workgroup per (sequence, KV head).  Finds the E = n - N rows with the
// largest (score, position) -- these are evicted; everything else is retained,
// so equal scores keep the lower position -- by an MSB-first 8-bit radix select
// over the 64-bit key (orderable score bits : position).  Positions are unique,
// so the threshold is exact and there are no ties left to break.
__device__ __forceinline__ uint32_t orderable(float s)
{
    const uint32_t b = __float_as_uint(s);
    return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}

struct SelectShared {
    uint32_t hist[256];
    uint32_t wave_tot[16];
    uint32_t sel_bin, sel_rank, sel_cnt, total_evicted;
};

__device__ __forceinline__ uint32_t block_exclusive_scan(uint32_t v, uint32_t *wave_tot, uint32_t *total)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    uint32_t inc = v;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const uint32_t t = __shfl_up(inc, off);
        if (lane >= off) inc += t;
    }
    __syncthreads();  // wave_tot free for reuse
    if (lane == 63) wave_tot[wave] = inc;
    __syncthreads();
    uint32_t base = 0, tot = 0;
    const int nw = blockDim.x >> 6;
    for (int w = 0; w < nw; ++w) {
        const uint32_t t = wave_tot[w];
        if (w < wave) base += t;
        tot += t;
    }
    *total = tot;
    return base + inc - v;
}

__global__ __launch_bounds__(SELECT_THREADS) void select_kernel(EvictParams p)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    __shared__ SelectShared sh;
    uint32_t *skey = reinterpret_cast<uint32_t *>(smem_raw);  // [n] orderable scores
    const int E = p.n - p.N;
    int32_t *lists = reinterpret_cast<int32_t *>(skey + p.n);  // FILL: holes[E], movers[E]

    const int bh = blockIdx.x, tid = threadIdx.x, lane = tid & 63;
    const float *sc = p.scores + (size_t)bh * p.cap;
    int32_t *pos = p.pos + (size_t)bh * p.cap;

    for (int i = tid; i < p.n; i += SELECT_THREADS) {
        uint32_t key = orderable(sc[i]);
        if (p.window_W > 0 && pos[i] >= p.window_pos_min) key = 0u;  // exempt: never a candidate
        skey[i] = key;
    }
    // contiguous ownership: thread t owns rows [t*S, t*S + S); S odd keeps LDS reads conflict free
    int S = (p.n + SELECT_THREADS - 1) / SELECT_THREADS;
    S |= 1;
    const int own0 = tid * S;
    const int own1 = min(p.n, own0 + S);

    uint64_t prefix = 0;  // resolved high bits of the threshold
    uint32_t rank = (uint32_t)E;
    int resolved = 0;  // number of resolved bits
    for (int pass = 0; pass < 8; ++pass) {
        const int shift = 56 - 8 * pass;
        for (int i = tid; i < 256; i += SELECT_THREADS) sh.hist[i] = 0;
        __syncthreads();
        for (int i = own0; i < own0 + S; ++i) {
            bool part = false;
            uint32_t digit = 0;
            if (i < own1) {
                const uint32_t hi = skey[i];
                if (pass < 4) {
                    part = pass == 0 || (hi >> (32 - 8 * pass)) == (uint32_t)(prefix);
                    digit = (hi >> (24 - 8 * pass)) & 255u;
                } else if (hi == (uint32_t)(prefix >> (8 * (pass - 4)))) {
                    const uint64_t key = ((uint64_t)hi << 32) | (uint32_t)pos[i];
                    part = (key >> (shift + 8)) == prefix;
                    digit = (uint32_t)(key >> shift) & 255u;
                }
            }
            // one aggregated add for the leader's digit (clustered scores), plain adds for the rest
            const uint64_t active = __ballot(part);
            if (active) {
                const int leader = __ffsll((unsigned long long)active) - 1;
                const uint32_t ld = __shfl(digit, leader);
                const uint64_t same = __ballot(part && digit == ld);
                if (lane == leader) atomicAdd(&sh.hist[ld], (uint32_t)__popcll(same));
                else if (part && digit != ld) atomicAdd(&sh.hist[digit], 1u);
            }
        }
        __syncthreads();
        if (tid < 64) {
            // bins 4*lane .. 4*lane+3; suffix sums from the top bin down
            const uint32_t c0 = sh.hist[4 * lane], c1 = sh.hist[4 * lane + 1], c2 = sh.hist[4 * lane + 2],
                           c3 = sh.hist[4 * lane + 3];
            const uint32_t mine = c0 + c1 + c2 + c3;
            uint32_t suf = mine;
#pragma unroll
            for (int off = 1; off < 64; off <<= 1) {
                const uint32_t t = __shfl_down(suf, off);
                if (lane + off < 64) suf += t;
            }
            const uint64_t reach = __ballot(suf >= rank);
            const int owner = 63 - __clzll((unsigned long long)reach);  // highest lane whose suffix reaches rank
            if (lane == owner) {
                uint32_t above = suf - mine;
                uint32_t bin, cnt;
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
        const bool done = sh.sel_cnt == rank;  // every key left in the bin is evicted
        __syncthreads();
        if (done) break;
    }

    // evicted <=> top `resolved` bits of the key >= prefix
    uint64_t evmask = 0;
    uint32_t nev = 0;
    for (int i = own0; i < own1; ++i) {
        const uint32_t hi = skey[i];
        bool ev;
        if (resolved <= 32) ev = (hi >> (32 - resolved)) >= (uint32_t)prefix;
        else {
            const uint64_t key = ((uint64_t)hi << 32) | (uint32_t)pos[i];
            ev = (key >> (64 - resolved)) >= prefix;
        }
        if (ev) {
            evmask |= 1ull << (i - own0);
            ++nev;
        }
    }

    if (p.layout == 1) {
        // FILL: k-th surviving row of [N, n) moves into the k-th evicted slot of [0, N)
        uint32_t nh = 0, nm = 0;
        for (int i = own0; i < own1; ++i) {
            const bool ev = (evmask >> (i - own0)) & 1;
            if (ev && i < p.N) ++nh;
            if (!ev && i >= p.N) ++nm;
        }
        uint32_t total;
        uint32_t base = block_exclusive_scan(nh | (nm << 16) | 0u, sh.wave_tot, &total);
        uint32_t tot_ev;
        (void)block_exclusive_scan(nev, sh.wave_tot, &tot_ev);
        uint32_t hb = base & 0xFFFFu, mb = base >> 16;
        int32_t *holes = lists, *movers = lists + E;
        const uint32_t nholes = total & 0xFFFFu, nmov = total >> 16;
        // an impossible count is reported and nothing is moved (keeps every index in range)
        const bool sane = tot_ev == (uint32_t)E && nholes == nmov && nholes <= (uint32_t)E;
        if (sane)
            for (int i = own0; i < own1; ++i) {
                const bool ev = (evmask >> (i - own0)) & 1;
                if (ev && i < p.N) holes[hb++] = i;
                if (!ev && i >= p.N) movers[mb++] = i;
            }
        __syncthreads();
        if (tid == 0 && !sane) atomicOr(p.status, STATUS_SELECT_COUNT);
        const int nmove = sane ? (int)nholes : 0;
        const int UPR = p.D / 8;
        uint16_t *kb = p.k + (size_t)bh * p.cap * p.D;
        uint16_t *vb = p.v + (size_t)bh * p.cap * p.D;
        for (int w = tid; w < nmove * UPR * 2; w += SELECT_THREADS) {
            const int r = w / (UPR * 2), rem = w % (UPR * 2);
            const int u = rem % UPR;
            uint16_t *base_ptr = rem < UPR ? kb : vb;
            const u32x4 val = *reinterpret_cast<const u32x4 *>(base_ptr + (size_t)movers[r] * p.D + u * 8);
            *reinterpret_cast<u32x4 *>(base_ptr + (size_t)holes[r] * p.D + u * 8) = val;
        }
        for (int r = tid; r < nmove; r += SELECT_THREADS) pos[holes[r]] = pos[movers[r]];
    } else {
        // ORDERED: kept row i moves to i - (evicted rows before i)
        uint32_t tot_ev;
        uint32_t eb = block_exclusive_scan(nev, sh.wave_tot, &tot_ev);
        if (tid == 0 && tot_ev != (uint32_t)E) atomicOr(p.status, STATUS_SELECT_COUNT);
        int32_t *dst = p.dstmap + (size_t)bh * p.cap;
        int32_t mypos[33];
        // positions are compacted here: all reads of pos precede all writes
        for (int i = own0, j = 0; i < own1; ++i, ++j) mypos[j] = pos[i];
        __syncthreads();
        for (int i = own0, j = 0; i < own1; ++i, ++j) {
            const bool ev = (evmask >> (i - own0)) & 1;
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

// --------------------------------------------------------------- ordered compaction
// Stable in-place shift.  One workgroup per (sequence, KV head) walks the rows in
// ascending chunks: a chunk's surviving rows are read into LDS, then written to
// their destinations, which lie at or before their sources, so nothing unread is
// overwritten.
__global__ __launch_bounds__(1024) void compact_ordered_kernel(EvictParams p)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    const int bh = blockIdx.x, tid = threadIdx.x;
    const int UPR = p.D / 8;
    u32x4 *stage = reinterpret_cast<u32x4 *>(smem_raw);  // [2][CHUNK_ROWS][UPR]
    uint16_t *kb = p.k + (size_t)bh * p.cap * p.D;
    uint16_t *vb = p.v + (size_t)bh * p.cap * p.D;
    const int32_t *dst = p.dstmap + (size_t)bh * p.cap;
    const int per_chunk = CHUNK_ROWS * UPR * 2;
    for (int r0 = 0; r0 < p.n; r0 += CHUNK_ROWS) {
        for (int w = tid; w < per_chunk; w += 1024) {
            const int which = w / (CHUNK_ROWS * UPR), rem = w % (CHUNK_ROWS * UPR);
            const int r = rem / UPR, u = rem % UPR;
            const int row = r0 + r;
            if (row < p.n && dst[row] >= 0 && dst[row] != row)
                stage[w] = *reinterpret_cast<const u32x4 *>((which ? vb : kb) + (size_t)row * p.D + u * 8);
        }
        __syncthreads();
        for (int w = tid; w < per_chunk; w += 1024) {
            const int which = w / (CHUNK_ROWS * UPR), rem = w % (CHUNK_ROWS * UPR);
            const int r = rem / UPR, u = rem % UPR;
            const int row = r0 + r;
            if (row < p.n) {
                const int d = dst[row];
                if (d >= 0 && d != row)
                    *reinterpret_cast<u32x4 *>((which ? vb : kb) + (size_t)d * p.D + u * 8) = stage[w];
            }
        }
        __syncthreads();
    }
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

__global__ void copy_scores_kernel(const float *src, float *dst, int cap, int n)
{
    const int bh = blockIdx.y;
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i < n) dst[(size_t)bh * n + i] = src[(size_t)bh * cap + i];
}

// ---------------------------------------------------------------------- launchers
hipError_t launch_append(const uint16_t *k_new, const uint16_t *v_new, uint16_t *k, uint16_t *v,
                         int32_t *pos, int BH, int cap, int D, int len, int Bt, int32_t pos0,
                         hipStream_t s)
{
    const int units = Bt * (D / 8);
    hipLaunchKernelGGL(append_kernel, dim3((units + 255) / 256, BH), dim3(256), 0, s, k_new, v_new, k, v, pos,
                       cap, D, len, Bt, pos0);
    return hipGetLastError();
}

hipError_t launch_anchor(const EvictParams &p, hipStream_t s)
{
    dim3 grid(p.nchunks, p.BH);
    if (p.D == 128) hipLaunchKernelGGL((anchor_kernel<128>), grid, dim3(256), 0, s, p);
    else if (p.D == 64) hipLaunchKernelGGL((anchor_kernel<64>), grid, dim3(256), 0, s, p);
    else return hipErrorInvalidValue;
    return hipGetLastError();
}

hipError_t launch_score(const EvictParams &p, hipStream_t s)
{
    dim3 grid(p.nchunks, p.BH);
    if (p.D == 128) hipLaunchKernelGGL((score_kernel<128>), grid, dim3(256), 0, s, p);
    else if (p.D == 64) hipLaunchKernelGGL((score_kernel<64>), grid, dim3(256), 0, s, p);
    else return hipErrorInvalidValue;
    return hipGetLastError();
}

size_t select_lds_bytes(int n, int N)
{
    const int E = n - N > 0 ? n - N : 0;
    return (size_t)n * 4 + (size_t)E * 8 + 16;
}

size_t compact_lds_bytes(int D) { return (size_t)2 * CHUNK_ROWS * (D / 8) * 16; }

hipError_t launch_select(const EvictParams &p, hipStream_t s)
{
    const size_t lds = select_lds_bytes(p.n, p.N);
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(select_kernel),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(select_kernel, dim3(p.BH), dim3(SELECT_THREADS), lds, s, p);
    return hipGetLastError();
}

hipError_t launch_compact_ordered(const EvictParams &p, hipStream_t s)
{
    const size_t lds = compact_lds_bytes(p.D);
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(compact_ordered_kernel),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(compact_ordered_kernel, dim3(p.BH), dim3(1024), lds, s, p);
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

hipError_t launch_copy_scores(const float *src, float *dst, int BH, int cap, int n, hipStream_t s)
{
    hipLaunchKernelGGL(copy_scores_kernel, dim3((n + 255) / 256, BH), dim3(256), 0, s, src, dst, cap, n);
    return hipGetLastError();
}

}  // namespace kd
