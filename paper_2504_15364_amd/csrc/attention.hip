// step_main: append (Eq. 5) + block attention over cache || block (Eq. 1-2) + anchor and cosine
// score of every key (Method, "Efficient Variant"; appendix "FLOP count of KeyDiff") for gfx950.
//
// Flash-style: the attention matrix is never materialised (Method, "Efficient
// Variant": KeyDiff needs no attention weights).  bf16 MFMA 32x32x16 for both
// contractions, fp32 online softmax.
//
// Work decomposition.  All G * Bt query rows that share one KV head form the M
// dimension (GQA packing): a workgroup of NW waves owns 32 * NQ * NW of them and a
// contiguous range of 64-key tiles (split-KV); the splits are merged by
// log-sum-exp in step_post (or the merge kernel).  Workgroup ids map KV heads
// round-robin so that the workgroups of one head share an XCD and its L2.
// Variants: HELP (few query rows: waves without one copy tiles and score rows), ALT on
// top of it (one wave's worth of rows: two waves take alternate key tiles), and the
// carrying kernel whose first workgroups run another cache's pending selection.
//
// Data path.  K and V tiles stream global -> LDS asynchronously
// (global_load_lds_dwordx4: lane i's 16 bytes land at LDS base + 16 i, no VGPRs)
// through a ring of STAGES buffers, so several tiles are in flight per CU while
// one is computed.  Both tiles are stored row-major with a 16-byte-unit XOR swizzle
// applied on the global side (a lane fetches the unit that belongs in its LDS slot).
// The queries take the same road once, at the start.
//
// Both contractions are computed transposed so that softmax statistics are
// per-lane scalars and P never leaves registers:
//   S^T = K Q^T   A = K rows (ds_read_b128), B = Q^T (registers)
//                 -> a lane holds one query column (lane % 32) and 16 keys
//   O^T = V^T P^T A = V^T, read from the row-major V tile with the LDS transpose
//                 read ds_read_b64_tr_b16 (a 16-lane group fetches 4 keys x 16 d and
//                 lane i receives column i); B = P^T: the S^T accumulator layout
//                 already is the B-operand layout once the 16 keys of a k-chunk are
//                 enumerated in accumulator order (keys 16c + 8a + 4h + r for
//                 k-slot 4a + r of lane half h), and the two transpose reads of an
//                 operand fetch exactly those two groups of 4 consecutive keys.
//
// The block's own rows are read straight from k_new / v_new; every workgroup
// copies a slice of them into the cache (the append).  Every workgroup also sums
// the block's keys in double (32 KB from L2) to form the key sum after this step
// and from it the anchor, and scores the rows of its K tiles while they sit in LDS,
// so the keys cross HBM once per step.
#include <type_traits>

#include "kd_kernels.h"
#include "kd_device.h"
#include "kd_select.h"
#include "kd_shift.h"

namespace kd {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ bf16x8 as_bf16x8(u32x4 v) { return __builtin_bit_cast(bf16x8, v); }

// The running reference max may lag the true row max by 2^SLACK before the accumulators are
// rescaled: weights then reach 2^64 and sums 2^64 * 32768 rows * |v|, far inside fp32 range, and
// bf16 / fp32 keep their relative precision at any magnitude, so the slack costs no accuracy; it
// makes the rescale (a pass over all accumulators) a once-per-row event instead of a per-tile one.
constexpr float RESCALE_SLACK = 64.f;
constexpr int STAGES = 4;             // LDS ring: tiles t - 1 and t in use, STAGES - 2 in flight

// Asynchronous 16-byte-per-lane copy global -> LDS.  `lds_base` is wave uniform; lane i writes
// bytes [16 i, 16 i + 16) above it.  Issued through asm so that the compiler does not force
// every outstanding copy to complete before the next LDS read; completion is awaited with
// explicit s_waitcnt vmcnt(N) (copies complete in issue order).
__device__ __forceinline__ void async_copy16(uint32_t lds_base, const void *gaddr)
{
    const uint32_t base = (uint32_t)__builtin_amdgcn_readfirstlane((int)lds_base);
    asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, off" : : "s"(base), "v"(gaddr) : "memory");
}
__device__ __forceinline__ void async_copy16(uint32_t lds_base, const void *gbase, uint32_t byte_off)
{
    const uint32_t base = (uint32_t)__builtin_amdgcn_readfirstlane((int)lds_base);
    const uint64_t g = (uint64_t)(uintptr_t)gbase;
    // readfirstlane returns a signed int: widen through uint32_t, or a low word with bit 31 set
    // would sign-extend into the high half of the address
    const uint32_t g_lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)g);
    const uint32_t g_hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(g >> 32));
    const uint64_t gu = ((uint64_t)g_hi << 32) | (uint64_t)g_lo;
    asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, %2" : : "s"(base), "v"(byte_off), "s"(gu) : "memory");
}

// max(a, b, c) without the NaN canonicalisation fmaxf carries (logits are finite or -inf)
__device__ __forceinline__ float max3_raw(float a, float b, float c)
{
    float r;
    asm("v_max3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
    return r;
}

// Lane i and lane i ^ 32 hold the two halves of a query's keys (accumulator rows 4 h + ...).  One
// v_permlane32_swap hands each the other's value without a trip through LDS: of the pair it
// returns, element 0 is x with its upper 32 lanes replaced by x's lower 32, element 1 is x with its
// lower 32 lanes replaced by x's upper 32, so in every lane the two elements are {x[i], x[i ^ 32]}.
__device__ __forceinline__ float max_halves(float x)
{
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return max3_raw(__uint_as_float(r[0]), __uint_as_float(r[1]), __uint_as_float(r[0]));
}
__device__ __forceinline__ float sum_halves(float x)
{
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

template <int N>
__device__ __forceinline__ void wait_copies()  // at most N of this wave's copies still in flight
{
    static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
    __builtin_amdgcn_s_waitcnt(0x0F70 | (N & 15) | ((N >> 4) << 14));
}

// the same for a count known only at run time (wave uniform, at most 24)
__device__ __forceinline__ void wait_copies_upto(int n)
{
    switch (n) {
#define KD_WAIT_CASE(N) case N: wait_copies<N>(); break;
        KD_WAIT_CASE(1) KD_WAIT_CASE(2) KD_WAIT_CASE(3) KD_WAIT_CASE(4) KD_WAIT_CASE(5) KD_WAIT_CASE(6)
        KD_WAIT_CASE(7) KD_WAIT_CASE(8) KD_WAIT_CASE(9) KD_WAIT_CASE(10) KD_WAIT_CASE(11) KD_WAIT_CASE(12)
        KD_WAIT_CASE(13) KD_WAIT_CASE(14) KD_WAIT_CASE(15) KD_WAIT_CASE(16) KD_WAIT_CASE(17) KD_WAIT_CASE(18)
        KD_WAIT_CASE(19) KD_WAIT_CASE(20) KD_WAIT_CASE(21) KD_WAIT_CASE(22) KD_WAIT_CASE(23) KD_WAIT_CASE(24)
#undef KD_WAIT_CASE
        default: wait_copies<0>(); break;
    }
}

// Loads into registers that the compiler is not told are loads: it neither counts them nor waits
// for them.  The registers hold the data only after an explicit wait (wait_copies: these loads and
// the copies complete in issue order) followed by loads_landed() on them, which is where the code
// that reads them takes them from.
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ u32x4 load16_async(const void *g)
{
    u32x4 v;
    asm volatile("global_load_dwordx4 %0, %1, off" : "=v"(v) : "v"(g) : "memory");
    return v;
}
__device__ __forceinline__ u32x2 load8_async(const void *g)
{
    u32x2 v;
    asm volatile("global_load_dwordx2 %0, %1, off" : "=v"(v) : "v"(g) : "memory");
    return v;
}
template <int A, int B>
__device__ __forceinline__ void loads_landed(u32x2 &x, u32x4 (&w)[A][B])
{
    asm volatile("" : "+v"(x) : : "memory");
#pragma unroll
    for (int i = 0; i < A; ++i)
#pragma unroll
        for (int j = 0; j < B; ++j) asm volatile("" : "+v"(w[i][j]) : : "memory");
}

// A workgroup is NW = 8 waves of NQ = 1 block of 32 query rows each (two waves per SIMD: with one wave
// of 64 rows per SIMD every vector, LDS and copy-issue latency lay open and the kernel was slower).
// HELP: some waves of a workgroup may have no query row at all (few query rows: decode); such a
// wave takes no part in the attention, it copies its share of every tile and scores rows.
constexpr int MAIN_WAVES = 8;
template <int D, bool HELP, bool ALT>
__device__ __forceinline__ void step_main_body(const StepParams &p, const int block_id)
{
    constexpr int NW = MAIN_WAVES;   // waves per workgroup
    constexpr int NQ = 1;            // 32-row query blocks per wave
    constexpr int NT = 64 * NW;   // threads
    constexpr int TM = 32 * NQ * NW;          // query rows per workgroup
    constexpr int UPR = D / 8;    // 16-byte units per K/V row
    constexpr int NC = D / 16;    // k-chunks of the first MFMA
    constexpr int NDB = D / 32;   // 32-wide d blocks of the output
    constexpr int ROWB = D * 2;   // bytes per row
    constexpr int TILE_B = TILE_KEYS * ROWB;  // bytes of one K (or V) tile
    constexpr int RPL = 64 / UPR;             // rows one wave-wide copy covers
    constexpr int CPT = TILE_KEYS / RPL;      // wave-wide copies per K (or V) tile
    constexpr int CPW = CPT / NW;             // ... per wave
    static_assert(CPW >= 1 && CPW * NW == CPT, "tile copies must divide over the waves");
    constexpr int LPW = 2 * CPW;              // copies per wave per tile (K and V)
    static_assert(2 * LPW < 64, "two tiles of copies in flight must fit the 6-bit counter");

    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];  // [STAGES][K tile | V tile]
    __shared__ double red[NW][4];       // |mu|^2 in pieces: one per 16-lane row of every wave
    __shared__ double bs_part[NW][D];   // per-wave column sums of the block's keys
    __shared__ double mu_s[D];          // the anchor: (key sum incl. this block) / n
    // (mu.k, |k|^2, row) of scored rows, staged per wave until 64 are there: the square root and the
    // division that finish a score are long instruction sequences, run once per 64 rows this way
    __shared__ double st_dot[NW][64], st_k2[NW][64];
    __shared__ int st_row[NW][64];
    KD_TL_DECL
    KD_TL(0);

    const int tid = threadIdx.x, lane = tid & 63;
    // the wave index as a scalar: what follows from it (buffer pieces, roles, branches) is then
    // scalar arithmetic and scalar branches instead of per-lane values and execution masks
    // (not in the alternating mode, whose two roles the compiler then turns into two copies of the
    // loop body and spills)
    const int wave = ALT ? tid >> 6 : __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l32 = lane & 31, h = lane >> 5;
    const int BH = p.batch * p.hkv;
    int id = block_id;
    const int bh = id % BH;
    id /= BH;
    const int mt = id % p.mtiles;
    const int sp = id / p.mtiles;
    const int b = bh / p.hkv, kvh = bh % p.hkv;
    const int Mtot = p.G * p.Bt;
    // Key range of this split.  A tile that takes rows of the block (causal mask, a second source,
    // decisions per copy) costs more than a plain tile of cached keys -- about 1.4 times by the
    // in-kernel stamps -- and the split that holds them would end last: the ranges are balanced with
    // such a tile counted as edge_cost (1 or 2) plain ones.
    const int tplain = min(p.ntiles, p.len / TILE_KEYS);
    const int ctotal = tplain + (p.ntiles - tplain) * p.edge_cost;
    auto tile_at = [&](int i) {   // first tile of split i
        const int c = (int)(((unsigned)i * (unsigned)ctotal) / (unsigned)p.splits);   // < 2^31: at most 512 splits x 1024 cost units
        return c <= tplain ? c : tplain + (c - tplain) / p.edge_cost;
    };
    const int t0 = tile_at(sp);
    const int t1 = sp + 1 == p.splits ? p.ntiles : tile_at(sp + 1);
    const int ntl = t1 - t0;
    KD_TL(13);  // arguments read, key range known

    const uint16_t *kcache = p.k + (size_t)bh * p.cap * D;
    const uint16_t *vcache = p.v + (size_t)bh * p.cap * D;
    const uint16_t *knew = p.k_new + (size_t)bh * p.Bt * D;
    const uint16_t *vnew = p.v_new + (size_t)bh * p.Bt * D;

    // ---- tile copies.  Wave w issues copies w, w + NW, ... of the K tile and of the V tile; copy s
    // fills LDS bytes [1024 s, 1024 s + 1024) of the tile = rows RPL s .. RPL s + RPL - 1.  Lane i
    // owns slot (row RPL s + i / UPR, unit i % UPR) and fetches the unit the swizzle puts there:
    //   K: unit ^ (row % UPR)          (LDS serves 256 bytes per clock to ds_read_b128: the 16 rows a
    //                                   clock covers must spread over 16 distinct 16-byte units)
    //   V: unit ^ 2 (row & 3)          (the 4 rows x 32 bytes of a transpose read do the same)
    const uint32_t lds0 = (uint32_t)(uintptr_t)smem;
    // Copy i of a wave covers rows RPL (wave + NW i) ..: NW RPL is a multiple of 8, so the swizzle
    // terms (row % UPR, row & 3) are those of copy 0 and copy i only adds i NW RPL rows.
    // ... or by half a period, which flips the top bit of the K swizzle: (row + UPR / 2) % UPR == (row % UPR) ^ (UPR / 2)
    static_assert((NW * RPL) % UPR == 0 || (NW * RPL) % UPR == UPR / 2, "the K swizzle of copy i must follow from that of copy 0");
    static_assert((NW * RPL) % 4 == 0, "the V swizzle of a lane must not depend on the copy index");
    constexpr int VSW = UPR / 4;     // V swizzle stride: unit ^ VSW (row & 3)
    constexpr int CSTEP = NW * RPL;  // rows between consecutive copies of one wave
    const int crow0 = RPL * wave + lane / UPR;   // row of copy 0 inside the tile
    const uint32_t koff0 = (uint32_t)(crow0 * ROWB + ((lane % UPR) ^ (crow0 & (UPR - 1))) * 16);
    const uint32_t voff0 = (uint32_t)(crow0 * ROWB + ((lane % UPR) ^ (VSW * (crow0 & 3))) * 16);
    auto koff_of = [&](int i) { return koff0 ^ (uint32_t)((((i * CSTEP) & (UPR - 1))) * 16); };  // copy i of the K tile
    // A tile is "whole" when its 64 rows are valid and come from one source (the cache, or the
    // block's k_new / v_new): then only the base pointer differs.  A partial tile (it straddles len
    // or n; at most two per step) takes per-row pointers; rows past n read row n - 1 -- finite
    // data whose logits are masked, so it is never zeroed.
    auto issue_copy = [&](int t, int c) {   // copy c of tile t: c < CPW K tile, else V tile
        const int r0 = t * TILE_KEYS;
        const bool isv = c >= CPW;
        const int i = isv ? c - CPW : c;
        const uint32_t dst = lds0 + (uint32_t)((t % STAGES) * 2 * TILE_B) + (isv ? TILE_B : 0) + 1024u * (wave + NW * i);
        const uint32_t off0 = isv ? voff0 : koff_of(i);
        const bool whole = r0 + TILE_KEYS <= p.len || (r0 >= p.len && r0 + TILE_KEYS <= p.n);
        if (whole) {
            const bool cached = r0 < p.len;
            const uint16_t *src = cached ? (isv ? vcache : kcache) + (size_t)r0 * D
                                         : (isv ? vnew : knew) + (size_t)(r0 - p.len) * D;
            async_copy16(dst, src + (size_t)i * CSTEP * D, off0);
        } else {
            const int rc = min(r0 + crow0 + i * CSTEP, p.n - 1);
            const uint16_t *src = rc < p.len ? (isv ? vcache : kcache) + (size_t)rc * D
                                             : (isv ? vnew : knew) + (size_t)(rc - p.len) * D;
            async_copy16(dst, reinterpret_cast<const char *>(src) + (off0 - crow0 * ROWB));
        }
    };

    // the same for a tile known to lie entirely in the cache: no decisions left, a handful of
    // scalar instructions per copy
    auto issue_copy_cached = [&](int t, int c) {
        const bool isv = c >= CPW;
        const int i = isv ? c - CPW : c;
        const uint32_t dst = lds0 + (uint32_t)((t % STAGES) * 2 * TILE_B) + (isv ? TILE_B : 0) + 1024u * (wave + NW * i);
        const uint16_t *src = (isv ? vcache : kcache) + ((size_t)t * TILE_KEYS + (size_t)i * CSTEP) * D;
        async_copy16(dst, src, isv ? voff0 : koff_of(i));
    };
    auto issue_tile = [&](int t) {
        if ((t + 1) * TILE_KEYS <= p.len) {   // uniform: the whole tile lies in the cache
#pragma unroll
            for (int c = 0; c < LPW; ++c) issue_copy_cached(t, c);
        } else {
#pragma unroll
            for (int c = 0; c < LPW; ++c) issue_copy(t, c);
        }
    };
    auto issue_half = [&](int t, bool vhalf) {   // the K tile (copies [0, CPW)) or the V tile (copies [CPW, LPW)) alone
        if ((t + 1) * TILE_KEYS <= p.len) {   // uniform: the whole tile lies in the cache
#pragma unroll
            for (int c = 0; c < CPW; ++c) issue_copy_cached(t, c + (vhalf ? CPW : 0));
        } else {
#pragma unroll
            for (int c = 0; c < CPW; ++c) issue_copy(t, c + (vhalf ? CPW : 0));
        }
    };

    // ---- anchor, part 1 (Method, "Efficient Variant"): key sum after this step = key sum before it +
    // the block's keys.  Every workgroup that scores forms it by itself (the block is 32 KB in L2); one
    // workgroup per head also stores it for step_post and the next step.  The block's rows are
    // requested first and consumed while the copies below fly.  These loads are written out as
    // instructions of their own: for a load of its own the compiler waits by counting the loads it
    // knows of, so with the copies (which it does not know of) issued behind it, it would wait for all
    // of them.  Their registers are handed to the code that reads them by loads_landed(), after an
    // explicit wait.
    const bool writer = sp == 0 && mt == 0;
    const bool need_sum = p.do_score != 0 || writer;
    constexpr int BROWS = NT / UPR;    // block rows per pass: UPR consecutive lanes share a row
    constexpr int BPASS = 4;           // passes loaded together (one batch)
    constexpr int BBATCH = 2;          // batches requested up front
    const int bu = tid % UPR, brl = tid / UPR;
    const int nbatch = !need_sum ? 0 : min(BBATCH, (p.Bt + BPASS * BROWS - 1) / (BPASS * BROWS));   // uniform
    u32x4 kw[BBATCH][BPASS];
    u32x2 ksum_raw = {0u, 0u};
#pragma unroll
    for (int bt = 0; bt < BBATCH; ++bt)
#pragma unroll
        for (int ps = 0; ps < BPASS; ++ps) kw[bt][ps] = u32x4{0u, 0u, 0u, 0u};
    auto request_rows = [&]() {
        ksum_raw = load8_async(p.ksum + (size_t)bh * D + (tid & (D - 1)));
#pragma unroll
        for (int bt = 0; bt < BBATCH; ++bt) {
            if (bt < nbatch) {
#pragma unroll
                for (int ps = 0; ps < BPASS; ++ps) {
                    const int j = min((bt * BPASS + ps) * BROWS + brl, p.Bt - 1);   // rows past the block: masked below
                    kw[bt][ps] = load16_async(knew + (size_t)j * D + bu * 8);
                }
            }
        }
    };
    if (need_sum) request_rows();
    // then the K half of tile t0 and the queries (what the first S^T reads), then the V half and tile
    // t0 + 1: one memory round trip covers all of it, and the order of arrival is the order of use
    if (ntl > 0) issue_half(t0, false);
    KD_TL(14);  // block rows and first K tile requested

    // ---- query rows of this lane (one per block): B operands of S^T = K Q^T, kept in registers.
    // Row m of a head is query (m / Bt, m % Bt) and the rows are contiguous in memory, so a wave's
    // 32 NQ rows are one block of memory: it is copied asynchronously, whole rows at a time, into
    // the wave's piece of the two ring buffers that tiles t0 + 2 and t0 + 3 will use later (with
    // the K swizzle), and read from there into registers.  Loading the B-operand layout directly
    // would touch 32 rows per instruction.
    // ALT (a HELP kernel whose workgroup has a single wave's worth of query rows: decode): waves 0 and 1
    // both hold those rows and take alternate key tiles -- in every step one of them forms S^T of its
    // next tile while the other turns the logits of its current tile into weights and multiplies
    // with V, so the two halves of a step run side by side on two SIMDs.  Each keeps its own
    // running maximum, row sum and output and writes them as a partial of its own: to the merge
    // the two look like two more key splits (p.psplits = 2 p.splits).
    static_assert(!ALT || HELP, "alternating waves are a mode of the kernel with helper waves");
    constexpr bool alt = ALT;
    const int wave_q = alt ? 0 : wave;                // whose query rows this wave holds
    int mrow[NQ], qg[NQ], qj[NQ], vis[NQ];
    bool valid[NQ];
    bf16x8 qreg[NQ][NC];
#pragma unroll
    for (int a = 0; a < NQ; ++a) {
        mrow[a] = mt * TM + wave_q * (32 * NQ) + 32 * a + l32;
        valid[a] = mrow[a] < Mtot;
        qg[a] = valid[a] ? mrow[a] / p.Bt : 0;
        qj[a] = valid[a] ? mrow[a] % p.Bt : 0;
        vis[a] = p.len + qj[a] + 1;  // rows [0, vis) are visible: all cached rows, block rows 0..j
    }
    const bool active = !HELP || (alt ? wave < 2 : mt * TM + wave * (32 * NQ) < Mtot);   // wave uniform
    constexpr int QROWS = 32 * NQ, QBYTES = QROWS * ROWB;
    static_assert(NW * QBYTES <= 2 * 2 * TILE_B && (2 * TILE_B) % QBYTES == 0, "query staging uses two ring buffers");
    const int qoff = wave * QBYTES, qhalf = qoff / (2 * TILE_B);
    unsigned char *qwave = smem + (size_t)((t0 + 2 + qhalf) % STAGES) * 2 * TILE_B + (qoff - qhalf * 2 * TILE_B);
    {
        const char *qhead = reinterpret_cast<const char *>(p.q + (size_t)(b * p.hq + kvh * p.G) * p.Bt * D);
        const int m0 = mt * TM + wave_q * QROWS;   // first row of the wave
        if (m0 + QROWS <= Mtot) {
            // every row exists: one base address for the wave, a 32-bit offset per lane and copy
            const int r0 = lane / UPR;
#pragma unroll
            for (int i = 0; i < QBYTES / 1024; ++i) {
                const int r = RPL * i + r0;
                async_copy16((uint32_t)(uintptr_t)qwave + 1024u * i, qhead + (size_t)m0 * ROWB,
                             (uint32_t)(r * ROWB + (((lane % UPR) ^ (r & (UPR - 1))) * 16)));
            }
        } else {
#pragma unroll
            for (int i = 0; i < QBYTES / 1024; ++i) {
                const int r = RPL * i + lane / UPR;                       // row inside the wave's block
                const int m = min(m0 + r, Mtot - 1);                      // rows past the end repeat the last one
                async_copy16((uint32_t)(uintptr_t)qwave + 1024u * i,
                             qhead + (size_t)m * ROWB + (((lane % UPR) ^ (r & (UPR - 1))) * 16));
            }
        }
    }
    KD_TL(15);  // queries requested
    if (ntl > 0) issue_half(t0, true);
    if (ntl > 1) issue_tile(t0 + 1);
    KD_TL(1);   // first two tiles and the queries requested

    // ---- anchor, part 2: the block's rows have landed when only the copies issued behind them remain
    constexpr int QCOPIES = 32 * NQ * ROWB / 1024;   // copies of a wave's query rows
    const int behind_rows = (ntl > 0 ? LPW : 0) + QCOPIES + (ntl > 1 ? LPW : 0);   // uniform
    double bacc[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) bacc[i] = 0.0;
    auto add_rows = [&](const u32x4 (&w)[BPASS], int j0) {   // rows j0 + pass * BROWS + brl of the block
#pragma unroll
        for (int ps = 0; ps < BPASS; ++ps) {
            const bool live = j0 + ps * BROWS + brl < p.Bt;
            double x[8];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const uint32_t wi = live ? w[ps][i] : 0u;   // (a row past the block adds zeros)
                x[2 * i] = bf16_lo(wi);
                x[2 * i + 1] = bf16_hi(wi);
            }
            double inv = 1.0;
            if (p.anchor_mode == 1) {  // unit keys (Eq. 7): x / |k_j|, a zero key adds nothing
                double k2 = 0.0;
#pragma unroll
                for (int i = 0; i < 8; ++i) k2 += x[i] * x[i];
                k2 = row_allreduce_f64<UPR>(k2);
                const double nk = sqrt(k2);
                inv = nk > 0.0 ? 1.0 / nk : 0.0;
            }
#pragma unroll
            for (int i = 0; i < 8; ++i) bacc[i] += (p.anchor_mode == 1) ? x[i] * inv : x[i];
        }
    };
    double ksum_before = 0.0;
    if (need_sum) {
        wait_copies_upto(behind_rows);
        loads_landed(ksum_raw, kw);
        ksum_before = __hiloint2double((int)ksum_raw[1], (int)ksum_raw[0]);
#pragma unroll
        for (int bt = 0; bt < BBATCH; ++bt)
            if (bt < nbatch) add_rows(kw[bt], bt * BPASS * BROWS);
        // a block of more rows than were requested up front (rare): batch by batch, each waiting for
        // everything in flight
        for (int j0 = BBATCH * BPASS * BROWS; j0 < p.Bt; j0 += BPASS * BROWS) {   // uniform
#pragma unroll
            for (int ps = 0; ps < BPASS; ++ps)
                kw[0][ps] = load16_async(knew + (size_t)min(j0 + ps * BROWS + brl, p.Bt - 1) * D + bu * 8);
            wait_copies<0>();
            loads_landed(ksum_raw, kw);
            add_rows(kw[0], j0);
        }
        // fold the lanes that hold the same unit (bu), then the waves
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            if constexpr (UPR == 16) bacc[i] = sum_over_rows_f64(bacc[i]);
            else {
#pragma unroll
                for (int off = UPR; off < 64; off <<= 1) bacc[i] += shfl_xor_f64(bacc[i], off);
            }
        }
        if (lane < UPR) {
#pragma unroll
            for (int i = 0; i < 8; ++i) bs_part[wave][bu * 8 + i] = bacc[i];
        }
        // (the per-wave sums are published by the barrier of the prologue below and added up after it)
    }
    KD_TL(2);   // block rows landed, summed and folded

    // ---- the queries go from LDS to registers (a wave reads only what its own copies wrote) once
    // they and the K half of tile t0 have landed.  With two tiles or more the V half and tile t0 + 1
    // may still fly: the first step of the loop waits for them.  A single tile has no such step.
    if (ntl > 1) wait_copies<CPW + LPW>();
    else wait_copies<0>();
    KD_TL(3);   // queries and first K tile landed
#pragma unroll
    for (int a = 0; a < NQ; ++a)
#pragma unroll
        for (int c = 0; c < NC; ++c)
            qreg[a][c] = as_bf16x8(*reinterpret_cast<const u32x4 *>(
                qwave + (32 * a + l32) * ROWB + (((2 * c + h) ^ (l32 & (UPR - 1))) * 16)));
    double ksum_after = 0.0;   // element tid of the new key sum (tid < D), stored at the end by the writer

    KD_TL(4);   // queries in registers, block sum folded
    f32x16 oacc[NQ][NDB];
    float mref[NQ], lrun[NQ][2];  // the row sum runs in two independent chains
#pragma unroll
    for (int a = 0; a < NQ; ++a) {
        mref[a] = -INFINITY;
        lrun[a][0] = lrun[a][1] = 0.f;
#pragma unroll
        for (int db = 0; db < NDB; ++db)
#pragma unroll
            for (int e = 0; e < 16; ++e) oacc[a][db][e] = 0.f;
    }

    // ---- LDS byte offsets of this lane's MFMA A operands.
    // K: row l32 of the key group, unit (2c + h) ^ (row & 7): the offset of k-chunk c is (offset of
    // chunk 0) ^ 32 c for c < 4; the key group and c >> 2 add constants.
    const int kof0 = l32 * ROWB + (h ^ (l32 & (UPR - 1))) * 16;
    // V (transpose read): the lane's 16-lane group fetches keys k0 .. k0 + 3 (k0 = 16 c + 4 h, + 8 for
    // the second read) x columns d0 .. d0 + 15 (d0 = 32 db + 16 (group & 1)); this lane supplies row
    // k0 + (lane % 16) / 4, columns d0 + 4 (lane % 4) .. + 3 and receives column d0 + lane % 16.
    // The swizzled unit is (4 db + 2 (group & 1) + (lane % 4) / 2) ^ 2 (row & 3) = (per-lane part) ^ 4 db.
    const int i16 = lane & 15, vrow = 4 * h + (i16 >> 2);
    const int vof0 =
        vrow * ROWB + (((2 * ((lane >> 4) & 1) + ((i16 & 3) >> 1)) ^ (VSW * (vrow & 3))) * 16) + (i16 & 1) * 8;

    // S^T of one 64-key tile for both query blocks: s[a][kg], kg = 32-key group
    auto qk_tile = [&](const unsigned char *tK, f32x16 (&s)[NQ][2]) {
        const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int kg = 0; kg < 2; ++kg)
#pragma unroll
            for (int c = 0; c < NC; ++c) {
                const bf16x8 ka = as_bf16x8(*reinterpret_cast<const u32x4 *>(
                    tK + ((kof0 ^ (c * 32)) + kg * 32 * ROWB)));
#pragma unroll
                for (int a = 0; a < NQ; ++a)
                    s[a][kg] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka, qreg[a][c], c == 0 ? zero : s[a][kg], 0, 0, 0);
            }
    };
    // causal mask of an edge tile: accumulator element e of group kg holds key
    // r0 + 32 kg + 4 h + 8 (e / 4) + e % 4
    auto mask_tile = [&](f32x16 (&s)[NQ][2], int r0) {
#pragma unroll
        for (int a = 0; a < NQ; ++a) {
            const int lim = vis[a] - r0 - 4 * h;
#pragma unroll
            for (int kg = 0; kg < 2; ++kg)
#pragma unroll
                for (int e = 0; e < 16; ++e)
                    s[a][kg][e] = (32 * kg + 8 * (e >> 2) + (e & 3)) < lim ? s[a][kg][e] : -INFINITY;
        }
    };
    // reference-max decision for a tile whose per-lane logit maxima are mloc: the reference only
    // moves when the tile max exceeds it by 2^SLACK (lazy rescale); then O and l are brought to
    // the new reference
    auto new_reference = [&](const float (&mloc)[NQ]) {
        float mtile[NQ];
        bool need[NQ];
#pragma unroll
        for (int a = 0; a < NQ; ++a) {
            mtile[a] = max_halves(mloc[a]) * p.scale_log2e;
            need[a] = mtile[a] > mref[a] + RESCALE_SLACK;
        }
        bool any = false;
#pragma unroll
        for (int a = 0; a < NQ; ++a) any = any || need[a];
        if (__builtin_amdgcn_ballot_w64(any) != 0) {
#pragma unroll
            for (int a = 0; a < NQ; ++a) {
                const float alpha = need[a] ? __builtin_amdgcn_exp2f(mref[a] - mtile[a]) : 1.f;
                mref[a] = need[a] ? mtile[a] : mref[a];
                lrun[a][0] *= alpha;
                lrun[a][1] *= alpha;
#pragma unroll
                for (int db = 0; db < NDB; ++db)
#pragma unroll
                    for (int e = 0; e < 16; ++e) oacc[a][db][e] *= alpha;
            }
        }
    };
    auto tile_max = [&](const f32x16 (&s)[NQ][2], float (&mloc)[NQ]) {
#pragma unroll
        for (int a = 0; a < NQ; ++a) {
            mloc[a] = max3_raw(s[a][0][0], s[a][1][0], s[a][0][0]);
#pragma unroll
            for (int e = 1; e < 16; ++e) mloc[a] = max3_raw(mloc[a], s[a][0][e], s[a][1][e]);
        }
    };
    // LDS fragment reads
    // fragment i = (key group i % 2, k-chunk i / 2): consecutive MFMAs alternate between the two
    // accumulators, so none waits for the result of the one before it
    auto read_k = [&](const unsigned char *tK, int i) {
        const int kg = i % 2, c = i / 2;
        return as_bf16x8(*reinterpret_cast<const u32x4 *>(
            tK + ((kof0 ^ (c * 32)) + kg * 32 * ROWB)));
    };
    auto read_v = [&](const unsigned char *tV, int j) {   // fragment j = (key chunk j / NDB, d block j % NDB)
        const int kc = j / NDB, db = j % NDB;
        const unsigned char *ap = tV + ((vof0 ^ (db * 64)) + kc * 16 * ROWB);
        const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3))) *)(ap));
        const s16x4 hi =
            __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3))) *)(ap + 8 * ROWB));
        return __builtin_bit_cast(bf16x8, (s16x8)__builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
    };
    // The 32 NQ exponentials a lane owes per tile are cut into 32 NQ / SL slices of SL: slice i covers
    // block (i / (8 / SL)) % NQ, 16-key chunk kc = i / (8 NQ / SL), accumulator elements
    // 8 (kc % 2) + SL (i % (8 / SL)) .. + SL - 1 of key group kc / 2.  A slice goes through three steps
    // one pipeline step apart, so that no instruction waits for the one before it: F scale and shift,
    // E exponential, C round to bf16 (the B operand of the second MFMA) and add the rounded weights to
    // the row sum.  Small slices spread the vector work evenly between the MFMAs: a wave gets the
    // matrix pipe every other MFMA slot, and what does not fit between two of its MFMAs delays the next.
    constexpr int SL = 2;              // exponentials per slice (2 or 4)
    constexpr int SPC = 8 / SL;        // slices per 16-key chunk and query block
    auto slice_F = [&](const f32x16 (&s)[NQ][2], int i, float (&arg)[SL]) {
        const int a = (i / SPC) % NQ, kc = i / (SPC * NQ), kg = kc >> 1, cc = kc & 1, part = i % SPC;
        const float nmuse = mref[a] == -INFINITY ? 0.f : -mref[a];
#pragma unroll
        for (int r = 0; r < SL; ++r) {
            arg[r] = __builtin_fmaf(s[a][kg][8 * cc + SL * part + r], p.scale_log2e, nmuse);
            asm volatile("" : "+v"(arg[r]));   // computed here, not where the optimiser finds its use
        }
    };
    auto slice_E = [&](const float (&arg)[SL], float (&ex)[SL]) {
#pragma unroll
        for (int r = 0; r < SL; ++r) {
            ex[r] = __builtin_amdgcn_exp2f(arg[r]);
            asm volatile("" : "+v"(ex[r]));
        }
    };
    auto slice_C = [&](const float (&ex)[SL], int i, bf16x8 (&pk)[NQ][4]) {
        const int a = (i / SPC) % NQ, kc = i / (SPC * NQ), part = i % SPC;
#pragma unroll
        for (int r = 0; r < SL / 2; ++r) {
            const int e0 = SL * part + 2 * r;   // element pair inside the 8 of this lane's chunk
            bf16x2 pr;
            pr[0] = (__bf16)ex[2 * r];
            pr[1] = (__bf16)ex[2 * r + 1];
            pk[a][kc][e0] = pr[0];
            pk[a][kc][e0 + 1] = pr[1];
            const bf16x2 one = {(__bf16)1.0f, (__bf16)1.0f};
            const int chain = (e0 >> 1) & 1;    // the row sum runs in two chains
            lrun[a][chain] = __builtin_amdgcn_fdot2_f32_bf16(pr, one, lrun[a][chain], false);
            asm volatile("" : "+v"(lrun[a][chain]));
        }
    };

    // ---- cosine score of the rows of one K tile (appendix "FLOP count of KeyDiff"), read from LDS
    // while the tile is there for the attention: s_i = mu.k_i / max(|mu| |k_i|, eps) in double on
    // the bf16 values, rounded once to float.  The query-row tiles of a head share the K tiles, so
    // tile t is scored by the workgroup with mt == t % mtiles.  UPR lanes share a row.
    int staged = 0;   // rows this wave has staged (wave uniform)
    // Generation phase (p.argmax_rec): the row to evict is the arg-max of the scores, so every lane keeps
    // the best of the rows it finishes as (orderable score bits << 32 | row), and whether it met the
    // same score bits on another row (then the token position has to decide, which the selection does
    // from all scores as before); the workgroup leaves one such record for the selection.
    unsigned long long am_best = 0;
    bool am_tie = false;
    auto am_merge = [](unsigned long long &best, bool &tie, unsigned long long ob, bool ot) {
        const uint32_t hb = (uint32_t)(best >> 32), ho = (uint32_t)(ob >> 32);
        if (ho > hb) {
            best = ob;
            tie = ot;
        } else if (ho == hb && ob != 0) {
            tie = tie || ot || ob != best;
            best = ob > best ? ob : best;
        }
    };
    auto flush_scores = [&]() {
        // same wave wrote and reads: the LDS accesses of one wave complete in order; the fences only
        // keep the compiler from moving the reads above the writes, and later writes above the reads
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        if (lane < staged) {
            const int row = st_row[wave][lane];
            if (row < p.n) {
                double nmu2 = 0.0;
#pragma unroll
                for (int w = 0; w < NW; ++w) nmu2 += (red[w][0] + red[w][1]) + (red[w][2] + red[w][3]);
                const float sc = finish_score(st_dot[wave][lane], st_k2[wave][lane], sqrt(nmu2), p.eps);
                p.scores[(size_t)bh * p.cap + row] = sc;
                if (p.scores_out) p.scores_out[(size_t)bh * p.n + row] = sc;
                if constexpr (HELP) am_merge(am_best, am_tie, ((unsigned long long)orderable(sc) << 32) | (uint32_t)row, false);
            }
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        staged = 0;
    };
    auto score_tile_fixed = [&](int t) {
        constexpr int RPP = 64 / UPR;            // rows per pass
        constexpr int PASSES = TILE_KEYS / NW / RPP;
        static_assert(PASSES >= 1, "a wave scores at least one pass of rows per tile");
        const unsigned char *tK = smem + (size_t)(t % STAGES) * 2 * TILE_B;
        const int u = lane % UPR, rl = lane / UPR;
        double mu8[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) mu8[i] = mu_s[u * 8 + i];
        double dotp[PASSES], k2p[PASSES];
#pragma unroll
        for (int ps = 0; ps < PASSES; ++ps) {
            const int r = wave * (TILE_KEYS / NW) + ps * RPP + rl;   // row inside the tile
            const u32x4 w = *reinterpret_cast<const u32x4 *>(tK + r * ROWB + ((u ^ (r & (UPR - 1))) * 16));
            // products of two bf16 values are exact in double, so fma(a, a, .) is the plain sum of
            // squares; mu.k takes one rounding per term either way
            double dot = 0.0, k2 = 0.0;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const double a = bf16_lo(w[i]), b = bf16_hi(w[i]);
                dot = __builtin_fma(mu8[2 * i], a, dot);
                k2 = __builtin_fma(a, a, k2);
                dot = __builtin_fma(mu8[2 * i + 1], b, dot);
                k2 = __builtin_fma(b, b, k2);
            }
            dotp[ps] = dot;
            k2p[ps] = k2;
        }
        if constexpr (UPR == 16 && PASSES == 2) {
            // lanes 0-3 of a row end with mu.k of pass 0, 4-7 with |k|^2 of pass 0, 8-11 and 12-15
            // with those of pass 1
            const double v = row_reduce_scatter4_f64(dotp[0], k2p[0], dotp[1], k2p[1], u);
            if ((u & 3) == 0) {
                const int ps = u >> 3;
                const int slot = staged + ps * RPP + rl;
                if (u & 4) st_k2[wave][slot] = v;
                else {
                    st_dot[wave][slot] = v;
                    st_row[wave][slot] = t * TILE_KEYS + wave * (TILE_KEYS / NW) + ps * RPP + rl;
                }
            }
        } else {
#pragma unroll
            for (int ps = 0; ps < PASSES; ++ps) {
                const double dot = row_allreduce_f64<UPR>(dotp[ps]), k2 = row_allreduce_f64<UPR>(k2p[ps]);
                if (u == 0) {
                    const int slot = staged + ps * RPP + rl;
                    st_dot[wave][slot] = dot;
                    st_k2[wave][slot] = k2;
                    st_row[wave][slot] = t * TILE_KEYS + wave * (TILE_KEYS / NW) + ps * RPP + rl;
                }
            }
        }
        staged += PASSES * RPP;
        if (staged + PASSES * RPP > 64) flush_scores();
    };
    // Which waves score when some have no query rows: only those, so that the waves carrying the
    // attention do not also carry the score.  A scoring wave takes the passes (RPP consecutive rows
    // each) sidx, sidx + nscore, ... of every tile its workgroup owns.
    const int nactive = !HELP ? NW : alt ? 2 : min(NW, (Mtot - mt * TM + 32 * NQ - 1) / (32 * NQ));
    const int nscore = nactive < NW ? NW - nactive : NW;
    const int sidx = nactive < NW ? wave - nactive : wave;   // negative: this wave does not score
    auto score_tile_shared = [&](int t) {
        constexpr int RPP = 64 / UPR;              // rows per pass
        constexpr int TPASS = TILE_KEYS / RPP;     // passes per tile
        if (sidx < 0) return;
        const unsigned char *tK = smem + (size_t)(t % STAGES) * 2 * TILE_B;
        const int u = lane % UPR, rl = lane / UPR;
        double mu8[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) mu8[i] = mu_s[u * 8 + i];
        auto partial = [&](int ps, double &dot, double &k2) {
            const int r = ps * RPP + rl;
            const u32x4 w = *reinterpret_cast<const u32x4 *>(tK + r * ROWB + ((u ^ (r & (UPR - 1))) * 16));
            dot = 0.0;
            k2 = 0.0;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const double a = bf16_lo(w[i]), b = bf16_hi(w[i]);
                dot = __builtin_fma(mu8[2 * i], a, dot);
                k2 = __builtin_fma(a, a, k2);
                dot = __builtin_fma(mu8[2 * i + 1], b, dot);
                k2 = __builtin_fma(b, b, k2);
            }
        };
        int ps = sidx;   // wave uniform
        if constexpr (UPR == 16) {
            // two passes at a time, see score_tile
            for (; ps + nscore < TPASS; ps += 2 * nscore) {
                double d0, q0, d1, q1;
                partial(ps, d0, q0);
                partial(ps + nscore, d1, q1);
                const double v = row_reduce_scatter4_f64(d0, q0, d1, q1, u);
                if ((u & 3) == 0) {
                    const int second = u >> 3;
                    const int slot = staged + second * RPP + rl;
                    if (u & 4) st_k2[wave][slot] = v;
                    else {
                        st_dot[wave][slot] = v;
                        st_row[wave][slot] = t * TILE_KEYS + (ps + second * nscore) * RPP + rl;
                    }
                }
                staged += 2 * RPP;
            }
        }
        for (; ps < TPASS; ps += nscore) {
            double dot, k2;
            partial(ps, dot, k2);
            dot = row_allreduce_f64<UPR>(dot);
            k2 = row_allreduce_f64<UPR>(k2);
            if (u == 0) {
                const int slot = staged + rl;
                st_dot[wave][slot] = dot;
                st_k2[wave][slot] = k2;
                st_row[wave][slot] = t * TILE_KEYS + ps * RPP + rl;
            }
            staged += RPP;
        }
        // room for the next tile's rows of this wave?
        if (staged + ((TPASS + nscore - 1) / nscore) * RPP > 64) flush_scores();
    };
    auto score_tile = [&](int t) {
        if constexpr (HELP) score_tile_shared(t);
        else score_tile_fixed(t);
    };
    const bool scoring = p.do_score != 0;

    const int tint = min(t1, max(t0, p.len / TILE_KEYS));  // tiles before it: every key cached, no mask
    f32x16 s[NQ][2];
    if (ntl > 0) {
        // ---- prologue: every wave has its queries in registers and its part of tiles t0, t0 + 1 in
        // LDS; the staging buffers are free for tile t0 + 2, which flies while S^T of tile t0 is formed
        __syncthreads();
        static_assert(STAGES == 4, "the prologue fills three of the four ring buffers");
        KD_TL(5);   // first barrier passed
        if (ntl > 2) issue_tile(t0 + 2);
        if (need_sum) {
            // the anchor: waves 0 .. D/64 - 1 form it while the others already work on tile t0
            double sq = 0.0;
            if (tid < D) {
                double tot = 0.0;
#pragma unroll
                for (int w = 0; w < NW; ++w) tot += bs_part[w][tid];
                ksum_after = ksum_before + tot;
                const double m = ksum_after / (double)p.n;
                mu_s[tid] = m;
                sq = m * m;
            }
            sq = row_allreduce_f64<16>(sq);
            if ((lane & 15) == 0) red[wave][lane >> 4] = sq;
        }
        KD_TL(6);   // anchor formed
        if (active && !(alt && wave == 1)) {   // (ALT: tile t0 is wave 0's; wave 1 starts with t0 + 1 inside the loop)
            qk_tile(smem + (size_t)(t0 % STAGES) * 2 * TILE_B, s);
            if (t0 >= tint) mask_tile(s, t0 * TILE_KEYS);
            float mloc[NQ];
            tile_max(s, mloc);
#pragma unroll
            for (int a = 0; a < NQ; ++a)   // first reference: nothing accumulated yet, nothing to rescale
                mref[a] = max_halves(mloc[a]) * p.scale_log2e;
        }
        // The anchor is complete before any row is scored: the barrier that opens the first step of
        // the loop publishes it; a range of a single tile has no such step.
        if (need_sum && ntl == 1) __syncthreads();
        KD_TL(7);   // logits of the first tile ready: the loop starts
    }
    // ---- the tile loop, software pipelined by hand (at most two waves share a SIMD: little else
    // hides a latency).  Iteration t:
    //   stage A  the 2 NC MFMA groups of S^T(t + 1), each issued with the K fragment read a few
    //            groups ahead, a share of the copies of tile t + 3 and of the exponentials of tile t;
    //   stage B  the 4 NDB MFMA groups of O^T += V^T P^T(t), each with the V^T fragment read a few
    //            groups ahead, the rest of the exponentials and one slice of the max scan of tile t + 1;
    //   then the cosine score of tile t's rows if this workgroup owns them.
    // The scheduling barriers pin that order.  Tiles t + 2 and t + 3 are in flight meanwhile.
    // COPY: 0 no tile left to fetch, 1 the tile to fetch lies entirely in the cache, 2 decide per copy
    auto step = [&](int t, f32x16 (&sc)[NQ][2], f32x16 (&sn)[NQ][2], auto next_tag, auto masked_tag, auto copy_tag) {
        constexpr bool NEXT = decltype(next_tag)::value, MASKED = decltype(masked_tag)::value;
        constexpr int COPY = decltype(copy_tag)::value;
        constexpr int NA = 2 * NC, NB = 4 * NDB;
        static_assert((NA == 16 && NB == 16) || (NA == 8 && NB == 8), "slice counts below assume D = 128 or 64");
        // The exponential slices are spread evenly over stage A and the first half of stage B (whose
        // second half multiplies with the weights computed last): group g runs in slot g SLOTS / NG,
        // slots [0, NA) being the steps of stage A and [NA, SLOTS) steps of stage B.
        constexpr int NS = 32 * NQ / SL;           // exponential slices per tile
        constexpr int SLOTS = NA + NB / 2;
        constexpr int SPG = NS > SLOTS ? 2 : 1;    // slices per group
        constexpr int NG = NS / SPG;
        auto slot_of = [](int g) { return g * SLOTS / NG; };
        // one pipeline beat: E of group g, C of group g - 1, F of group g + 1
        auto beat = [&](int g, float (&arg)[2][SPG][SL], float (&ex)[2][SPG][SL], bf16x8 (&pk)[NQ][4]) {
            if (g < NG) {
#pragma unroll
                for (int e = 0; e < SPG; ++e) slice_E(arg[g & 1][e], ex[g & 1][e]);
            }
            if (g > 0) {
#pragma unroll
                for (int e = 0; e < SPG; ++e) slice_C(ex[(g - 1) & 1][e], SPG * (g - 1) + e, pk);
            }
            if (g + 1 < NG) {
#pragma unroll
                for (int e = 0; e < SPG; ++e) slice_F(sc, SPG * (g + 1) + e, arg[(g + 1) & 1][e]);
            }
        };
        constexpr int KAHEAD = 2, VAHEAD = 2;  // fragment reads run this many MFMA groups ahead (deeper spills)
        const unsigned char *tV = smem + (size_t)(t % STAGES) * 2 * TILE_B + TILE_B;
        const unsigned char *tK = smem + (size_t)((t + 1) % STAGES) * 2 * TILE_B;
        bf16x8 pk[NQ][4];
        bf16x8 kf[KAHEAD + 1], vf[VAHEAD + 1];
        float arg[2][SPG][SL], ex[2][SPG][SL];
        if (NEXT) {
            // tile t + 1 has landed when at most the copies of tile t + 2 remain; the barrier
            // publishes every wave's part and retires the buffer tile t - 1 used
            if (t + 2 < t1) wait_copies<LPW>();
            else wait_copies<0>();
            __syncthreads();
        }
#ifdef KD_TIMELINE
        if (t == t0 + 2) KD_TL(16);   // step t0 + 2: barrier passed
        if (t == t0 + 3) KD_TL(20);
#endif
        if (HELP && !active) {
            if (NEXT) {
#pragma unroll
                for (int c = 0; c < LPW; ++c) {
                    if (COPY == 1) issue_copy_cached(t + STAGES - 1, c);
                    if (COPY == 2 && t + STAGES - 1 < t1) issue_copy(t + STAGES - 1, c);
                }
            }
            if (scoring && t % p.mtiles == mt) score_tile(t);
            return;
        }
        if constexpr (ALT) {
            // this wave's half of the step: the tile after this one is mine -> its logits; this tile is
            // mine -> its weights and the product with V
            auto fetch_ahead = [&]() {
                if (NEXT) {
#pragma unroll
                    for (int c = 0; c < LPW; ++c) {
                        if (COPY == 1) issue_copy_cached(t + STAGES - 1, c);
                        if (COPY == 2 && t + STAGES - 1 < t1) issue_copy(t + STAGES - 1, c);
                    }
                }
            };
            const bool mine = ((t - t0) & 1) == wave;   // wave uniform
            if (mine) {
                // per 16-key chunk: its V^T fragments are requested, its weights formed (the MFMAs of
                // the chunk before run meanwhile), then its MFMAs issued
                constexpr int SPK = NS / 4;   // slices per chunk (NQ == 1)
                static_assert(NQ == 1, "the alternating mode is written for one query block per wave");
                bf16x8 vfr[2][NDB];
#pragma unroll
                for (int db = 0; db < NDB; ++db) vfr[0][db] = read_v(tV, db);
#pragma unroll
                for (int kc = 0; kc < 4; ++kc) {
                    if (kc + 1 < 4) {
#pragma unroll
                        for (int db = 0; db < NDB; ++db) vfr[(kc + 1) & 1][db] = read_v(tV, (kc + 1) * NDB + db);
                    }
                    // the chunk's slices step by step, not slice by slice: the SPK instructions of a step
                    // are independent of each other, so none waits for the one before it (this wave is
                    // alone on its SIMD for the length of the chain)
                    float fa[SPK][SL], fe[SPK][SL];
#pragma unroll
                    for (int i = 0; i < SPK; ++i) slice_F(s, kc * SPK + i, fa[i]);
#pragma unroll
                    for (int i = 0; i < SPK; ++i) slice_E(fa[i], fe[i]);
#pragma unroll
                    for (int i = 0; i < SPK; ++i) slice_C(fe[i], kc * SPK + i, pk);
#pragma unroll
                    for (int db = 0; db < NDB; ++db)
                        oacc[0][db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vfr[kc & 1][db], pk[0][kc], oacc[0][db], 0, 0, 0);
                    __builtin_amdgcn_sched_barrier(0);
                }
            } else if (NEXT) {
                qk_tile(tK, s);
                if (MASKED) mask_tile(s, (t + 1) * TILE_KEYS);
                float mloc[NQ];
                tile_max(s, mloc);
                new_reference(mloc);
            }
            // the wave's share of the copies of tile t + 3 goes out after its half of the step, not before it: a
            // copy can sit in front of a full memory queue for a third of the time the half takes, and the
            // step ends when the slower of the two waves is done (the tile is not needed for two more steps)
            fetch_ahead();
#ifdef KD_TIMELINE
            if (t == t0 + 2) KD_TL(17);   // wave 0: weights and product with V of its tile done
            if (t == t0 + 3) KD_TL(21);   // wave 0: logits of its next tile done
#endif
            return;
        } else {
        if (NEXT) {
#pragma unroll
            for (int i = 0; i < KAHEAD; ++i) kf[i] = read_k(tK, i);
        }
#pragma unroll
        for (int e = 0; e < SPG; ++e) slice_F(sc, e, arg[0][e]);
        const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int i = 0; i < NA; ++i) {
            if (NEXT) {
                if (i + KAHEAD < NA) kf[(i + KAHEAD) % (KAHEAD + 1)] = read_k(tK, i + KAHEAD);
                const int kg = i % 2, c = i / 2;
#pragma unroll
                for (int a = 0; a < NQ; ++a)
                    sn[a][kg] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[i % (KAHEAD + 1)], qreg[a][c],
                                                                        c == 0 ? zero : sn[a][kg], 0, 0, 0);
            }
            if (i >= NA - VAHEAD) vf[i - (NA - VAHEAD)] = read_v(tV, i - (NA - VAHEAD));
            if (NEXT) {
                // the copies of tile t + 3 (into the buffer the barrier above retired), a few per
                // step: issued in one burst they would fill the memory pipeline's queue and stall
                // this wave -- the only one feeding this SIMD's matrix pipe
#pragma unroll
                for (int c = i * LPW / NA; c < (i + 1) * LPW / NA; ++c) {
                    if (COPY == 1) issue_copy_cached(t + STAGES - 1, c);
                    if (COPY == 2 && t + STAGES - 1 < t1) issue_copy(t + STAGES - 1, c);
                }
            }
#pragma unroll
            for (int g = 0; g < NG; ++g)
                if (slot_of(g) == i) beat(g, arg, ex, pk);
            __builtin_amdgcn_sched_barrier(0);
        }
#ifdef KD_TIMELINE
        if (t == t0 + 2) KD_TL(17);   // stage A done
        if (t == t0 + 3) KD_TL(21);
#endif
        if (NEXT && MASKED) mask_tile(sn, (t + 1) * TILE_KEYS);
        float mch[NQ][2];  // max scan of tile t + 1 in two chains per block
#pragma unroll
        for (int j = 0; j < NB; ++j) {
            if (j + VAHEAD < NB) vf[(j + VAHEAD) % (VAHEAD + 1)] = read_v(tV, j + VAHEAD);
            // remaining exponential groups; the last beat only rounds the last group's weights
#pragma unroll
            for (int g = 0; g <= NG; ++g)
                if ((g < NG ? slot_of(g) : slot_of(NG - 1) + 1) == NA + j) beat(g, arg, ex, pk);
            const int kc = j / NDB, db = j % NDB;
#pragma unroll
            for (int a = 0; a < NQ; ++a)
                oacc[a][db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[j % (VAHEAD + 1)], pk[a][kc], oacc[a][db], 0, 0, 0);
            if (NEXT) {
                constexpr int PER = 16 / NB;  // accumulator elements per step (both key groups at once)
#pragma unroll
                for (int a = 0; a < NQ; ++a)
#pragma unroll
                    for (int r = 0; r < PER; ++r) {
                        const int e = PER * j + r;
                        mch[a][e & 1] = e < 2 ? max3_raw(sn[a][0][e], sn[a][1][e], sn[a][0][e])
                                              : max3_raw(mch[a][e & 1], sn[a][0][e], sn[a][1][e]);
                    }
            }
            __builtin_amdgcn_sched_barrier(0);
        }
#ifdef KD_TIMELINE
        if (t == t0 + 2) KD_TL(18);   // stage B done
        if (t == t0 + 3) KD_TL(22);
#endif
        // tile t is still in its buffer (recycled in the next iteration): score its rows
        if (scoring && t % p.mtiles == mt) score_tile(t);
#ifdef KD_TIMELINE
        if (t == t0 + 2) KD_TL(19);   // tile scored (if this workgroup owns it)
        if (t == t0 + 3) KD_TL(23);
#endif
        float mloc[NQ];
#pragma unroll
        for (int a = 0; a < NQ; ++a) mloc[a] = NEXT ? max3_raw(mch[a][0], mch[a][1], mch[a][0]) : 0.f;
        if (NEXT) {
            new_reference(mloc);
        }
        }   // !ALT
    };
    // Four loops, so that the common iterations carry no decisions: (1) tile t + 1 unmasked and tile
    // t + 3 entirely cached; (2) tile t + 1 unmasked, nothing left to fetch; (3) the general case
    // (edge tiles: causal mask, rows from the block, partial tiles); then the last tile.
    using T_ = std::true_type;
    using F_ = std::false_type;
    // The logits of tile t + 1 are formed in one array while those of tile t are consumed from the
    // other; the hot loop runs two steps per iteration with the roles swapped, the other loops move
    // the new logits back (32 register moves per lane that the hot loop is spared).
    f32x16 s2[NQ][2];
    auto step1 = [&](int t, auto next_tag, auto masked_tag, auto copy_tag) {
        step(t, s, s2, next_tag, masked_tag, copy_tag);
        if (!ALT && decltype(next_tag)::value) {   // (alternating waves keep their logits in s throughout)
#pragma unroll
            for (int a = 0; a < NQ; ++a) {
                s[a][0] = s2[a][0];
                s[a][1] = s2[a][1];
            }
        }
    };
    int t = t0;
    const int lim1 = min(tint, t1);
    for (; t + STAGES < lim1; t += 2) {
        step(t, s, s2, T_{}, F_{}, std::integral_constant<int, 1>{});
        step(t + 1, s2, s, T_{}, F_{}, std::integral_constant<int, 1>{});
    }
    for (; t + STAGES - 1 < lim1; ++t) step1(t, T_{}, F_{}, std::integral_constant<int, 1>{});
    if (t + STAGES - 1 >= t1)
        for (; t + 1 < tint; ++t) step1(t, T_{}, F_{}, std::integral_constant<int, 0>{});
    for (; t + 1 < t1; ++t) step1(t, T_{}, T_{}, std::integral_constant<int, 2>{});

    KD_TL(8);   // all steps but the last done
    // ---- append (Eq. 5): this workgroup's slice of the block's rows.  The attention reads the
    // block straight from k_new / v_new, so nothing waits for the append: when the slice is small
    // its loads are issued here, fly during the last tile, and are stored after it.
    const int W = p.mtiles * p.splits, widx = sp * p.mtiles + mt;
    const int j0 = (int)(((unsigned)widx * (unsigned)p.Bt) / (unsigned)W), j1 = (int)(((unsigned)(widx + 1) * (unsigned)p.Bt) / (unsigned)W);
    const int arows = j1 - j0;
    const bool small = arows * UPR * 2 <= NT;
    u32x4 aval = {0u, 0u, 0u, 0u};
    if (small && tid < arows * UPR * 2) {
        const int which = tid >= arows * UPR, rem = tid - which * arows * UPR;
        aval = *reinterpret_cast<const u32x4 *>((which ? vnew : knew) + (size_t)(j0 + rem / UPR) * D + (rem % UPR) * 8);
    }

    if (ntl > 0) step1(t, F_{}, F_{}, std::integral_constant<int, 0>{});
    KD_TL(9);   // last tile done

    // ---- output: stored first, so that the write latency runs under the score flush and the append
    if (active && p.psplits > 1) {
        // Partials leave in the accumulator's own layout, as whole 512-byte slabs with no detour
        // through LDS: slab (db, jj) of a 32-row block holds, for lane (h, l32), the four values
        // d = 32 db + 8 jj + 4 h .. + 3 of row l32.  Only the merge reads them, in the same order, in
        // the next launch and on other compute units: the stores go through to memory at once
        // (device-scope relaxed atomics) instead of waiting in L2 for the write-back at the end of
        // the kernel (measured: 0.5 us off the kernel; the same for scores and row sums cost time).
        constexpr int SLABS = D / 8;
        const int nblk = (Mtot + 31) / 32;
#pragma unroll
        for (int a = 0; a < NQ; ++a) {
            const float lsum = lrun[a][0] + lrun[a][1];
            const float ltot = sum_halves(lsum);
            const float inv = ltot > 0.f ? 1.f / ltot : 0.f;   // a row of a split may see no key at all
            const int blk = (mt * TM + wave_q * (32 * NQ)) / 32 + a;
            const int spo = alt ? 2 * sp + wave : sp;   // ALT: the two waves' results are two partials
            _Float16 *base = p.part_o + ((((size_t)spo * BH + bh) * nblk + blk) * SLABS * 64 + lane) * 4;
#pragma unroll
            for (int db = 0; db < NDB; ++db)
#pragma unroll
                for (int jj = 0; jj < 4; ++jj) {
                    f16x4 o;
#pragma unroll
                    for (int r = 0; r < 4; ++r) o[r] = (_Float16)(oacc[a][db][4 * jj + r] * inv);
                    __hip_atomic_store(reinterpret_cast<uint64_t *>(base + (size_t)(4 * db + jj) * 64 * 4),
                                       __builtin_bit_cast(uint64_t, o), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                }
            if (h == 0 && valid[a]) p.part_ml[(size_t)spo * BH * Mtot + (size_t)bh * Mtot + mrow[a]] = make_float2(mref[a], ltot);
        }
    } else if (active) {
        // A single split writes the bf16 output itself.  Accumulator element e of d-block db is
        // d = 32 db + 8 (e / 4) + 4 h + e % 4 of query l32: 8-byte pieces of 32 different rows, which as
        // direct stores would cost one memory transaction per piece.  Each wave transposes its 32 NQ
        // rows through a private piece of LDS (the two ring buffers no tile occupies after the last
        // barrier) and stores whole rows, 16 bytes per lane.
        constexpr int WROWS = 32 * NQ, WBYTES = WROWS * ROWB;
        static_assert(NW * WBYTES <= 2 * 2 * TILE_B, "the transposition uses two ring buffers");
        // stages (t1 + 1) % STAGES and t1 % STAGES: tiles t1 - 3 and t1 - 4 (or never filled)
        const int region = wave * WBYTES;
        auto stage_ptr = [&](int off) {   // byte `off` of the 2-buffer scratch area
            const int half = off / (2 * TILE_B);
            return smem + (size_t)((t1 + 1 - half + STAGES) % STAGES) * 2 * TILE_B + (off - half * 2 * TILE_B);
        };
#pragma unroll
        for (int a = 0; a < NQ; ++a) {
            const float lsum = lrun[a][0] + lrun[a][1];
            const float ltot = sum_halves(lsum);
            const float inv = ltot > 0.f ? 1.f / ltot : 0.f;
            const int row = 32 * a + l32;
#pragma unroll
            for (int db = 0; db < NDB; ++db)
#pragma unroll
                for (int jj = 0; jj < 4; ++jj) {
                    // 16-byte unit 4 db + jj of the row, swizzled by the row; lane half h takes 8 bytes
                    unsigned char *dst = stage_ptr(region + row * ROWB + (((4 * db + jj) ^ (row & (UPR - 1))) * 16) + 8 * h);
                    bf16x4 o;
#pragma unroll
                    for (int r = 0; r < 4; ++r) o[r] = (__bf16)(oacc[a][db][4 * jj + r] * inv);
                    *reinterpret_cast<bf16x4 *>(dst) = o;
                }
        }
        // rows of this wave: m = mbase .. mbase + WROWS - 1, contiguous in `out`
        const int mbase = mt * TM + wave_q * WROWS;
        unsigned char *gbase = reinterpret_cast<unsigned char *>(p.out + ((size_t)(b * p.hq + kvh * p.G) * p.Bt + mbase) * D);
        constexpr int RPI = 1024 / ROWB;   // rows one wave-wide 16-byte-per-lane store covers
#pragma unroll
        for (int i = 0; i < WBYTES / 1024; ++i) {
            const int row = RPI * i + lane / UPR, unit = lane % UPR;
            const u32x4 val = *reinterpret_cast<const u32x4 *>(stage_ptr(region + row * ROWB + ((unit ^ (row & (UPR - 1))) * 16)));
            if (mbase + row < Mtot) *reinterpret_cast<u32x4 *>(gbase + (size_t)row * ROWB + unit * 16) = val;
        }
    }

    KD_TL(10);  // output stores issued
    if (small) {
        if (tid < arows * UPR * 2) {
            const int which = tid >= arows * UPR, rem = tid - which * arows * UPR;
            *reinterpret_cast<u32x4 *>((which ? p.v : p.k) + ((size_t)bh * p.cap + p.len + j0 + rem / UPR) * D + (rem % UPR) * 8) = aval;
        }
    } else {
        for (int u = tid; u < arows * UPR * 2; u += NT) {
            const int which = u >= arows * UPR, rem = u - which * arows * UPR;
            const int j = j0 + rem / UPR, unit = rem % UPR;
            const u32x4 val = *reinterpret_cast<const u32x4 *>((which ? vnew : knew) + (size_t)j * D + unit * 8);
            *reinterpret_cast<u32x4 *>((which ? p.v : p.k) + ((size_t)bh * p.cap + p.len + j) * D + unit * 8) = val;
        }
    }
    for (int j = j0 + tid; j < j1; j += NT) p.pos[(size_t)bh * p.cap + p.len + j] = p.pos0 + j;
    // the key sum after this step, for step_post and for the next step
    if (writer && tid < D) p.ksum_next[(size_t)bh * D + tid] = ksum_after;

    if (scoring) flush_scores();   // last: the square roots and divisions run while the stores above complete
    if constexpr (HELP) {
        if (scoring && p.argmax_rec) {   // uniform
#pragma unroll
            for (int off = 1; off < 64; off <<= 1) {
                const uint32_t lo = __shfl_xor((uint32_t)am_best, off), hi = __shfl_xor((uint32_t)(am_best >> 32), off);
                const bool ot = __shfl_xor((int)am_tie, off) != 0;
                am_merge(am_best, am_tie, ((unsigned long long)hi << 32) | lo, ot);
            }
            unsigned long long *wrec = reinterpret_cast<unsigned long long *>(&st_dot[0][0]);   // staging is over
            __syncthreads();
            if (lane == 0) {
                wrec[2 * wave] = am_best;
                wrec[2 * wave + 1] = am_tie ? 1ull : 0ull;
            }
            __syncthreads();
            if (tid == 0) {
                unsigned long long b0 = 0;
                bool t0_ = false;
                for (int w = 0; w < NW; ++w) am_merge(b0, t0_, wrec[2 * w], wrec[2 * w + 1] != 0);
                unsigned long long *rec = p.argmax_rec + ((size_t)bh * p.splits + sp) * 2;
                rec[0] = b0;
                rec[1] = t0_ ? 1ull : 0ull;
            }
        }
    }
    KD_TL(11);  // append stored, scores flushed
#ifdef KD_TIMELINE
    __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0): the stores of this wave have been acknowledged
    KD_TL(12);
    if (threadIdx.x == 0) {
        kd_tl[30] = (unsigned long long)ntl;
        kd_tl[31] = 1;   // record kind: attention workgroup
    }
    KD_TL_DUMP(p.timeline, blockIdx.x);
#endif
}

template <int D, bool HELP, bool ALT>
__global__ __launch_bounds__(64 * MAIN_WAVES) void step_main_kernel(StepParams p)
{
    warm_arguments<sizeof(StepParams)>();
    step_main_body<D, HELP, ALT>(p, (int)blockIdx.x);
}

// step_main with passengers (8-wave workgroups, with or without helper waves, not the alternating
// mode): the first `ncarry` workgroups run the pending selection and
// compaction of another cache (one head each, parameters `cy`), the rest are the workgroups of
// step_main proper.  A selection is a chain of short dependent stages that keeps one compute unit
// busy per head for about half as long as the attention keeps the others busy: launched this way
// it costs no time of its own.  The two caches share nothing, so no ordering between the two
// kinds of workgroup is needed.
// cy_res: the passengers work on LDS copies of their head's scores and positions (the launch then
// asks for the dynamic LDS that takes)
template <int D, bool HELP>
__global__ __launch_bounds__(CARRY_THREADS) void step_main_carry_kernel(StepParams p, StepParams cy, int ncarry, int cy_res)
{
    warm_arguments<2 * sizeof(StepParams) + 8>();   // both parameter blocks: the role is not known yet
    if ((int)blockIdx.x < ncarry) {
        extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
        PostShared &sh = *reinterpret_cast<PostShared *>(smem);
        unsigned char *dyn = smem + carry_shared_bytes();
        if (cy_res) select_and_compact<D, true, CARRY_THREADS>(cy, sh, dyn, (int)blockIdx.x);
        else select_and_compact<D, false, CARRY_THREADS>(cy, sh, dyn, (int)blockIdx.x);
        return;
    }
    step_main_body<D, HELP, false>(p, (int)blockIdx.x - ncarry);
}

// The same with a third kind of workgroup behind the selection's: `ride.nshift` workgroups that shift
// the rows of an ORDERED cache whose selection ran in an earlier launch (kd_shift.h).  The shift is
// bound by memory traffic the attention leaves unused; it holds the compute units the plan left to
// it for about as long as the attention holds the others.  A kernel of its own, so that the
// launches without a shift keep their code as it is.  (Not for launches with helper waves: their
// attention body leaves no registers to spare, and with this kernel's larger argument block it spilled.)
// (The workgroup counts come first in the argument block, in one cache line: a workgroup finds its role
// with a single trip to the freshly written, cold argument memory instead of one per count.)
struct RideCounts {
    int ncarry, cy_res, nshift;
};
template <int D>
__global__ __launch_bounds__(CARRY_THREADS) void step_main_ride_kernel(RideCounts cnt, StepParams p, StepParams cy, ShiftRide ride)
{
    warm_arguments<sizeof(RideCounts) + 2 * sizeof(StepParams)>();
    const int ncarry = cnt.ncarry, cy_res = cnt.cy_res, nshift = cnt.nshift;
    if ((int)blockIdx.x < ncarry) {
        extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
        PostShared &sh = *reinterpret_cast<PostShared *>(smem);
        unsigned char *dyn = smem + carry_shared_bytes();
        if (cy_res) select_and_compact<D, true, CARRY_THREADS>(cy, sh, dyn, (int)blockIdx.x);
        else select_and_compact<D, false, CARRY_THREADS>(cy, sh, dyn, (int)blockIdx.x);
        return;
    }
    if ((int)blockIdx.x < ncarry + nshift) {
        const int i = (int)blockIdx.x - ncarry, heads = ride.p.batch * ride.p.hkv;
        shift_range<D, CARRY_THREADS>(ride.p, ride.flags, ride.nchunks, ride.epoch, i % heads, i / heads, ride.parts);
        return;
    }
    step_main_body<D, false, false>(p, (int)blockIdx.x - ncarry - nshift);
}

static size_t main_lds_bytes(int D) { return (size_t)STAGES * 2 * TILE_KEYS * D * 2; }
// dynamic LDS the carrying kernel may ask for: what 160 KB per compute unit leaves next to the
// static tables of the attention body (below 20 KB)
constexpr size_t CARRY_DYN_MAX = 140 * 1024;
static size_t carry_need(const StepParams &cy, bool resident)
{
    return carry_shared_bytes() + select_dyn_bytes(cy.n, cy.N, cy.cap, cy.lists_in_lds != 0, resident);
}

hipError_t configure_main_kernels()
{
    hipError_t e;
#define KD_SET(fn, D)                                                                              \
    e = hipFuncSetAttribute(reinterpret_cast<const void *>(fn), hipFuncAttributeMaxDynamicSharedMemorySize, \
                            (int)main_lds_bytes(D));                                               \
    if (e != hipSuccess) return e;
    KD_SET((step_main_kernel<128, false, false>), 128)
    KD_SET((step_main_kernel<128, true, false>), 128)
    KD_SET((step_main_kernel<128, true, true>), 128)
    KD_SET((step_main_kernel<64, false, false>), 64)
    KD_SET((step_main_kernel<64, true, false>), 64)
    KD_SET((step_main_kernel<64, true, true>), 64)
#undef KD_SET
#define KD_SET(fn)                                                                                  \
    e = hipFuncSetAttribute(reinterpret_cast<const void *>(fn), hipFuncAttributeMaxDynamicSharedMemorySize, \
                            (int)CARRY_DYN_MAX);                                                    \
    if (e != hipSuccess) return e;
    KD_SET((step_main_carry_kernel<128, false>))
    KD_SET((step_main_carry_kernel<128, true>))
    KD_SET((step_main_carry_kernel<64, false>))
    KD_SET((step_main_carry_kernel<64, true>))
    KD_SET((step_main_ride_kernel<128>))
    KD_SET((step_main_ride_kernel<64>))
#undef KD_SET
    return hipSuccess;
}

// workgroups whose last waves have no query row at all run the variant in which those waves help
static bool main_runs_help(const StepParams &p) { return p.mtiles * 32 * p.NW - p.G * p.Bt >= 32; }

hipError_t launch_step_main(const StepParams &p, hipStream_t s)
{
    const int grid = p.batch * p.hkv * p.mtiles * p.splits;
    const size_t lds = main_lds_bytes(p.D);
    const bool help = main_runs_help(p);
    const bool alt = p.psplits != p.splits;   // two waves share the key tiles: planned only for 8-wave helper launches
    if (alt && !(help && p.NW == 8 && p.psplits == 2 * p.splits)) return hipErrorInvalidValue;
#define KD_GO(DD)                                                                                          \
    if (help) hipLaunchKernelGGL((step_main_kernel<DD, true, false>), dim3(grid), dim3(64 * MAIN_WAVES), lds, s, p);  \
    else hipLaunchKernelGGL((step_main_kernel<DD, false, false>), dim3(grid), dim3(64 * MAIN_WAVES), lds, s, p);
    if (alt && p.D == 128) hipLaunchKernelGGL((step_main_kernel<128, true, true>), dim3(grid), dim3(512), lds, s, p);
    else if (alt && p.D == 64) hipLaunchKernelGGL((step_main_kernel<64, true, true>), dim3(grid), dim3(512), lds, s, p);
    else if (p.D == 128 && p.NW == MAIN_WAVES) { KD_GO(128) }
    else if (p.D == 64 && p.NW == MAIN_WAVES) { KD_GO(64) }
#undef KD_GO
    else return hipErrorInvalidValue;
    return hipGetLastError();
}

bool can_carry(const StepParams &p, const StepParams &cy)
{
    const int ncarry = cy.batch * cy.hkv;
    return p.NW == 8 && p.psplits == p.splits && p.D == cy.D && cy.do_evict && cy.n <= 32 * CARRY_THREADS &&
           carry_need(cy, false) <= CARRY_DYN_MAX && ncarry > 0;
}

hipError_t launch_step_main_carry(const StepParams &p, const StepParams &cy, hipStream_t s)
{
    if (!can_carry(p, cy)) return hipErrorInvalidValue;
    const int ncarry = cy.batch * cy.hkv;
    const int grid = ncarry + p.batch * p.hkv * p.mtiles * p.splits;
    StepParams cyl = cy;
#ifdef KD_TIMELINE
    cyl.timeline = p.timeline;   // one record per workgroup of the launch, passengers first
#endif
    const int res = carry_need(cy, true) <= CARRY_DYN_MAX && !cy.argmax_rec ? 1 : 0;
    const size_t need = carry_need(cy, res != 0);
    const size_t lds = need > main_lds_bytes(p.D) ? need : main_lds_bytes(p.D);
    const bool help = main_runs_help(p);
#define KD_GO(DD)                                                                                                   \
    if (help) hipLaunchKernelGGL((step_main_carry_kernel<DD, true>), dim3(grid), dim3(CARRY_THREADS), lds, s, p, cyl, ncarry, res); \
    else hipLaunchKernelGGL((step_main_carry_kernel<DD, false>), dim3(grid), dim3(CARRY_THREADS), lds, s, p, cyl, ncarry, res);
    if (p.D == 128) { KD_GO(128) }
    else if (p.D == 64) { KD_GO(64) }
#undef KD_GO
    else return hipErrorInvalidValue;
    return hipGetLastError();
}

bool can_host_shift(const StepParams &p, const StepParams &shifted)
{
    const int E = shifted.n - shifted.N;
    return p.NW == 8 && p.psplits == p.splits && !main_runs_help(p) && p.D == shifted.D && E > 0 && E <= ORD_ROWS;
}

hipError_t launch_step_main_ride(const StepParams &p, const StepParams *cy, const ShiftRide &ride, hipStream_t s)
{
    if (!can_host_shift(p, ride.p) || ride.nshift < 1 || ride.parts < 1) return hipErrorInvalidValue;
    if (cy && !can_carry(p, *cy)) return hipErrorInvalidValue;
    const int ncarry = cy ? cy->batch * cy->hkv : 0;
    const int grid = ncarry + ride.nshift + p.batch * p.hkv * p.mtiles * p.splits;
    StepParams cyl = cy ? *cy : p;
#ifdef KD_TIMELINE
    cyl.timeline = p.timeline;   // one record per workgroup of the launch that stamps (the shifting ones do not)
#endif
    const int res = cy && carry_need(*cy, true) <= CARRY_DYN_MAX && !cy->argmax_rec ? 1 : 0;
    const size_t need = cy ? carry_need(*cy, res != 0) : 0;
    const size_t lds = need > main_lds_bytes(p.D) ? need : main_lds_bytes(p.D);
    const RideCounts cnt{ncarry, res, ride.nshift};
    if (p.D == 128) hipLaunchKernelGGL((step_main_ride_kernel<128>), dim3(grid), dim3(CARRY_THREADS), lds, s, cnt, p, cyl, ride);
    else if (p.D == 64) hipLaunchKernelGGL((step_main_ride_kernel<64>), dim3(grid), dim3(CARRY_THREADS), lds, s, cnt, p, cyl, ride);
    else return hipErrorInvalidValue;
    return hipGetLastError();
}

}  // namespace kd
