// step_main: append + block attention over cache || block (Eq. 5, Eq. 1-2) for gfx950.
//
// Flash-style: the attention matrix is never materialised (Method, "Efficient
// Variant": KeyDiff needs no attention weights).  bf16 MFMA 32x32x16 for both
// contractions, fp32 online softmax.
//
// Work decomposition.  All G * Bt query rows that share one KV head form the M
// dimension (GQA packing): a workgroup of NW waves owns 32 * NW of them and a
// contiguous range of 64-key tiles (split-KV); the splits are merged by
// log-sum-exp in step_post.  Workgroup ids map KV heads round-robin so that the
// workgroups of one head share an XCD and its L2.
//
// Data path.  K and V tiles stream global -> LDS asynchronously
// (global_load_lds_dwordx4: lane i's 16 bytes land at LDS base + 16 i, no VGPRs)
// through a ring of STAGES buffers, so several tiles are in flight per CU while
// one is computed.  Both tiles are stored row-major with a 16-byte-unit XOR swizzle
// applied on the global side (a lane fetches the unit that belongs in its LDS slot).
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
// copies a slice of them into the cache (the append) and adds that slice to the
// running key sum the anchor is derived from.
#include <type_traits>

#include "kd_kernels.h"

namespace kd {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ bf16x8 as_bf16x8(u32x4 v) { return __builtin_bit_cast(bf16x8, v); }

constexpr float RESCALE_SLACK = 8.f;  // the running reference max may lag the true max by 2^8
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

template <int N>
__device__ __forceinline__ void wait_copies()  // at most N of this wave's copies still in flight
{
    static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
    __builtin_amdgcn_s_waitcnt(0x0F70 | (N & 15) | ((N >> 4) << 14));
}

template <int D, int NW>
__global__ __launch_bounds__(64 * NW) void step_main_kernel(StepParams p)
{
    constexpr int NT = 64 * NW;   // threads; each wave owns 32 query rows
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

    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];  // [STAGES][K tile | V tile]
    __shared__ double red[NW];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, h = lane >> 5;
    const int BH = p.batch * p.hkv;
    int id = blockIdx.x;
    const int bh = id % BH;
    id /= BH;
    const int mt = id % p.mtiles;
    const int sp = id / p.mtiles;
    const int b = bh / p.hkv, kvh = bh % p.hkv;
    const int Mtot = p.G * p.Bt;
    const int t0 = (int)(((long)sp * p.ntiles) / p.splits);
    const int t1 = (int)(((long)(sp + 1) * p.ntiles) / p.splits);

    const uint16_t *kcache = p.k + (size_t)bh * p.cap * D;
    const uint16_t *vcache = p.v + (size_t)bh * p.cap * D;
    const uint16_t *knew = p.k_new + (size_t)bh * p.Bt * D;
    const uint16_t *vnew = p.v_new + (size_t)bh * p.Bt * D;

    // ---- query row of this lane: B operand of S^T = K Q^T, kept in registers
    const int m = mt * (32 * NW) + wave * 32 + l32;
    const bool valid = m < Mtot;
    const int qg = valid ? m / p.Bt : 0, qj = valid ? m % p.Bt : 0;
    const int vis = p.len + qj + 1;  // rows [0, vis) are visible: all cached rows, block rows 0..j
    bf16x8 qreg[NC];
    {
        const uint16_t *qp = p.q + ((size_t)(b * p.hq + kvh * p.G + qg) * p.Bt + qj) * D;
#pragma unroll
        for (int c = 0; c < NC; ++c) {
            u32x4 z = {0u, 0u, 0u, 0u};
            if (valid) z = *reinterpret_cast<const u32x4 *>(qp + 16 * c + 8 * h);
            qreg[c] = as_bf16x8(z);
        }
    }

    // ---- append (Eq. 5): this workgroup's slice of the block's rows, and the key sum
    {
        const int W = p.mtiles * p.splits, widx = sp * p.mtiles + mt;
        const int j0 = (int)(((long)widx * p.Bt) / W), j1 = (int)(((long)(widx + 1) * p.Bt) / W);
        const int rows = j1 - j0;
        for (int u = tid; u < rows * UPR * 2; u += NT) {
            const int which = u / (rows * UPR), rem = u % (rows * UPR);
            const int j = j0 + rem / UPR, unit = rem % UPR;
            const u32x4 val = *reinterpret_cast<const u32x4 *>((which ? vnew : knew) + (size_t)j * D + unit * 8);
            *reinterpret_cast<u32x4 *>((which ? p.v : p.k) + ((size_t)bh * p.cap + p.len + j) * D + unit * 8) = val;
        }
        for (int j = j0 + tid; j < j1; j += NT) p.pos[(size_t)bh * p.cap + p.len + j] = p.pos0 + j;
        double acc = 0.0;
        for (int j = j0; j < j1; ++j) {
            double x = 0.0;
            if (tid < D) x = (double)__uint_as_float((uint32_t)knew[(size_t)j * D + tid] << 16);
            if (p.anchor_mode == 1) {  // unit keys (Eq. 7): x / |k_j|, a zero key adds nothing
                double k2 = x * x;
#pragma unroll
                for (int off = 1; off < 64; off <<= 1) {
                    int lo = __shfl_xor(__double2loint(k2), off), hi = __shfl_xor(__double2hiint(k2), off);
                    k2 += __hiloint2double(hi, lo);
                }
                __syncthreads();
                if (lane == 0) red[wave] = k2;
                __syncthreads();
                double tot = 0.0;
#pragma unroll
                for (int w = 0; w < NW; ++w) tot += red[w];
                const double nk = sqrt(tot);
                x = nk > 0.0 ? x * (1.0 / nk) : 0.0;
            }
            acc += x;
        }
        if (tid < D && rows > 0) unsafeAtomicAdd(p.ksum + (size_t)bh * D + tid, acc);
    }

    f32x16 oacc[NDB];
    float mref = -INFINITY, lrun = 0.f;
#pragma unroll
    for (int db = 0; db < NDB; ++db)
#pragma unroll
        for (int e = 0; e < 16; ++e) oacc[db][e] = 0.f;

    // ---- tile copies.  Wave w issues copies w, w + NW, ... of the K tile and of the V tile; copy s
    // fills LDS bytes [1024 s, 1024 s + 1024) of the tile = rows RPL s .. RPL s + RPL - 1.  Lane i
    // owns slot (row RPL s + i / UPR, unit i % UPR) and fetches the unit the swizzle puts there:
    //   K: unit ^ (row & 7)            (ds_read_b128 of 8 consecutive rows hits 32 banks once)
    //   V: unit ^ 2 (row & 3)          (the 4 rows x 32 bytes of a transpose read do the same)
    const uint32_t lds0 = (uint32_t)(uintptr_t)smem;
    uint32_t koff[CPW], voff[CPW];  // byte offset of this lane's unit inside a whole tile in memory
    int crow[CPW];                  // its row inside the tile
#pragma unroll
    for (int i = 0; i < CPW; ++i) {
        const int s = wave + NW * i;
        const int row = RPL * s + lane / UPR, su = lane % UPR;
        crow[i] = row;
        koff[i] = (uint32_t)(row * ROWB + ((su ^ (row & 7)) & (UPR - 1)) * 16);
        voff[i] = (uint32_t)(row * ROWB + ((su ^ (2 * (row & 3))) & (UPR - 1)) * 16);
    }
    // A tile is "whole" when its 64 rows are valid and come from one source (the cache, or the
    // block's k_new / v_new): then only the base pointer differs.  A partial tile (it straddles len
    // or n; at most two per step) takes per-row pointers; rows past n read row n - 1 -- finite
    // data whose logits are masked, so it is never zeroed.
    auto issue_tile = [&](int t) {
        const int r0 = t * TILE_KEYS;
        const uint32_t kdst = lds0 + (uint32_t)((t % STAGES) * 2 * TILE_B), vdst = kdst + TILE_B;
        const bool whole = r0 + TILE_KEYS <= p.len || (r0 >= p.len && r0 + TILE_KEYS <= p.n);
        if (whole) {
            const bool cached = r0 < p.len;
            const uint16_t *kt = cached ? kcache + (size_t)r0 * D : knew + (size_t)(r0 - p.len) * D;
            const uint16_t *vt = cached ? vcache + (size_t)r0 * D : vnew + (size_t)(r0 - p.len) * D;
#pragma unroll
            for (int i = 0; i < CPW; ++i) async_copy16(kdst + 1024u * (wave + NW * i), kt, koff[i]);
#pragma unroll
            for (int i = 0; i < CPW; ++i) async_copy16(vdst + 1024u * (wave + NW * i), vt, voff[i]);
        } else {
#pragma unroll
            for (int i = 0; i < CPW; ++i) {
                const int rc = min(r0 + crow[i], p.n - 1);
                const uint16_t *src = rc < p.len ? kcache + (size_t)rc * D : knew + (size_t)(rc - p.len) * D;
                async_copy16(kdst + 1024u * (wave + NW * i),
                             reinterpret_cast<const char *>(src) + (koff[i] - crow[i] * ROWB));
            }
#pragma unroll
            for (int i = 0; i < CPW; ++i) {
                const int rc = min(r0 + crow[i], p.n - 1);
                const uint16_t *src = rc < p.len ? vcache + (size_t)rc * D : vnew + (size_t)(rc - p.len) * D;
                async_copy16(vdst + 1024u * (wave + NW * i),
                             reinterpret_cast<const char *>(src) + (voff[i] - crow[i] * ROWB));
            }
        }
    };

    // ---- LDS byte offsets of this lane's MFMA A operands.
    // K: row l32 of the key group, unit (2c + h) ^ (row & 7): the offset of k-chunk c is (offset of
    // chunk 0) ^ 32 c for c < 4; the key group and c >> 2 add constants.
    const int kof0 = l32 * ROWB + (h ^ (l32 & 7)) * 16;
    // V (transpose read): the lane's 16-lane group fetches keys k0 .. k0 + 3 (k0 = 16 c + 4 h, + 8 for
    // the second read) x columns d0 .. d0 + 15 (d0 = 32 db + 16 (group & 1)); this lane supplies row
    // k0 + (lane % 16) / 4, columns d0 + 4 (lane % 4) .. + 3 and receives column d0 + lane % 16.
    // The swizzled unit is (4 db + 2 (group & 1) + (lane % 4) / 2) ^ 2 (row & 3) = (per-lane part) ^ 4 db.
    const int i16 = lane & 15, vrow = 4 * h + (i16 >> 2);
    const int vof0 =
        vrow * ROWB + (((2 * ((lane >> 4) & 1) + ((i16 & 3) >> 1)) ^ (2 * (vrow & 3))) * 16) + (i16 & 1) * 8;

    // One 64-key tile.  Operand reads are issued a phase ahead of the MFMAs that consume them so
    // that LDS latency hides behind matrix and vector work: K operands of both 32-key groups, then
    // the V^T operands of group 0 while S is still in the matrix pipe; one reference-max decision
    // per tile; then a straight-line block (softmax 0, PV 0, softmax 1, PV 1) in which the PV MFMAs
    // of one group overlap the exponentials of the other.
    auto read_k = [&](const unsigned char *tK, int kg, bf16x8 (&ka)[NC]) {
#pragma unroll
        for (int c = 0; c < NC; ++c)
            ka[c] = as_bf16x8(*reinterpret_cast<const u32x4 *>(
                tK + ((kof0 ^ ((c & 3) * 32)) + kg * 32 * ROWB + (c >> 2) * 128)));
    };
    auto read_v = [&](const unsigned char *tV, int kg, bf16x8 (&va)[NDB][2]) {
#pragma unroll
        for (int db = 0; db < NDB; ++db)
#pragma unroll
            for (int cc = 0; cc < 2; ++cc) {
                const unsigned char *a = tV + ((vof0 ^ (db * 64)) + (2 * kg + cc) * 16 * ROWB);
                const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3))) *)(a));
                const s16x4 hi =
                    __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3))) *)(a + 8 * ROWB));
                va[db][cc] = __builtin_bit_cast(bf16x8, (s16x8)__builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
            }
    };
    auto qk = [&](const bf16x8 (&ka)[NC]) {
        const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        f32x16 acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[0], qreg[0], zero, 0, 0, 0);
#pragma unroll
        for (int c = 1; c < NC; ++c) acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[c], qreg[c], acc, 0, 0, 0);
        return acc;
    };
    // exponentials of one group -> bf16 B operands; the row sum adds the rounded weights the
    // second MFMA multiplies with
    auto softmax = [&](const f32x16 &sacc, float nmuse, bf16x8 (&pk)[2]) {
#pragma unroll
        for (int cc = 0; cc < 2; ++cc) {
            bf16x8 v;
#pragma unroll
            for (int i = 0; i < 8; ++i)
                v[i] = (__bf16)__builtin_amdgcn_exp2f(__builtin_fmaf(sacc[8 * cc + i], p.scale_log2e, nmuse));
            pk[cc] = v;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                bf16x2 pr = {v[2 * i], v[2 * i + 1]};
                const bf16x2 one = {(__bf16)1.0f, (__bf16)1.0f};
                lrun = __builtin_amdgcn_fdot2_f32_bf16(pr, one, lrun, false);
            }
        }
    };
    auto pv = [&](const bf16x8 (&va)[NDB][2], const bf16x8 (&pk)[2]) {
#pragma unroll
        for (int cc = 0; cc < 2; ++cc)
#pragma unroll
            for (int db = 0; db < NDB; ++db)
                oacc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va[db][cc], pk[cc], oacc[db], 0, 0, 0);
    };
    // first half of a tile: S^T of both key groups (+ causal mask on edge tiles)
    auto s_phase = [&](const unsigned char *tK, int r0, f32x16 &s0, f32x16 &s1, auto masked_tag) {
        constexpr bool MASKED = decltype(masked_tag)::value;
        bf16x8 ka0[NC], ka1[NC];
        read_k(tK, 0, ka0);
        read_k(tK, 1, ka1);
        s0 = qk(ka0);
        s1 = qk(ka1);
        if (MASKED) {
            // accumulator element e of group kg holds key r0 + 32 kg + 4 h + 8 (e / 4) + e % 4
            const int lim = vis - r0 - 4 * h;
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                s0[e] = (8 * (e >> 2) + (e & 3)) < lim ? s0[e] : -INFINITY;
                s1[e] = (32 + 8 * (e >> 2) + (e & 3)) < lim ? s1[e] : -INFINITY;
            }
        }
    };
    // second half: reference-max decision, exponentials, O^T += V^T P^T
    auto pv_phase = [&](const unsigned char *tV, const f32x16 &s0, const f32x16 &s1) {
        bf16x8 va0[NDB][2], va1[NDB][2];
        read_v(tV, 0, va0);
        float mloc = fmaxf(s0[0], s1[0]);
#pragma unroll
        for (int e = 1; e < 16; ++e) mloc = fmaxf(mloc, fmaxf(s0[e], s1[e]));
        mloc = fmaxf(mloc, __shfl_xor(mloc, 32));
        const float mtile = mloc * p.scale_log2e;
        // lazy rescale: the reference max only moves when the tile max exceeds it by 2^SLACK
        const bool need = mtile > mref + RESCALE_SLACK;
        if (__builtin_amdgcn_ballot_w64(need) != 0) {
            const float alpha = need ? __builtin_amdgcn_exp2f(mref - mtile) : 1.f;
            mref = need ? mtile : mref;
            lrun *= alpha;
#pragma unroll
            for (int db = 0; db < NDB; ++db)
#pragma unroll
                for (int e = 0; e < 16; ++e) oacc[db][e] *= alpha;
        }
        const float nmuse = mref == -INFINITY ? 0.f : -mref;
        bf16x8 pk0[2], pk1[2];
        softmax(s0, nmuse, pk0);
        read_v(tV, 1, va1);
        pv(va0, pk0);
        softmax(s1, nmuse, pk1);
        pv(va1, pk1);
    };

    // Pin the query registers here: their global loads must not be pending when the tile loop
    // starts (the explicit copy waits below count outstanding memory operations).
#pragma unroll
    for (int c = 0; c < NC; ++c) {
        u32x4 qv = __builtin_bit_cast(u32x4, qreg[c]);
        asm volatile("" : "+v"(qv));
        qreg[c] = as_bf16x8(qv);
    }

    // ---- the ring.  Waves [0, NW/2) ("early") run both halves of tile t in iteration t; waves
    // [NW/2, NW) ("late") -- the second wave on each SIMD -- run the second half one iteration
    // behind: [second half of t - 1, first half of t].  The per-tile barrier would otherwise keep
    // all waves in the same phase, and the two waves of a SIMD would queue for the same pipe
    // (matrix, vector or LDS) instead of overlapping MFMAs with exponentials.  The V tile of
    // t - 1 therefore stays live during iteration t: with STAGES buffers, STAGES - 2 tiles are
    // in flight.
    const bool late = wave >= NW / 2;
    const int ntl = t1 - t0;
#pragma unroll
    for (int i = 0; i < STAGES - 2; ++i)
        if (i < ntl) issue_tile(t0 + i);
    const int tint = min(t1, max(t0, p.len / TILE_KEYS));  // tiles before it: every key cached, no mask
    f32x16 sp0, sp1;  // S of the previous tile (late waves)
    auto step = [&](int t, auto masked_tag) {
        // this wave's copies of tile t have landed when at most the copies of the later tile in
        // flight remain; the barrier then publishes every wave's part and retires tile t - 2
        if (t + 1 < t1) wait_copies<LPW>();
        else wait_copies<0>();
        __syncthreads();
        if (t + STAGES - 2 < t1) issue_tile(t + STAGES - 2);  // into the buffer tile t - 2 left
        const unsigned char *tK = smem + (size_t)(t % STAGES) * 2 * TILE_B;
        if (!late) {
            f32x16 s0, s1;
            s_phase(tK, t * TILE_KEYS, s0, s1, masked_tag);
            pv_phase(tK + TILE_B, s0, s1);
        } else {
            if (t > t0) pv_phase(smem + (size_t)((t - 1) % STAGES) * 2 * TILE_B + TILE_B, sp0, sp1);
            s_phase(tK, t * TILE_KEYS, sp0, sp1, masked_tag);
        }
    };
    static_assert(STAGES == 4, "the wait ladder in step() assumes two tiles in flight");
    // interior and edge tiles run in separate loops so that the rare masked path does not weigh on
    // the register allocation of the hot one
    for (int t = t0; t < tint; ++t) step(t, std::false_type{});
    for (int t = tint; t < t1; ++t) step(t, std::true_type{});
    if (late && ntl > 0) pv_phase(smem + (size_t)((t1 - 1) % STAGES) * 2 * TILE_B + TILE_B, sp0, sp1);

    // ---- epilogue: accumulator element e of d-block db is d = 32 db + 8 (e/4) + 4 h + e%4
    const float ltot = lrun + __shfl_xor(lrun, 32);
    if (!valid) return;
    if (p.splits == 1) {
        uint16_t *op = p.out + ((size_t)(b * p.hq + kvh * p.G + qg) * p.Bt + qj) * D;
        const float inv = 1.f / ltot;
#pragma unroll
        for (int db = 0; db < NDB; ++db)
#pragma unroll
            for (int jj = 0; jj < 4; ++jj) {
                bf16x4 o;
#pragma unroll
                for (int r = 0; r < 4; ++r) o[r] = (__bf16)(oacc[db][4 * jj + r] * inv);
                *reinterpret_cast<bf16x4 *>(op + 32 * db + 8 * jj + 4 * h) = o;
            }
    } else {
        const size_t row = (size_t)sp * BH * Mtot + (size_t)bh * Mtot + m;
        float *po = p.part_o + row * D;
#pragma unroll
        for (int db = 0; db < NDB; ++db)
#pragma unroll
            for (int jj = 0; jj < 4; ++jj) {
                float4 o = make_float4(oacc[db][4 * jj], oacc[db][4 * jj + 1], oacc[db][4 * jj + 2],
                                       oacc[db][4 * jj + 3]);
                *reinterpret_cast<float4 *>(po + 32 * db + 8 * jj + 4 * h) = o;
            }
        if (h == 0) p.part_ml[row] = make_float2(mref, ltot);
    }
}

static size_t main_lds_bytes(int D) { return (size_t)STAGES * 2 * TILE_KEYS * D * 2; }

hipError_t configure_main_kernels()
{
    hipError_t e;
#define KD_SET(fn, D)                                                                              \
    e = hipFuncSetAttribute(reinterpret_cast<const void *>(fn), hipFuncAttributeMaxDynamicSharedMemorySize, \
                            (int)main_lds_bytes(D));                                               \
    if (e != hipSuccess) return e;
    KD_SET((step_main_kernel<128, 8>), 128)
    KD_SET((step_main_kernel<128, 4>), 128)
    KD_SET((step_main_kernel<64, 8>), 64)
    KD_SET((step_main_kernel<64, 4>), 64)
#undef KD_SET
    return hipSuccess;
}

hipError_t launch_step_main(const StepParams &p, hipStream_t s)
{
    const int grid = p.batch * p.hkv * p.mtiles * p.splits;
    const size_t lds = main_lds_bytes(p.D);
    if (p.D == 128 && p.NW == 8) hipLaunchKernelGGL((step_main_kernel<128, 8>), dim3(grid), dim3(512), lds, s, p);
    else if (p.D == 128 && p.NW == 4) hipLaunchKernelGGL((step_main_kernel<128, 4>), dim3(grid), dim3(256), lds, s, p);
    else if (p.D == 64 && p.NW == 8) hipLaunchKernelGGL((step_main_kernel<64, 8>), dim3(grid), dim3(512), lds, s, p);
    else if (p.D == 64 && p.NW == 4) hipLaunchKernelGGL((step_main_kernel<64, 4>), dim3(grid), dim3(256), lds, s, p);
    else return hipErrorInvalidValue;
    return hipGetLastError();
}

}  // namespace kd
