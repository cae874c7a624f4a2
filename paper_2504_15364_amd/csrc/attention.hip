// step_main: append + block attention over cache || block (Eq. 5, Eq. 1-2) for gfx950.
//
// Flash-style: the attention matrix is never materialised (Method, "Efficient
// Variant": KeyDiff needs no attention weights).  bf16 MFMA 32x32x16 for both
// contractions, fp32 online softmax, K/V tiles double-buffered in LDS.
//
// Work decomposition.  All G * Bt query rows that share one KV head form the M
// dimension (GQA packing): a workgroup of NW waves owns 32 * NW of them and a
// contiguous range of 64-key tiles (split-KV); the splits are merged by
// log-sum-exp in step_post.  Workgroup ids map KV heads round-robin so that the
// workgroups of one head share an XCD and its L2.
//
// Both contractions are computed transposed so that softmax statistics are
// per-lane scalars and P never leaves registers:
//   S^T = K Q^T   A = K tile rows (LDS, row-major), B = Q^T (registers)
//                 -> a lane holds one query column (lane % 32) and 16 keys
//   O^T = V^T P^T A = V^T (LDS, transposed while staging), B = P^T: the S^T
//                 accumulator layout already is the B-operand layout once the 16
//                 keys of a k-chunk are enumerated in accumulator order; V^T is
//                 stored with the matching key permutation.
//
// The block's own rows are read straight from k_new / v_new; every workgroup
// copies a slice of them into the cache (the append) and adds that slice to the
// running key sum the anchor is derived from.
#include "kd_kernels.h"

namespace kd {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ bf16x8 as_bf16x8(u32x4 v) { return __builtin_bit_cast(bf16x8, v); }

constexpr float RESCALE_SLACK = 8.f;  // the running reference max may lag the true max by 2^8

// Key permutation inside a 16-key chunk of V^T.  An S^T accumulator of lane
// half h holds keys 8j + 4h + r (j = 0..3, r = 0..3) of its 32-key group; the
// k-chunk c of the second MFMA takes j in {2c, 2c+1}, i.e. keys
// 16c + 8a + 4h + r (a = 0,1).  Its 8 k-slots per half must be contiguous in
// LDS: key (c, a, h, r) is stored at slot 16c + 8h + 4a + r.

template <int D, int NW>
__global__ __launch_bounds__(64 * NW) void step_main_kernel(StepParams p)
{
    constexpr int NT = 64 * NW;  // threads; each wave owns 32 query rows
    constexpr int UPR = D / 8;   // 16-byte units per K/V row
    constexpr int NC = D / 16;   // k-chunks of the first MFMA
    constexpr int NDB = D / 32;  // 32-wide d blocks of the output
    constexpr int KLOADS = (TILE_KEYS * UPR) / NT;
    constexpr int TILE_ELEMS = TILE_KEYS * D;
    static_assert(KLOADS >= 1, "tile staging needs at least one K unit per thread");

    extern __shared__ __attribute__((aligned(16))) uint16_t smem[];
    uint16_t *sK = smem;                    // [2][TILE_KEYS][D]   swizzled rows
    uint16_t *sVT = smem + 2 * TILE_ELEMS;  // [2][D][TILE_KEYS]   transposed, permuted, swizzled
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

    f32x16 oacc[NDB];
    float mref = -INFINITY, lrun = 0.f;
#pragma unroll
    for (int db = 0; db < NDB; ++db)
#pragma unroll
        for (int e = 0; e < 16; ++e) oacc[db][e] = 0.f;

    // ---- tile staging: global -> registers (prefetch) -> LDS (double buffered)
    u32x4 kpre[KLOADS], vpre[4];
    const int v_db = tid % UPR, v_kq = tid / UPR;  // V item: 4 consecutive keys x one 16-byte unit
    const bool v_active = tid < 16 * UPR;

    auto row_ptr = [&](const uint16_t *cache, const uint16_t *fresh, int row) -> const uint16_t * {
        return row < p.len ? cache + (size_t)row * D : fresh + (size_t)(row - p.len) * D;
    };

    auto prefetch = [&](int t) {
        const int r0 = t * TILE_KEYS;
#pragma unroll
        for (int pp = 0; pp < KLOADS; ++pp) {
            const int idx = tid + NT * pp;
            const int row = r0 + idx / UPR, unit = idx % UPR;
            u32x4 z = {0u, 0u, 0u, 0u};
            if (row < p.n) z = *reinterpret_cast<const u32x4 *>(row_ptr(kcache, knew, row) + unit * 8);
            kpre[pp] = z;
        }
        if (v_active) {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int row = r0 + 4 * v_kq + i;
                u32x4 z = {0u, 0u, 0u, 0u};
                if (row < p.n) z = *reinterpret_cast<const u32x4 *>(row_ptr(vcache, vnew, row) + v_db * 8);
                vpre[i] = z;
            }
        }
    };

    auto stage = [&](int buf) {
        uint16_t *dK = sK + buf * TILE_ELEMS, *dV = sVT + buf * TILE_ELEMS;
#pragma unroll
        for (int pp = 0; pp < KLOADS; ++pp) {
            const int idx = tid + NT * pp;
            const int row = idx / UPR, unit = idx % UPR;
            const int su = unit ^ (row & 7);
            *reinterpret_cast<u32x4 *>(dK + row * D + su * 8) = kpre[pp];
        }
        if (v_active) {
            const int c = v_kq >> 2, q4 = v_kq & 3, a = q4 >> 1, hh = q4 & 1;
            const int unit = 2 * c + hh;
#pragma unroll
            for (int w = 0; w < 4; ++w) {
#pragma unroll
                for (int bsel = 0; bsel < 2; ++bsel) {
                    const int R = 8 * v_db + 2 * w + bsel;  // d index = row of V^T
                    uint32_t lo, hi;
                    if (bsel == 0) {
                        lo = (vpre[0][w] & 0xFFFFu) | (vpre[1][w] << 16);
                        hi = (vpre[2][w] & 0xFFFFu) | (vpre[3][w] << 16);
                    } else {
                        lo = (vpre[0][w] >> 16) | (vpre[1][w] & 0xFFFF0000u);
                        hi = (vpre[2][w] >> 16) | (vpre[3][w] & 0xFFFF0000u);
                    }
                    const int su = unit ^ ((R ^ (R >> 3)) & 7);
                    u32x2 val = {lo, hi};
                    *reinterpret_cast<u32x2 *>(dV + R * TILE_KEYS + su * 8 + a * 4) = val;
                }
            }
        }
    };

    if (t0 < t1) {
        prefetch(t0);
        stage(0);
        if (t0 + 1 < t1) prefetch(t0 + 1);
    }
    int cur = 0;
    for (int t = t0; t < t1; ++t) {
        __syncthreads();  // tile t is staged; the other buffer is no longer read
        if (t + 1 < t1) {
            stage(cur ^ 1);
            if (t + 2 < t1) prefetch(t + 2);  // in flight during this tile and the next staging
        }
        const uint16_t *tK = sK + cur * TILE_ELEMS, *tV = sVT + cur * TILE_ELEMS;
        cur ^= 1;

        const int r0 = t * TILE_KEYS;
        const bool need_mask = r0 + TILE_KEYS > p.len;

        // ---- per 32-key group: S^T = K Q^T, online softmax (per lane = per query column),
        //      then O^T += V^T P^T
#pragma unroll
        for (int kg = 0; kg < 2; ++kg) {
            f32x16 sacc;
            {
                const int row = 32 * kg + l32;
#pragma unroll
                for (int c = 0; c < NC; ++c) {
                    const int su = (2 * c + h) ^ (row & 7);
                    const bf16x8 a = as_bf16x8(*reinterpret_cast<const u32x4 *>(tK + row * D + su * 8));
                    if (c == 0) {
                        const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
                        sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qreg[c], zero, 0, 0, 0);
                    } else {
                        sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qreg[c], sacc, 0, 0, 0);
                    }
                }
            }
            float mloc = -INFINITY;
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                float x = sacc[e];
                if (need_mask) {
                    const int key = r0 + 32 * kg + 8 * (e >> 2) + 4 * h + (e & 3);
                    x = key < vis ? x : -INFINITY;
                    sacc[e] = x;
                }
                mloc = fmaxf(mloc, x);
            }
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
            float lsum = 0.f;
            bf16x8 pk[2];
#pragma unroll
            for (int cc = 0; cc < 2; ++cc) {
                bf16x8 v;
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    const float pe = __builtin_amdgcn_exp2f(__builtin_fmaf(sacc[8 * cc + i], p.scale_log2e, nmuse));
                    lsum += pe;
                    v[i] = (__bf16)pe;
                }
                pk[cc] = v;
            }
            lrun += lsum;
#pragma unroll
            for (int db = 0; db < NDB; ++db) {
                const int R = 32 * db + l32;
#pragma unroll
                for (int cc = 0; cc < 2; ++cc) {
                    const int su = (2 * (2 * kg + cc) + h) ^ ((R ^ (R >> 3)) & 7);
                    const bf16x8 a = as_bf16x8(*reinterpret_cast<const u32x4 *>(tV + R * TILE_KEYS + su * 8));
                    oacc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pk[cc], oacc[db], 0, 0, 0);
                }
            }
        }
    }

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

static size_t main_lds_bytes(int D) { return (size_t)4 * TILE_KEYS * D * 2; }

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
