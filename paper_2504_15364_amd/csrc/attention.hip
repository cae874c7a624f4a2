// Block attention over cache || block (Eq. 1-2 of the paper) for gfx950.
//
// Flash-style: the attention matrix is never materialised (the paper's point in
// Method, "Efficient Variant": KeyDiff needs no attention weights).  bf16 MFMA
// 32x32x16 for both contractions, fp32 online softmax, K/V tiles staged in LDS.
//
// Work decomposition.  All G * Bt query rows that share one KV head form the M
// dimension (GQA packing): a workgroup of 4 waves owns 128 * NQ of them and a
// contiguous range of 64-key tiles (split-KV); partial results of the splits are
// merged by log-sum-exp in merge_kernel.  Workgroup ids map KV heads round-robin
// so that all workgroups of one head land on the same XCD and share its L2.
//
// Both contractions are computed transposed so that softmax statistics are
// per-lane scalars and P never leaves registers:
//   S^T = K Q^T   A = K tile rows (LDS, row-major), B = Q^T (registers)
//                 -> lane holds query column (lane % 32), 16 keys
//   O^T = V^T P^T A = V^T (LDS, stored transposed at tile load), B = P^T
//                 -> the accumulator layout of S^T is already the B-operand
//                    layout of the second MFMA once the 16 keys of a k-chunk are
//                    enumerated in accumulator order; V^T is stored with the
//                    matching key permutation.
#include "kd_kernels.h"

namespace kd {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ bf16x8 as_bf16x8(u32x4 v)
{
    return __builtin_bit_cast(bf16x8, v);
}

// Key permutation inside a 16-key chunk of V^T.  An S^T accumulator of lane
// half h holds keys 8j + 4h + r (j = 0..3, r = 0..3) of its 32-key group; the
// k-chunk c of the second MFMA takes j in {2c, 2c+1}, i.e. keys
// 16c + 8a + 4h + r (a = 0,1).  Its 8 k-slots per half must be contiguous in
// LDS: key (c, a, h, r) is stored at slot 16c + 8h + 4a + r.

template <int D, int NQ>
__global__ __launch_bounds__(256) void attn_kernel(AttnParams p)
{
    constexpr int UPR = D / 8;   // 16-byte units per K/V row
    constexpr int NC = D / 16;   // k-chunks of the first MFMA
    constexpr int NDB = D / 32;  // 32-wide d blocks of the output
    constexpr int KLOADS = (TILE_KEYS * UPR) / 256;

    __shared__ __attribute__((aligned(16))) uint16_t sK[TILE_KEYS * D];
    __shared__ __attribute__((aligned(16))) uint16_t sVT[D * TILE_KEYS];

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

    const uint16_t *kbase = p.k + (size_t)bh * p.cap * D;
    const uint16_t *vbase = p.v + (size_t)bh * p.cap * D;

    // ---- query rows of this lane: B operand of S^T = K Q^T, kept in registers
    int mrow[NQ], vis[NQ];
    bf16x8 qreg[NQ][NC];
#pragma unroll
    for (int s = 0; s < NQ; ++s) {
        const int m = mt * (128 * NQ) + wave * (32 * NQ) + s * 32 + l32;
        const bool valid = m < Mtot;
        const int g = valid ? m / p.Bt : 0, j = valid ? m % p.Bt : 0;
        mrow[s] = valid ? m : -1;
        vis[s] = p.len + j + 1;  // rows [0, vis) are visible: all cached rows, block rows 0..j
        const uint16_t *qp = p.q + ((size_t)(b * p.hq + kvh * p.G + g) * p.Bt + j) * D;
#pragma unroll
        for (int c = 0; c < NC; ++c) {
            u32x4 z = {0u, 0u, 0u, 0u};
            if (valid) z = *reinterpret_cast<const u32x4 *>(qp + 16 * c + 8 * h);
            qreg[s][c] = as_bf16x8(z);
        }
    }

    f32x16 oacc[NQ][NDB];
    float mrun[NQ], lrun[NQ];
#pragma unroll
    for (int s = 0; s < NQ; ++s) {
        mrun[s] = -INFINITY;
        lrun[s] = 0.f;
#pragma unroll
        for (int db = 0; db < NDB; ++db)
#pragma unroll
            for (int e = 0; e < 16; ++e) oacc[s][db][e] = 0.f;
    }

    // ---- tile staging: global -> registers (prefetch) -> LDS
    u32x4 kpre[KLOADS], vpre[4];
    const int v_db = tid % UPR, v_kq = tid / UPR;  // V item: 4 consecutive keys x one 16-byte unit
    const bool v_active = tid < 16 * UPR;

    auto prefetch = [&](int t) {
        const int r0 = t * TILE_KEYS;
#pragma unroll
        for (int pp = 0; pp < KLOADS; ++pp) {
            const int idx = tid + 256 * pp;
            const int row = idx / UPR, unit = idx % UPR;
            u32x4 z = {0u, 0u, 0u, 0u};
            if (r0 + row < p.n) z = *reinterpret_cast<const u32x4 *>(kbase + (size_t)(r0 + row) * D + unit * 8);
            kpre[pp] = z;
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int row = r0 + 4 * v_kq + i;
            u32x4 z = {0u, 0u, 0u, 0u};
            if (v_active && row < p.n) z = *reinterpret_cast<const u32x4 *>(vbase + (size_t)row * D + v_db * 8);
            vpre[i] = z;
        }
    };

    auto stage = [&]() {
#pragma unroll
        for (int pp = 0; pp < KLOADS; ++pp) {
            const int idx = tid + 256 * pp;
            const int row = idx / UPR, unit = idx % UPR;
            const int su = unit ^ (row & 7);
            *reinterpret_cast<u32x4 *>(sK + row * D + su * 8) = kpre[pp];
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
                    *reinterpret_cast<u32x2 *>(sVT + R * TILE_KEYS + su * 8 + a * 4) = val;
                }
            }
        }
    };

    if (t0 < t1) prefetch(t0);
    for (int t = t0; t < t1; ++t) {
        __syncthreads();  // everyone finished reading the previous tile
        stage();
        __syncthreads();
        if (t + 1 < t1) prefetch(t + 1);  // loads fly while this tile is computed

        const int r0 = t * TILE_KEYS;
        // ---- S^T = K Q^T
        f32x16 sacc[NQ][2];
#pragma unroll
        for (int s = 0; s < NQ; ++s)
#pragma unroll
            for (int kg = 0; kg < 2; ++kg)
#pragma unroll
                for (int e = 0; e < 16; ++e) sacc[s][kg][e] = 0.f;
#pragma unroll
        for (int kg = 0; kg < 2; ++kg) {
            const int row = 32 * kg + l32;
#pragma unroll
            for (int c = 0; c < NC; ++c) {
                const int su = (2 * c + h) ^ (row & 7);
                const bf16x8 a = as_bf16x8(*reinterpret_cast<const u32x4 *>(sK + row * D + su * 8));
#pragma unroll
                for (int s = 0; s < NQ; ++s)
                    sacc[s][kg] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qreg[s][c], sacc[s][kg], 0, 0, 0);
            }
        }

        // ---- online softmax, per lane = per query column
        const bool need_mask = r0 + TILE_KEYS > p.len;
        bf16x8 pk[NQ][4];
#pragma unroll
        for (int s = 0; s < NQ; ++s) {
            float mloc = -INFINITY;
#pragma unroll
            for (int kg = 0; kg < 2; ++kg)
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    float x = sacc[s][kg][e] * p.scale_log2e;
                    if (need_mask) {
                        const int key = r0 + 32 * kg + 8 * (e >> 2) + 4 * h + (e & 3);
                        x = key < vis[s] ? x : -INFINITY;
                    }
                    sacc[s][kg][e] = x;
                    mloc = fmaxf(mloc, x);
                }
            mloc = fmaxf(mloc, __shfl_xor(mloc, 32));
            const float mnew = fmaxf(mrun[s], mloc);
            const float muse = mnew == -INFINITY ? 0.f : mnew;
            const float alpha = __builtin_amdgcn_exp2f(mrun[s] - muse);
            mrun[s] = mnew;
            float lsum = 0.f;
#pragma unroll
            for (int kg = 0; kg < 2; ++kg)
#pragma unroll
                for (int cc = 0; cc < 2; ++cc) {
                    bf16x8 v;
#pragma unroll
                    for (int i = 0; i < 8; ++i) {
                        const float pe = __builtin_amdgcn_exp2f(sacc[s][kg][8 * cc + i] - muse);
                        lsum += pe;
                        v[i] = (__bf16)pe;
                    }
                    pk[s][2 * kg + cc] = v;
                }
            lrun[s] = lrun[s] * alpha + lsum;
#pragma unroll
            for (int db = 0; db < NDB; ++db)
#pragma unroll
                for (int e = 0; e < 16; ++e) oacc[s][db][e] *= alpha;
        }

        // ---- O^T += V^T P^T
#pragma unroll
        for (int db = 0; db < NDB; ++db) {
            const int R = 32 * db + l32;
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const int su = (2 * c + h) ^ ((R ^ (R >> 3)) & 7);
                const bf16x8 a = as_bf16x8(*reinterpret_cast<const u32x4 *>(sVT + R * TILE_KEYS + su * 8));
#pragma unroll
                for (int s = 0; s < NQ; ++s)
                    oacc[s][db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pk[s][c], oacc[s][db], 0, 0, 0);
            }
        }
    }

    // ---- epilogue: accumulator element e of d-block db is d = 32 db + 8 (e/4) + 4 h + e%4
#pragma unroll
    for (int s = 0; s < NQ; ++s) {
        const float ltot = lrun[s] + __shfl_xor(lrun[s], 32);
        const int m = mrow[s];
        if (m < 0) continue;
        if (p.splits == 1) {
            const int g = m / p.Bt, j = m % p.Bt;
            uint16_t *op = p.out + ((size_t)(b * p.hq + kvh * p.G + g) * p.Bt + j) * D;
            const float inv = 1.f / ltot;
#pragma unroll
            for (int db = 0; db < NDB; ++db)
#pragma unroll
                for (int jj = 0; jj < 4; ++jj) {
                    typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
                    bf16x4 o;
#pragma unroll
                    for (int r = 0; r < 4; ++r) o[r] = (__bf16)(oacc[s][db][4 * jj + r] * inv);
                    *reinterpret_cast<bf16x4 *>(op + 32 * db + 8 * jj + 4 * h) = o;
                }
        } else {
            const size_t row = (size_t)sp * BH * Mtot + (size_t)bh * Mtot + m;
            float *po = p.part_o + row * D;
#pragma unroll
            for (int db = 0; db < NDB; ++db)
#pragma unroll
                for (int jj = 0; jj < 4; ++jj) {
                    float4 o = make_float4(oacc[s][db][4 * jj], oacc[s][db][4 * jj + 1],
                                           oacc[s][db][4 * jj + 2], oacc[s][db][4 * jj + 3]);
                    *reinterpret_cast<float4 *>(po + 32 * db + 8 * jj + 4 * h) = o;
                }
            if (h == 0) p.part_ml[row] = make_float2(mrun[s], ltot);
        }
    }
}

// Log-sum-exp merge of the split-KV partials: one thread per (row, 4 outputs).
template <int D>
__global__ __launch_bounds__(256) void merge_kernel(AttnParams p)
{
    const int BH = p.batch * p.hkv;
    const int Mtot = p.G * p.Bt;
    const size_t rows = (size_t)BH * Mtot;
    const size_t gid = (size_t)blockIdx.x * 256 + threadIdx.x;
    const int d4 = (int)(gid % (D / 4));
    const size_t row = gid / (D / 4);
    if (row >= rows) return;
    float mx = -INFINITY;
    for (int s = 0; s < p.splits; ++s) mx = fmaxf(mx, p.part_ml[(size_t)s * rows + row].x);
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    float L = 0.f;
    for (int s = 0; s < p.splits; ++s) {
        const float2 ml = p.part_ml[(size_t)s * rows + row];
        const float w = ml.x == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(ml.x - mx);
        const float4 o = *reinterpret_cast<const float4 *>(p.part_o + ((size_t)s * rows + row) * D + 4 * d4);
        acc.x += w * o.x;
        acc.y += w * o.y;
        acc.z += w * o.z;
        acc.w += w * o.w;
        L += w * ml.y;
    }
    const float inv = 1.f / L;
    const int bh = (int)(row / Mtot), m = (int)(row % Mtot);
    const int b = bh / p.hkv, kvh = bh % p.hkv;
    const int g = m / p.Bt, j = m % p.Bt;
    typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
    bf16x4 o;
    o[0] = (__bf16)(acc.x * inv);
    o[1] = (__bf16)(acc.y * inv);
    o[2] = (__bf16)(acc.z * inv);
    o[3] = (__bf16)(acc.w * inv);
    *reinterpret_cast<bf16x4 *>(p.out + ((size_t)(b * p.hq + kvh * p.G + g) * p.Bt + j) * D + 4 * d4) = o;
}

hipError_t launch_attention(const AttnParams &p, int D, int NQ, hipStream_t s)
{
    const int grid = p.batch * p.hkv * p.mtiles * p.splits;
    if (D == 128 && NQ == 2) hipLaunchKernelGGL((attn_kernel<128, 2>), dim3(grid), dim3(256), 0, s, p);
    else if (D == 128 && NQ == 1) hipLaunchKernelGGL((attn_kernel<128, 1>), dim3(grid), dim3(256), 0, s, p);
    else if (D == 64 && NQ == 2) hipLaunchKernelGGL((attn_kernel<64, 2>), dim3(grid), dim3(256), 0, s, p);
    else if (D == 64 && NQ == 1) hipLaunchKernelGGL((attn_kernel<64, 1>), dim3(grid), dim3(256), 0, s, p);
    else return hipErrorInvalidValue;
    return hipGetLastError();
}

hipError_t launch_merge(const AttnParams &p, int D, hipStream_t s)
{
    const size_t threads = (size_t)p.batch * p.hkv * p.G * p.Bt * (D / 4);
    const int grid = (int)((threads + 255) / 256);
    if (D == 128) hipLaunchKernelGGL((merge_kernel<128>), dim3(grid), dim3(256), 0, s, p);
    else if (D == 64) hipLaunchKernelGGL((merge_kernel<64>), dim3(grid), dim3(256), 0, s, p);
    else return hipErrorInvalidValue;
    return hipGetLastError();
}

}  // namespace kd
