// The ORDERED layout's stable row shift for workgroups that own a RANGE of chunks: the form in which
// the shift rides in an attention launch (step_main_carry), on the few compute units the attention
// leaves to it.  Kept row i moves to dst[i] = i - (evicted rows before i) <= i, down by at most
// E = n - N rows; here E <= ORD_ROWS, so the rows of chunk c land in chunks c - 1 and c.
//
// A workgroup takes the chunks [c0, c1) of one head from the top down, with the next two chunks
// already requested while it stores one: chunk c is stored once chunk c - 1 is in registers (its
// own registers, or -- for its lowest chunk -- those of the workgroup below, which says so with a
// flag as soon as it has read its top chunk).  A workgroup therefore only ever waits for the first
// thing another workgroup does, whatever order they start in; the wait is bounded and reports a
// timeout in the status word instead of hanging.
#pragma once
#include "kd_kernels.h"
#include "kd_device.h"

namespace kd {

template <int D, int THREADS>
__device__ __forceinline__ void shift_range(const StepParams &p, int32_t *flags, int nchunks, int32_t epoch, int bh,
                                            int part, int parts)
{
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    constexpr int UPR = D / 8;
    constexpr int UPT = ORD_ROWS * UPR * 2 / THREADS;   // 16-byte units (K and V) per thread and chunk
    static_assert(UPT * THREADS == ORD_ROWS * UPR * 2, "a chunk must divide over the threads");
    static_assert(UPT < 64, "the wait below names UPT outstanding operations in a 6-bit field");
    const int tid = threadIdx.x;
    const int c0 = (int)(((long)part * nchunks) / parts), c1 = (int)(((long)(part + 1) * nchunks) / parts);
    if (c0 >= c1) return;   // uniform
    uint16_t *kb = p.k + (size_t)bh * p.cap * D;
    uint16_t *vb = p.v + (size_t)bh * p.cap * D;
    const int32_t *dst = p.dstmap + (size_t)bh * p.cap;
    int32_t *myflags = flags + (size_t)bh * nchunks;

    u32x4 va[UPT], vb2[UPT], vc[UPT];
    int da[UPT], db[UPT], dc[UPT];
    auto load = [&](int chunk, u32x4 (&val)[UPT], int (&drow)[UPT]) {
        const int r0 = chunk * ORD_ROWS;
#pragma unroll
        for (int q = 0; q < UPT; ++q) {
            const int w = q * THREADS + tid;
            const int which = w >= ORD_ROWS * UPR, rem = w - which * ORD_ROWS * UPR;
            const int row = min(r0 + rem / UPR, p.n - 1), u = rem % UPR;   // rows past n repeat the last one (never stored)
            val[q] = *reinterpret_cast<const u32x4 *>((which ? vb : kb) + (size_t)row * D + u * 8);
            const int d = dst[row];
            drow[q] = (r0 + rem / UPR < p.n && d >= 0 && d != row) ? d : -1;
        }
    };
    auto store = [&](const u32x4 (&val)[UPT], const int (&drow)[UPT]) {
#pragma unroll
        for (int q = 0; q < UPT; ++q) {
            const int w = q * THREADS + tid;
            const int which = w >= ORD_ROWS * UPR, rem = w - which * ORD_ROWS * UPR;
            if (drow[q] >= 0)
                *reinterpret_cast<u32x4 *>((which ? vb : kb) + (size_t)drow[q] * D + (rem % UPR) * 8) = val[q];
        }
    };
    // Chunk c may be stored when chunk c - 1 has been read by every thread that reads it.  Loads complete
    // in issue order and the chunk requested after c - 1 is at least UPT load instructions per thread (its
    // 16-byte row pieces; how many loads of the destination map the compiler makes of the rest is its
    // business), so "at most UPT memory operations outstanding" means c - 1 has landed in this thread
    // (stores in flight only make the count stricter), and the barrier extends that to the workgroup.
    auto ready_to_store = [&](int c, int later_chunks) {
        asm volatile("" ::: "memory");
        if (later_chunks >= 1) __builtin_amdgcn_s_waitcnt(0x0F70 | (UPT & 15) | ((UPT >> 4) << 14));
        else __builtin_amdgcn_s_waitcnt(0x0F70);
        asm volatile("" ::: "memory");
        __syncthreads();
        if (c == c1 - 1 && tid == 0)   // the top chunk is in registers: the workgroup above may overwrite its rows
            __hip_atomic_store(&myflags[c], epoch, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (c == c0 && c > 0) {        // the lowest chunk writes into the top chunk of the workgroup below
            if (tid == 0) {
                int spins = 0;
                while (__hip_atomic_load(&myflags[c - 1], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != epoch) {
                    if (++spins > ORD_SPIN_LIMIT) {
                        atomicOr(p.status, STATUS_ORDER_TIMEOUT);
                        break;
                    }
                    __builtin_amdgcn_s_sleep(8);
                }
            }
            __syncthreads();
        }
    };
    // three register sets in rotation: chunk c in one, c - 1 in the next, c - 2 requested into the third
    int c = c1 - 1;
    load(c, va, da);
    if (c - 1 >= c0) load(c - 1, vb2, db);
    while (true) {
        if (c - 2 >= c0) load(c - 2, vc, dc);
        ready_to_store(c, c - 2 >= c0 ? 1 : 0);
        store(va, da);
        if (--c < c0) break;
        if (c - 2 >= c0) load(c - 2, va, da);
        ready_to_store(c, c - 2 >= c0 ? 1 : 0);
        store(vb2, db);
        if (--c < c0) break;
        if (c - 2 >= c0) load(c - 2, vb2, db);
        ready_to_store(c, c - 2 >= c0 ? 1 : 0);
        store(vc, dc);
        if (--c < c0) break;
    }
}

}  // namespace kd
