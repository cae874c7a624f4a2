// Device helpers shared by the kernels: bf16 -> double, and double-precision lane exchanges.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

// Phase timeline (profiling build, -DKD_TIMELINE): thread 0 of a workgroup stamps the constant
// 100 MHz wall clock into LDS at named points and the workgroup stores its 32 stamps at the end.
// The product build compiles all of it away.
#ifdef KD_TIMELINE
#define KD_TL_DECL                                                  \
    __shared__ unsigned long long kd_tl[32];                        \
    if (threadIdx.x == 0) {                                         \
        for (int i_ = 0; i_ < 32; ++i_) kd_tl[i_] = 0;              \
    }
#define KD_TL(i)                                                    \
    do {                                                            \
        if (threadIdx.x == 0) kd_tl[(i)] = wall_clock64();          \
    } while (0)
#define KD_TL_DUMP(dst, wg)                                                                      \
    do {                                                                                         \
        __syncthreads();                                                                         \
        if ((dst) && threadIdx.x < 32) (dst)[(size_t)(wg) * 32 + threadIdx.x] = kd_tl[threadIdx.x]; \
    } while (0)
#else
#define KD_TL_DECL
#define KD_TL(i) do { } while (0)
#define KD_TL_DUMP(dst, wg) do { } while (0)
#endif

namespace kd {

// The argument block of a launch was written by the host just before it and lies in no cache: every 64
// bytes of it that a workgroup touches for the first time cost a trip to memory, and the compiler reads
// the fields of a parameter structure where they are needed, one such trip after another (measured on
// the attention launch: 1 us).  warm_arguments<BYTES>() requests one word of each cache line of the
// first BYTES bytes at once, ahead of everything else, and waits for them: later reads find the lines
// in the scalar cache.  (At most 8 lines; the words themselves are not used.)
template <size_t BYTES>
__device__ __forceinline__ void warm_arguments()
{
    constexpr int LINES = (int)((BYTES + 63) / 64) < 8 ? (int)((BYTES + 63) / 64) : 8;
    const char *ka = (const char *)__builtin_amdgcn_kernarg_segment_ptr();
    uint32_t d[LINES];
#pragma unroll
    for (int i = 0; i < LINES; ++i) asm volatile("s_load_dword %0, %1, %2" : "=s"(d[i]) : "s"(ka), "n"(64 * i));
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
    for (int i = 0; i < LINES; ++i) asm volatile("" : : "s"(d[i]));   // the destination registers stay reserved until here
}

// Asynchronous 16-byte-per-lane copy global -> LDS (no registers).  `lds_base` is uniform over the
// active lanes; lane i writes bytes [16 i, 16 i + 16) above it.  Issued through asm, so the compiler
// does not count it: completion is awaited with an explicit s_waitcnt vmcnt (copies complete in
// issue order, together with the wave's other loads).
__device__ __forceinline__ void lds_copy16(uint32_t lds_base, const void *gaddr)
{
    const uint32_t base = (uint32_t)__builtin_amdgcn_readfirstlane((int)lds_base);
    asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, off" : : "s"(base), "v"(gaddr) : "memory");
}

__device__ __forceinline__ double bf16_lo(uint32_t w) { return (double)__uint_as_float(w << 16); }
__device__ __forceinline__ double bf16_hi(uint32_t w) { return (double)__uint_as_float(w & 0xFFFF0000u); }

__device__ __forceinline__ double shfl_xor_f64(double x, int m)
{
    int lo = __double2loint(x), hi = __double2hiint(x);
    lo = __shfl_xor(lo, m);
    hi = __shfl_xor(hi, m);
    return __hiloint2double(hi, lo);
}

// x + (x of another lane of the same 16-lane row), by a DPP control word
template <int CTRL>
__device__ __forceinline__ double dpp_add_f64(double x)
{
    const int lo = __builtin_amdgcn_update_dpp(0, __double2loint(x), CTRL, 0xF, 0xF, false);
    const int hi = __builtin_amdgcn_update_dpp(0, __double2hiint(x), CTRL, 0xF, 0xF, false);
    return x + __hiloint2double(hi, lo);
}

// sum over the LANES (8 or 16) consecutive lanes that share one key row; every lane gets the
// total.  Quad exchanges, then mirrors inside the half row and the row: each step pairs a lane
// with one that holds the sum of a different, equally sized group.
template <int LANES>
__device__ __forceinline__ double row_allreduce_f64(double x)
{
    static_assert(LANES == 8 || LANES == 16, "a key row spans 8 or 16 lanes");
    x = dpp_add_f64<0xB1>(x);                    // quad_perm [1,0,3,2]
    x = dpp_add_f64<0x4E>(x);                    // quad_perm [2,3,0,1]
    x = dpp_add_f64<0x141>(x);                   // row_half_mirror: lane i <-> 7 - i
    if (LANES == 16) x = dpp_add_f64<0x140>(x);  // row_mirror: lane i <-> 15 - i
    return x;
}


// x + (x of lane ^ 16) + (x of lane ^ 32) + (x of lane ^ 48): the sum over the four 16-lane rows of a
// wave, position by position, without a trip through LDS (every lane gets the total).
// v_permlane16_swap exchanges the odd rows of its first operand with the even rows of its second:
// given x twice, the pair it returns holds {x of the even row, x of the odd row} of the lane's row
// pair in every lane; v_permlane32_swap does the same with the two halves of the wave.
__device__ __forceinline__ double sum_over_rows_f64(double x)
{
    auto pair_sum = [](double v, bool halves) {
        const uint32_t lo = (uint32_t)__double2loint(v), hi = (uint32_t)__double2hiint(v);
        const auto a = halves ? __builtin_amdgcn_permlane32_swap(lo, lo, false, false)
                              : __builtin_amdgcn_permlane16_swap(lo, lo, false, false);
        const auto b = halves ? __builtin_amdgcn_permlane32_swap(hi, hi, false, false)
                              : __builtin_amdgcn_permlane16_swap(hi, hi, false, false);
        return __hiloint2double((int)b[0], (int)a[0]) + __hiloint2double((int)b[1], (int)a[1]);
    };
    return pair_sum(pair_sum(x, false), true);
}

// the double another lane holds, fetched by a DPP control word (rows of 16 lanes)
template <int CTRL>
__device__ __forceinline__ double dpp_fetch_f64(double x)
{
    const int lo = __builtin_amdgcn_update_dpp(0, __double2loint(x), CTRL, 0xF, 0xF, false);
    const int hi = __builtin_amdgcn_update_dpp(0, __double2hiint(x), CTRL, 0xF, 0xF, false);
    return __hiloint2double(hi, lo);
}

// Four quantities, each spread over the 16 lanes of a row, summed with 5 additions per lane instead
// of 16: the lanes first split the quantities between them (lane bit 3, then bit 2, decides which
// a lane keeps; it hands the others to a partner on the other side of that bit and adds what the
// partner hands over), then the four lanes left with the same quantity finish among themselves.
// On return lanes 4k .. 4k + 3 of every row hold the full sum of quantity k.
__device__ __forceinline__ double row_reduce_scatter4_f64(double q0, double q1, double q2, double q3, int u)
{
    const bool b3 = (u & 8) != 0, b2 = (u & 4) != 0;
    double k0 = b3 ? q2 : q0, k1 = b3 ? q3 : q1;          // kept
    const double s0 = b3 ? q0 : q2, s1 = b3 ? q1 : q3;    // handed to lane u ^ 8
    k0 += dpp_fetch_f64<0x128>(s0);                       // row_ror:8
    k1 += dpp_fetch_f64<0x128>(s1);
    double k = b2 ? k1 : k0;
    const double s = b2 ? k0 : k1;                        // handed to lane 7 - u of the half row
    k += dpp_fetch_f64<0x141>(s);                         // row_half_mirror
    k += dpp_fetch_f64<0xB1>(k);                          // quad_perm [1,0,3,2]
    k += dpp_fetch_f64<0x4E>(k);                          // quad_perm [2,3,0,1]
    return k;
}

// The canonical score of one key (appendix "FLOP count of KeyDiff"): mu.k / max(|mu| |k|, eps) in
// IEEE double, rounded once to float; + 0 folds -0 into +0.  Every kernel that scores calls this.
__device__ __forceinline__ float finish_score(double dot, double k2, double nmu, double eps)
{
    double den = nmu * sqrt(k2);
    if (den < eps) den = eps;
    return (float)(dot / den) + 0.0f;
}

}  // namespace kd
