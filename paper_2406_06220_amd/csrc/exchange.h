// How the workgroups of a cluster exchange data and wait for each other: agent-scope relaxed
// atomics that are served at the device's coherence point, packed (value, index) cells for
// atomic maxima, the split barrier, and the small list / split helpers of the label loop.
// Included by decode.hip only.
#ifndef TDT_EXCHANGE_H
#define TDT_EXCHANGE_H

#include "tdt_internal.h"
#include "decode_state.h"

namespace tdt {
namespace {

// ---- number formats
// two consecutive matrix entries: the load as it comes from memory, and its conversion
template <typename WT> struct W2;
template <> struct W2<float> {
    typedef float2 Raw;
    __device__ static Raw load(const float *p) { return *reinterpret_cast<const float2 *>(p); }
    __device__ static float2 cvt(Raw r) { return r; }
};
template <> struct W2<uint16_t> {
    typedef uint32_t Raw;
    __device__ static Raw load(const uint16_t *p) { return *reinterpret_cast<const uint32_t *>(p); }
    __device__ static float2 cvt(Raw u) { return make_float2(__uint_as_float(u << 16), __uint_as_float(u & 0xffff0000u)); }
};

// hardware exponential and reciprocal: about 1e-7 absolute error on a value in (0, 1)
__device__ inline float fast_sigmoid(float x) { return __frcp_rn(1.0f + __expf(-x)); }

// ---- reductions across lanes on the data-parallel-primitive path of the vector ALU (no LDS
// round trip per step, unlike a shuffle).  Rows are the four groups of 16 lanes of a wavefront:
// row_shr:n hands lane i the value of lane i - n of its row (the identity where there is none);
// row_bcast:15 hands every lane of rows 1 and 3 the value of lane 15 of the row before.  After
// the five steps lane 31 holds the reduction over lanes 0..31 and lane 63 that over lanes
// 32..63; a sixth step (row_bcast:31) would leave the whole wavefront's in lane 63.
template <int CTRL, int ROW_MASK> __device__ inline float dpp_move(float identity, float v)
{
    return __int_as_float(__builtin_amdgcn_update_dpp(__float_as_int(identity), __float_as_int(v), CTRL, ROW_MASK,
                                                      0xf, false));
}
template <int CTRL, int ROW_MASK> __device__ inline int dpp_move(int identity, int v)
{
    return __builtin_amdgcn_update_dpp(identity, v, CTRL, ROW_MASK, 0xf, false);
}
// op over each half of the wavefront; the result is valid in lanes 31 and 63
template <typename T, typename Op> __device__ inline T half_reduce(T v, T identity, Op op)
{
    v = op(v, dpp_move<0x111, 0xf>(identity, v));   // row_shr:1
    v = op(v, dpp_move<0x112, 0xf>(identity, v));   // row_shr:2
    v = op(v, dpp_move<0x114, 0xf>(identity, v));   // row_shr:4
    v = op(v, dpp_move<0x118, 0xf>(identity, v));   // row_shr:8
    v = op(v, dpp_move<0x142, 0xa>(identity, v));   // row_bcast:15 into rows 1 and 3
    return v;
}
// the value lane 31 holds, in lanes 0..31, and the value lane 63 holds, in lanes 32..63
__device__ inline float half_broadcast(float v, int lane)
{
    const float lo = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 31));
    const float hi = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 63));
    return lane < 32 ? lo : hi;
}
// sum over the whole wavefront, valid in lane 63
__device__ inline float wave_sum(float v)
{
    v = half_reduce(v, 0.0f, [](float a, float b) { return a + b; });
    return v + dpp_move<0x143, 0xc>(0.0f, v);   // row_bcast:31 into rows 2 and 3
}

// ---- coherent exchange primitives (see the header comment)
#define TDT_AGENT __HIP_MEMORY_SCOPE_AGENT
#define TDT_GLOBAL __attribute__((address_space(1)))
// Loads through a pointer that is known to point to device memory.  The compiler cannot see that
// for pointers that went through structures and selections and then emits flat loads, which count
// against the LDS counter as well: every wait for an LDS access would then wait for them too.
__device__ inline uint4 ldg_u4(const uint4 *p)
{
    typedef unsigned v4u __attribute__((ext_vector_type(4)));
    const v4u v = *(const TDT_GLOBAL v4u *)p;
    return make_uint4(v.x, v.y, v.z, v.w);
}
__device__ inline float ldg_f(const float *p) { return *(const TDT_GLOBAL float *)p; }

__device__ inline float ld_co(const float *p)
{
    return __hip_atomic_load((const TDT_GLOBAL float *)p, __ATOMIC_RELAXED, TDT_AGENT);
}
__device__ inline void st_co(float *p, float v)
{
    __hip_atomic_store((TDT_GLOBAL float *)p, v, __ATOMIC_RELAXED, TDT_AGENT);
}
__device__ inline float2 ld_co2(const float *p)   // p 8-byte aligned
{
    const unsigned long long u =
        __hip_atomic_load((const TDT_GLOBAL unsigned long long *)p, __ATOMIC_RELAXED, TDT_AGENT);
    return make_float2(__uint_as_float((unsigned)u), __uint_as_float((unsigned)(u >> 32)));
}
// Four floats of a row that other workgroups wrote in an earlier phase, with one 16-byte load
// of agent scope.  An atomic load is 8 bytes at most, and the compute unit takes in agent-scope
// 8-byte loads at half the rate of 16-byte ones (27 against 55 bytes a clock, measured); a raw
// buffer load carries the same scope bit (sc1: what an agent-scope relaxed atomic load compiles
// to) on a 16-byte access.  The four floats need not arrive as one unit: a row is only read
// after the group barrier that follows its last store.  `row` must be the same in every lane
// (the buffer descriptor lives in scalar registers); offsets at or beyond `n` floats read zeros.
__device__ inline float4 ld_co4(const float *row, int n, int k)
{
    typedef unsigned v4u __attribute__((ext_vector_type(4)));
    const __amdgpu_buffer_rsrc_t rs =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(row), 0, n * (int)sizeof(float), 0x00020000);
    const v4u v = __builtin_amdgcn_raw_buffer_load_b128(rs, k * (int)sizeof(float), 0, 16 /* sc1 */);
    return make_float4(__uint_as_float(v.x), __uint_as_float(v.y), __uint_as_float(v.z), __uint_as_float(v.w));
}
__device__ inline unsigned long long ld_co64(const unsigned long long *p)
{
    return __hip_atomic_load((const TDT_GLOBAL unsigned long long *)p, __ATOMIC_RELAXED, TDT_AGENT);
}
__device__ inline void st_co64(unsigned long long *p, unsigned long long v)
{
    __hip_atomic_store((TDT_GLOBAL unsigned long long *)p, v, __ATOMIC_RELAXED, TDT_AGENT);
}

// (logit, index) packed so that an unsigned 64-bit maximum is "largest logit,
// lowest index on ties"; zero is below every packed value
__device__ inline unsigned long long pack_best(float v, int idx)
{
    unsigned u = __float_as_uint(v + 0.0f);   // -0 and +0 compare equal: make them one pattern
    u = (u & 0x80000000u) ? ~u : (u | 0x80000000u);
    return ((unsigned long long)u << 32) | (unsigned long long)(0xffffffffu - (unsigned)idx);
}
__device__ inline int unpack_index(unsigned long long p) { return (int)(0xffffffffu - (unsigned)p); }
__device__ inline float unpack_value(unsigned long long p)
{
    unsigned u = (unsigned)(p >> 32);
    u = (u & 0x80000000u) ? (u & 0x7fffffffu) : ~u;
    return __uint_as_float(u);
}

// Barrier over the C workgroups of one cluster, in two halves.  Every workgroup owns one
// flag word, a cache line apart from the next.  To arrive it stores the barrier's sequence
// number there, after all its earlier coherent stores have completed.  To wait, its first
// wavefront polls the flags of all C members (lane l reads member l, l + 64, ...) until they
// have reached that number, while the other wavefronts rest at the workgroup barrier: little
// polling traffic, no read-modify-write and no tree.  Work that does not depend on what the
// other workgroups wrote (setting up the next work item, fetching weights) goes between the
// two halves and hides the flags' way through memory.  Every wait is bounded: on a timeout,
// or when another workgroup has flagged an abort, the wait returns false and the caller
// leaves the kernel.
struct BarrierInfo {
    unsigned *flags;   // the cluster's flags, kBarrierStride words apart
    unsigned *mine;    // where this workgroup announces its arrivals: its flag -- or, in the self-test
                       // of the time-out path, a spare word nobody reads
    unsigned epoch;    // barriers arrived at so far (the same in every thread of the cluster)
};

__device__ inline void barrier_arrive(BarrierInfo &bi, int C)
{
    // every coherent store / atomic of this wavefront has completed ...
    TR(30);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    TR(31);
    __syncthreads();   // ... and so have those of the whole workgroup
    TR(32);
    const unsigned epoch = ++bi.epoch;
    if (C > 1 && threadIdx.x == 0) __hip_atomic_store(bi.mine, epoch, __ATOMIC_RELAXED, TDT_AGENT);
}

// ends with a workgroup barrier
__device__ inline bool barrier_wait(HypShared &S, const BarrierInfo &bi, int *abort_flag, int C,
                                    long long timeout_ticks)
{
    TR(34);
    const unsigned epoch = bi.epoch;
    if (C > 1 && threadIdx.x < 64) {
        const int lane = threadIdx.x;
        const long long t0 = wall_clock64();
        unsigned spins = 0;
        for (;;) {
            bool all = true;
            for (int base = 0; base < C; base += 64) {   // uniform
                const int idx = base + lane;
                const unsigned f = __hip_atomic_load(bi.flags + (size_t)(idx < C ? idx : 0) * kBarrierStride,
                                                     __ATOMIC_RELAXED, TDT_AGENT);
                all = all && (idx >= C || (int)(f - epoch) >= 0);
            }
            if (__ballot(!all) == 0ull) break;
            if ((++spins & 31u) == 0u) {
                int stop = 0;
                if (lane == 0) {
                    if (__hip_atomic_load(abort_flag, __ATOMIC_RELAXED, TDT_AGENT)) {
                        stop = 1;
                    } else if (wall_clock64() - t0 > timeout_ticks) {
                        __hip_atomic_store(abort_flag, 1, __ATOMIC_RELAXED, TDT_AGENT);
                        stop = 1;
                    }
                }
                if (__shfl(stop, 0, 64)) {
                    if (lane == 0) S.aborted = 1;
                    break;
                }
            }
        }
    }
    __syncthreads();
    TR(33);
    return S.aborted == 0;
}

__device__ inline bool cluster_barrier(HypShared &S, BarrierInfo &bi, int *abort_flag, int C,
                                       long long timeout_ticks)
{
    barrier_arrive(bi, C);
    return barrier_wait(S, bi, abort_flag, C, timeout_ticks);
}

// list[0..n) = indices g < G with flag[g] set, ascending.  All threads call it.
__device__ inline void build_list(HypShared &S, const unsigned char *flag, int G, int *list,
                                  int *n_out)
{
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const bool f = tid < G && flag[tid] != 0;
    const unsigned long long m = __ballot(f);
    if (lane == 0) S.wave_cnt[wave] = __popcll(m);
    __syncthreads();
    int off = 0, total = 0;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
        const int c = S.wave_cnt[w];
        if (w < wave) off += c;
        total += c;
    }
    if (f) list[off + __popcll(m & ((1ull << lane) - 1ull))] = tid;
    if (tid == 0) *n_out = total;
    __syncthreads();
}

// build_list for two flag arrays at once (one pair of workgroup barriers for both)
__device__ inline void build_two_lists(HypShared &S, int G, const unsigned char *flag_a, int *list_a, int *n_a,
                                       const unsigned char *flag_b, int *list_b, int *n_b)
{
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const bool fa = tid < G && flag_a[tid] != 0, fb = tid < G && flag_b[tid] != 0;
    const unsigned long long ma = __ballot(fa), mb = __ballot(fb);
    if (lane == 0) {
        S.wave_cnt[wave] = __popcll(ma);
        S.wave_cnt2[wave] = __popcll(mb);
    }
    __syncthreads();
    int off_a = 0, tot_a = 0, off_b = 0, tot_b = 0;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
        const int ca = S.wave_cnt[w], cb = S.wave_cnt2[w];
        if (w < wave) { off_a += ca; off_b += cb; }
        tot_a += ca;
        tot_b += cb;
    }
    const unsigned long long below = (1ull << lane) - 1ull;
    if (fa) list_a[off_a + __popcll(ma & below)] = tid;
    if (fb) list_b[off_b + __popcll(mb & below)] = tid;
    if (tid == 0) {
        *n_a = tot_a;
        *n_b = tot_b;
    }
    __syncthreads();
}

// deal `n_units` column tiles to the workgroups left after `n_row_tiles` took theirs
__device__ inline void split_tiles(int C, int n_row_tiles, int n_units, int max_groups, int &n_groups,
                                   int &per_group)
{
    int g = C / (n_row_tiles > 0 ? n_row_tiles : 1);
    if (g < 1) g = 1;
    if (g > max_groups) g = max_groups;
    if (g > n_units) g = n_units;
    per_group = (n_units + g - 1) / g;
    n_groups = (n_units + per_group - 1) / per_group;
}

}  // namespace
}  // namespace tdt

#endif
