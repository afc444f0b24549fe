// The small-M GEMM every heavy phase of the decode kernel is made of: 16 activation rows staged
// in LDS (split exactly into three bfloat16 planes for the matrix cores) against 16-column
// tiles of a weight matrix; run_item drives one work item through staging, products and
// epilogue.  Included by decode.hip only.
#ifndef TDT_TILE_GEMM_H
#define TDT_TILE_GEMM_H

#include <type_traits>

#include "tdt_internal.h"
#include "decode_state.h"
#include "exchange.h"

namespace tdt {
namespace {

// ---------------------------------------------------------------------------
// Activation tile in LDS and the two tile-GEMM back ends (both on the matrix cores)
// ---------------------------------------------------------------------------
// bfloat16 weights: three bfloat16 planes [3][RT][ldb] with hi + lo + lo2 == x.
// float32 weights:  one float plane [RT][ldb].
template <typename WT> struct ActTile;

template <> struct ActTile<uint16_t> {
    uint16_t *planes;
    int ldb;   // elements per row (multiple of 8, padded)
    __host__ __device__ static int row_elems(int kseg_max) { return ((kseg_max + 31) / 32) * 32 + 8; }
    // x == hi + lo + lo2 exactly, each term a bfloat16: hi and lo are x and the first
    // remainder truncated to their top 16 bits (a truncated term keeps the sign, so each
    // remainder is exact and shorter by at least 8 significant bits); the second
    // remainder has at most 8 significant bits left and is a bfloat16 as it stands
    __device__ static void split3(float x, unsigned &hi, unsigned &lo, unsigned &lo2)
    {
        hi = __float_as_uint(x) & 0xffff0000u;
        const float r1 = x - __uint_as_float(hi);
        lo = __float_as_uint(r1) & 0xffff0000u;
        const float r2 = r1 - __uint_as_float(lo);
        lo2 = __float_as_uint(r2);
    }
    __device__ void store2(int i, int k, float2 v) const
    {
        unsigned a[3], b[3];
        split3(v.x, a[0], a[1], a[2]);
        split3(v.y, b[0], b[1], b[2]);
#pragma unroll
        for (int pl = 0; pl < 3; ++pl)   // element k in the low half, k + 1 in the high half
            *reinterpret_cast<unsigned *>(planes + ((size_t)pl * RT + i) * ldb + k) =
                (a[pl] >> 16) | (b[pl] & 0xffff0000u);
    }
    // four consecutive inputs k .. k+3 (k a multiple of 4): one 8-byte store per plane
    __device__ void store4(int i, int k, float4 v) const
    {
        unsigned a[3], b[3], c[3], d[3];
        split3(v.x, a[0], a[1], a[2]);
        split3(v.y, b[0], b[1], b[2]);
        split3(v.z, c[0], c[1], c[2]);
        split3(v.w, d[0], d[1], d[2]);
#pragma unroll
        for (int pl = 0; pl < 3; ++pl)
            *reinterpret_cast<uint2 *>(planes + ((size_t)pl * RT + i) * ldb + k) =
                make_uint2((a[pl] >> 16) | (b[pl] & 0xffff0000u), (c[pl] >> 16) | (d[pl] & 0xffff0000u));
    }
};

template <> struct ActTile<float> {
    float *planes;
    int ldb;   // floats per row: padded by 16 bytes so that 16-byte reads of 16 rows meet different banks
    __host__ __device__ static int row_elems(int kseg_max) { return ((kseg_max + 31) / 32) * 32 + 4; }
    __device__ void store2(int i, int k, float2 v) const
    {
        *reinterpret_cast<float2 *>(planes + (size_t)i * ldb + k) = v;
    }
    __device__ void store4(int i, int k, float4 v) const
    {
        *reinterpret_cast<float4 *>(planes + (size_t)i * ldb + k) = v;
    }
};

// stage one K segment: with c = ctx(i) computed once per row, mix(c, k, load(c, k)) gives the
// two inputs (k, k+1) of row i; the tail up to a multiple of 32 is zero-filled.  load only
// loads and mix only computes: all loads of a wavefront are issued before the first loaded
// value is used, so that their latencies overlap (a use between two loads makes the
// compiler wait for the first load before it issues the second, and so does a load inside
// a block that depends on the lane).  For the same reason load is called for every step of a
// row -- steps beyond K re-read the last step -- and what it returned there is dropped
// afterwards.  Rows beyond nrows are skipped altogether (the condition is the same for all
// lanes of a wavefront): the tile keeps whatever those rows held, their products are never
// looked at, and a row of the product depends on no other row of the tile.
// RB: rows of a wavefront whose loads are in flight together (all RT / kWaves of them, or fewer
// where a row's loads take many registers; the rounds then follow each other).
template <typename WT, int KIT, int RB, typename CtxF, typename LoadF, typename MixF>
__device__ inline void stage_segment_impl(const ActTile<WT> &A, int K, int nrows, CtxF ctx, LoadF load, MixF mix)
{
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int Kpad = ((K + 31) / 32) * 32;
    constexpr int RPW = RT / kWaves;    // rows per wavefront
    static_assert(RPW % RB == 0, "rows per round must divide the rows of a wavefront");
#pragma unroll
    for (int i0 = 0; i0 < RPW; i0 += RB) {
        decltype(ctx(0)) c[RB];
#pragma unroll
        for (int ii = 0; ii < RB; ++ii) {
            const int i = wave + (i0 + ii) * kWaves;
            c[ii] = ctx(i < nrows ? i : 0);
        }
        decltype(load(c[0], 0)) v[RB][KIT];
#pragma unroll
        for (int ii = 0; ii < RB; ++ii)
            if (wave + (i0 + ii) * kWaves < nrows) {
#pragma unroll
                for (int kk = 0; kk < KIT; ++kk) {
                    const int k = lane * 2 + kk * 128;
                    v[ii][kk] = load(c[ii], k < K ? k : K - 2);
                }
            }
        __builtin_amdgcn_sched_barrier(0);
        TR(60);
#if TDT_TRACE
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        TR(61);
#endif
#pragma unroll
        for (int ii = 0; ii < RB; ++ii)
            if (wave + (i0 + ii) * kWaves < nrows) {
#pragma unroll
                for (int kk = 0; kk < KIT; ++kk) {
                    const int i = wave + (i0 + ii) * kWaves, k = lane * 2 + kk * 128;
                    const float2 x = mix(c[ii], k < K ? k : K - 2, v[ii][kk]);
                    if (k < Kpad) A.store2(i, k, make_float2(k < K ? x.x : 0.0f, k < K ? x.y : 0.0f));
                }
            }
    }
}

template <typename WT, int RB = RT / kWaves, typename CtxF, typename LoadF, typename MixF>
__device__ inline void stage_segment(const ActTile<WT> &A, int K, int nrows, CtxF ctx, LoadF load, MixF mix)
{
    // 64 lanes x 2 inputs per step: pick the unrolling that covers K without spare loads
    if (K <= 640) stage_segment_impl<WT, 5, RB>(A, K, nrows, ctx, load, mix);
    else stage_segment_impl<WT, KSEG / 128, RB>(A, K, nrows, ctx, load, mix);
}

// The same with four inputs (16 bytes) per lane and step: mix(c, k, load(c, k)) gives inputs
// k .. k+3 of row i.  For sources that plain loads may read (what the kernel itself does not
// write): a compute unit takes in 16-byte-per-lane loads at nearly twice the rate of
// 8-byte-per-lane ones (measured: 53 against 30 bytes a clock).
template <typename WT, int KIT, int RB, typename CtxF, typename LoadF, typename MixF>
__device__ inline void stage_segment4_impl(const ActTile<WT> &A, int K, int nrows, CtxF ctx, LoadF load, MixF mix)
{
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int Kpad = ((K + 31) / 32) * 32;
    constexpr int RPW = RT / kWaves;
    static_assert(RPW % RB == 0, "rows per round must divide the rows of a wavefront");
#pragma unroll
    for (int i0 = 0; i0 < RPW; i0 += RB) {
        decltype(ctx(0)) c[RB];
#pragma unroll
        for (int ii = 0; ii < RB; ++ii) {
            const int i = wave + (i0 + ii) * kWaves;
            c[ii] = ctx(i < nrows ? i : 0);
        }
        decltype(load(c[0], 0)) v[RB][KIT];
#pragma unroll
        for (int ii = 0; ii < RB; ++ii)
            if (wave + (i0 + ii) * kWaves < nrows) {
#pragma unroll
                for (int kk = 0; kk < KIT; ++kk) {
                    const int k = lane * 4 + kk * 256;
                    v[ii][kk] = load(c[ii], k < K ? k : K - 4);
                }
            }
        __builtin_amdgcn_sched_barrier(0);
        TR(60);
#if TDT_TRACE
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        TR(61);
#endif
#pragma unroll
        for (int ii = 0; ii < RB; ++ii)
            if (wave + (i0 + ii) * kWaves < nrows) {
#pragma unroll
                for (int kk = 0; kk < KIT; ++kk) {
                    const int i = wave + (i0 + ii) * kWaves, k = lane * 4 + kk * 256;
                    const float4 x = mix(c[ii], k < K ? k : K - 4, v[ii][kk]);
                    // (K is a multiple of 8: the four inputs lie on one side of it)
                    if (k < Kpad) A.store4(i, k, k < K ? x : make_float4(0.0f, 0.0f, 0.0f, 0.0f));
                }
            }
    }
}

template <typename WT, int RB = RT / kWaves, typename CtxF, typename LoadF, typename MixF>
__device__ inline void stage_segment4(const ActTile<WT> &A, int K, int nrows, CtxF ctx, LoadF load, MixF mix)
{
    // 64 lanes x 4 inputs per step: pick the unrolling that covers K without spare loads
    if (K <= 512) stage_segment4_impl<WT, 2, RB>(A, K, nrows, ctx, load, mix);
    else if (K <= 768) stage_segment4_impl<WT, 3, RB>(A, K, nrows, ctx, load, mix);
    else stage_segment4_impl<WT, KSEG / 256, RB>(A, K, nrows, ctx, load, mix);
}

// accumulators of one wavefront for one 16x16 tile
template <typename WT> struct Accum;
template <> struct Accum<uint16_t> {
    f32x4 c;   // lane l: column l % 16, rows (l / 16) * 4 + e
    __device__ void clear() { c = f32x4{0.0f, 0.0f, 0.0f, 0.0f}; }
};
template <> struct Accum<float> {
    f32x4 c;   // same layout
    __device__ void clear() { c = f32x4{0.0f, 0.0f, 0.0f, 0.0f}; }
};

// matrix-core back end: this wavefront adds its share (k-steps kpart, kpart + ksplit, ...)
// of one segment to the 16x16 tile whose 16 weight rows are given per lane (l % 16).
// The first chunk of weight fragments can be fetched ahead (before the activations are
// staged) with weight_prefetch.
#ifndef TDT_CH
#define TDT_CH 5
#endif
constexpr int CH = TDT_CH;   // weight fragments in flight per wavefront

struct WeightCursor {
    const uint4 *fr;   // this lane's 16 bytes of the first fragment of the tile's stretch
    int kq, n_my, last;   // last: the stretch's last step
};

// tile: the column tile's index in the matrix's fragment-major copy
__device__ inline WeightCursor weight_cursor(const Seg &sg, int tile, int kpart, int ksplit, int lane)
{
    WeightCursor wc;
    wc.kq = (lane >> 4) * 8;
    wc.fr = static_cast<const uint4 *>(sg.w) + ((size_t)tile * sg.nst + (sg.k0 >> 5)) * 64 + lane;
    const int nsteps = (sg.K + 31) / 32;
    wc.last = nsteps - 1;
    // ksplit is a power of two
    wc.n_my = nsteps > kpart ? (nsteps - kpart + ksplit - 1) >> __builtin_ctz(ksplit) : 0;
    return wc;
}

// Loads are unconditional (a step beyond the stretch re-reads its last fragment) and nothing
// uses a fragment before all CH loads have been issued.  A wavefront's load is one contiguous KiB.
__device__ inline void weight_prefetch(const WeightCursor &wc, const Seg &, int kpart, int ksplit, int c0,
                                       uint4 (&b)[CH])
{
#pragma unroll
    for (int j = 0; j < CH; ++j) {
        const int s = kpart + (c0 + j) * ksplit;
        b[j] = ldg_u4(wc.fr + (size_t)min(s, wc.last) * 64);
    }
    __builtin_amdgcn_sched_barrier(0);
}

// the products of one chunk of CH k-steps (from step c0 of this wavefront's share) with the
// weight fragments b.  Nothing is masked: the fragment-major copy holds zeros beyond the end of
// a row (K no multiple of 32) and in columns that are padding, and the tile is zero from K up
// to a multiple of 32 as well.  A step beyond the wavefront's share reads, as its
// activation fragment, the padding at the end of each tile row, which nothing ever writes and
// which is zero from the start of the kernel.  The activation fragments of step j + 1 are
// requested from LDS before the products of step j are issued.
__device__ inline void chunk_products(const uint16_t *arow, size_t plane, int zoff, int kq, int kpart, int ksplit,
                                      int c0, int n_my, const uint4 (&b)[CH], f32x4 &acc0, f32x4 &acc1, f32x4 &acc2)
{
    auto aoff = [&](int c) { return c < n_my ? (kpart + c * ksplit) * 32 + kq : zoff; };
    bf16x8 x[2][3];
    {
        const uint16_t *a = arow + aoff(c0);
        x[0][0] = *reinterpret_cast<const bf16x8 *>(a);
        x[0][1] = *reinterpret_cast<const bf16x8 *>(a + plane);
        x[0][2] = *reinterpret_cast<const bf16x8 *>(a + 2 * plane);
    }
    __builtin_amdgcn_sched_group_barrier(0x100, 3, 0);   // (the schedule: these three reads first)
#pragma unroll
    for (int j = 0; j < CH; ++j) {
        if (j + 1 < CH) {
            const uint16_t *a = arow + aoff(c0 + j + 1);
            x[(j + 1) & 1][0] = *reinterpret_cast<const bf16x8 *>(a);
            x[(j + 1) & 1][1] = *reinterpret_cast<const bf16x8 *>(a + plane);
            x[(j + 1) & 1][2] = *reinterpret_cast<const bf16x8 *>(a + 2 * plane);
        }
        const bf16x8 bv = *reinterpret_cast<const bf16x8 *>(&b[j]);
        acc0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(x[j & 1][0], bv, acc0, 0, 0, 0);
        acc1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(x[j & 1][1], bv, acc1, 0, 0, 0);
        acc2 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(x[j & 1][2], bv, acc2, 0, 0, 0);
        // keep that order in the schedule: the next step's three LDS reads, then this step's products
        if (j + 1 < CH) __builtin_amdgcn_sched_group_barrier(0x100, 3, 0);
        __builtin_amdgcn_sched_group_barrier(0x008, 3, 0);
    }
}

// b holds the wavefront's first chunk of weight fragments, b2 its second (if it has one): the
// first was requested before the item waited for its rows, the second as soon as the registers
// of the staged rows were free again, so that it travels while the first is multiplied.
// Further chunks are requested into a buffer as soon as its products have been issued.
__device__ inline void tile_accumulate(const ActTile<uint16_t> &A, const Seg &sg, const WeightCursor &wc,
                                       int kpart, int ksplit, uint4 (&b)[CH], uint4 (&b2)[CH], f32x4 &acc, int lane)
{
    const uint16_t *arow = A.planes + (size_t)(lane & 15) * A.ldb;
    const size_t plane = (size_t)RT * A.ldb;
    const int zoff = A.ldb - 8;
    const int n_my = __builtin_amdgcn_readfirstlane(wc.n_my);   // the same in every lane
    // One accumulator per plane of the split: three independent chains of products instead of
    // one, added up at the end.
    f32x4 acc1 = f32x4{0.0f, 0.0f, 0.0f, 0.0f}, acc2 = acc1;
    for (int c0 = 0; c0 < n_my; c0 += 2 * CH) {
        chunk_products(arow, plane, zoff, wc.kq, kpart, ksplit, c0, n_my, b, acc, acc1, acc2);
        if (c0 + 2 * CH < n_my) weight_prefetch(wc, sg, kpart, ksplit, c0 + 2 * CH, b);
        TR(50);
        if (c0 + CH < n_my) {
            chunk_products(arow, plane, zoff, wc.kq, kpart, ksplit, c0 + CH, n_my, b2, acc, acc1, acc2);
            if (c0 + 3 * CH < n_my) weight_prefetch(wc, sg, kpart, ksplit, c0 + 3 * CH, b2);
        }
    }
    // smallest terms first
    acc = acc + (acc1 + acc2);
}

template <typename WT> struct Backend;
template <> struct Backend<uint16_t> {
    struct Pre {   // weight fragments fetched before the activations can be read
        WeightCursor wc;
        uint4 b[CH], b2[CH];
    };
    // first chunk: requested before the item waits for the rows it depends on
    template <typename RowF>
    __device__ static void prefetch(Pre &pre, const Seg &sg, RowF, int, int tile, int kpart, int ksplit, int lane)
    {
        pre.wc = weight_cursor(sg, tile, kpart, ksplit, lane);
        weight_prefetch(pre.wc, sg, kpart, ksplit, 0, pre.b);
    }
    // second chunk: requested once the registers of the staged rows are free again
    __device__ static void prefetch_more(Pre &pre, const Seg &sg, int kpart, int ksplit)
    {
        if (__builtin_amdgcn_readfirstlane(pre.wc.n_my) > CH) weight_prefetch(pre.wc, sg, kpart, ksplit, CH, pre.b2);
    }
    template <typename RowF>
    __device__ static void accumulate(const ActTile<uint16_t> &A, const Seg &sg, RowF, int, int kpart, int ksplit,
                                      Accum<uint16_t> &acc, int lane, Pre &pre)
    {
        tile_accumulate(A, sg, pre.wc, kpart, ksplit, pre.b, pre.b2, acc.c, lane);
    }
    __device__ static void spill(HypShared &S, const Accum<uint16_t> &acc, int wave, int lane)
    {
#pragma unroll
        for (int e = 0; e < 4; ++e) S.cpart[wave][(lane >> 4) * 4 + e][lane & 15] = acc.c[e];
    }
    __device__ static int ksplit_for(int n_ct) { return n_ct <= 1 ? 8 : n_ct <= 2 ? 4 : n_ct <= 4 ? 2 : 1; }
};
// float32 weights: the float32 matrix-core product (v_mfma_f32_16x16x4_f32: exact products,
// float32 accumulation).  A lane holds four consecutive inputs of its weight row / activation
// row (one 16-byte load each) and feeds them to four MFMAs; a step covers 16 inputs.
template <> struct Backend<float> {
    struct Pre {
        const float *wr;   // this lane's weight row at its quarter of a step (row 0 if the column is padding)
        bool live;
        int kq, n_my;
        float4 b[CH];
    };
    __device__ static void fetch(Pre &pre, const Seg &sg, int kpart, int ksplit, int c0)
    {
#pragma unroll
        for (int j = 0; j < CH; ++j) {   // unconditional, clamped into the row; masked where used
            const int k = (kpart + (c0 + j) * ksplit) * 16 + pre.kq;
            pre.b[j] = *reinterpret_cast<const float4 *>(pre.wr + (k < sg.K ? k : sg.K - 4));
        }
        __builtin_amdgcn_sched_barrier(0);
    }
    template <typename RowF>
    __device__ static void prefetch(Pre &pre, const Seg &sg, RowF rowidx, int ct, int, int kpart, int ksplit, int lane)
    {
        const long long wrow = rowidx(ct, lane & 15);
        pre.kq = (lane >> 4) * 4;
        pre.live = wrow >= 0;
        pre.wr = static_cast<const float *>(sg.w) + (pre.live ? wrow : 0) * sg.wld + sg.k0;
        const int nsteps = (sg.K + 15) / 16;
        pre.n_my = nsteps > kpart ? (nsteps - kpart + ksplit - 1) >> __builtin_ctz(ksplit) : 0;
        fetch(pre, sg, kpart, ksplit, 0);
    }
    __device__ static void prefetch_more(Pre &, const Seg &, int, int) {}
    template <typename RowF>
    __device__ static void accumulate(const ActTile<float> &A, const Seg &sg, RowF, int, int kpart, int ksplit,
                                      Accum<float> &acc, int lane, Pre &pre)
    {
        const float *a0 = A.planes + (size_t)(lane & 15) * A.ldb + pre.kq;
        for (int c0 = 0; c0 < pre.n_my; c0 += CH) {
            if (c0 > 0) fetch(pre, sg, kpart, ksplit, c0);
#pragma unroll
            for (int j = 0; j < CH; ++j) {
                if (c0 + j < pre.n_my) {
                    const int s = kpart + (c0 + j) * ksplit;
                    // the tile is zero beyond K up to a multiple of 32, so only the weights need the mask
                    const bool ok = pre.live && s * 16 + pre.kq < sg.K;
                    const float4 x = *reinterpret_cast<const float4 *>(a0 + s * 16);
                    acc.c = __builtin_amdgcn_mfma_f32_16x16x4f32(x.x, ok ? pre.b[j].x : 0.0f, acc.c, 0, 0, 0);
                    acc.c = __builtin_amdgcn_mfma_f32_16x16x4f32(x.y, ok ? pre.b[j].y : 0.0f, acc.c, 0, 0, 0);
                    acc.c = __builtin_amdgcn_mfma_f32_16x16x4f32(x.z, ok ? pre.b[j].z : 0.0f, acc.c, 0, 0, 0);
                    acc.c = __builtin_amdgcn_mfma_f32_16x16x4f32(x.w, ok ? pre.b[j].w : 0.0f, acc.c, 0, 0, 0);
                }
            }
        }
    }
    __device__ static void spill(HypShared &S, const Accum<float> &acc, int wave, int lane)
    {
#pragma unroll
        for (int e = 0; e < 4; ++e) S.cpart[wave][(lane >> 4) * 4 + e][lane & 15] = acc.c[e];
    }
    __device__ static int ksplit_for(int n_ct) { return n_ct <= 1 ? 8 : n_ct <= 2 ? 4 : n_ct <= 4 ? 2 : 1; }
};

// One work item: all K segments of the staged rows against n_ct column tiles, a round of
// (8 / ksplit) column tiles at a time.
//   tile0                          the item's first column tile, counted in column tiles of the
//                                  whole matrix (where the fragment-major copy keeps it)
//   stage(seg)                     stages Seg seg of the item's rows (stage_segment)
//   rowidx(ct, j)    -> long long  weight row of column j of column tile ct, -1 if none
//   pre(ct0, n)                    called by all threads at the start of a round, before the
//                                  rows are staged: issues loads whose latency should hide there
//   park(ct0, n)                   called by all threads after the round's products, before the
//                                  barrier that precedes epi: may put what pre loaded into LDS
//   wait()                         called by all threads once, before the first rows are staged
//                                  (after the first weights have been requested); must contain
//                                  a workgroup barrier
//   epi(ct0, n, ksplit)            called by all threads once S.cpart holds round results:
//                                  tile slot t (< n) is the sum over kp < ksplit of
//                                  S.cpart[t * ksplit + kp]; S.bias[t * 16 + j] is
//                                  bias[rowidx(ct0 + t, j)]
// With one segment the rows are staged once; with several they are staged again for
// every round.
template <typename WT, typename StageF, typename RowF, typename PreF, typename ParkF, typename EpiF, typename WaitF>
__device__ inline void run_item(HypShared &S, const ActTile<WT> &A, const PhaseInputs &in, int tile0, int n_ct,
                                const float *__restrict__ bias, const float *any_floats, StageF stage,
                                RowF rowidx, PreF pre_round, ParkF park, EpiF epi, WaitF wait)
{
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int nseg = in.count();
    // The bias load below is unconditional, so that it is issued with the other loads of the
    // item: where there is no bias, any_floats must be a readable float array that covers every
    // index rowidx can return.
    const float *bias_or_any = bias ? bias : static_cast<const float *>(any_floats);
    const int ksplit = Backend<WT>::ksplit_for(n_ct);
    const int ksh = __builtin_ctz(ksplit);    // ksplit is 1, 2, 4 or 8
    const int tpr = kWaves >> ksh;            // column tiles per round
    const int tslot = wave >> ksh, kpart = wave & (ksplit - 1);
    for (int base = 0; base < n_ct; base += tpr) {
        const int ct = base + tslot;
        const bool mine = ct < n_ct;
        Accum<WT> acc;
        acc.clear();
        // bias of column (threadIdx.x % 16) of tile slot (threadIdx.x / 16): the load is issued
        // here, unconditionally, and parked in LDS only after the rows have been staged
        float bias_v;
        {
            const int bt = (int)(threadIdx.x % (kWaves * CT)) / CT, bj = (int)threadIdx.x % CT;
            const long long r = base + bt < n_ct ? rowidx(base + bt, bj) : -1;
            bias_v = bias_or_any[r >= 0 ? r : 0];
            if (r < 0 || !bias) bias_v = 0.0f;
        }
        TR(10);
        pre_round(base, min(tpr, n_ct - base));
        TR(11);
        for (int sgi = 0; sgi < nseg; ++sgi) {
            const Seg sg = in.get(sgi);
            long long tq = 0;
            if (TDT_FINE_TIMERS && threadIdx.x == 0) tq = wall_clock64();
            typename Backend<WT>::Pre pre;
            // the weights do not depend on the activations: fetch the first of them now
            if (mine) Backend<WT>::prefetch(pre, sg, rowidx, ct, tile0 + ct, kpart, ksplit, lane);
            TR(12);
            if (nseg > 1 || base == 0) {
                // previous readers of the tile are done
                if (base == 0 && sgi == 0) wait();
                else __syncthreads();
                TR(13);
                stage(sg);
                if (mine) Backend<WT>::prefetch_more(pre, sg, kpart, ksplit);
                TR(14);
                __syncthreads();
                TR(15);
            }
            else if (mine) Backend<WT>::prefetch_more(pre, sg, kpart, ksplit);
            if (TDT_FINE_TIMERS && threadIdx.x == 0) { const long long n = wall_clock64(); S.tk_fine[S.fine_phase][0] += n - tq; tq = n; }
            if (mine) Backend<WT>::accumulate(A, sg, rowidx, ct, kpart, ksplit, acc, lane, pre);
            TR(16);
            if (TDT_FINE_TIMERS && threadIdx.x == 0) S.tk_fine[S.fine_phase][1] += wall_clock64() - tq;
        }
        long long tq = 0;
        if (TDT_FINE_TIMERS && threadIdx.x == 0) tq = wall_clock64();
        if (mine) Backend<WT>::spill(S, acc, wave, lane);
        if (threadIdx.x < kWaves * CT) S.bias[threadIdx.x] = bias_v;
        park(base, min(tpr, n_ct - base));
        TR(17);
        __syncthreads();
        TR(18);
        epi(base, min(tpr, n_ct - base), ksplit);
        TR(19);
        __syncthreads();
        TR(20);
        if (TDT_FINE_TIMERS && threadIdx.x == 0) S.tk_fine[S.fine_phase][2] += wall_clock64() - tq;
    }
}

// ---------------------------------------------------------------------------
// The streaming joint pass (bfloat16 weights, one stretch of the reduction).  The 16 rows are
// staged once; then every wavefront walks groups of WTW column tiles of its own (group wave,
// wave + 8, ...) with no workgroup barrier in between.  An activation fragment read from LDS is
// multiplied by WTW weight fragments (the reads of the activations from LDS, not the matrix
// cores, bound a wavefront that takes one tile at a time).  Weight fragments travel in chunks of
// WKS k-steps (WKS * WTW fragments) through two register buffers, one being multiplied while the
// other is on its way, across group borders.  A lane holds column l % 16 and rows
// (l / 16) * 4 .. + 3 of each tile of its wavefront's current group and keeps running statistics
// of those four rows over all its tiles -- largest label logit, its column, the sum of
// exp(logit - largest), largest duration logit and its class -- so that no logit ever goes
// through LDS; they are reduced across the 16 lanes of a row (DPP rotations) and across the
// wavefronts (LDS) once per work item.  Ties: a lane walks its columns in ascending order and
// keeps the first maximum; across lanes and wavefronts the lowest column among equals wins.
// ---------------------------------------------------------------------------
#ifndef TDT_WIDE_TW
#define TDT_WIDE_TW 1
#endif
#ifndef TDT_WIDE_KS
#define TDT_WIDE_KS 8
#endif
constexpr int WTW = TDT_WIDE_TW;   // column tiles per group
constexpr int WKS = TDT_WIDE_KS;   // k-steps per chunk

// what thread i (< 16) of the workgroup holds for row i of the tile after wide_item
struct WideRowStats {
    float m, s, dm;   // largest label logit, sum of exp(logit - m) over the item's label columns, largest duration logit
    int a, da;        // their columns (label; duration class)
};

// v combined over the 16 lanes of its row by rotations: every lane ends up with the result
template <typename T, typename Op> __device__ inline T row_allreduce(T v, Op op)
{
    v = op(v, dpp_move<0x121, 0xf>(v, v));   // row_ror:1
    v = op(v, dpp_move<0x122, 0xf>(v, v));   // row_ror:2
    v = op(v, dpp_move<0x124, 0xf>(v, v));   // row_ror:4
    v = op(v, dpp_move<0x128, 0xf>(v, v));   // row_ror:8
    return v;
}

// one chunk of weight fragments in flight, with the biases of its group's columns
struct WideChunk {
    uint4 b[WKS][WTW];
    float bias[WTW];
};

template <typename StageF, typename WaitF>
__device__ inline void wide_item(HypShared &S, const ActTile<uint16_t> &A, const Seg &sg, int tile0, int n_ct, int V,
                                 int O, const float *__restrict__ bias, StageF stage, WaitF wait, WideRowStats &out)
{
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int kq = (lane >> 4) * 8;
    const int nsteps = (sg.K + 31) / 32;
    const int nch = (nsteps + WKS - 1) / WKS;                        // chunks per group of tiles
    const int n_grp = (n_ct + WTW - 1) / WTW;
    const int my_groups = n_grp > wave ? (n_grp - wave + kWaves - 1) / kWaves : 0;
    const int total = my_groups * nch;                               // chunks of this wavefront
    const uint4 *wbase = static_cast<const uint4 *>(sg.w) + (size_t)(sg.k0 >> 5) * 64 + lane;
    // chunk (t, ci) of this wavefront: tiles tile0 + (wave + t * 8) * WTW + u, k-steps ci * WKS ...
    // (a tile beyond the item, a column beyond the matrix: a valid row, results never looked at)
    auto fetch = [&](int t, int ci, WideChunk &w) __attribute__((always_inline)) {
        const int s0 = ci * WKS;
#pragma unroll
        for (int u = 0; u < WTW; ++u) {
            const int tl = (wave + t * kWaves) * WTW + u;
            const int col = (tile0 + tl) * CT + (lane & 15);
            const int cc = tl < n_ct && col < O ? col : 0;
            const uint4 *fr = wbase + (size_t)(tl < n_ct ? tile0 + tl : tile0) * sg.nst * 64;
            w.bias[u] = bias[cc];
#pragma unroll
            for (int j = 0; j < WKS; ++j) w.b[j][u] = ldg_u4(fr + (size_t)min(s0 + j, nsteps - 1) * 64);
        }
    };
    WideChunk wA, wB;
    int ft = 0, fci = 0;   // the next chunk to request
    auto fetch_next = [&](WideChunk &w) __attribute__((always_inline)) {
        fetch(ft, fci, w);
        {   // (selections, not branches with stores: those would put the counters into memory)
            const bool wrap = fci + 1 == nch;
            ft += wrap ? 1 : 0;
            fci = wrap ? 0 : fci + 1;
        }
    };
    if (total > 0) fetch_next(wA);   // before the rows this item depends on have arrived
    TR(70);
    wait();
    stage();
    __syncthreads();
    TR(71);

    const uint16_t *arow = A.planes + (size_t)(lane & 15) * A.ldb;
    const size_t plane = (size_t)RT * A.ldb;
    const int zoff = A.ldb - 8;   // a row's padding: zeros (see chunk_products)
    // one accumulator per plane of the split: three independent chains of products per tile
    // instead of one (a product that waits for the one before it takes several times as long)
    f32x4 acc[WTW][3];
#pragma unroll
    for (int u = 0; u < WTW; ++u)
#pragma unroll
        for (int pl = 0; pl < 3; ++pl) acc[u][pl] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
    float rm[4], rs[4], rdm[4];
    int ra[4], rda[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        rm[e] = rdm[e] = -INFINITY;
        rs[e] = 0.0f;
        ra[e] = rda[e] = 0x7fffffff;
    }
    int ct_ = 0, cci = 0;   // the chunk being multiplied
    // The activation fragments of step j of the chunk.  A chunk that lies inside the reduction
    // (every chunk when the joint width is a multiple of 32 * WKS) reads them at constant offsets
    // from three per-lane addresses computed once per chunk; otherwise every step is checked
    // against the end of the reduction (a step beyond it reads the zero padding).
    // The fragments of the chunk after this one are requested one k-step at a time, between the
    // products: a wavefront that asks for a whole chunk at once sits in the compute unit's queue
    // for the address path (64 bytes a clock for all eight wavefronts: 0.36 us per chunk measured)
    // while its matrix core idles.
    auto products = [&](const WideChunk &w, WideChunk &wn, auto whole_tag) __attribute__((always_inline)) {
        constexpr bool kWhole = decltype(whole_tag)::value;
        const int s0 = cci * WKS;
        // the chunk to request (uniform)
        const int ns0 = fci * WKS;
        const uint4 *nfr[WTW];
#pragma unroll
        for (int u = 0; u < WTW; ++u) {
            const int tl = (wave + ft * kWaves) * WTW + u;
            const int col = (tile0 + tl) * CT + (lane & 15);
            nfr[u] = wbase + (size_t)(tl < n_ct ? tile0 + tl : tile0) * sg.nst * 64;
            wn.bias[u] = ldg_f(bias + (tl < n_ct && col < O ? col : 0));
        }
        {   // (selections, not branches with stores: those would put the counters into memory)
            const bool wrap = fci + 1 == nch;
            ft += wrap ? 1 : 0;
            fci = wrap ? 0 : fci + 1;
        }
        const uint16_t *a0 = arow + (size_t)s0 * 32 + kq;
        auto frag = [&](int j, int pl) -> const uint16_t * {
            if constexpr (kWhole) return a0 + pl * plane + j * 32;
            else return arow + (s0 + j < nsteps ? (s0 + j) * 32 + kq : zoff) + pl * plane;
        };
        bf16x8 x[2][3];
#pragma unroll
        for (int pl = 0; pl < 3; ++pl) x[0][pl] = *reinterpret_cast<const bf16x8 *>(frag(0, pl));
        __builtin_amdgcn_sched_group_barrier(0x100, 3, 0);   // (the schedule: these three reads first)
#pragma unroll
        for (int j = 0; j < WKS; ++j) {
            if (j + 1 < WKS) {
#pragma unroll
                for (int pl = 0; pl < 3; ++pl)
                    x[(j + 1) & 1][pl] = *reinterpret_cast<const bf16x8 *>(frag(j + 1, pl));
            }
            // consecutive products go to different accumulators
#pragma unroll
            for (int pl = 0; pl < 3; ++pl)
#pragma unroll
                for (int u = 0; u < WTW; ++u)
                    acc[u][pl] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                        x[j & 1][pl], *reinterpret_cast<const bf16x8 *>(&w.b[j][u]), acc[u][pl], 0, 0, 0);
#pragma unroll
            for (int u = 0; u < WTW; ++u) wn.b[j][u] = ldg_u4(nfr[u] + (size_t)min(ns0 + j, nsteps - 1) * 64);
            // keep that order in the schedule: the next step's three LDS reads, this step's
            // products, the request for the next chunk's fragments of this step
            if (j + 1 < WKS) __builtin_amdgcn_sched_group_barrier(0x100, 3, 0);
            __builtin_amdgcn_sched_group_barrier(0x008, 3 * WTW, 0);
            __builtin_amdgcn_sched_group_barrier(0x020, WTW, 0);
        }
    };
    // the products of one chunk; at the end of a group the logits of this lane update the statistics
    auto chunk = [&](const WideChunk &w, WideChunk &wn) __attribute__((always_inline)) {
        if ((cci + 1) * WKS <= nsteps) products(w, wn, std::true_type{});   // uniform over the wavefront
        else products(w, wn, std::false_type{});
        if (cci == nch - 1) {   // uniform over the wavefront: the group is complete
#pragma unroll
            for (int u = 0; u < WTW; ++u) {
                const int tl = (wave + ct_ * kWaves) * WTW + u;
                const int col = tl < n_ct ? (tile0 + tl) * CT + (lane & 15) : O;   // O: no column
                const f32x4 sum = acc[u][0] + (acc[u][1] + acc[u][2]);   // smallest terms first
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const float v = sum[e] + w.bias[u];
                    if (col <= V) {
                        if (v > rm[e]) {
                            rs[e] = (rs[e] > 0.0f ? rs[e] * __expf(rm[e] - v) : 0.0f) + 1.0f;
                            rm[e] = v;
                            ra[e] = col;
                        } else {
                            rs[e] += __expf(v - rm[e]);
                        }
                    } else if (col < O && v > rdm[e]) {
                        rdm[e] = v;
                        rda[e] = col - (V + 1);
                    }
                }
#pragma unroll
                for (int pl = 0; pl < 3; ++pl) acc[u][pl] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
            }
        }
        {
            const bool last = cci == nch - 1;
            ct_ += last ? 1 : 0;
            cci = last ? 0 : cci + 1;
        }
    };
    // Every chunk requests the one after it (beyond the wavefront's last chunk: a valid fragment
    // again), so the number of loads in flight is the same at every wait.
    int c = 0;
    for (; c + 2 <= total; c += 2) {
        chunk(wA, wB);
        TR(72);
        chunk(wB, wA);
        TR(72);
    }
    if (c < total) chunk(wA, wB);
    TR(73);

    // ---- one reduction per work item: across the 16 lanes of a row, then across the wavefronts
    auto fmax2 = [](float x, float y) { return fmaxf(x, y); };
    auto imin2 = [](int x, int y) { return min(x, y); };
    auto fadd2 = [](float x, float y) { return x + y; };
    float *wstat = &S.cpart[0][0][0];   // [kWaves][RT][5], the partial-result scratch is not in use here
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const float m = row_allreduce(rm[e], fmax2);
        const int a = row_allreduce(rm[e] == m ? ra[e] : 0x7fffffff, imin2);
        const float sl = rs[e] > 0.0f ? rs[e] * __expf(rm[e] - m) : 0.0f;
        const float sr = row_allreduce(sl, fadd2);
        const float dm = row_allreduce(rdm[e], fmax2);
        const int da = row_allreduce(rdm[e] == dm ? rda[e] : 0x7fffffff, imin2);
        if ((lane & 15) == 0) {
            float *w = wstat + ((size_t)wave * RT + (lane >> 4) * 4 + e) * 5;
            w[0] = m;
            w[1] = __int_as_float(a);
            w[2] = sr;
            w[3] = dm;
            w[4] = __int_as_float(da);
        }
    }
    __syncthreads();
    out.m = out.dm = -INFINITY;
    out.s = 0.0f;
    out.a = out.da = 0x7fffffff;
    if (threadIdx.x < RT) {
        const int i = threadIdx.x;
        for (int w8 = 0; w8 < kWaves; ++w8) {   // wavefronts hold interleaved tiles: lowest column among equals
            const float *w = wstat + ((size_t)w8 * RT + i) * 5;
            const float m = w[0], sr = w[2], dm = w[3];
            const int a = __float_as_int(w[1]), da = __float_as_int(w[4]);
            if (sr > 0.0f) {
                if (m > out.m) {
                    out.s = (out.s > 0.0f ? out.s * __expf(out.m - m) : 0.0f) + sr;
                    out.m = m;
                    out.a = a;
                } else {
                    out.s += sr * __expf(m - out.m);
                    if (m == out.m && a < out.a) out.a = a;
                }
            }
            if (dm > out.dm || (dm == out.dm && da < out.da)) {
                out.dm = dm;
                out.da = da;
            }
        }
    }
    __syncthreads();   // the scratch is free again
    TR(74);
}

__device__ inline float cpart_sum(const HypShared &S, int t, int ksplit, int i, int j)
{
    float v = S.cpart[t * ksplit][i][j];
    for (int kp = 1; kp < ksplit; ++kp) v += S.cpart[t * ksplit + kp][i][j];
    return v;
}

}  // namespace
}  // namespace tdt

#endif
