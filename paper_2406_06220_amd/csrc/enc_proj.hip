// Dense projections computed once per call, before the label loop starts:
//   encoder projection (paper Sec. 3.4; the precomputation at line 2 of Algorithm 3)
//     out[r][n] = sum_k enc[r][k] * w_enc[n][k] + b_enc[n]
//   and, with the same kernel, what the predictor side can tabulate per label: the first LSTM
//   layer's input product w_ih[0] * emb[label] + b_lstm[0], or -- for a stateless predictor,
//   whose output is nothing but embeddings of the last labels -- its whole projection into the
//   joint space, one table per context position: w_pred[:, c*E .. (c+1)*E) * emb_c[label]
//   (the last table with b_pred added).
// A dense contraction over all B*T frames, so it runs on the matrix cores:
// bf16 operands, fp32 accumulation, fp32 output (v_mfma_f32_32x32x16_bf16).
// Both operands are K-contiguous ("NT" GEMM), which is the layout the MFMA lane
// mapping wants: lane l supplies row (l % 32), k-slice (l / 32) * 8 .. + 7.
#include "tdt_internal.h"

#include <mutex>
#include <type_traits>

namespace tdt {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

namespace {

constexpr int BM = 128, BN = 128, BK = 64;   // workgroup tile
constexpr int GEMM_THREADS = 256;            // 4 wavefronts, each a 64x64 sub-tile

// A tile row is 128 bytes, half of the 64 four-byte LDS banks; rows r and r + 1 lie in different
// halves.  16-byte chunk c of row r is stored at chunk c ^ ((r >> 1) & 7), so that the 16 rows a
// quarter of a wavefront reads for one k-slice (same c, consecutive r) fall on 16 different
// chunk positions, i.e. on all 64 banks.
__device__ inline int lds_off(int row, int chunk) { return row * BK + ((chunk ^ ((row >> 1) & 7)) << 3); }

// One product C = A * W^T + bias and the workgroups it takes.  Rows of W are ldw apart (a
// slice of the columns of a wider matrix can be multiplied); bias may be null.
// With `lens` the rows are the frames of B utterances of T frames each, of which only the first
// min(max(lens[b], 0), T) of utterance b are multiplied (Alg. 3 line 2 projects the encoder
// output; frames beyond an utterance's length are never looked at, so they are neither read nor
// written): the workgroups then walk the valid frames in order, 128 at a time, and M = B * T only
// bounds their number.
struct LinearProblem {
    const uint16_t *A, *W;
    const float *bias;
    float *C;
    long long M;
    int N, K, ldw, group;
    const int32_t *lens;
    int B, T;
    unsigned blocks;
};
constexpr int kMaxProblems = 3;   // products one preparation launch can hold
struct LinearBatch {
    LinearProblem q[kMaxProblems];
};

// Which frames rows m0 .. m0 + ROWS - 1 of the packed sequence of valid frames are: row_of[i] =
// b * T + t, or -1 beyond the last valid frame.  Called by all THREADS threads of a workgroup;
// returns false (for all of them) if the tile holds no valid frame at all.  Every thread sums a
// stretch of the utterances' lengths, the stretches' sums are scanned across the workgroup, and
// each row finds its utterance by a search over the stretches and a walk through its stretch.
template <int ROWS, int THREADS = GEMM_THREADS>
__device__ inline bool valid_row_map(const int32_t *lens, int B, int T, long long m0, long long *row_of, int *scan,
                                     int *wsum)
{
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int per = (B + THREADS - 1) / THREADS;
    const int b_lo = min(tid * per, B), b_hi = min(b_lo + per, B);
    int mine = 0;   // B * T < 2^31, so every sum of lengths fits an int
    for (int b = b_lo; b < b_hi; ++b) mine += min(max(lens[b], 0), T);
    int v = mine;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const int t = __shfl_up(v, off, 64);
        if (lane >= off) v += t;
    }
    if (lane == 63) wsum[wave] = v;
    __syncthreads();
    int base = 0, total = 0;
#pragma unroll
    for (int w = 0; w < THREADS / 64; ++w) {
        if (w < wave) base += wsum[w];
        total += wsum[w];
    }
    scan[tid] = base + v - mine;   // valid frames before stretch tid
    __syncthreads();
    if (m0 >= total) return false;
    if (tid < ROWS) {
        const long long m = m0 + tid;
        long long src = -1;
        if (m < total) {
            int lo = 0, hi = THREADS - 1;   // the last stretch that starts at or before m
            while (lo < hi) {
                const int mid = (lo + hi + 1) >> 1;
                if (scan[mid] <= m) lo = mid; else hi = mid - 1;
            }
            long long before = scan[lo];
            int b = min(lo * per, B);
            for (;; ++b) {   // ends, because m < total
                const int len = min(max(lens[b], 0), T);
                if (m < before + len) break;
                before += len;
            }
            src = (long long)b * T + (m - before);
        }
        row_of[tid] = src;
    }
    return true;
}

// the 128 x 128 output tile of workgroup `block` (of q.blocks) of one product
__device__ inline void gemm_tile_bf16(const LinearProblem &q, unsigned block)
{
    const uint16_t *__restrict__ A = q.A;
    const uint16_t *__restrict__ W = q.W;
    const float *__restrict__ bias = q.bias;
    float *__restrict__ C = q.C;
    const long long M = q.M;
    const int N = q.N, K = q.K, ldw = q.ldw, group = q.group;
    // the operand tiles (two buffers each) and, once the products are done, the output tile on
    // its way to memory share one block of LDS
    constexpr int CLD = BN + 4;   // floats per row of the output tile (padded: rows 8 apart meet other banks)
    constexpr size_t kTileBytes = 2 * (size_t)(BM + BN) * BK * sizeof(uint16_t);
    constexpr size_t kOutBytes = (size_t)BM * CLD * sizeof(float);
    __shared__ __align__(16) unsigned char lds_raw[kOutBytes > kTileBytes ? kOutBytes : kTileBytes];
    uint16_t (*As)[BM * BK] = reinterpret_cast<uint16_t (*)[BM * BK]>(lds_raw);
    uint16_t (*Bs)[BN * BK] = reinterpret_cast<uint16_t (*)[BN * BK]>(lds_raw + 2 * (size_t)BM * BK * sizeof(uint16_t));
    float *Cs = reinterpret_cast<float *>(lds_raw);
    __shared__ long long row_of[BM];   // source / destination row of each row of the tile, -1: none
    __shared__ int scan[GEMM_THREADS], wsum[GEMM_THREADS / 64];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    // 1-D grid.  Consecutive workgroups go to consecutive XCDs, each with an L2 of its own, so
    // the workgroups that share a row tile of `A` (all its column tiles) are given to one XCD:
    // row tiles are dealt round robin to the XCDs, and the j-th workgroup of an XCD takes
    // column tile j % nt_n of that XCD's (j / nt_n)-th row tile.  `A` then comes from HBM once
    // instead of once per XCD; `W` is small and stays in every L2.
    const int nt_n = (N + BN - 1) / BN;
    const long long j = block / kXcds;
    const long long mt = (j / nt_n) * kXcds + block % kXcds;
    const long long m0 = mt * BM;
    const int n0 = (int)(j % nt_n) * BN;
    if (m0 >= M) return;   // the last round of row tiles may be partial (uniform over the workgroup)
    if (q.lens) {
        if (!valid_row_map<BM>(q.lens, q.B, q.T, m0, row_of, scan, wsum)) return;   // uniform
    } else if (tid < BM) {
        row_of[tid] = m0 + tid < M ? m0 + tid : -1;
    }
    __syncthreads();

    f32x16 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;

    // Two register sets and two LDS buffers: K tile kt is multiplied from LDS while tile kt + 1
    // sits in (or is still on its way into) one register set and tile kt + 2 is being requested
    // into the other -- at this kernel's few hundred bytes per flop-microsecond it is the number
    // of bytes in flight per compute unit that decides how much of the HBM rate it gets.
    uint4 ra[2][4], rb[2][4];
    // What this thread loads of every K tile: 16-byte chunk kc of four rows of each operand.
    // The loads themselves are unconditional -- a row or chunk that does not exist is read from
    // one that does (row 0, the last chunk) and replaced by zeros on its way into LDS -- because
    // a load inside a block that depends on the lane makes the compiler wait for every load
    // still in flight before it issues the next, and the two K tiles in flight become one.
    const int kc = tid & 7;
    const uint16_t *a_src[4], *w_src[4];
    bool a_ok[4], w_ok[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int row = (tid + j * GEMM_THREADS) >> 3;
        const long long ar = row_of[row];
        const int n = n0 + row;
        a_ok[j] = ar >= 0;
        w_ok[j] = n < N;
        a_src[j] = A + (a_ok[j] ? ar : 0) * K;
        w_src[j] = W + (long long)(w_ok[j] ? n : 0) * ldw;
    }
    auto load_tiles = [&](int k0, uint4 (&xa)[4], uint4 (&xb)[4]) {
        const int k = min(k0 + kc * 8, K - 8);   // K is a multiple of 8
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            xa[j] = *reinterpret_cast<const uint4 *>(a_src[j] + k);
            xb[j] = *reinterpret_cast<const uint4 *>(w_src[j] + k);
        }
    };
    auto store_tiles = [&](int buf, int k0, const uint4 (&xa)[4], const uint4 (&xb)[4]) {
        const bool k_ok = k0 + kc * 8 < K;
        // (masks, not a choice between two values: a choice between the register set and a
        // constant becomes a choice between two addresses, which puts the set into scratch memory)
        auto keep = [](uint4 v, bool ok) {
            const unsigned m = ok ? 0xffffffffu : 0u;
            return make_uint4(v.x & m, v.y & m, v.z & m, v.w & m);
        };
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int row = (tid + j * GEMM_THREADS) >> 3;
            *reinterpret_cast<uint4 *>(As[buf] + lds_off(row, kc)) = keep(xa[j], a_ok[j] && k_ok);
            *reinterpret_cast<uint4 *>(Bs[buf] + lds_off(row, kc)) = keep(xb[j], w_ok[j] && k_ok);
        }
    };
    auto products = [&](int buf) {
#pragma unroll
        for (int s = 0; s < BK / 16; ++s) {
            const int chunk = s * 2 + (lane >> 5);
            bf16x8 a[2], b[2];
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                const int ar = wm * 64 + i * 32 + (lane & 31);
                const int br = wn * 64 + i * 32 + (lane & 31);
                a[i] = *reinterpret_cast<const bf16x8 *>(As[buf] + lds_off(ar, chunk));
                b[i] = *reinterpret_cast<const bf16x8 *>(Bs[buf] + lds_off(br, chunk));
            }
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
        }
    };

    // The same products with the requests for a later K tile dealt out between them, one after
    // every two products (step s asks for the thread's s-th chunk of both operands), so that
    // the compute unit's address path takes them one by one instead of eight in a row.
    auto products_and_loads = [&](int buf, int k0, uint4 (&xa)[4], uint4 (&xb)[4]) __attribute__((always_inline)) {
        static_assert(BK / 16 == 4, "one chunk of each operand per k step");
        const int k = min(k0 + kc * 8, K - 8);
#pragma unroll
        for (int s = 0; s < BK / 16; ++s) {
            const int chunk = s * 2 + (lane >> 5);
            bf16x8 a[2], b[2];
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                const int ar = wm * 64 + i * 32 + (lane & 31);
                const int br = wn * 64 + i * 32 + (lane & 31);
                a[i] = *reinterpret_cast<const bf16x8 *>(As[buf] + lds_off(ar, chunk));
                b[i] = *reinterpret_cast<const bf16x8 *>(Bs[buf] + lds_off(br, chunk));
            }
            acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[0], b[0], acc[0][0], 0, 0, 0);
            acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[0], b[1], acc[0][1], 0, 0, 0);
            xa[s] = *reinterpret_cast<const uint4 *>(a_src[s] + k);
            acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[1], b[0], acc[1][0], 0, 0, 0);
            acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[1], b[1], acc[1][1], 0, 0, 0);
            xb[s] = *reinterpret_cast<const uint4 *>(w_src[s] + k);
            __builtin_amdgcn_sched_group_barrier(0x100, 4, 0);   // the step's four fragments from LDS
            __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);   // two products
            __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);   // one request
            __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);
            __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
        }
    };

    const int nk = (K + BK - 1) / BK;
    load_tiles(0, ra[0], rb[0]);
    if (nk > 1) load_tiles(BK, ra[1], rb[1]);
    store_tiles(0, 0, ra[0], rb[0]);
    __syncthreads();
    // Two K tiles per trip, so that the register sets are named at compile time; one workgroup
    // barrier per K tile (the buffer written after the products was last read before the
    // previous barrier).  The trips that have all their tiles run without a branch: behind a
    // branch, even a uniform one, the compiler no longer knows how many loads are in flight and
    // waits for all of them where the older set would do.  (The fence keeps the older set's way
    // into LDS behind the products.)
    int kt = 0;
    for (; kt + 4 <= nk; kt += 2) {
        products_and_loads(0, (kt + 2) * BK, ra[0], rb[0]);
        __builtin_amdgcn_sched_barrier(0);
        store_tiles(1, (kt + 1) * BK, ra[1], rb[1]);
        __syncthreads();
        products_and_loads(1, (kt + 3) * BK, ra[1], rb[1]);
        __builtin_amdgcn_sched_barrier(0);
        store_tiles(0, (kt + 2) * BK, ra[0], rb[0]);
        __syncthreads();
    }
    for (; kt < nk; kt += 2) {   // the last one to three tiles
        if (kt + 2 < nk) load_tiles((kt + 2) * BK, ra[0], rb[0]);
        products(0);
        if (kt + 1 < nk) store_tiles(1, (kt + 1) * BK, ra[1], rb[1]);
        __syncthreads();
        if (kt + 1 < nk) {
            if (kt + 3 < nk) load_tiles((kt + 3) * BK, ra[1], rb[1]);
            products(1);
            if (kt + 2 < nk) store_tiles(0, (kt + 2) * BK, ra[0], rb[0]);
            __syncthreads();
        }
    }

    // accumulator register e of lane l is row 8*(e/4) + 4*(l/32) + e%4, column l%32
    if (group > 0) {
        // outputs regrouped column by column (the LSTM table): scattered four-byte stores
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const int n = n0 + wn * 64 + j * 32 + (lane & 31);
                if (n >= N) continue;
                const float bn = bias ? bias[n] : 0.0f;
                const int nc = (n % group) * (N / group) + n / group;
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const long long dst = row_of[wm * 64 + i * 32 + (e >> 2) * 8 + (lane >> 5) * 4 + (e & 3)];
                    if (dst >= 0) C[dst * N + nc] = acc[i][j][e] + bn;
                }
            }
        return;
    }
    // The output tile goes through LDS so that it leaves as whole rows: a lane then stores 16
    // bytes, half a wavefront one 512-byte row, and the row's destination is looked up once per
    // row instead of once per element.  (The operand tiles are dead: every wavefront has passed
    // the barrier that followed the last products.)
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int r = wm * 64 + i * 32 + (e >> 2) * 8 + (lane >> 5) * 4 + (e & 3);
                Cs[r * CLD + wn * 64 + j * 32 + (lane & 31)] = acc[i][j][e];
            }
    __syncthreads();
    {
        const int c4 = (lane & 31) * 4;                 // this lane's four columns of the tile
        const int n = n0 + c4;
        float4 bn = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
        if (bias && n < N) {                            // N is a multiple of 8, so n + 3 < N too
            bn = *reinterpret_cast<const float4 *>(bias + n);
        }
#pragma unroll 4
        for (int it = 0; it < BM / (2 * GEMM_THREADS / 64); ++it) {
            const int r = (it * (GEMM_THREADS / 64) + wave) * 2 + (lane >> 5);
            const long long dst = row_of[r];
            float4 v = *reinterpret_cast<const float4 *>(Cs + r * CLD + c4);
            v.x += bn.x;
            v.y += bn.y;
            v.z += bn.z;
            v.w += bn.w;
            if (dst >= 0 && n < N) *reinterpret_cast<float4 *>(C + dst * N + n) = v;
        }
    }
}

__global__ __launch_bounds__(GEMM_THREADS, 2) void enc_proj_bf16_kernel(LinearProblem q)
{
    gemm_tile_bf16(q, blockIdx.x);
}

// ---------------------------------------------------------------------------
// The same product for large problems: 256 x 256 output tile, 8 wavefronts, each 128 x 64
// ---------------------------------------------------------------------------
// With 64 x 64 outputs a wavefront every MFMA needs one 16-byte fragment per lane from LDS, and
// the LDS of a compute unit (128 bytes a clock) is busy four fifths of the K loop while the
// matrix cores are busy half of it.  At 128 x 64 outputs a wavefront six fragments feed eight
// MFMAs, and a 256 x 256 tile stores half as many operand bytes per product.  One workgroup of
// 8 wavefronts per compute unit (two a SIMD), two LDS buffers of 64 KB, one register set that
// is requested during one K tile and stored to LDS during the next.
constexpr int GM = 256, GN = 256, BIG_THREADS = 512;
constexpr int BIG_OUT_ROWS = 64;          // rows of the output tile in LDS at a time
constexpr int BIG_CLD = GN + 4;           // floats per row of that part
struct BigShared {
    long long row_of[GM];
    int scan[BIG_THREADS], wsum[BIG_THREADS / 64];
};
constexpr size_t kBigTileBytes = 2 * (size_t)(GM + GN) * BK * sizeof(uint16_t);
static_assert((size_t)BIG_OUT_ROWS * BIG_CLD * sizeof(float) <= kBigTileBytes, "the output parts reuse the operand buffers");
constexpr size_t kBigLdsBytes = kBigTileBytes + sizeof(BigShared);

__global__ __launch_bounds__(BIG_THREADS, 1) void enc_proj_bf16_big_kernel(LinearProblem q)
{
    extern __shared__ __align__(16) unsigned char big_lds[];
    const uint16_t *__restrict__ A = q.A;
    const uint16_t *__restrict__ W = q.W;
    const float *__restrict__ bias = q.bias;
    float *__restrict__ C = q.C;
    const long long M = q.M;
    const int N = q.N, K = q.K, ldw = q.ldw;
    uint16_t *const As = reinterpret_cast<uint16_t *>(big_lds);                     // [2][GM * BK]
    uint16_t *const Bs = As + 2 * GM * BK;                                          // [2][GN * BK]
    float *const Cs = reinterpret_cast<float *>(big_lds);
    BigShared &sh = *reinterpret_cast<BigShared *>(big_lds + kBigTileBytes);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 2, wn = wave & 3;
    // the die-aware order of tiles of the 128 x 128 kernel
    const unsigned block = blockIdx.x;
    const int nt_n = (N + GN - 1) / GN;
    const long long jb = block / kXcds;
    const long long mt = (jb / nt_n) * kXcds + block % kXcds;
    const long long m0 = mt * GM;
    const int n0 = (int)(jb % nt_n) * GN;
    if (m0 >= M) return;   // uniform over the workgroup
    if (q.lens) {
        if (!valid_row_map<GM, BIG_THREADS>(q.lens, q.B, q.T, m0, sh.row_of, sh.scan, sh.wsum)) return;   // uniform
    } else if (tid < GM) {
        sh.row_of[tid] = m0 + tid < M ? m0 + tid : -1;
    }
    __syncthreads();

    f32x16 acc[4][2];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;

    // this thread's part of every K tile: 16-byte chunk kc of four rows of each operand
    // (unconditional loads, zeros by mask: see the 128 x 128 kernel)
    const int kc = tid & 7;
    const uint16_t *a_src[4], *w_src[4];
    bool a_ok[4], w_ok[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int row = (tid + j * BIG_THREADS) >> 3;
        const long long ar = sh.row_of[row];
        const int n = n0 + row;
        a_ok[j] = ar >= 0;
        w_ok[j] = n < N;
        a_src[j] = A + (a_ok[j] ? ar : 0) * K;
        w_src[j] = W + (long long)(w_ok[j] ? n : 0) * ldw;
    }
    uint4 xa[4], xb[4];
    auto keep = [](uint4 v, bool ok) {   // (a mask, not a choice: see the 128 x 128 kernel)
        const unsigned m = ok ? 0xffffffffu : 0u;
        return make_uint4(v.x & m, v.y & m, v.z & m, v.w & m);
    };
    // chunk idx (0..3 of A, 4..7 of W) of the register set: its request, and its way into LDS
    auto request = [&](int idx, int k) __attribute__((always_inline)) {
        if (idx < 4) xa[idx] = *reinterpret_cast<const uint4 *>(a_src[idx] + k);
        else xb[idx - 4] = *reinterpret_cast<const uint4 *>(w_src[idx - 4] + k);
    };
    auto to_lds = [&](int idx, int buf, bool k_ok) __attribute__((always_inline)) {
        const int row = (tid + (idx & 3) * BIG_THREADS) >> 3;
        if (idx < 4) *reinterpret_cast<uint4 *>(As + buf * (GM * BK) + lds_off(row, kc)) = keep(xa[idx], a_ok[idx] && k_ok);
        else *reinterpret_cast<uint4 *>(Bs + buf * (GN * BK) + lds_off(row, kc)) = keep(xb[idx - 4], w_ok[idx - 4] && k_ok);
    };
    // The products of the K tile in buffer `buf`.  Between the products of its first two k steps
    // the register set (K tile kt + 1, requested during the tile before) goes into the other
    // buffer, between those of its last two the set is requested again for K tile kt + 2: one
    // LDS store or one request after every two products, so that neither the stores nor the
    // requests stand between two K tiles, where all wavefronts would do them at the same time
    // with the matrix cores idle.
    auto products = [&](int buf, auto stores, auto loads, int k_store, int k_load) __attribute__((always_inline)) {
        constexpr bool STORES = decltype(stores)::value, LOADS = decltype(loads)::value;
        const uint16_t *const Ab = As + buf * (GM * BK), *const Bb = Bs + buf * (GN * BK);
        const bool k_ok = k_store + kc * 8 < K;
        const int k = min(k_load + kc * 8, K - 8);
#pragma unroll
        for (int s = 0; s < BK / 16; ++s) {
            const int chunk = s * 2 + (lane >> 5);
            bf16x8 a[4], b[2];
#pragma unroll
            for (int i = 0; i < 4; ++i)
                a[i] = *reinterpret_cast<const bf16x8 *>(Ab + lds_off(wm * 128 + i * 32 + (lane & 31), chunk));
#pragma unroll
            for (int j = 0; j < 2; ++j)
                b[j] = *reinterpret_cast<const bf16x8 *>(Bb + lds_off(wn * 64 + j * 32 + (lane & 31), chunk));
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                acc[i][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[0], acc[i][0], 0, 0, 0);
                acc[i][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[1], acc[i][1], 0, 0, 0);
                if (STORES && s < 2) to_lds(s * 4 + i, buf ^ 1, k_ok);
                if (LOADS && s >= 2) request((s - 2) * 4 + i, k);
            }
            __builtin_amdgcn_sched_group_barrier(0x100, 6, 0);   // the step's six fragments from LDS
            if ((STORES && s < 2) || (LOADS && s >= 2)) {
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);                  // two products
                    if (s < 2) __builtin_amdgcn_sched_group_barrier(0x200, 1, 0);       // one LDS store
                    else __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);             // or one request
                }
            } else {
                __builtin_amdgcn_sched_group_barrier(0x008, 8, 0);
            }
        }
    };

    const int nk = (K + BK - 1) / BK;
#pragma unroll
    for (int idx = 0; idx < 8; ++idx) request(idx, min(kc * 8, K - 8));
#pragma unroll
    for (int idx = 0; idx < 8; ++idx) to_lds(idx, 0, kc * 8 < K);
    if (nk > 1) {
#pragma unroll
        for (int idx = 0; idx < 8; ++idx) request(idx, min(BK + kc * 8, K - 8));
    }
    __syncthreads();
    // one workgroup barrier per K tile: the buffer written during the products of tile kt was
    // last read before the barrier that ended tile kt - 1.  The trips that store and request
    // run without a branch.
    const std::true_type yes{};
    const std::false_type no{};
    int kt = 0;
    for (; kt + 2 < nk; ++kt) {
        products(kt & 1, yes, yes, (kt + 1) * BK, (kt + 2) * BK);
        __syncthreads();
    }
    if (kt + 1 < nk) {
        products(kt & 1, yes, no, (kt + 1) * BK, 0);
        __syncthreads();
        ++kt;
    }
    products(kt & 1, no, no, 0, 0);
    __syncthreads();   // the operand buffers are dead: the output tile passes through them

    // accumulator register e of lane l is row 8*(e/4) + 4*(l/32) + e%4, column l%32.  The tile
    // leaves in four parts of 64 rows, each as whole rows: a wavefront stores one 1024-byte row.
    const int c4 = lane * 4;
    const int n = n0 + c4;
    float4 bn = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
    if (bias && n < N) bn = *reinterpret_cast<const float4 *>(bias + n);   // N is a multiple of 8
#pragma unroll
    for (int part = 0; part < GM / BIG_OUT_ROWS; ++part) {
        if (part > 0) __syncthreads();   // the part before has left LDS
        if (wm == part / 2) {
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j)
#pragma unroll
                    for (int e = 0; e < 16; ++e) {
                        const int r = i * 32 + (e >> 2) * 8 + (lane >> 5) * 4 + (e & 3);
                        Cs[r * BIG_CLD + wn * 64 + j * 32 + (lane & 31)] = acc[(part & 1) * 2 + i][j][e];
                    }
        }
        __syncthreads();
#pragma unroll 4
        for (int it = 0; it < BIG_OUT_ROWS / (BIG_THREADS / 64); ++it) {
            const int r = it * (BIG_THREADS / 64) + wave;
            const long long dst = sh.row_of[part * BIG_OUT_ROWS + r];
            float4 v = *reinterpret_cast<const float4 *>(Cs + r * BIG_CLD + c4);
            v.x += bn.x;
            v.y += bn.y;
            v.z += bn.z;
            v.w += bn.w;
            if (dst >= 0 && n < N) *reinterpret_cast<float4 *>(C + dst * N + n) = v;
        }
    }
}

// ---------------------------------------------------------------------------
// fragment-major copies of the streamed matrices
// ---------------------------------------------------------------------------
struct PackJob {
    const uint16_t *src;
    uint4 *dst;
    int N, K, gate_h;   // gate_h > 0: LSTM gate matrix of gate_h hidden units
    int steps;
    long long first, pieces;   // 16-byte pieces: its first in the batch, how many
};
constexpr int kMaxPackJobs = 3 + 2 * TDT_MAX_LSTM_LAYERS;
struct PackBatch {
    PackJob j[kMaxPackJobs];
    int n;
    long long pieces;
};

// block `blk` of `nblk` blocks of 256 threads copies its share of the pieces
__device__ inline void pack_pieces(const PackBatch &b, unsigned blk, unsigned nblk)
{
    for (long long piece = (long long)blk * 256 + threadIdx.x; piece < b.pieces; piece += (long long)nblk * 256) {
        int ji = 0;
        while (ji + 1 < b.n && piece >= b.j[ji + 1].first) ++ji;
        const PackJob &q = b.j[ji];
        const long long local = piece - q.first;
        const int lane = (int)(local & 63);
        const long long frag = local >> 6;
        const int step = (int)(frag % q.steps), tile = (int)(frag / q.steps);
        const int j = lane & 15, k = step * 32 + (lane >> 4) * 8;
        long long row;
        if (q.gate_h > 0) {
            const int unit = tile * 4 + (j >> 2);
            row = unit < q.gate_h ? (long long)(j & 3) * q.gate_h + unit : -1;
        } else {
            row = tile * 16 + j < q.N ? tile * 16 + j : -1;
        }
        uint4 v = make_uint4(0, 0, 0, 0);
        if (row >= 0 && k < q.K) v = *reinterpret_cast<const uint4 *>(q.src + row * q.K + k);   // K % 8 == 0
        q.dst[local] = v;
    }
}

__global__ __launch_bounds__(256) void pack_weights_kernel(PackBatch b) { pack_pieces(b, blockIdx.x, gridDim.x); }

PackBatch pack_batch(const tdt_weights_t *w, const PackedLayout &pl, bool on_the_fly, void *packed)
{
    PackBatch b{};
    if (w->dtype != 1 || pl.total == 0) return b;
    const bool lstm = w->pred_kind == TDT_PRED_LSTM;
    auto add = [&](const void *src, const PackedMatrix &m, int N, int K, int gate_h) {
        PackJob &q = b.j[b.n++];
        q.src = static_cast<const uint16_t *>(src);
        q.dst = reinterpret_cast<uint4 *>(static_cast<char *>(packed) + m.offset);
        q.N = N;
        q.K = K;
        q.gate_h = gate_h;
        q.steps = m.steps;
        q.first = b.pieces;
        q.pieces = (long long)m.tiles * m.steps * 64;
        b.pieces += q.pieces;
    };
    // what a call does not multiply by stays unpacked: the encoder projection and, with a
    // stateless predictor, its projection are products of the kernel only when it projects on the fly
    if (on_the_fly) add(w->w_enc, pl.w_enc, w->h_joint, w->d_enc, 0);
    if (on_the_fly || lstm) add(w->w_pred, pl.w_pred, w->h_joint, w->h_pred, 0);
    add(w->w_out, pl.w_out, w->vocab + 1 + w->n_dur, w->h_joint, 0);
    for (int l = 0; lstm && l < w->pred_layers; ++l) {
        if (l > 0) add(w->w_ih[l], pl.w_ih[l], 4 * w->h_pred, w->h_pred, w->h_pred);
        add(w->w_hh[l], pl.w_hh[l], 4 * w->h_pred, w->h_pred, w->h_pred);
    }
    return b;
}
unsigned pack_blocks_for(const PackBatch &b)
{
    const long long blocks = (b.pieces + 255) / 256;
    return (unsigned)(blocks < 1024 ? blocks : 1024);
}

// Everything a decode call needs before its decode kernel, in one launch: the encoder
// projection, the per-label tables of the predictor side (a product with blocks == 0 is
// absent), and the clearing of the workspace's zero region and of the statistics.  The tasks
// are independent; a workgroup takes its task from its index.  Every product's workgroup count
// is a multiple of the number of dies, so each keeps its die-aware order of tiles.
__global__ __launch_bounds__(GEMM_THREADS, 2) void prepare_bf16_kernel(LinearBatch batch, PackBatch pack,
                                                                   unsigned pack_blocks, uint4 *zero, size_t n16,
                                                                   long long *out_stats)
{
    unsigned b = blockIdx.x, used = 0;
#pragma unroll
    for (int i = 0; i < kMaxProblems; ++i) {
        if (b < batch.q[i].blocks) {
            gemm_tile_bf16(batch.q[i], b);
            return;
        }
        b -= batch.q[i].blocks;
        used += batch.q[i].blocks;
    }
    if (b < pack_blocks) {   // the fragment-major copies of the matrices the decode kernel streams
        pack_pieces(pack, b, pack_blocks);
        return;
    }
    b -= pack_blocks;
    used += pack_blocks;
    const unsigned zb = b, nzb = gridDim.x - used;
    for (size_t i = (size_t)zb * GEMM_THREADS + threadIdx.x; i < n16; i += (size_t)nzb * GEMM_THREADS)
        zero[i] = make_uint4(0, 0, 0, 0);
    if (out_stats && zb == 0 && threadIdx.x < TDT_STAT_COUNT) out_stats[threadIdx.x] = 0;
}

// float32 models (small): classic 64x64 tile, 4x4 outputs per thread.  lens as in LinearProblem
// (null: all M rows).
__global__ __launch_bounds__(GEMM_THREADS) void enc_proj_f32_kernel(
    const float *__restrict__ A, const float *__restrict__ W, const float *__restrict__ bias,
    float *__restrict__ C, long long M, int N, int K, int ldw, int group, const int32_t *lens, int B, int T)
{
    __shared__ float As[16][65];
    __shared__ float Ws[16][65];
    __shared__ long long row_of[64];
    __shared__ int scan[GEMM_THREADS], wsum[GEMM_THREADS / 64];
    const int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;
    const int nt_n = (N + 63) / 64;
    const long long m0 = (long long)(blockIdx.x / nt_n) * 64;
    const int n0 = (blockIdx.x % nt_n) * 64;
    if (lens) {
        if (!valid_row_map<64>(lens, B, T, m0, row_of, scan, wsum)) return;   // uniform
    } else if (tid < 64) {
        row_of[tid] = m0 + tid < M ? m0 + tid : -1;
    }
    __syncthreads();
    float acc[4][4] = {};
    for (int k0 = 0; k0 < K; k0 += 16) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int idx = tid + j * 256;
            const int row = idx >> 4, kk = idx & 15;
            const int k = k0 + kk;
            const long long m = row_of[row];
            const int n = n0 + row;
            As[kk][row] = (m >= 0 && k < K) ? A[m * K + k] : 0.0f;
            Ws[kk][row] = (n < N && k < K) ? W[(long long)n * ldw + k] : 0.0f;
        }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < 16; ++kk) {
            float a[4], w[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) a[i] = As[kk][ty * 4 + i];
#pragma unroll
            for (int j = 0; j < 4; ++j) w[j] = Ws[kk][tx * 4 + j];
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], w[j], acc[i][j]);
        }
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const long long m = row_of[ty * 4 + i];
        if (m < 0) continue;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int n = n0 + tx * 4 + j;
            if (n < N) C[m * N + (group > 0 ? (n % group) * (N / group) + n / group : n)] = acc[i][j] + (bias ? bias[n] : 0.0f);
        }
    }
}

}  // namespace

static LinearProblem linear_problem(const void *a, int64_t rows, int K, const void *w, int ldw, int N,
                                    const float *bias, int group, float *out)
{
    LinearProblem q{};
    q.A = static_cast<const uint16_t *>(a);
    q.W = static_cast<const uint16_t *>(w);
    q.bias = bias;
    q.C = out;
    q.M = rows;
    q.N = N;
    q.K = K;
    q.ldw = ldw;
    q.group = group;
    const long long row_tiles = (rows + BM - 1) / BM, rounds = (row_tiles + kXcds - 1) / kXcds;
    q.blocks = (unsigned)(rounds * kXcds * ((N + BN - 1) / BN));
    return q;
}

// Large products with a column count that 256-column tiles divide take the 256 x 256 kernel
// (a launch of its own: it has its own workgroup size and LDS footprint).
static bool takes_big_tiles(int64_t rows, int N, int group)
{
    return group == 0 && N % GN == 0 && rows >= 32768;
}

static hipError_t launch_big_tiles(LinearProblem q, hipStream_t stream)
{
    static std::mutex mu;
    static bool ready[64] = {};
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= 64) return hipErrorInvalidDevice;
    {
        std::lock_guard<std::mutex> lock(mu);
        if (!ready[dev]) {
            e = hipFuncSetAttribute(reinterpret_cast<const void *>(enc_proj_bf16_big_kernel),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, (int)kBigLdsBytes);
            if (e != hipSuccess) return e;
            ready[dev] = true;
        }
    }
    const long long row_tiles = (q.M + GM - 1) / GM, rounds = (row_tiles + kXcds - 1) / kXcds;
    q.blocks = (unsigned)(rounds * kXcds * ((q.N + GN - 1) / GN));
    hipLaunchKernelGGL(enc_proj_bf16_big_kernel, dim3(q.blocks), dim3(BIG_THREADS), kBigLdsBytes, stream, q);
    return hipGetLastError();
}

hipError_t launch_prepare_bf16(const void *enc, const int32_t *enc_len, int B, int T, const tdt_weights_t *w,
                               float *enc_proj, float *emb_gates, float *pred_tab, const PackedLayout &pl,
                               bool on_the_fly, void *packed, void *zero_begin, size_t zero_bytes,
                               long long *out_stats, hipStream_t stream)
{
    LinearBatch batch{};
    int n = 0;
    // (B == 0: no encoder projection in this launch)
    batch.q[n] = linear_problem(enc, (int64_t)B * T, w->d_enc, w->w_enc, w->d_enc, w->h_joint, w->b_enc, 0, enc_proj);
    batch.q[n].lens = enc_len;
    batch.q[n].B = B;
    batch.q[n].T = T;
    if (takes_big_tiles((int64_t)B * T, w->h_joint, 0)) {
        const hipError_t e = launch_big_tiles(batch.q[n], stream);
        if (e != hipSuccess) return e;
        batch.q[n].blocks = 0;   // not part of the launch below
    }
    ++n;
    if (w->pred_kind == TDT_PRED_LSTM) {   // stored [label][unit][gate]
        batch.q[n++] = linear_problem(w->emb, w->vocab + 1, w->emb_dim, w->w_ih[0], w->emb_dim, 4 * w->h_pred,
                                      w->b_lstm[0], w->h_pred, emb_gates);
    } else if (pred_tab) {
        const size_t E = (size_t)w->emb_dim, rows_tab = (size_t)w->vocab + 1;
        for (int c = 0; c < w->pred_layers; ++c)
            batch.q[n++] = linear_problem(static_cast<const uint16_t *>(w->emb) + c * rows_tab * E, (int64_t)rows_tab,
                                          w->emb_dim, static_cast<const uint16_t *>(w->w_pred) + c * E, w->h_pred,
                                          w->h_joint, c == w->pred_layers - 1 ? w->b_pred : nullptr, 0,
                                          pred_tab + c * rows_tab * w->h_joint);
    }
    unsigned blocks = 0;
    for (int i = 0; i < n; ++i) blocks += batch.q[i].blocks;
    const size_t n16 = zero_bytes / 16;
    size_t zb = (n16 + GEMM_THREADS - 1) / GEMM_THREADS;
    if (zb > 256) zb = 256;
    if (zb < 1) zb = 1;
    const PackBatch pack = pack_batch(w, pl, on_the_fly, packed);
    const unsigned pb = pack.pieces > 0 ? pack_blocks_for(pack) : 0;
    hipLaunchKernelGGL(prepare_bf16_kernel, dim3(blocks + pb + (unsigned)zb), dim3(GEMM_THREADS), 0, stream, batch,
                       pack, pb, static_cast<uint4 *>(zero_begin), n16, out_stats);
    return hipGetLastError();
}

hipError_t launch_linear(const void *a, int64_t rows, int K, const void *w, int ldw, int N, const float *bias,
                         int dtype, int group, float *out, hipStream_t stream)
{
    if (rows <= 0) return hipSuccess;
    if (dtype == 1) {
        const LinearProblem q = linear_problem(a, rows, K, w, ldw, N, bias, group, out);
        if (takes_big_tiles(rows, N, group)) return launch_big_tiles(q, stream);
        hipLaunchKernelGGL(enc_proj_bf16_kernel, dim3(q.blocks), dim3(GEMM_THREADS), 0, stream, q);
    } else {
        dim3 grid((unsigned)(((N + 63) / 64) * ((rows + 63) / 64)));
        hipLaunchKernelGGL(enc_proj_f32_kernel, grid, dim3(GEMM_THREADS), 0, stream, static_cast<const float *>(a),
                           static_cast<const float *>(w), bias, out, (long long)rows, N, K, ldw, group,
                           static_cast<const int32_t *>(nullptr), 0, 0);
    }
    return hipGetLastError();
}

hipError_t launch_encoder_projection_valid(const void *enc, const int32_t *enc_len, int B, int T,
                                           const tdt_weights_t *w, float *out, hipStream_t stream)
{
    const int64_t rows = (int64_t)B * T;
    if (rows <= 0) return hipSuccess;
    if (w->dtype == 1) {
        LinearProblem q = linear_problem(enc, rows, w->d_enc, w->w_enc, w->d_enc, w->h_joint, w->b_enc, 0, out);
        q.lens = enc_len;
        q.B = B;
        q.T = T;
        if (takes_big_tiles(rows, w->h_joint, 0)) return launch_big_tiles(q, stream);
        hipLaunchKernelGGL(enc_proj_bf16_kernel, dim3(q.blocks), dim3(GEMM_THREADS), 0, stream, q);
    } else {
        dim3 grid((unsigned)(((w->h_joint + 63) / 64) * ((rows + 63) / 64)));
        hipLaunchKernelGGL(enc_proj_f32_kernel, grid, dim3(GEMM_THREADS), 0, stream, static_cast<const float *>(enc),
                           static_cast<const float *>(w->w_enc), w->b_enc, out, (long long)rows, w->h_joint,
                           w->d_enc, w->d_enc, 0, enc_len, B, T);
    }
    return hipGetLastError();
}

hipError_t launch_encoder_projection(const void *enc, int64_t rows, const tdt_weights_t *w,
                                     float *out, hipStream_t stream)
{
    return launch_linear(enc, rows, w->d_enc, w->w_enc, w->d_enc, w->h_joint, w->b_enc, w->dtype, 0, out, stream);
}

namespace {
PackedMatrix place(size_t &off, int tiles, int K)
{
    PackedMatrix m;
    m.offset = off;
    m.tiles = tiles;
    m.steps = (K + 31) / 32;
    off += (size_t)m.tiles * m.steps * 1024;
    return m;
}
}  // namespace

PackedLayout packed_layout(const tdt_weights_t *w)
{
    PackedLayout pl{};
    size_t off = 0;
    if (w->dtype != 1) return pl;
    const bool lstm = w->pred_kind == TDT_PRED_LSTM;
    pl.w_enc = place(off, (w->h_joint + 15) / 16, w->d_enc);
    pl.w_pred = place(off, (w->h_joint + 15) / 16, w->h_pred);
    pl.w_out = place(off, (w->vocab + 1 + w->n_dur + 15) / 16, w->h_joint);
    for (int l = 0; lstm && l < w->pred_layers; ++l) {
        // the first layer's input product is a per-label table: its matrix is not streamed
        if (l > 0) pl.w_ih[l] = place(off, (w->h_pred + 3) / 4, w->h_pred);
        pl.w_hh[l] = place(off, (w->h_pred + 3) / 4, w->h_pred);
    }
    pl.total = off;
    return pl;
}


// the copies in a launch of their own (calls that reuse the projections of an earlier call)
hipError_t launch_pack_weights(const tdt_weights_t *w, const PackedLayout &pl, bool on_the_fly, void *packed,
                               hipStream_t stream)
{
    const PackBatch b = pack_batch(w, pl, on_the_fly, packed);
    if (b.pieces == 0) return hipSuccess;
    hipLaunchKernelGGL(pack_weights_kernel, dim3(pack_blocks_for(b)), dim3(256), 0, stream, b);
    return hipGetLastError();
}

// stateless predictor, float32 models: the per-label tables of the projected predictor output
hipError_t launch_pred_tables(const tdt_weights_t *w, float *pred_tab, hipStream_t stream)
{
    const size_t E = (size_t)w->emb_dim, rows_tab = (size_t)w->vocab + 1;
    const size_t esz = w->dtype == 1 ? 2 : 4;
    for (int c = 0; c < w->pred_layers; ++c) {
        const hipError_t e = launch_linear(
            static_cast<const char *>(w->emb) + c * rows_tab * E * esz, (int64_t)rows_tab, w->emb_dim,
            static_cast<const char *>(w->w_pred) + c * E * esz, w->h_pred, w->h_joint,
            c == w->pred_layers - 1 ? w->b_pred : nullptr, w->dtype, 0, pred_tab + c * rows_tab * w->h_joint, stream);
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

}  // namespace tdt
