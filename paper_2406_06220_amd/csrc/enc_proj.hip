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

namespace tdt {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

namespace {

constexpr int BM = 128, BN = 128, BK = 64;   // workgroup tile
constexpr int GEMM_THREADS = 256;            // 4 wavefronts, each a 64x64 sub-tile

// 16-byte chunk index c of a row is stored at chunk (c ^ (row & 7)) so that the
// 32 rows a wavefront reads for one k-slice spread over all LDS banks.
__device__ inline int lds_off(int row, int chunk) { return row * BK + ((chunk ^ (row & 7)) << 3); }

// One product C = A * W^T + bias and the workgroups it takes.  Rows of W are ldw apart (a
// slice of the columns of a wider matrix can be multiplied); bias may be null.
struct LinearProblem {
    const uint16_t *A, *W;
    const float *bias;
    float *C;
    long long M;
    int N, K, ldw, group;
    unsigned blocks;
};
constexpr int kMaxProblems = 3;   // products one preparation launch can hold
struct LinearBatch {
    LinearProblem q[kMaxProblems];
};

// the 128 x 128 output tile of workgroup `block` (of q.blocks) of one product
__device__ inline void gemm_tile_bf16(const LinearProblem &q, unsigned block)
{
    const uint16_t *__restrict__ A = q.A;
    const uint16_t *__restrict__ W = q.W;
    const float *__restrict__ bias = q.bias;
    float *__restrict__ C = q.C;
    const long long M = q.M;
    const int N = q.N, K = q.K, ldw = q.ldw, group = q.group;
    __shared__ __align__(16) uint16_t As[BM * BK];
    __shared__ __align__(16) uint16_t Bs[BN * BK];
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

    f32x16 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;

    uint4 ra[4], rb[4];
    auto load_tiles = [&](int k0) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int c = tid + j * GEMM_THREADS;   // 0..1023
            const int row = c >> 3, kc = c & 7;
            const int k = k0 + kc * 8;
            const long long m = m0 + row;
            const int n = n0 + row;
            ra[j] = (m < M && k < K) ? *reinterpret_cast<const uint4 *>(A + m * K + k)
                                     : make_uint4(0, 0, 0, 0);
            rb[j] = (n < N && k < K) ? *reinterpret_cast<const uint4 *>(W + (long long)n * ldw + k)
                                     : make_uint4(0, 0, 0, 0);
        }
    };
    auto store_tiles = [&]() {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int c = tid + j * GEMM_THREADS;
            const int row = c >> 3, kc = c & 7;
            *reinterpret_cast<uint4 *>(As + lds_off(row, kc)) = ra[j];
            *reinterpret_cast<uint4 *>(Bs + lds_off(row, kc)) = rb[j];
        }
    };

    const int nk = (K + BK - 1) / BK;
    load_tiles(0);
    for (int kt = 0; kt < nk; ++kt) {
        store_tiles();
        __syncthreads();
        if (kt + 1 < nk) load_tiles((kt + 1) * BK);
#pragma unroll
        for (int s = 0; s < BK / 16; ++s) {
            const int chunk = s * 2 + (lane >> 5);
            bf16x8 a[2], b[2];
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                const int ar = wm * 64 + i * 32 + (lane & 31);
                const int br = wn * 64 + i * 32 + (lane & 31);
                a[i] = *reinterpret_cast<const bf16x8 *>(As + lds_off(ar, chunk));
                b[i] = *reinterpret_cast<const bf16x8 *>(Bs + lds_off(br, chunk));
            }
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
        }
        __syncthreads();
    }

    // accumulator register e of lane l is row 8*(e/4) + 4*(l/32) + e%4, column l%32
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int n = n0 + wn * 64 + j * 32 + (lane & 31);
            if (n >= N) continue;
            const float bn = bias ? bias[n] : 0.0f;
            const int nc = group > 0 ? (n % group) * (N / group) + n / group : n;
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const long long m = m0 + wm * 64 + i * 32 + (e >> 2) * 8 + (lane >> 5) * 4 + (e & 3);
                if (m < M) C[m * N + nc] = acc[i][j][e] + bn;
            }
        }
}

__global__ __launch_bounds__(GEMM_THREADS) void enc_proj_bf16_kernel(LinearProblem q)
{
    gemm_tile_bf16(q, blockIdx.x);
}

// Everything a decode call needs before its decode kernel, in one launch: the encoder
// projection, the per-label tables of the predictor side (a product with blocks == 0 is
// absent), and the clearing of the workspace's zero region and of the statistics.  The tasks
// are independent; a workgroup takes its task from its index.  Every product's workgroup count
// is a multiple of the number of dies, so each keeps its die-aware order of tiles.
__global__ __launch_bounds__(GEMM_THREADS) void prepare_bf16_kernel(LinearBatch batch, uint4 *zero, size_t n16,
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
    const unsigned zb = b, nzb = gridDim.x - used;
    for (size_t i = (size_t)zb * GEMM_THREADS + threadIdx.x; i < n16; i += (size_t)nzb * GEMM_THREADS)
        zero[i] = make_uint4(0, 0, 0, 0);
    if (out_stats && zb == 0 && threadIdx.x < TDT_STAT_COUNT) out_stats[threadIdx.x] = 0;
}

// float32 models (small): classic 64x64 tile, 4x4 outputs per thread.
__global__ __launch_bounds__(256) void enc_proj_f32_kernel(
    const float *__restrict__ A, const float *__restrict__ W, const float *__restrict__ bias,
    float *__restrict__ C, long long M, int N, int K, int ldw, int group)
{
    __shared__ float As[16][65];
    __shared__ float Ws[16][65];
    const int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;
    const int nt_n = (N + 63) / 64;
    const long long m0 = (long long)(blockIdx.x / nt_n) * 64;
    const int n0 = (blockIdx.x % nt_n) * 64;
    float acc[4][4] = {};
    for (int k0 = 0; k0 < K; k0 += 16) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int idx = tid + j * 256;
            const int row = idx >> 4, kk = idx & 15;
            const int k = k0 + kk;
            const long long m = m0 + row;
            const int n = n0 + row;
            As[kk][row] = (m < M && k < K) ? A[m * K + k] : 0.0f;
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
        const long long m = m0 + ty * 4 + i;
        if (m >= M) continue;
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

hipError_t launch_prepare_bf16(const void *enc, int64_t rows, const tdt_weights_t *w, float *enc_proj,
                               float *emb_gates, float *pred_tab, void *zero_begin, size_t zero_bytes,
                               long long *out_stats, hipStream_t stream)
{
    LinearBatch batch{};
    int n = 0;
    batch.q[n++] = linear_problem(enc, rows, w->d_enc, w->w_enc, w->d_enc, w->h_joint, w->b_enc, 0, enc_proj);
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
    hipLaunchKernelGGL(prepare_bf16_kernel, dim3(blocks + (unsigned)zb), dim3(GEMM_THREADS), 0, stream, batch,
                       static_cast<uint4 *>(zero_begin), n16, out_stats);
    return hipGetLastError();
}

hipError_t launch_linear(const void *a, int64_t rows, int K, const void *w, int ldw, int N, const float *bias,
                         int dtype, int group, float *out, hipStream_t stream)
{
    if (rows <= 0) return hipSuccess;
    if (dtype == 1) {
        const LinearProblem q = linear_problem(a, rows, K, w, ldw, N, bias, group, out);
        hipLaunchKernelGGL(enc_proj_bf16_kernel, dim3(q.blocks), dim3(GEMM_THREADS), 0, stream, q);
    } else {
        dim3 grid((unsigned)(((N + 63) / 64) * ((rows + 63) / 64)));
        hipLaunchKernelGGL(enc_proj_f32_kernel, grid, dim3(256), 0, stream, static_cast<const float *>(a),
                           static_cast<const float *>(w), bias, out, (long long)rows, N, K, ldw, group);
    }
    return hipGetLastError();
}

hipError_t launch_encoder_projection(const void *enc, int64_t rows, const tdt_weights_t *w,
                                     float *out, hipStream_t stream)
{
    return launch_linear(enc, rows, w->d_enc, w->w_enc, w->d_enc, w->h_joint, w->b_enc, w->dtype, 0, out, stream);
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
