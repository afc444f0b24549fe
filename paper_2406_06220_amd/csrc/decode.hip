// Device-resident label-looping greedy decoder (paper Algorithm 3, Sec. 3.2;
// TDT variant Sec. 3.3; batched hypothesis arrays Sec. 3.1).
//
// One persistent kernel runs the whole decode.  Its workgroups are split into
// clusters; a cluster owns a contiguous slice of the batch and runs the label
// loop for it on its own, so clusters never wait for each other.  Inside a
// cluster every workgroup keeps an identical copy of the small per-hypothesis
// control state (frame index, symbols at this frame, last labels, length,
// score) in LDS and updates it with the same deterministic code, so that loop
// control needs no host and no extra exchange; the heavy phases are split over
// the cluster's workgroups and separated by cluster-wide barriers:
//
//   P  predictor step     LSTM layer(s) for the hypotheses that are still active
//                         (Alg. 3 line 6; the state is kept for every row)
//   Q  predictor projection into the joint space (Sec. 3.4)
//   J  joint pass         relu(enc_proj[b, t..t+W) + pred_proj[b]) . w_out, scored
//                         for a window of W upcoming frames of every hypothesis
//                         that still searches for its next non-blank label
//                         (Alg. 3 lines 7-9 and 13-15; the predictor output is
//                         constant during that search, so the frames of the
//                         inner loop can be scored together and the first
//                         non-blank taken -- same result, fewer dependent steps)
//   D  decision           every workgroup reads the per-row argmax cells that the
//                         joint pass filled with atomic maxima, walks the window (Alg. 3 lines 10-11,
//                         16-19; TDT: the step is the predicted duration),
//                         appends the label (line 20) and updates its copy of
//                         the control state.
//
// Exchange between workgroups.  Data one workgroup writes for another (hidden and
// cell state, projected predictor output, per-row argmax cells, softmax partials,
// barrier counters) is written and read only with agent-scope relaxed atomic
// stores / loads / RMWs, which the hardware performs at the device's coherence
// point, bypassing the per-CU L1 and the per-XCD L2.  A producer waits for the
// completion of its stores (s_waitcnt vmcnt(0)) before it arrives at a barrier;
// a consumer issues its loads after it has seen the barrier complete.  No
// cache-wide write-back or invalidate is ever needed, which keeps a barrier at
// about a microsecond.  Weights and enc_proj are written before the kernel
// starts and are read through the caches as usual.
//
// Arithmetic: float32 activations times float32 or bfloat16 weights with
// float32 accumulation on the vector ALUs; a wavefront owns one output column,
// its 64 lanes split the reduction dimension, 16 rows are processed per pass.
#include <math.h>

#include "tdt_internal.h"

namespace tdt {
namespace {

constexpr int RT = 16;   // rows of one staged activation tile

struct HypShared {
    int len[kMaxHypsPerCluster];
    int time[kMaxHypsPerCluster];
    int sym[kMaxHypsPerCluster];
    int last[kMaxHypsPerCluster];
    int last2[kMaxHypsPerCluster];
    int out_len[kMaxHypsPerCluster];
    int status[kMaxHypsPerCluster];
    float score[kMaxHypsPerCluster];
    unsigned char active[kMaxHypsPerCluster];
    unsigned char need[kMaxHypsPerCluster];
    int act_list[kMaxHypsPerCluster];
    int need_list[kMaxHypsPerCluster];
    int n_act, n_need;
    int wave_cnt[kWaves];
    int durations[TDT_MAX_DURATIONS];
    float wstats[kWaves][RT][5];
    int row_a[kMaxRowsPerPass];     // per joint row: argmax label (V = blank)
    int row_d[kMaxRowsPerPass];     //                frame step of the argmax duration class
    float row_m[kMaxRowsPerPass];   //                largest label logit
    int dec_w[kMaxHypsPerCluster];  // per searching hypothesis: window offset the walk stopped at
    unsigned char dec_found[kMaxHypsPerCluster];   // ... on a non-blank label
    unsigned epoch;
    int aborted;
};

template <typename WT> __device__ inline float2 load_w2(const WT *p);
template <> __device__ inline float2 load_w2<float>(const float *p)
{
    return *reinterpret_cast<const float2 *>(p);
}
template <> __device__ inline float2 load_w2<uint16_t>(const uint16_t *p)
{
    const uint32_t u = *reinterpret_cast<const uint32_t *>(p);
    return make_float2(__uint_as_float(u << 16), __uint_as_float(u & 0xffff0000u));
}
template <typename WT> __device__ inline float load_w1(const WT *p);
template <> __device__ inline float load_w1<float>(const float *p) { return *p; }
template <> __device__ inline float load_w1<uint16_t>(const uint16_t *p)
{
    return __uint_as_float(((uint32_t)*p) << 16);
}

// acc[i] += sum over this lane's k of act[i][k] * w[k]   (K even; lanes take pairs)
template <typename WT>
__device__ inline void wave_dot(const float *act, int ld, int K, const WT *__restrict__ w,
                                float (&acc)[RT], int lane)
{
    for (int k = lane * 2; k < K; k += 128) {
        const float2 wv = load_w2<WT>(w + k);
#pragma unroll
        for (int i = 0; i < RT; ++i) {
            const float2 a = *reinterpret_cast<const float2 *>(act + i * ld + k);
            acc[i] = fmaf(a.x, wv.x, acc[i]);
            acc[i] = fmaf(a.y, wv.y, acc[i]);
        }
    }
}

// after this every lane holds the wavefront-wide sums; returns the one of row `lane`
__device__ inline float wave_reduce_select(float (&acc)[RT], int lane)
{
    float mine = 0.0f;
#pragma unroll
    for (int i = 0; i < RT; ++i) {
        float v = acc[i];
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
        if (lane == i) mine = v;
    }
    return mine;
}

__device__ inline float sigmoidf_dev(float x) { return 1.0f / (1.0f + expf(-x)); }

// ---- coherent exchange primitives (see the header comment)
#define TDT_AGENT __HIP_MEMORY_SCOPE_AGENT
__device__ inline float ld_co(const float *p) { return __hip_atomic_load(p, __ATOMIC_RELAXED, TDT_AGENT); }
__device__ inline void st_co(float *p, float v) { __hip_atomic_store(p, v, __ATOMIC_RELAXED, TDT_AGENT); }
__device__ inline float2 ld_co2(const float *p)   // p 8-byte aligned
{
    const unsigned long long u =
        __hip_atomic_load(reinterpret_cast<const unsigned long long *>(p), __ATOMIC_RELAXED, TDT_AGENT);
    return make_float2(__uint_as_float((unsigned)u), __uint_as_float((unsigned)(u >> 32)));
}
__device__ inline unsigned long long ld_co64(const unsigned long long *p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, TDT_AGENT);
}
__device__ inline void st_co64(unsigned long long *p, unsigned long long v)
{
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, TDT_AGENT);
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

// Barrier over the C workgroups of one cluster.  Counters only grow: the n-th
// barrier waits for n * (arrivals per barrier).  Clusters of more than
// kBarrierGroup workgroups arrive on one of 8 first-level counters (by rank
// modulo 8, i.e. by XCD when the cluster spans the chip); the last arrival of a
// group arrives on the root counter, on which everybody waits.  Every wait is
// bounded: on a timeout, or when another workgroup has flagged an abort, the
// barrier returns false and the caller leaves the kernel.
struct BarrierInfo {
    unsigned *root;    // root counter of this cluster
    unsigned *group;   // first-level counter of this workgroup's group (null if flat)
    unsigned group_size, root_arrivals;
};

__device__ inline bool cluster_barrier(HypShared &S, const BarrierInfo &bi, int *abort_flag, int C,
                                       long long timeout_ticks)
{
    // every coherent store / atomic of this wavefront has completed ...
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();   // ... and so have those of the whole workgroup
    if (threadIdx.x == 0) {
        int ab = 0;
        if (C > 1) {
            S.epoch += 1;
            if (bi.group) {
                const unsigned old = __hip_atomic_fetch_add(bi.group, 1u, __ATOMIC_RELAXED, TDT_AGENT);
                if (old + 1u == S.epoch * bi.group_size)
                    __hip_atomic_fetch_add(bi.root, 1u, __ATOMIC_RELAXED, TDT_AGENT);
            } else {
                __hip_atomic_fetch_add(bi.root, 1u, __ATOMIC_RELAXED, TDT_AGENT);
            }
            const unsigned target = S.epoch * bi.root_arrivals;
            const long long t0 = wall_clock64();
            unsigned spins = 0;
            while (__hip_atomic_load(bi.root, __ATOMIC_RELAXED, TDT_AGENT) < target) {
                if ((++spins & 63u) == 0u) {
                    if (__hip_atomic_load(abort_flag, __ATOMIC_RELAXED, TDT_AGENT)) { ab = 1; break; }
                    if (wall_clock64() - t0 > timeout_ticks) {
                        __hip_atomic_store(abort_flag, 1, __ATOMIC_RELAXED, TDT_AGENT);
                        ab = 1;
                        break;
                    }
                }
            }
        }
        S.aborted = ab;
    }
    __syncthreads();
    return S.aborted == 0;
}

// list[0..n) = indices g < G with flag[g] set, ascending.  All threads call it.
__device__ inline void build_list(HypShared &S, const unsigned char *flag, int G, int *list,
                                  int *n_out)
{
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
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

// split `n_cols` columns over the workgroups left after `n_tiles` row tiles took theirs
__device__ inline void split_columns(int C, int n_tiles, int n_cols, int max_groups, int &n_groups,
                                     int &per_group)
{
    int g = C / (n_tiles > 0 ? n_tiles : 1);
    if (g < 1) g = 1;
    if (g > max_groups) g = max_groups;
    if (g > n_cols) g = n_cols;
    per_group = (n_cols + g - 1) / g;
    n_groups = (n_cols + per_group - 1) / per_group;
}

template <typename WT>
__global__ __launch_bounds__(kThreads, 1) void decode_kernel(DecodeParams p)
{
    extern __shared__ __align__(16) float act[];
    __shared__ HypShared S;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int ncl = p.n_clusters;
    const int cl = blockIdx.x % ncl, rank = blockIdx.x / ncl, C = gridDim.x / ncl;
    const int b0 = cl * p.hyps_per_cluster;
    int G = p.B - b0;
    if (G > p.hyps_per_cluster) G = p.hyps_per_cluster;
    if (G <= 0) return;   // the whole cluster leaves together

    const int B = p.B, T = p.T, H = p.H, V = p.V, D = p.D, O = p.O;
    const int Hp = p.h_pred, E = p.emb_dim, L = p.pred_layers;
    const bool lstm = p.pred_kind == TDT_PRED_LSTM;

    BarrierInfo bi;
    bi.root = p.barrier + (size_t)cl * kBarrierStride;
    if (C > kBarrierGroup) {
        const int n_groups = 8, grp = rank % n_groups;
        bi.group = p.barrier + ((size_t)kMaxGrid + cl + (size_t)ncl * grp) * kBarrierStride;
        bi.group_size = (unsigned)((C - grp + n_groups - 1) / n_groups);
        bi.root_arrivals = (unsigned)n_groups;
    } else {
        bi.group = nullptr;
        bi.group_size = 0;
        bi.root_arrivals = (unsigned)C;
    }
    LsePartial *const pbase = p.partials + (size_t)cl * (kPartialEntries / ncl);
    const int rows_cap = p.rows_per_cluster;
    unsigned long long *const rl_base = p.row_lab + (size_t)cl * kRowBufs * rows_cap;
    unsigned long long *const rd_base = p.row_dur + (size_t)cl * kRowBufs * rows_cap;
    const int max_cg = min(kMaxColGroups, kPartialEntries / ncl / kMaxRowsPerPass);

    // ---- Alg. 3 lines 3-4: empty hypotheses, time 0, everyone with frames is active
    for (int g = tid; g < G; g += kThreads) {
        int len = p.enc_len[b0 + g];
        int st = 0;
        if (len < 0) { len = 0; st = TDT_HYP_LEN_CLAMPED; }
        if (len > T) { len = T; st = TDT_HYP_LEN_CLAMPED; }
        S.len[g] = len;
        S.time[g] = 0;
        S.sym[g] = 0;
        S.last[g] = V;    // start-of-sequence label
        S.last2[g] = V;
        S.out_len[g] = 0;
        S.status[g] = st;
        S.score[g] = 0.0f;
        S.active[g] = len > 0;
        S.need[g] = 0;
    }
    if (tid < TDT_MAX_DURATIONS) S.durations[tid] = p.durations[tid];
    if (tid == 0) { S.epoch = 0; S.aborted = 0; }
    __syncthreads();

    long long st_pred_pass = 0, st_pred_rows = 0, st_joint_pass = 0, st_joint_rows = 0, st_outer = 0;
    int pp = 0;          // which half of hbuf holds the current hidden state
    unsigned jpass = 0;  // joint passes so far (selects the exchange buffers)
    bool ok = true;

    while (ok) {   // ---- Alg. 3 line 5: while any hypothesis is active
        build_list(S, S.active, G, S.act_list, &S.n_act);
        const int n_act = S.n_act;
        if (n_act == 0) break;
        ++st_outer;
        ++st_pred_pass;
        st_pred_rows += n_act;
        const int n_tiles_a = (n_act + RT - 1) / RT;

        // ---- P: predictor step (Alg. 3 line 6)
        if (lstm) {
            for (int l = 0; l < L && ok; ++l) {
                const int in_dim = l == 0 ? E : Hp, ld = in_dim + Hp;
                const WT *w_ih = static_cast<const WT *>(p.w_ih[l]);
                const WT *w_hh = static_cast<const WT *>(p.w_hh[l]);
                const float *bl = p.b_lstm[l];
                const float *h_cur = p.hbuf + ((size_t)pp * L + l) * B * Hp;
                float *h_next = p.hbuf + ((size_t)(pp ^ 1) * L + l) * B * Hp;
                const float *x_prev = l > 0 ? p.hbuf + ((size_t)(pp ^ 1) * L + (l - 1)) * B * Hp : nullptr;
                float *cst = p.cbuf + (size_t)l * B * Hp;
                int n_ug, upg;
                split_columns(C, n_tiles_a, Hp, Hp, n_ug, upg);
                for (int it = rank; it < n_tiles_a * n_ug; it += C) {
                    const int ti = it / n_ug, ug = it % n_ug;
                    const int nrows = min(RT, n_act - ti * RT);
                    for (int i = wave; i < RT; i += kWaves) {
                        float *row = act + i * ld;
                        if (i < nrows) {
                            const int g = S.act_list[ti * RT + i];
                            const size_t hb = (size_t)(b0 + g) * Hp;
                            if (l == 0) {
                                const WT *e = static_cast<const WT *>(p.emb) + (size_t)S.last[g] * E;
                                for (int k = lane; k < E; k += 64) row[k] = load_w1<WT>(e + k);
                            } else {
                                for (int k = lane * 2; k < Hp; k += 128)
                                    *reinterpret_cast<float2 *>(row + k) = ld_co2(x_prev + hb + k);
                            }
                            for (int k = lane * 2; k < Hp; k += 128)
                                *reinterpret_cast<float2 *>(row + in_dim + k) = ld_co2(h_cur + hb + k);
                        } else {
                            for (int k = lane; k < ld; k += 64) row[k] = 0.0f;
                        }
                    }
                    __syncthreads();
                    const int u_end = min(Hp, (ug + 1) * upg);
                    for (int u = ug * upg + wave; u < u_end; u += kWaves) {
                        float gate[4];
#pragma unroll
                        for (int q = 0; q < 4; ++q) {
                            float acc[RT];
#pragma unroll
                            for (int i = 0; i < RT; ++i) acc[i] = 0.0f;
                            const size_t r = (size_t)q * Hp + u;
                            wave_dot<WT>(act, ld, in_dim, w_ih + r * in_dim, acc, lane);
                            wave_dot<WT>(act + in_dim, ld, Hp, w_hh + r * Hp, acc, lane);
                            gate[q] = wave_reduce_select(acc, lane) + bl[r];
                        }
                        if (lane < nrows) {
                            const int g = S.act_list[ti * RT + lane];
                            const size_t o = (size_t)(b0 + g) * Hp + u;
                            const float ig = sigmoidf_dev(gate[0]), fg = sigmoidf_dev(gate[1]);
                            const float gg = tanhf(gate[2]), og = sigmoidf_dev(gate[3]);
                            const float cn = fg * ld_co(cst + o) + ig * gg;
                            st_co(cst + o, cn);
                            st_co(h_next + o, og * tanhf(cn));
                        }
                    }
                    __syncthreads();
                }
                ok = cluster_barrier(S, bi, p.abort_flag, C, p.timeout_ticks);
            }
            if (!ok) break;
        }

        // ---- Q: predictor output into the joint space (Sec. 3.4)
        {
            const WT *w_pred = static_cast<const WT *>(p.w_pred);
            const float *dec_src = lstm ? p.hbuf + ((size_t)(pp ^ 1) * L + (L - 1)) * B * Hp : nullptr;
            int n_cg, cpg;
            split_columns(C, n_tiles_a, H, H, n_cg, cpg);
            for (int it = rank; it < n_tiles_a * n_cg; it += C) {
                const int ti = it / n_cg, cg = it % n_cg;
                const int nrows = min(RT, n_act - ti * RT);
                for (int i = wave; i < RT; i += kWaves) {
                    float *row = act + i * Hp;
                    if (i < nrows) {
                        const int g = S.act_list[ti * RT + i];
                        if (lstm) {
                            const size_t hb = (size_t)(b0 + g) * Hp;
                            for (int k = lane * 2; k < Hp; k += 128)
                                *reinterpret_cast<float2 *>(row + k) = ld_co2(dec_src + hb + k);
                        } else {
                            // table L-1 embeds the newest label, table 0 the older one
                            const WT *emb = static_cast<const WT *>(p.emb);
                            for (int c = 0; c < L; ++c) {
                                const int tok = (c == L - 1) ? S.last[g] : S.last2[g];
                                const WT *e = emb + ((size_t)c * (V + 1) + tok) * E;
                                for (int k = lane; k < E; k += 64) row[c * E + k] = load_w1<WT>(e + k);
                            }
                        }
                    } else {
                        for (int k = lane; k < Hp; k += 64) row[k] = 0.0f;
                    }
                }
                __syncthreads();
                const int c_end = min(H, (cg + 1) * cpg);
                for (int n = cg * cpg + wave; n < c_end; n += kWaves) {
                    float acc[RT];
#pragma unroll
                    for (int i = 0; i < RT; ++i) acc[i] = 0.0f;
                    wave_dot<WT>(act, Hp, Hp, w_pred + (size_t)n * Hp, acc, lane);
                    const float v = wave_reduce_select(acc, lane) + p.b_pred[n];
                    if (lane < nrows)
                        st_co(p.pred_proj + (size_t)(b0 + S.act_list[ti * RT + lane]) * H + n, v);
                }
                __syncthreads();
            }
            ok = cluster_barrier(S, bi, p.abort_flag, C, p.timeout_ticks);
            if (!ok) break;
        }

        // every active hypothesis now searches for its next non-blank label
        for (int g = tid; g < G; g += kThreads) S.need[g] = S.active[g];
        __syncthreads();
        build_list(S, S.need, G, S.need_list, &S.n_need);

        // ---- inner loop (Alg. 3 line 12): joint passes until nobody searches any more
        while (S.n_need > 0) {
            const int n_need = S.n_need;
            int Kw = p.window > 0 ? p.window : 256 / n_need;
            if (Kw < 4 && p.window <= 0) Kw = 4;
            if (Kw > kMaxWindow) Kw = kMaxWindow;
            if (Kw * n_need > rows_cap) Kw = rows_cap / n_need;
            const int M = n_need * Kw;
            const int n_tiles = (M + RT - 1) / RT;
            int n_cg, cpg;
            split_columns(C, n_tiles, O, max_cg, n_cg, cpg);
            LsePartial *pbuf = pbase + (size_t)(jpass & 1u) * kPartialEntries;
            unsigned long long *row_lab = rl_base + (size_t)(jpass % kRowBufs) * rows_cap;
            unsigned long long *row_dur = rd_base + (size_t)(jpass % kRowBufs) * rows_cap;
            {   // clear the argmax cells of the next pass; their last readers finished before
                // the barrier that precedes this pass
                unsigned long long *nl = rl_base + (size_t)((jpass + 1) % kRowBufs) * rows_cap;
                unsigned long long *nd = rd_base + (size_t)((jpass + 1) % kRowBufs) * rows_cap;
                for (int r = rank * kThreads + tid; r < rows_cap; r += C * kThreads) {
                    st_co64(nl + r, 0ull);
                    if (D > 0) st_co64(nd + r, 0ull);
                }
            }
            ++jpass;
            ++st_joint_pass;
            st_joint_rows += M;

            // ---- J: joint network on M rows
            const WT *w_out = static_cast<const WT *>(p.w_out);
            for (int it = rank; it < n_tiles * n_cg; it += C) {
                const int ti = it / n_cg, cg = it % n_cg;
                for (int i = wave; i < RT; i += kWaves) {
                    float *row = act + i * H;
                    const int r = ti * RT + i;
                    bool valid = r < M;
                    int g = 0, f = 0;
                    if (valid) {
                        g = S.need_list[r / Kw];
                        f = S.time[g] + r % Kw;
                        valid = f < S.len[g];
                    }
                    if (valid) {
                        const float *ep = p.enc_proj + ((size_t)(b0 + g) * T + f) * H;
                        const float *pj = p.pred_proj + (size_t)(b0 + g) * H;
                        for (int k = lane * 2; k < H; k += 128) {
                            const float2 e2 = *reinterpret_cast<const float2 *>(ep + k);
                            const float2 p2 = ld_co2(pj + k);
                            *reinterpret_cast<float2 *>(row + k) =
                                make_float2(fmaxf(e2.x + p2.x, 0.0f), fmaxf(e2.y + p2.y, 0.0f));
                        }
                    } else {
                        for (int k = lane; k < H; k += 64) row[k] = 0.0f;
                    }
                }
                __syncthreads();
                // running statistics of row `lane` over this wavefront's columns
                float mlab = -INFINITY, slab = 0.0f, mdur = -INFINITY;
                int alab = 0, adur = 0;
                const int c_end = min(O, (cg + 1) * cpg);
                for (int n = cg * cpg + wave; n < c_end; n += kWaves) {
                    float acc[RT];
#pragma unroll
                    for (int i = 0; i < RT; ++i) acc[i] = 0.0f;
                    wave_dot<WT>(act, H, H, w_out + (size_t)n * H, acc, lane);
                    const float logit = wave_reduce_select(acc, lane) + p.b_out[n];
                    if (n <= V) {
                        if (logit > mlab) {
                            slab = slab * expf(mlab - logit) + 1.0f;
                            mlab = logit;
                            alab = n;
                        } else {
                            slab += expf(logit - mlab);
                        }
                    } else if (logit > mdur) {
                        mdur = logit;
                        adur = n - (V + 1);
                    }
                }
                if (lane < RT) {
                    float *ws = S.wstats[wave][lane];
                    ws[0] = mlab;
                    ws[1] = __int_as_float(alab);
                    ws[2] = slab;
                    ws[3] = mdur;
                    ws[4] = __int_as_float(adur);
                }
                __syncthreads();
                if (wave == 0 && lane < RT && ti * RT + lane < M) {
                    float m = -INFINITY, s = 0.0f, dm = -INFINITY;
                    int a = 0, da = 0;
#pragma unroll
                    for (int w = 0; w < kWaves; ++w) {
                        const float *ws = S.wstats[w][lane];
                        const float wm = ws[0], wsum = ws[2], wd = ws[3];
                        const int wa = __float_as_int(ws[1]), wda = __float_as_int(ws[4]);
                        if (wsum > 0.0f) {   // the wavefront saw at least one label column
                            if (wm > m || (wm == m && wa < a)) {
                                s = (s > 0.0f ? s * expf(m - wm) : 0.0f) + wsum;
                                m = wm;
                                a = wa;
                            } else {
                                s += wsum * expf(wm - m);
                            }
                        }
                        if (wd > dm || (wd == dm && wd > -INFINITY && wda < da)) {
                            dm = wd;
                            da = wda;
                        }
                    }
                    const int r = ti * RT + lane;
                    if (s > 0.0f)
                        __hip_atomic_fetch_max(row_lab + r, pack_best(m, a), __ATOMIC_RELAXED, TDT_AGENT);
                    if (dm > -INFINITY)
                        __hip_atomic_fetch_max(row_dur + r, pack_best(dm, da), __ATOMIC_RELAXED, TDT_AGENT);
                    const unsigned long long lp = (unsigned long long)__float_as_uint(m) |
                                                  ((unsigned long long)__float_as_uint(s) << 32);
                    st_co64(reinterpret_cast<unsigned long long *>(pbuf + (size_t)r * n_cg + cg), lp);
                }
                __syncthreads();
            }
            ok = cluster_barrier(S, bi, p.abort_flag, C, p.timeout_ticks);
            if (!ok) break;

            // ---- D: every workgroup takes the same decisions from the same cells
            // D1: one coherent load per row, all rows in flight together
            for (int r = tid; r < M; r += kThreads) {
                const unsigned long long best = ld_co64(row_lab + r);
                unsigned long long bd = 0ull;
                if (D > 0) bd = ld_co64(row_dur + r);
                S.row_a[r] = best ? unpack_index(best) : V;
                S.row_m[r] = unpack_value(best);
                S.row_d[r] = D > 0 ? S.durations[unpack_index(bd) & (TDT_MAX_DURATIONS - 1)] : 0;
            }
            __syncthreads();
            // D2: walk each searching hypothesis through its window
            for (int q = wave; q < n_need; q += kWaves) {
                const int g = S.need_list[q];
                const int nv = min(Kw, S.len[g] - S.time[g]);   // >= 1: a searching row has frames left
                int a = V, dstep = 0;
                if (lane < nv) {
                    a = S.row_a[q * Kw + lane];
                    dstep = S.row_d[q * Kw + lane];
                }
                int w = 0;
                bool found = false;
                if (D == 0) {   // Alg. 3 lines 10 / 18: a blank moves one frame on
                    const unsigned long long nb = __ballot(lane < nv && a != V);
                    if (nb) { found = true; w = __ffsll((long long)nb) - 1; } else { w = nv; }
                } else {        // Sec. 3.3: the step comes from the duration head
                    while (w < nv) {
                        if (__shfl(a, w, 64) != V) { found = true; break; }
                        const int dd = __shfl(dstep, w, 64);
                        w += dd > 0 ? dd : 1;
                    }
                }
                if (lane == 0) {
                    S.dec_w[q] = w;
                    S.dec_found[q] = found;
                }
            }
            __syncthreads();
            // D3: softmax denominator of each chosen row, then the state update (Alg. 3 line 20,
            // Sec. 3.1 add_results); a segment of seg lanes serves one hypothesis
            {
                int seg = 1;
                while (seg < n_cg) seg <<= 1;   // <= kMaxColGroups = 64
                const int per_round = kThreads / seg;
                for (int base = 0; base < n_need; base += per_round) {
                    const int q = base + tid / seg, cg = tid % seg;
                    const bool live = q < n_need;
                    const bool found = live && S.dec_found[q];
                    const int w = live ? S.dec_w[q] : 0;
                    float part = 0.0f;
                    if (found && cg < n_cg) {
                        const unsigned long long u = ld_co64(
                            reinterpret_cast<const unsigned long long *>(pbuf + (size_t)(q * Kw + w) * n_cg + cg));
                        const float pm = __uint_as_float((unsigned)u), ps = __uint_as_float((unsigned)(u >> 32));
                        if (ps > 0.0f) part = ps * expf(pm - S.row_m[q * Kw + w]);
                    }
                    for (int off = seg >> 1; off > 0; off >>= 1) part += __shfl_xor(part, off, 64);
                    if (live && cg == 0) {
                        const int g = S.need_list[q];
                        const int t0 = S.time[g], len = S.len[g];
                        int sym = (w > 0 || !found) ? 0 : S.sym[g];
                        if (found) {
                            const int k = S.row_a[q * Kw + w];
                            int dk = S.row_d[q * Kw + w];
                            const int frame = t0 + w, n = S.out_len[g];
                            if (rank == 0) {
                                p.out_labels[(size_t)(b0 + g) * p.u_cap + n] = k;
                                p.out_frames[(size_t)(b0 + g) * p.u_cap + n] = frame;
                            }
                            S.score[g] -= logf(part);   // log_softmax at the maximum = -log(sum exp(l - max))
                            S.out_len[g] = n + 1;
                            S.last2[g] = S.last[g];
                            S.last[g] = k;
                            sym += 1;
                            if (dk == 0 && sym >= p.max_symbols) dk = 1;
                            int t1 = frame;
                            if (dk > 0) { t1 = frame + dk; sym = 0; }
                            S.time[g] = t1;
                            bool act_now = t1 < len;
                            if (n + 1 >= p.u_cap) { act_now = false; S.status[g] |= TDT_HYP_TRUNCATED; }
                            S.active[g] = act_now;
                            S.need[g] = 0;
                        } else {
                            const int t1 = t0 + w;
                            S.time[g] = t1;
                            S.active[g] = t1 < len;
                            S.need[g] = t1 < len;
                        }
                        S.sym[g] = sym;
                    }
                }
            }
            __syncthreads();
            build_list(S, S.need, G, S.need_list, &S.n_need);
        }
        if (!ok) break;
        pp ^= 1;
    }

    // ---- results of this cluster's hypotheses
    if (rank == 0) {
        for (int g = tid; g < G; g += kThreads) {
            p.out_len[b0 + g] = S.out_len[g];
            p.out_score[b0 + g] = S.score[g];
            p.out_status[b0 + g] = S.status[g];
        }
        if (tid == 0 && p.out_stats) {
            atomicAdd((unsigned long long *)&p.out_stats[TDT_STAT_PRED_PASSES], (unsigned long long)st_pred_pass);
            atomicAdd((unsigned long long *)&p.out_stats[TDT_STAT_PRED_ROWS], (unsigned long long)st_pred_rows);
            atomicAdd((unsigned long long *)&p.out_stats[TDT_STAT_JOINT_PASSES], (unsigned long long)st_joint_pass);
            atomicAdd((unsigned long long *)&p.out_stats[TDT_STAT_JOINT_ROWS], (unsigned long long)st_joint_rows);
            atomicMax((unsigned long long *)&p.out_stats[TDT_STAT_OUTER_MAX], (unsigned long long)st_outer);
            if (!ok) atomicAdd((unsigned long long *)&p.out_stats[TDT_STAT_ABORT], 1ull);
        }
    }
}

__global__ void init_kernel(uint4 *zero, size_t n16, long long *out_stats)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += stride)
        zero[i] = make_uint4(0, 0, 0, 0);
    if (out_stats && blockIdx.x == 0 && threadIdx.x < TDT_STAT_COUNT) out_stats[threadIdx.x] = 0;
}

size_t lds_bytes_for(const tdt_weights_t *w)
{
    int kmax = w->h_joint;
    if (w->h_pred > kmax) kmax = w->h_pred;
    if (w->pred_kind == TDT_PRED_LSTM) {
        if (w->emb_dim + w->h_pred > kmax) kmax = w->emb_dim + w->h_pred;
        if (w->pred_layers > 1 && 2 * w->h_pred > kmax) kmax = 2 * w->h_pred;
    }
    return (size_t)RT * kmax * sizeof(float);
}

}  // namespace

hipError_t launch_init(void *zero_begin, size_t zero_bytes, long long *out_stats, hipStream_t stream)
{
    const size_t n16 = zero_bytes / 16;
    int blocks = (int)((n16 + 255) / 256);
    if (blocks > 1024) blocks = 1024;
    if (blocks < 1) blocks = 1;
    hipLaunchKernelGGL(init_kernel, dim3(blocks), dim3(256), 0, stream,
                       static_cast<uint4 *>(zero_begin), n16, out_stats);
    return hipGetLastError();
}

int decode_max_grid(int dtype, size_t *lds_bytes_out, const tdt_weights_t *w)
{
    const size_t lds = lds_bytes_for(w);
    if (lds_bytes_out) *lds_bytes_out = lds;
    const void *fn = dtype == 1 ? (const void *)decode_kernel<uint16_t> : (const void *)decode_kernel<float>;
    if (hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess) {
        (void)hipGetLastError();
        return 0;
    }
    int dev = 0, n_cu = 0, per_cu = 0;
    if (hipGetDevice(&dev) != hipSuccess) return 0;
    if (hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return 0;
    hipError_t e = dtype == 1
        ? hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, decode_kernel<uint16_t>, kThreads, lds)
        : hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, decode_kernel<float>, kThreads, lds);
    if (e != hipSuccess || per_cu < 1) {
        (void)hipGetLastError();
        return 0;
    }
    int grid = n_cu;   // one workgroup per compute unit
    if (grid > kMaxGrid) grid = kMaxGrid;
    return grid;
}

hipError_t launch_decode(const DecodeParams &p, int dtype, int grid, hipStream_t stream)
{
    tdt_weights_t w{};
    w.h_joint = p.H;
    w.h_pred = p.h_pred;
    w.emb_dim = p.emb_dim;
    w.pred_kind = p.pred_kind;
    w.pred_layers = p.pred_layers;
    const size_t lds = lds_bytes_for(&w);
    DecodeParams pc = p;
    void *args[] = {&pc};
    const void *fn = dtype == 1 ? (const void *)decode_kernel<uint16_t> : (const void *)decode_kernel<float>;
    // cooperative launch: the runtime refuses a grid whose workgroups cannot all be
    // resident at once, which is what the cluster barriers rely on
    return hipLaunchCooperativeKernel(fn, dim3(grid), dim3(kThreads), args, (unsigned)lds, stream);
}

}  // namespace tdt
