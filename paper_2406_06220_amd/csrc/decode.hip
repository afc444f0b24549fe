// Device-resident label-looping greedy decoder (paper Algorithm 3, Sec. 3.2;
// TDT variant Sec. 3.3; batched hypothesis arrays Sec. 3.1).
//
// One persistent kernel runs the whole decode.  Its workgroups are split into
// clusters; a cluster owns a share of the batch (dealt by length) and runs the
// label loop for it on its own, so clusters never wait for each other.  Inside a
// cluster every workgroup keeps an identical copy of the small per-hypothesis
// control state (frame index, symbols at this frame, last labels, length,
// score) in LDS and updates it with the same deterministic code, so that loop
// control needs no host and no extra exchange; the heavy phases are split over
// the cluster's workgroups and separated by cluster-wide barriers:
//
//   P  predictor step     LSTM layer(s) for the hypotheses that are still active
//                         (Alg. 3 line 6; the state is kept for every row).  The
//                         first layer is only a cell update here: its input
//                         product is a per-label table row, its recurrent product
//                         was formed in phase Q of the previous label.
//   Q  products with the new predictor state: the projection into the joint
//                         space (Sec. 3.4) and W_hh . h of the first LSTM layer
//                         for the next label, which does not depend on that label
//   J  joint pass         relu(enc_proj[b, t..t+W) + pred_proj[b]) . w_out, scored
//                         for a window of W upcoming frames of every hypothesis
//                         that still searches for its next non-blank label
//                         (Alg. 3 lines 7-9 and 13-15; the predictor output is
//                         constant during that search, so the frames of the
//                         inner loop can be scored together and the first
//                         non-blank taken -- same result, fewer dependent steps)
//   D  decision           every workgroup reads the per-row argmax cells that the
//                         joint pass filled with atomic maxima, walks the window
//                         (Alg. 3 lines 10-11, 16-19; TDT: the step is the
//                         predicted duration), appends the label (line 20) and
//                         updates its copy of the control state.
//
// Each heavy phase is a small-M GEMM: 16 activation rows (a "row tile") against
// a slice of weight columns, cut into 16-column tiles.  A work item is (row
// tile, group of column tiles); items are dealt round-robin to the cluster's
// workgroups.  Activations are float32; bfloat16 weights run on the matrix
// cores (v_mfma_f32_16x16x32_bf16) with every activation split exactly into
// three bfloat16 terms (hi + lo + lo2 == x), so products are exact and only the
// float32 summation order differs from a scalar reference.  float32 weights
// (small models) run on the float32 matrix-core product (v_mfma_f32_16x16x4_f32).
//
// Exchange between workgroups.  Data one workgroup writes for another (hidden and
// cell state, projected predictor output, per-row argmax cells, softmax partials,
// barrier flags) is written and read only with agent-scope relaxed atomic
// stores / loads / RMWs, which the hardware performs at the device's coherence
// point, bypassing the per-CU L1 and the per-XCD L2.  A producer waits for the
// completion of its stores (s_waitcnt vmcnt(0)) before it arrives at a barrier;
// a consumer issues its loads after it has seen the barrier complete.  No
// cache-wide write-back or invalidate is ever needed, which keeps a barrier at
// about a microsecond.  Weights and enc_proj are written before the kernel
// starts and are read through the caches as usual.
#include <math.h>

#include <mutex>

#include "tdt_internal.h"
#include "decode_state.h"
#include "exchange.h"
#include "tile_gemm.h"

#if TDT_TRACE
// profiling builds only: copies the recorded time line (see TR in decode_state.h) to the host
extern "C" int tdt_debug_trace(long long *out, int n)
{
    return (int)hipMemcpyFromSymbol(out, HIP_SYMBOL(g_trace), (size_t)n * sizeof(long long));
}
#endif

#ifndef TDT_TIMER_GROUP
#define TDT_TIMER_GROUP 0   // the hypothesis group whose phase timers a build with TDT_PHASE_TIMERS reports
#endif

namespace tdt {
namespace {

// CHUNKED: the call decodes the next chunk of longer utterances (tdt_greedy_decode_chunk);
// compiled apart so that whole-utterance decoding carries none of its bookkeeping.
// FRAMELOOP: the conventional order of the loops the paper compares against (Algorithm 2,
// batched frame-looping), on the same phases: every step runs the predictor for every active
// hypothesis, scores one frame each, and keeps the new predictor state only where the step
// emitted a label.  Same hypotheses; there to measure what the re-ordering is worth.
// ONTHEFLY: no projections ahead of the loops (the arrangement Sec. 3.4 compares against): every
// joint pass first projects the encoder frames and the predictor outputs of its own rows.
// WIDEJ: the joint pass streams the output matrix (for output layers of many thousands of columns,
// where a work item holds a hundred column tiles and the pass is bound by how fast a compute unit
// can pull its share of the matrix): every wavefront walks column tiles of its own, with many
// weight fragments in flight and no workgroup barrier between tiles, and keeps running argmax /
// softmax statistics per lane that are reduced once per work item (wide_item in tile_gemm.h).
template <typename WT, bool CHUNKED, bool FRAMELOOP, bool ONTHEFLY, bool WIDEJ = false>
__global__ __launch_bounds__(kThreads, 1) void decode_kernel(DecodeParams p)
{
    extern __shared__ __align__(16) unsigned char dyn_lds[];
    __shared__ HypShared S;

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int ncl = p.n_clusters;
    const int C = gridDim.x / ncl;
    // Workgroups go to the chip's kXcds dies round-robin by blockIdx, and each die has its own
    // L2.  A workgroup's rank decides which weight columns it multiplies, so a die should host
    // the SAME ranks of every cluster: then its L2 holds an eighth of the matrices whatever the
    // number of clusters (with one cluster per die each L2 would have to hold all of them, which
    // it cannot, and every pass would fetch them again).  A die has gridDim / 8 slots; `per`
    // ranks of every cluster are aligned that way (ranks die * per .. die * per + per - 1), the
    // few ranks left over when the cluster size is no multiple of 8 take the remaining slots,
    // and a slot beyond those stays empty (the grid is rounded up to a multiple of 8).
    int cl, rank;
    if (gridDim.x % kXcds == 0) {
        const int die = blockIdx.x % kXcds, j = blockIdx.x / kXcds;
        const int per = (int)(gridDim.x / kXcds) / ncl;
        if (j < per * ncl) {
            cl = j % ncl;
            rank = die * per + j / ncl;
        } else {
            const int e = (j - per * ncl) * kXcds + die;
            if (e >= ncl * (C - kXcds * per)) return;   // an empty slot: not part of any cluster
            cl = e % ncl;
            rank = kXcds * per + e / ncl;
        }
    } else {
        cl = blockIdx.x % ncl;
        rank = blockIdx.x / ncl;
    }
    const int B = p.B, T = p.T, H = p.H, V = p.V, D = p.D, O = p.O;
    // the label head: outputs 0 .. VL (a multi-blank model's big blanks follow the blank V)
    const int VL = p.VL;
    const bool big_blanks = p.multi_blank != 0;
    // Which hypotheses this cluster decodes.  A cluster runs as long as its longest utterance
    // and costs more per step the more of its hypotheses are still active, so the clusters are
    // made alike: the batch is ranked by length (longest first, ties by index) and dealt in
    // rounds of ncl that alternate direction (0 .. ncl-1, ncl-1 .. 0, ...), so that no cluster
    // always gets the longest of a round.  Every workgroup ranks the whole batch itself
    // (B^2 / 512 comparisons per thread, up to kMaxRankedBatch).  Workspace rows are
    // addressed by (cluster, slot): row b0 + g; only enc_len, enc_proj and the outputs see
    // the caller's index S.gid[g].
    const int b0 = cl * p.hyps_per_cluster;
    const int Bw = ncl * p.hyps_per_cluster;   // rows of the per-hypothesis workspace arrays (>= B)
    const bool ranked = ncl > 1 && B <= kMaxRankedBatch;
    int G;
    if (ranked) {
        const int full = B / ncl, rem = B % ncl;   // the last, partial round has rem members
        const int pos_in_last = (full & 1) ? ncl - 1 - cl : cl;
        G = full + (pos_in_last < rem ? 1 : 0);
    } else {
        G = B - b0;
        if (G > p.hyps_per_cluster) G = p.hyps_per_cluster;
    }
    if (G <= 0) return;   // the whole cluster leaves together
    if (ranked) {
        int *lens = reinterpret_cast<int *>(dyn_lds);   // the activation tile is not in use yet
        for (int b = tid; b < B; b += kThreads) lens[b] = min(max(p.enc_len[b], 0), p.T);
        __syncthreads();
        for (int b = tid; b < B; b += kThreads) {
            const int lb = lens[b];
            int r = 0;
            for (int b2 = 0; b2 < B; ++b2) {
                const int l2 = lens[b2];
                r += (l2 > lb || (l2 == lb && b2 < b)) ? 1 : 0;
            }
            const int round = r / ncl, pos = r - round * ncl;
            if (((round & 1) ? ncl - 1 - pos : pos) == cl) S.gid[round] = b;
        }
    } else {
        for (int g = tid; g < G; g += kThreads) S.gid[g] = b0 + g;
    }
    __syncthreads();

    // A value that is the same in every lane of the wavefront (e.g. read from LDS at an address that
    // depends on the wavefront only), moved to a scalar register: what is computed from it -- row
    // pointers above all -- then runs on the scalar unit and loads take a scalar base address.
    auto uni = [](int v) { return __builtin_amdgcn_readfirstlane(v); };
    const int Hp = p.h_pred, E = p.emb_dim, L = p.pred_layers;
    const bool lstm = p.pred_kind == TDT_PRED_LSTM;
    // the activation tile starts out as zeros: rows a work item does not stage keep what they
    // held, and although nothing ever looks at their products they should be numbers
    for (int i = tid; i < p.lds_bytes / 16; i += kThreads)
        reinterpret_cast<uint4 *>(dyn_lds)[i] = make_uint4(0, 0, 0, 0);
    __syncthreads();

    ActTile<WT> A;
    A.planes = reinterpret_cast<decltype(A.planes)>(dyn_lds);
    A.ldb = ActTile<WT>::row_elems(p.kseg_max);

    BarrierInfo bi;
    bi.flags = p.barrier + (size_t)cl * C * kBarrierStride;
    bi.mine = bi.flags + (size_t)rank * kBarrierStride;
    // self-test (compiled into the frame-looping variant only, to keep it out of the kernels that
    // are benchmarked): this workgroup never announces its arrivals, so the waits of its cluster
    // run out
    if constexpr (FRAMELOOP)
        if (p.selftest_stall && cl == 0 && rank == 0) bi.mine = p.barrier + (size_t)kMaxGrid * kBarrierStride;
    bi.epoch = 0;
    LsePartial *const pbase = p.partials + (size_t)cl * (kPartialEntries / ncl);
    const int rows_cap = p.rows_per_cluster;
    unsigned long long *const rl_base = p.row_lab + (size_t)cl * kRowBufs * rows_cap;
    unsigned long long *const rd_base = p.row_dur + (size_t)cl * kRowBufs * rows_cap;
    const int max_cg = min(kMaxColGroups, kPartialEntries / ncl / kMaxRowsPerPass);

    constexpr bool chunked = CHUNKED;
    // ---- Alg. 3 lines 3-4: empty hypotheses, time 0, everyone with frames is active
    for (int g = tid; g < G; g += kThreads) {
        int len = p.enc_len[S.gid[g]];
        int st = 0;
        if (len < 0) { len = 0; st = TDT_HYP_LEN_CLAMPED; }
        if (len > T) { len = T; st = TDT_HYP_LEN_CLAMPED; }
        // A chunk of a longer utterance takes up what the previous chunk left: the frames
        // its last step reached past its end, and the labels the predictor saw last.
        int t0 = 0, last = V, last2 = V;   // V: the start-of-sequence label
        bool started = false;
        if (chunked) {
            const int b = S.gid[g];
            started = p.st_started[b] != 0;
            t0 = max(p.st_time[b], 0);
            if (started) {
                last = min(max(p.st_last[b], 0), V);
                last2 = min(max(p.st_last2[b], 0), V);
            }
        }
        const bool active = t0 < len;
        S.len[g] = len;
        S.time[g] = t0;
        S.sym[g] = 0;
        S.last[g] = last;
        S.last2[g] = last2;
        S.out_len[g] = 0;
        S.status[g] = st;
        S.score[g] = 0.0f;
        S.active[g] = active;
        S.need[g] = active && !started;   // who takes the first predictor step
        S.started[g] = started || active;
        S.took_part[g] = active;
        S.hpar[g] = 1;
        S.commit[g] = 1;   // the start-of-sequence step is kept
    }
    if (tid < TDT_MAX_DURATIONS) S.durations[tid] = p.durations[tid];
    if (tid == 0) {
#if TDT_TRACE
        g_tr_n = 0;
        g_tr_on = 0;
#endif
        S.aborted = 0;
        S.pend_n = 0;
        S.pend_ncg = 0;
        S.fine_phase = 0;
        for (int a = 0; a < 3; ++a)
            for (int b = 0; b < 3; ++b) S.tk_fine[a][b] = 0;
    }
    __syncthreads();

    enum { kTkP = 0, kTkQ, kTkJ, kTkD, kTkBar };
    if (tid == 0) {
        for (int a = 0; a < 5; ++a) S.tk[a] = 0;
        S.tk_last = S.tk_start = wall_clock64();
    }
    // work counters: the same in every thread, so they live in scalar registers
    long long st_pred_passes = 0, st_pred_rows = 0, st_joint_passes = 0, st_joint_rows = 0;
    // Thread 0 books the time since the last call -- in profiling builds only: every call is a
    // clock read and an LDS update that the other wavefronts wait for at the next barrier, about
    // ten of them per label.
    auto lap = [&](int bucket) {
        if (TDT_PHASE_TIMERS && tid == 0) {
            const long long now = wall_clock64();
            S.tk[bucket] += now - S.tk_last;
            S.tk_last = now;
        }
    };
    // softmax partials of the rows chosen in the last decision step, still to be summed
    unsigned long long pend_u[kDeferPerWave];
#pragma unroll
    for (int j = 0; j < kDeferPerWave; ++j) pend_u[j] = 0ull;
    auto finish_scores = [&]() {   // all threads; the loads were issued a phase ago
        const int n = uni(S.pend_n), ncg = uni(S.pend_ncg);
#pragma unroll
        for (int j = 0; j < kDeferPerWave; ++j) {
            const int q = wave + j * kWaves;
            if (q < n && S.pend_found[q]) {   // uniform over the wavefront
                float part = 0.0f;
                if (lane < ncg) {
                    const float pm = __uint_as_float((unsigned)pend_u[j]);
                    const float ps = __uint_as_float((unsigned)(pend_u[j] >> 32));
                    if (ps > 0.0f) part = ps * expf(pm - S.pend_m[q]);
                }
                part = wave_sum(part);
                // log_softmax at the maximum = -log(sum exp(l - max))
                if (lane == 63) S.score[S.pend_g[q]] -= logf(part);
            }
        }
        __syncthreads();
        if (tid == 0) S.pend_n = 0;
    };
    // Automatic window: as many rows as give every workgroup at most one joint work item of at
    // most `tiles_per_item` column tiles (then one round, all wavefronts busy).  Unless the
    // caller fixes it, a work item takes 8 column tiles, one a wavefront, in groups of five
    // hypotheses or more (the longer windows save more joint passes than the longer items cost:
    // measured 2 to 5 % at 6 to 13 hypotheses a group) and 4 in smaller groups (1 to 2 % the
    // other way), more (up to 8) where the group's hypotheses with the smallest window of 4
    // frames would otherwise make more items than there are workgroups.
    int auto_rows;
    {
        const int NT = (O + CT - 1) / CT;
        int tiles_per_item = p.joint_tiles;
        if (tiles_per_item <= 0) {
            const int row_tiles_min = (G * 4 + RT - 1) / RT;
            const int groups_fit = max(1, C / row_tiles_min);
            tiles_per_item = G >= 5 ? 8 : min(8, max(4, (NT + groups_fit - 1) / groups_fit));
        }
        const int groups = (NT + tiles_per_item - 1) / tiles_per_item;
        auto_rows = max(1, C / groups) * RT;
    }
    // streaming joint pass: dies the group's workgroups are spread over, workgroups per die, this
    // one's die and place on it, column tiles per die and this die's first
    const int wide_ndie = C >= kXcds ? kXcds : C, wide_per = C / wide_ndie;
    const int wide_die = rank / wide_per, wide_j = rank - wide_die * wide_per;
    const int wide_ntd_all = ((O + CT - 1) / CT + wide_ndie - 1) / wide_ndie;
    const int wide_t0 = wide_die * wide_ntd_all;
    const int wide_ntd = max(0, min(wide_ntd_all, (O + CT - 1) / CT - wide_t0));   // this die's column tiles
    // How a joint pass is cut depends only on how many hypotheses search: tabulated here, one
    // thread per count, so that a pass looks it up instead of dividing.
    for (int n = tid + 1; n <= G; n += kThreads) {
        const int NT = (O + CT - 1) / CT;
        int Kw = FRAMELOOP ? 1 : p.window;   // Alg. 2 looks at one frame per step
        if (Kw <= 0) {
            Kw = auto_rows / n;
            if (Kw < 3) Kw = 3;   // (2, 4 and 5 measured no better on any benchmark model)
            // the row tiles this window needs are paid for whole: as many frames as fill them
            const int fill = (n * Kw + RT - 1) / RT * RT / n;
            if (fill > Kw) Kw = fill;
        }
        if (Kw > kMaxWindow) Kw = kMaxWindow;
        if (Kw * n > rows_cap) Kw = rows_cap / n;
        const int n_tiles = (n * Kw + RT - 1) / RT;
        int n_cg, tpg;
        split_tiles(C, n_tiles, NT, max_cg, n_cg, tpg);
        JointPlan jp;
        jp.w_lo = jp.w_hi = 0;
        if constexpr (WIDEJ) {
            // The streaming pass deals its work die by die: die d of the chip multiplies by the same
            // eighth of the output matrix's column tiles in every pass, whatever the number of row
            // tiles, so that this eighth stays in the die's L2 (the whole matrix does not fit it,
            // and every row tile of every group streams it).  The workgroups a group has on a die
            // share (row tile, column tile) pairs of that die, row tile by row tile; a workgroup's
            // share is the range [w_lo, w_hi) of them and may span two row tiles.  Every workgroup
            // that takes part owns one softmax partial per row, so n_cg is their number.
            const int total = n_tiles * wide_ntd, chunk = (total + wide_per - 1) / wide_per;
            n_cg = wide_ndie * wide_per;
            if (rank < n_cg) {
                jp.w_lo = min(total, wide_j * chunk);
                jp.w_hi = min(total, jp.w_lo + chunk);
            }
        }
        jp.Kw = (short)Kw;
        jp.rcp_kw = ((1 << 20) + Kw - 1) / Kw;   // (r * rcp_kw) >> 20 == r / Kw for r < 16384, Kw <= 64
        jp.n_tiles = (short)n_tiles;
        jp.n_cg = (short)n_cg;
        jp.tpg = tpg;
        jp.ti0 = (short)(rank / n_cg);   // this workgroup's first work item (rank), if it has one
        jp.cg0 = rank % n_cg;
        S.jplan[n] = jp;
    }
    __syncthreads();
    int pp = 0;          // which half of hbuf holds the current hidden state
    bool first = true;   // the first label-loop iteration of this call
    unsigned jpass = 0;  // joint passes so far (selects the exchange buffers)
    bool ok = true;
    // A barrier this workgroup has arrived at but not yet waited for, and the timer bucket of
    // the phase that runs meanwhile.  The wait happens where the next phase first needs what
    // the other workgroups wrote: before its first rows are staged (run_item's wait hook), or
    // after its item loop in a workgroup that got no item.
    bool bar_pending = false;
    int phase_bucket = kTkP;
    auto finish_barrier = [&]() {
        lap(phase_bucket);
        ok = barrier_wait(S, bi, p.abort_flag, C, p.timeout_ticks) && ok;
        lap(kTkBar);
        bar_pending = false;
    };
    auto wait_hook = [&]() {
        if (bar_pending) finish_barrier();   // uniform over the workgroup
        else __syncthreads();
    };

    // The list of active hypotheses is rebuilt by the decision step together with the list of those
    // that still search; the loop top builds it only where that has not happened (first iteration;
    // the chunked and frame-looping forms, which change the flags between the two).
    constexpr bool kPlain = !CHUNKED && !FRAMELOOP;
    bool have_act = false;
    // the split of phase Q's column tiles, kept while the number of row tiles stays the same
    int q_for_tiles = -1, q_tpg = 1, q_ga = 0, q_gb = 0;
    while (ok) {   // ---- Alg. 3 line 5: while any hypothesis is active
        if (!(kPlain && have_act)) build_list(S, S.active, G, S.act_list, &S.n_act);
        // (what every lane reads from the same LDS word is uniform, but the compiler cannot know:
        // counts and plans go through readfirstlane, so that the loops and branches they steer
        // are scalar and the waits for loads in flight behind them stay exact)
        const int n_act = uni(S.n_act);
        if (n_act == 0) break;
        st_pred_passes += 1;
        const int n_tiles_a = (n_act + RT - 1) / RT;
        // Who takes the predictor step: every active hypothesis -- except in the first
        // iteration of a chunk, where the hypotheses that bring a state along keep it and
        // only those at their start of sequence step.
        const int *plist = S.act_list;
        int n_p = n_act;
        if (chunked && first) {
            build_list(S, S.need, G, S.need_list, &S.n_need);
            plist = S.need_list;
            n_p = uni(S.n_need);
            if (lstm) {
                // the state brought along goes where this iteration's step would have put it
                const int per = L * Hp;
                for (int idx = rank * kThreads + tid; idx < n_act * per; idx += C * kThreads) {
                    const int i = idx / per, r = idx - i * per, l = r / Hp, u = r - l * Hp;
                    const int g = S.act_list[i];
                    if (!S.need[g]) {
                        const size_t src = ((size_t)l * B + S.gid[g]) * Hp + u;
                        const size_t dst = ((size_t)l * Bw + b0 + g) * Hp + u;
                        st_co(p.hbuf + (size_t)L * Bw * Hp + dst, p.st_h[src]);
                        st_co(p.cbuf + dst, p.st_c[src]);
                    }
                }
            }
            first = false;
        }
        if (chunked)
            for (int i = tid; i < n_act; i += kThreads) S.hpar[S.act_list[i]] = (unsigned char)(pp ^ 1);
        const int n_tiles_p = (n_p + RT - 1) / RT;

#if TDT_TRACE
        if (tid == 0) g_tr_on = (st_pred_passes >= 20 && st_pred_passes < 24);
#endif
        TR(1);
        // ---- P: predictor step (Alg. 3 line 6)
        st_pred_rows += n_p;
        if (TDT_FINE_TIMERS && tid == 0) S.fine_phase = 0;
        phase_bucket = kTkP;
        if (lstm) {
            {
                // Layer 0 needs no product here.  W_ih * emb[label] + b is a row of the table that
                // the host-side call built before this kernel, and W_hh * h was computed right
                // after h itself (phase Q of the previous label, below), before the label was
                // known.  What is left is the cell update, one thread per (hypothesis, unit).
                float *h_next = p.hbuf + ((size_t)(pp ^ 1) * L) * Bw * Hp;
                float *cst = p.cbuf;
                const int total = n_p * Hp;
                const int per_wg = (total + C - 1) / C;
                const int c_end = min(total, (rank + 1) * per_wg);
                for (int c = rank * per_wg + tid; c < c_end; c += kThreads) {
                    const int i = c / Hp, unit = c - i * Hp;
                    const int g = plist[i];
                    const size_t o = (size_t)(b0 + g) * Hp + unit;
                    const float2 r01 = ld_co2(p.rgate + o * 4), r23 = ld_co2(p.rgate + o * 4 + 2);
                    const float4 t4 =
                        *reinterpret_cast<const float4 *>(p.emb_gates + ((size_t)S.last[g] * Hp + unit) * 4);
                    const float c_old = ld_co(cst + o);
                    const float ig = fast_sigmoid(r01.x + t4.x), fg = fast_sigmoid(r01.y + t4.y);
                    const float gg = 2.0f * fast_sigmoid(2.0f * (r23.x + t4.z)) - 1.0f;
                    const float og = fast_sigmoid(r23.y + t4.w);
                    const float cn = fg * c_old + ig * gg;
                    if (FRAMELOOP && !S.commit[g]) {
                        // Alg. 2: the step was computed, but the last decision was a blank, so
                        // the old state stays (it moves to the other half of the buffer)
                        st_co(h_next + o, ld_co(p.hbuf + (size_t)pp * L * Bw * Hp + o));
                    } else {
                        st_co(cst + o, cn);
                        st_co(h_next + o, og * (2.0f * fast_sigmoid(2.0f * cn) - 1.0f));
                    }
                }
                if (bar_pending) finish_barrier();
                if (!ok) break;
                lap(kTkP);
                barrier_arrive(bi, C);
                bar_pending = true;
            }
            for (int l = 1; l < L && ok; ++l) {   // deeper layers: [W_ih, W_hh] . [h of the layer below, own h]
                const float *bl = p.b_lstm[l];
                const float *h_cur = p.hbuf + ((size_t)pp * L + l) * Bw * Hp;
                float *h_next = p.hbuf + ((size_t)(pp ^ 1) * L + l) * Bw * Hp;
                const float *x_prev = p.hbuf + ((size_t)(pp ^ 1) * L + (l - 1)) * Bw * Hp;
                float *cst = p.cbuf + (size_t)l * Bw * Hp;
                PhaseInputs in;
                in.w0 = p.w_ih[l];
                in.K0 = Hp;
                in.w1 = p.w_hh[l];
                in.K1 = Hp;
                const int NT = (Hp + 3) / 4;   // a column tile = 4 hidden units x 4 gates
                int n_ug, tpg;
                split_tiles(C, n_tiles_p, NT, NT, n_ug, tpg);
                for (int it = rank; it < n_tiles_p * n_ug; it += C) {
                    const int ti = it / n_ug, ug = it % n_ug;
                    const int nrows = min(RT, n_p - ti * RT);
                    const int tile0 = ug * tpg, n_ct = min(tpg, NT - tile0);
                    // A round holds up to 8 tiles x 16 rows x 16 pre-activations (4 units x 4 gates
                    // a tile): entry idx = tid + e * 512 is (tile slot idx / 256, row idx / 16 % 16,
                    // column idx % 16), so the four gates of a unit sit in four neighbouring lanes.
                    float c_old[kTabPerThread];   // the unit's cell value (used by the lane of gate 0)
                    run_item<WT>(
                        S, A, in, tile0, n_ct, bl, bl,
                        [&](const Seg &sg) {
                            const int k0 = sg.k0;
                            const float *src = sg.part == 1 ? h_cur : x_prev;
                            const int K = sg.K;
                            stage_segment4<WT>(
                                A, K, nrows,
                                [&](int i) { return src + (size_t)(b0 + uni(plist[ti * RT + i])) * Hp + k0; },
                                [K](const float *row, int k) { return ld_co4(row, K, k); },
                                [](const float *, int, float4 v) { return v; });
                        },
                        [&](int ct, int j) -> long long {
                            const int unit = (tile0 + ct) * 4 + (j >> 2);
                            return unit < Hp ? (long long)(j & 3) * Hp + unit : -1;
                        },
                        [&](int base, int) {   // loads only; their values are used in the epilogue
#pragma unroll
                            for (int e = 0; e < kTabPerThread; ++e) {
                                const int idx = tid + e * kThreads;
                                const int t = idx >> 8, i = (idx >> 4) & 15, j = idx & 15;
                                const int unit = (tile0 + base + t) * 4 + (j >> 2);
                                const int g = plist[ti * RT + (i < nrows ? i : 0)];
                                c_old[e] = ld_co(cst + (size_t)(b0 + g) * Hp + (unit < Hp ? unit : 0));
                            }
                        },
                        [&](int, int) {},
                        [&](int base, int n, int ksplit) {
#pragma unroll
                            for (int e = 0; e < kTabPerThread; ++e) {
                                const int idx = tid + e * kThreads;
                                const int t = idx >> 8, i = (idx >> 4) & 15, j = idx & 15, q = j & 3;
                                if (t < n) {   // uniform over the wavefront
                                    const int unit = (tile0 + base + t) * 4 + (j >> 2);
                                    const float pre = cpart_sum(S, t, ksplit, i, j) + S.bias[t * CT + j];
                                    // gates 0, 1, 3: sigmoid(x); gate 2: tanh(x) = 2 sigmoid(2x) - 1
                                    const float sg = fast_sigmoid(q == 2 ? 2.0f * pre : pre);
                                    const float act = q == 2 ? 2.0f * sg - 1.0f : sg;
                                    const float fg = __shfl_down(act, 1, 4), gg = __shfl_down(act, 2, 4);
                                    const float og = __shfl_down(act, 3, 4);
                                    if (q == 0 && i < nrows && unit < Hp) {
                                        const float cn = fg * c_old[e] + act * gg;
                                        const int g = plist[ti * RT + i];
                                        const size_t o = (size_t)(b0 + g) * Hp + unit;
                                        if (FRAMELOOP && !S.commit[g]) {
                                            st_co(h_next + o, ld_co(h_cur + o));
                                        } else {
                                            st_co(cst + o, cn);
                                            st_co(h_next + o, og * (2.0f * fast_sigmoid(2.0f * cn) - 1.0f));
                                        }
                                    }
                                }
                            }
                        },
                        wait_hook);
                }
                if (bar_pending) finish_barrier();
                if (!ok) break;
                lap(kTkP);
                barrier_arrive(bi, C);
                bar_pending = true;
            }
            if (!ok) break;
        }

        TR(2);
        // ---- Q: everything that is a product with the new predictor state of an LSTM: its
        // projection into the joint space (Sec. 3.4), and the recurrent part W_hh * h of the first
        // layer's next step.  Two sections of column tiles, each with its matrix and its input.
        // (A stateless predictor has no such phase: its projected output is a sum of per-label
        // table rows that the joint pass reads directly.)
        if (TDT_FINE_TIMERS && tid == 0) S.fine_phase = 1;
        phase_bucket = kTkQ;
        if (lstm) {
            const float *src_a = p.hbuf + ((size_t)(pp ^ 1) * L + (L - 1)) * Bw * Hp;
            const float *src_b = p.hbuf + ((size_t)(pp ^ 1) * L) * Bw * Hp;
            // (projections on the fly: only the recurrent product is left here)
            const int NT_A = ONTHEFLY ? 0 : (H + CT - 1) / CT, NT_B = (Hp + 3) / 4;
            if (n_tiles_a != q_for_tiles) {
                // fewest tiles per work item that give every workgroup at most one item
                int t = max(1, ((NT_A + NT_B) * n_tiles_a + C - 1) / C);
                while (((NT_A + t - 1) / t + (NT_B + t - 1) / t) * n_tiles_a > C && t < NT_A + NT_B) ++t;
                q_tpg = t;
                q_ga = (NT_A + t - 1) / t;
                q_gb = (NT_B + t - 1) / t;
                q_for_tiles = n_tiles_a;
            }
            const int tpg = q_tpg, g_a = q_ga, g_b = q_gb;
            const int n_grp = g_a + g_b;
            for (int it = rank; it < n_tiles_a * n_grp; it += C) {
                int ti = 0, grp = it;   // one row tile: the item index is the group
                if (n_tiles_a > 1) {
                    ti = it / n_grp;
                    grp = it - ti * n_grp;
                }
                const bool sec_b = grp >= g_a;
                const int nrows = min(RT, n_act - ti * RT);
                const int tile0 = (sec_b ? grp - g_a : grp) * tpg;
                const int n_ct = min(tpg, (sec_b ? NT_B : NT_A) - tile0);
                const float *src = sec_b ? src_b : src_a;
                PhaseInputs in;
                in.w0 = sec_b ? p.w_hh[0] : p.w_pred;
                in.K0 = Hp;
                in.w1 = nullptr;
                in.K1 = 0;
                run_item<WT>(
                    // the recurrent section has no bias of its own; its placeholder must still
                    // cover the section's 4 * h_pred weight rows (run_item reads it unconditionally)
                    S, A, in, tile0, n_ct, sec_b ? nullptr : p.b_pred, sec_b ? p.b_lstm[0] : p.b_pred,
                    [&](const Seg &sg) {
                        const int k0 = sg.k0;
                        const int K = sg.K;
                        stage_segment4<WT>(
                            A, K, nrows,
                            [&](int i) { return src + (size_t)(b0 + uni(S.act_list[ti * RT + i])) * Hp + k0; },
                            [K](const float *row, int k) { return ld_co4(row, K, k); },
                            [](const float *, int, float4 v) { return v; });
                    },
                    [&](int ct, int j) -> long long {
                        if (sec_b) {   // a column tile = 4 hidden units x 4 gates
                            const int unit = (tile0 + ct) * 4 + (j >> 2);
                            return unit < Hp ? (long long)(j & 3) * Hp + unit : -1;
                        }
                        const int n = (tile0 + ct) * CT + j;
                        return n < H ? n : -1;
                    },
                    [&](int, int) {},
                    [&](int, int) {},
                    [&](int base, int n, int ksplit) {
                        for (int idx = tid; idx < n * RT * CT; idx += kThreads) {
                            const int t = idx >> 8, i = (idx >> 4) & 15, j = idx & 15;
                            if (i >= nrows) continue;
                            const size_t b = (size_t)(b0 + S.act_list[ti * RT + i]);
                            const float v = cpart_sum(S, t, ksplit, i, j) + S.bias[t * CT + j];
                            if (sec_b) {   // [hypothesis][unit][gate]
                                const int unit = (tile0 + base + t) * 4 + (j >> 2);
                                if (unit < Hp) st_co(p.rgate + (b * Hp + unit) * 4 + (j & 3), v);
                            } else {
                                const int col = (tile0 + base + t) * CT + j;
                                if (col < H) st_co(p.pred_proj + b * H + col, v);
                            }
                        }
                    },
                    wait_hook);
            }
            if (bar_pending) finish_barrier();
            if (!ok) break;
            lap(kTkQ);
            barrier_arrive(bi, C);
            bar_pending = true;
        }

        if (TDT_FINE_TIMERS && tid == 0) S.fine_phase = 2;
        phase_bucket = kTkJ;
        if (FRAMELOOP) {
            // Alg. 2 is frame-synchronous: the batch looks at one frame index at a time, and a
            // hypothesis that has already moved past it waits for the others
            if (tid == 0) S.t_sync = 0x7fffffff;
            __syncthreads();
            for (int g = tid; g < G; g += kThreads)
                if (S.active[g]) atomicMin(&S.t_sync, S.time[g]);
            __syncthreads();
        }
        // Every active hypothesis now searches for its next non-blank label: the first joint pass
        // of the iteration takes the list of active hypotheses as it stands (the search flags of
        // everybody else are clear, and the decision step sets those of the listed ones).
        const int *jl = S.act_list;   // who searches in the coming pass
        int n_need = n_act;
        if constexpr (!kPlain) {
            for (int g = tid; g < G; g += kThreads) {
                bool a = S.active[g];
                if (a && chunked && (S.time[g] >= S.len[g] || (S.status[g] & TDT_HYP_TRUNCATED))) {
                    a = false;   // had only stayed for the predictor step of its last label
                    S.active[g] = 0;
                }
                if (FRAMELOOP) {
                    a = a && S.time[g] == S.t_sync;
                    S.commit[g] = 0;   // this step's predictor pass has used it; a new label sets it again
                }
                S.need[g] = a;
            }
            __syncthreads();
            build_list(S, S.need, G, S.need_list, &S.n_need);
            jl = S.need_list;
            n_need = uni(S.n_need);
        }

        // ---- inner loop (Alg. 3 line 12): joint passes until nobody searches any more
        while (n_need > 0) {
            const int NT = (O + CT - 1) / CT;
            JointPlan jp = S.jplan[n_need];
            jp.Kw = (short)uni(jp.Kw);
            jp.n_tiles = (short)uni(jp.n_tiles);
            jp.n_cg = (short)uni(jp.n_cg);
            jp.ti0 = (short)uni(jp.ti0);
            jp.tpg = uni(jp.tpg);
            jp.cg0 = uni(jp.cg0);
            jp.rcp_kw = uni(jp.rcp_kw);
            jp.w_lo = uni(jp.w_lo);
            jp.w_hi = uni(jp.w_hi);
            const int Kw = jp.Kw, n_tiles = jp.n_tiles, n_cg = jp.n_cg, tpg = jp.tpg;
            const int M = n_need * Kw;
            LsePartial *pbuf = pbase + (size_t)(jpass & 1u) * kPartialEntries;
            unsigned long long *row_lab = rl_base + (size_t)(jpass % kRowBufs) * rows_cap;
            unsigned long long *row_dur = rd_base + (size_t)(jpass % kRowBufs) * rows_cap;
            // argmax cells to clear while this pass's barrier completes: those of the pass after
            // the next (see below)
            unsigned long long *clear_lab = rl_base + (size_t)((jpass + 2) % kRowBufs) * rows_cap;
            unsigned long long *clear_dur = rd_base + (size_t)((jpass + 2) % kRowBufs) * rows_cap;
            ++jpass;
            st_joint_passes += 1;
            st_joint_rows += M;

            if constexpr (ONTHEFLY) {
                // ---- the projections of this pass's rows into the joint space, as Sec. 3.4 has
                // them without precomputation: the M (hypothesis, frame) rows of the encoder output
                // and the predictor outputs of the n_need searching hypotheses
                const int NT_H = (H + CT - 1) / CT;
                const int n_tiles_n = (n_need + RT - 1) / RT, rt_all = n_tiles + n_tiles_n;
                int tpe = max(1, (NT_H * rt_all + C - 1) / C);
                while (((NT_H + tpe - 1) / tpe) * rt_all > C && tpe < NT_H) ++tpe;
                const int g_e = (NT_H + tpe - 1) / tpe;
                const float *src_h = lstm ? p.hbuf + ((size_t)(pp ^ 1) * L + (L - 1)) * Bw * Hp : nullptr;
                for (int it = rank; it < rt_all * g_e; it += C) {
                    const int ti_all = it / g_e, grp = it % g_e;
                    const bool sec_p = ti_all >= n_tiles;   // a tile of predictor outputs
                    const int ti = sec_p ? ti_all - n_tiles : ti_all;
                    const int nrows = min(RT, (sec_p ? n_need : M) - ti * RT);
                    const int tile0 = grp * tpe, n_ct = min(tpe, NT_H - tile0);
                    PhaseInputs ein;
                    ein.w0 = sec_p ? p.w_pred : p.w_enc;
                    ein.K0 = sec_p ? Hp : p.d_enc;
                    ein.w1 = nullptr;
                    ein.K1 = 0;
                    // frame of joint row r, or -1 if it lies beyond its hypothesis' last frame
                    auto row_frame = [&](int r, int &g) {
                        const int q = r / Kw;
                        g = jl[q];
                        const int f = S.time[g] + (r - q * Kw);
                        return f < S.len[g] ? f : -1;
                    };
                    run_item<WT>(
                        S, A, ein, tile0, n_ct, sec_p ? p.b_pred : p.b_enc, p.b_pred,
                        [&](const Seg &sg) {
                            const int k0 = sg.k0;
                            if (!sec_p) {
                                stage_segment<WT>(
                                    A, sg.K, nrows,
                                    [&](int i) {
                                        int g;
                                        const int f = row_frame(ti * RT + i, g);
                                        EncRow c;
                                        c.valid = f >= 0;
                                        c.row = static_cast<const WT *>(p.enc) +
                                                ((size_t)S.gid[g] * T + (c.valid ? f : 0)) * p.d_enc + k0;
                                        return c;
                                    },
                                    [](const EncRow &c, int k) { return W2<WT>::load(static_cast<const WT *>(c.row) + k); },
                                    [](const EncRow &c, int, typename W2<WT>::Raw v) {
                                        const float2 x = W2<WT>::cvt(v);
                                        return make_float2(c.valid ? x.x : 0.0f, c.valid ? x.y : 0.0f);
                                    });
                            } else if (lstm) {
                                const int K = sg.K;
                                stage_segment4<WT>(
                                    A, K, nrows,
                                    [&](int i) { return src_h + (size_t)(b0 + uni(jl[ti * RT + i])) * Hp + k0; },
                                    [K](const float *row, int k) { return ld_co4(row, K, k); },
                                    [](const float *, int, float4 v) { return v; });
                            } else {
                                stage_segment<WT>(
                                    A, sg.K, nrows,
                                    [&](int i) {
                                        const int g = jl[ti * RT + i];
                                        return make_int2(S.last[g], S.last2[g]);
                                    },
                                    [&](int2 lab, int k) {
                                        const int kk = k0 + k, c = kk / E;
                                        const int tok = (c == L - 1) ? lab.x : lab.y;
                                        return W2<WT>::load(static_cast<const WT *>(p.emb) +
                                                            ((size_t)c * (V + 1) + tok) * E + (kk - c * E));
                                    },
                                    [](int2, int, typename W2<WT>::Raw v) { return W2<WT>::cvt(v); });
                            }
                        },
                        [&](int ct, int j) -> long long {
                            const int n = (tile0 + ct) * CT + j;
                            return n < H ? n : -1;
                        },
                        [&](int, int) {},
                        [&](int, int) {},
                        [&](int base, int n, int ksplit) {
                            for (int idx = tid; idx < n * RT * CT; idx += kThreads) {
                                const int t = idx >> 8, i = (idx >> 4) & 15, j = idx & 15;
                                const int col = (tile0 + base + t) * CT + j;
                                if (i >= nrows || col >= H) continue;
                                const float v = cpart_sum(S, t, ksplit, i, j) + S.bias[t * CT + j];
                                if (sec_p) {
                                    st_co(p.pred_proj + (size_t)(b0 + jl[ti * RT + i]) * H + col, v);
                                } else {
                                    int g;
                                    const int f = row_frame(ti * RT + i, g);
                                    if (f >= 0) st_co(p.enc_proj + ((size_t)S.gid[g] * T + f) * H + col, v);
                                }
                            }
                        },
                        wait_hook);
                }
                if (bar_pending) finish_barrier();
                if (!ok) break;
                lap(kTkQ);
                barrier_arrive(bi, C);
                bar_pending = true;
            }

            TR(3);
            // ---- J: joint network on M rows
            PhaseInputs in;
            in.w0 = p.w_out;
            in.K0 = H;
            in.w1 = nullptr;
            in.K1 = 0;
            // staging of row tile ti of this pass: relu(projected encoder frame + projected predictor output)
            auto stage_joint = [&](const Seg &sg, int ti) {
                        const int k0 = sg.k0;
                        const int nrows = min(RT, M - ti * RT);
                        // where row i of the tile reads its projected encoder frame and its projected
                        // predictor output (the row is the same in all lanes of the wavefront)
                        auto row_of = [&](int i) {
                            const int r = ti * RT + i;
                            const int q = (r * jp.rcp_kw) >> 20;   // r / Kw
                            const int g = uni(jl[q]);
                            const int f = uni(S.time[g]) + (r - q * Kw);
                            JointRow c;
                            c.valid = f < uni(S.len[g]);
                            c.enc = p.enc_proj + ((size_t)uni(S.gid[g]) * T + (c.valid ? f : 0)) * H + k0;
                            c.pred = c.pred2 = nullptr;
                            c.g = g;
                            return c;
                        };
                        if (!p.pred_tab) {
                            // the predictor output was projected by this iteration's phase Q (or, on
                            // the fly, by the phase before this pass): coherent loads
                            stage_segment4<WT>(
                                A, sg.K, nrows,
                                [&](int i) {
                                    JointRow c = row_of(i);
                                    c.pred = p.pred_proj + (size_t)(b0 + c.g) * H + k0;
                                    return c;
                                },
                                [K = sg.K](const JointRow &c, int k) {
                                    EncPred4 v;
                                    if constexpr (ONTHEFLY) v.e = ld_co4(c.enc, K, k);   // written a phase ago
                                    else v.e = *reinterpret_cast<const float4 *>(c.enc + k);
                                    v.p = ld_co4(c.pred, K, k);
                                    return v;
                                },
                                [](const JointRow &c, int, EncPred4 v) {
                                    return make_float4(c.valid ? fmaxf(v.e.x + v.p.x, 0.0f) : 0.0f,
                                                       c.valid ? fmaxf(v.e.y + v.p.y, 0.0f) : 0.0f,
                                                       c.valid ? fmaxf(v.e.z + v.p.z, 0.0f) : 0.0f,
                                                       c.valid ? fmaxf(v.e.w + v.p.w, 0.0f) : 0.0f);
                                });
                        } else if (L == 1) {
                            // stateless predictor, one label of context: a row of its table
                            // (nothing here is written by the kernel: plain 16-byte loads)
                            stage_segment4<WT>(
                                A, sg.K, nrows,
                                [&](int i) {
                                    JointRow c = row_of(i);
                                    c.pred = p.pred_tab + (size_t)uni(S.last[c.g]) * H + k0;
                                    return c;
                                },
                                [](const JointRow &c, int k) {
                                    EncPred4 v;
                                    v.e = *reinterpret_cast<const float4 *>(c.enc + k);
                                    v.p = *reinterpret_cast<const float4 *>(c.pred + k);
                                    return v;
                                },
                                [](const JointRow &c, int, EncPred4 v) {
                                    return make_float4(c.valid ? fmaxf(v.e.x + v.p.x, 0.0f) : 0.0f,
                                                       c.valid ? fmaxf(v.e.y + v.p.y, 0.0f) : 0.0f,
                                                       c.valid ? fmaxf(v.e.z + v.p.z, 0.0f) : 0.0f,
                                                       c.valid ? fmaxf(v.e.w + v.p.w, 0.0f) : 0.0f);
                                });
                        } else {
                            // two labels of context: the older label's row of table 0 plus the newest
                            // label's row of table 1 (which carries the bias) is the projected output
                            // (three loads per slot: one row of the wavefront at a time)
                            stage_segment4<WT, 1>(
                                A, sg.K, nrows,
                                [&](int i) {
                                    JointRow c = row_of(i);
                                    c.pred = p.pred_tab + (size_t)uni(S.last2[c.g]) * H + k0;
                                    c.pred2 = p.pred_tab + ((size_t)(V + 1) + uni(S.last[c.g])) * H + k0;
                                    return c;
                                },
                                [](const JointRow &c, int k) {
                                    EncPred4x2 v;
                                    v.e = *reinterpret_cast<const float4 *>(c.enc + k);
                                    v.p = *reinterpret_cast<const float4 *>(c.pred + k);
                                    v.p2 = *reinterpret_cast<const float4 *>(c.pred2 + k);
                                    return v;
                                },
                                [](const JointRow &c, int, EncPred4x2 v) {
                                    return make_float4(c.valid ? fmaxf(v.e.x + (v.p.x + v.p2.x), 0.0f) : 0.0f,
                                                       c.valid ? fmaxf(v.e.y + (v.p.y + v.p2.y), 0.0f) : 0.0f,
                                                       c.valid ? fmaxf(v.e.z + (v.p.z + v.p2.z), 0.0f) : 0.0f,
                                                       c.valid ? fmaxf(v.e.w + (v.p.w + v.p2.w), 0.0f) : 0.0f);
                                });
                        }
                                };
            if constexpr (WIDEJ) {
                // the streaming form: this workgroup's share of its die's (row tile, column tile)
                // pairs, one row tile (staged once) at a time
                const Seg sg = in.get(0);   // H <= KSEG: one stretch
                const int ti_lo = jp.w_lo / max(wide_ntd, 1), ti_hi = jp.w_hi > jp.w_lo ? (jp.w_hi - 1) / max(wide_ntd, 1) : -1;
                if (rank < n_cg) {
                    // rows of row tiles this workgroup does not touch: an empty softmax partial
                    for (int r = tid; r < M; r += kThreads) {
                        const int t = r / RT;
                        if (jp.w_hi <= jp.w_lo || t < ti_lo || t > ti_hi)
                            st_co64(reinterpret_cast<unsigned long long *>(pbuf + (size_t)r * n_cg + rank), 0ull);
                    }
                }
                for (int idx = jp.w_lo; idx < jp.w_hi;) {
                    const int ti = idx / wide_ntd, c0 = idx - ti * wide_ntd;
                    const int n_ct = min(wide_ntd - c0, jp.w_hi - idx);
                    WideRowStats ws;
                    wide_item(S, A, sg, wide_t0 + c0, n_ct, VL, O, p.b_out, [&]() { stage_joint(sg, ti); }, wait_hook, ws);
                    if (tid < RT && ti * RT + tid < M) {   // thread i holds row i of the tile
                        const int r = ti * RT + tid;
                        if (ws.s > 0.0f)
                            __hip_atomic_fetch_max(row_lab + r, pack_best(ws.m, ws.a), __ATOMIC_RELAXED, TDT_AGENT);
                        if (ws.dm > -INFINITY)
                            __hip_atomic_fetch_max(row_dur + r, pack_best(ws.dm, ws.da), __ATOMIC_RELAXED, TDT_AGENT);
                        const unsigned long long lp = (unsigned long long)__float_as_uint(ws.m) |
                                                      ((unsigned long long)__float_as_uint(ws.s) << 32);
                        st_co64(reinterpret_cast<unsigned long long *>(pbuf + (size_t)r * n_cg + rank), lp);
                    }
                    idx += n_ct;
                }
            }
            for (int it = rank; !WIDEJ && it < n_tiles * n_cg; it += C) {
                int ti = jp.ti0, cg = jp.cg0;   // the first item is tabulated
                if (it != rank) {
                    ti = it / n_cg;
                    cg = it - ti * n_cg;
                }
                const int tile0 = cg * tpg, n_ct = min(tpg, NT - tile0);
                // running statistics of row tid / 32 over this item's columns (lanes 31 and 63)
                float rm = -INFINITY, rs = 0.0f, rdm = -INFINITY;
                int ra = 0, rda = 0;
                run_item<WT>(
                    S, A, in, tile0, n_ct, p.b_out, p.b_out,
                    [&](const Seg &sg) { stage_joint(sg, ti); },
                    [&](int ct, int j) -> long long {
                        const int n = (tile0 + ct) * CT + j;
                        return n < O ? n : -1;
                    },
                    [&](int, int) {},
                    [&](int, int) {},
                    [&](int base, int n, int ksplit) {
                        // 32 consecutive lanes share row i and deal the round's n * 16 columns
                        // round-robin; lower columns win ties, so the first maximum is kept
                        const int i = tid >> 5, sub = tid & 31;
                        float lg[kWaves * CT / 32];
                        float m = -INFINITY, dm = -INFINITY;
                        int a = 0x7fffffff, da = 0x7fffffff;
#pragma unroll
                        for (int e = 0; e < kWaves * CT / 32; ++e) {
                            const int c = sub + 32 * e;
                            lg[e] = -INFINITY;
                            if (c < n * CT) {
                                const int t = c >> 4, j = c & 15;
                                const int col = (tile0 + base + t) * CT + j;
                                const float logit = cpart_sum(S, t, ksplit, i, j) + S.bias[c];
                                if (col <= VL) {
                                    lg[e] = logit;
                                    if (logit > m) { m = logit; a = col; }
                                } else if (col < O && logit > dm) {
                                    dm = logit;
                                    da = col - (VL + 1);
                                }
                            }
                        }
                        // the row's maximum (in every lane of the half-wavefront), then the lowest
                        // column that reaches it and the sum of exp(logit - maximum) (in lane 31)
                        auto fmax2 = [](float x, float y) { return fmaxf(x, y); };
                        auto imin2 = [](int x, int y) { return min(x, y); };
                        const float mrow = half_broadcast(half_reduce(m, -INFINITY, fmax2), lane);
                        a = half_reduce(m == mrow ? a : 0x7fffffff, 0x7fffffff, imin2);
                        float s = 0.0f;
#pragma unroll
                        for (int e = 0; e < kWaves * CT / 32; ++e)
                            if (lg[e] > -INFINITY) s += __expf(lg[e] - mrow);
                        s = half_reduce(s, 0.0f, [](float x, float y) { return x + y; });
                        if (D > 0) {   // the duration head, the same way
                            const float drow = half_broadcast(half_reduce(dm, -INFINITY, fmax2), lane);
                            da = half_reduce(dm == drow ? da : 0x7fffffff, 0x7fffffff, imin2);
                            dm = drow;
                        }
                        m = mrow;
                        if (sub == 31) {   // rounds ascend through the columns: '>' keeps the first maximum
                            if (s > 0.0f) {
                                if (m > rm) {
                                    rs = (rs > 0.0f ? rs * __expf(rm - m) : 0.0f) + s;
                                    rm = m;
                                    ra = a;
                                } else {
                                    rs += s * __expf(m - rm);
                                }
                            }
                            if (D > 0 && dm > rdm) {
                                rdm = dm;
                                rda = da;
                            }
                        }
                    },
                    wait_hook);
                if ((tid & 31) == 31 && ti * RT + (tid >> 5) < M) {
                    const int r = ti * RT + (tid >> 5);
                    if (rs > 0.0f)
                        __hip_atomic_fetch_max(row_lab + r, pack_best(rm, ra), __ATOMIC_RELAXED, TDT_AGENT);
                    if (rdm > -INFINITY)
                        __hip_atomic_fetch_max(row_dur + r, pack_best(rdm, rda), __ATOMIC_RELAXED, TDT_AGENT);
                    const unsigned long long lp = (unsigned long long)__float_as_uint(rm) |
                                                  ((unsigned long long)__float_as_uint(rs) << 32);
                    st_co64(reinterpret_cast<unsigned long long *>(pbuf + (size_t)r * n_cg + cg), lp);
                }
            }
            if (bar_pending) finish_barrier();
            if (!ok) break;
            TR(22);
            lap(kTkJ);
            barrier_arrive(bi, C);
            // While the arrivals travel: clear the argmax cells of the pass after the next.  Of
            // the four rotating buffers that one was last read by the decision step two passes
            // ago, which every workgroup had left before it arrived at the previous pass's
            // barrier; and its next writers start behind the next pass's barrier, at which this
            // workgroup arrives only after these stores have completed.
            for (int r = rank * kThreads + tid; r < rows_cap; r += C * kThreads) {
                st_co64(clear_lab + r, 0ull);
                if (D > 0) st_co64(clear_dur + r, 0ull);
            }
            // ... and add the score terms the previous pass left pending (their loads were
            // complete before the arrival)
            finish_scores();
            ok = barrier_wait(S, bi, p.abort_flag, C, p.timeout_ticks);
            lap(kTkBar);
            if (!ok) break;

            TR(4);
            // ---- D: every workgroup takes the same decisions from the same cells
            // D1: one coherent load per row, all rows in flight together
            {
                unsigned long long best[kMaxRowsPerPass / kThreads], bd[kMaxRowsPerPass / kThreads];
#pragma unroll
                for (int e = 0; e < kMaxRowsPerPass / kThreads; ++e) {
                    const int r = tid + e * kThreads;
                    best[e] = bd[e] = 0ull;
                    if (e * kThreads < M) {   // uniform
                        best[e] = ld_co64(row_lab + (r < M ? r : 0));
                        if (D > 0) bd[e] = ld_co64(row_dur + (r < M ? r : 0));
                    }
                }
#pragma unroll
                for (int e = 0; e < kMaxRowsPerPass / kThreads; ++e) {
                    const int r = tid + e * kThreads;
                    if (r < M) {
                        const int a = best[e] ? unpack_index(best[e]) : V;
                        S.row_a[r] = a;
                        S.row_m[r] = unpack_value(best[e]);
                        // the frame step that goes with the row's decision: from the duration head
                        // (Sec. 3.3), or -- multi-blank -- from the chosen symbol itself: the blank
                        // one frame, big blank i its increment, a label none
                        int step = 0;
                        if (D > 0) step = S.durations[unpack_index(bd[e]) & (TDT_MAX_DURATIONS - 1)];
                        else if (big_blanks) step = a < V ? 0 : a == V ? 1 : S.durations[(a - V - 1) & (TDT_MAX_DURATIONS - 1)];
                        S.row_d[r] = step;
                    }
                }
            }
            __syncthreads();
            TR(40);
            // the walk through the window of one searching hypothesis (all lanes of a wavefront)
            auto walk = [&](int q, int &w) -> bool {
                const int g = jl[q];
                const int nv = min(Kw, S.len[g] - S.time[g]);   // >= 1: a searching row has frames left
                int a = V, dstep = 0;
                if (lane < nv) {
                    a = S.row_a[q * Kw + lane];
                    dstep = S.row_d[q * Kw + lane];
                }
                w = 0;
                bool found = false;
                if (D == 0 && !big_blanks) {   // Alg. 3 lines 10 / 18: a blank moves one frame on
                    const unsigned long long nb = __ballot(lane < nv && a != V);
                    if (nb) { found = true; w = __ffsll((long long)nb) - 1; } else { w = nv; }
                } else {        // Sec. 3.3: the step comes from the duration head (or the big blank)
                    while (w < nv) {
                        if (__shfl(a, w, 64) < V) { found = true; break; }
                        const int dd = __shfl(dstep, w, 64);
                        w += dd > 0 ? dd : 1;
                    }
                }
                return found;
            };
            // the state update of one hypothesis (one thread): Alg. 3 line 20, Sec. 3.1 add_results
            auto apply = [&](int q, bool found, int w) {
                const int g = jl[q];
                const int t0 = S.time[g], len = S.len[g];
                int sym = (w > 0 || !found) ? 0 : S.sym[g];
                if (found) {
                    const int k = S.row_a[q * Kw + w];
                    int dk = S.row_d[q * Kw + w];
                    const int frame = t0 + w, n = S.out_len[g];
                    if (rank == 0) {
                        p.out_labels[(size_t)S.gid[g] * p.u_cap + n] = k;
                        p.out_frames[(size_t)S.gid[g] * p.u_cap + n] = frame;
                    }
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
                    // In a chunk a hypothesis that is done still takes the predictor step of its
                    // last label, so that the state it carries on has seen it.
                    S.active[g] = act_now || chunked;
                    S.need[g] = 0;
                    if (FRAMELOOP) S.commit[g] = 1;
                } else {
                    if (FRAMELOOP) S.commit[g] = 0;
                    const int t1 = t0 + w;
                    S.time[g] = t1;
                    S.active[g] = t1 < len;
                    S.need[g] = t1 < len;
                }
                S.sym[g] = sym;
            };
            if (n_need <= kDeferred) {
                // D2: a wavefront per hypothesis walks, updates the state and only issues the
                // loads of the chosen row's softmax partials; the score term is added later
#pragma unroll
                for (int j = 0; j < kDeferPerWave; ++j) {
                    const int q = wave + j * kWaves;
                    if (q < n_need) {   // uniform over the wavefront
                        int w;
                        const bool found = walk(q, w);
                        pend_u[j] = 0ull;
                        if (found && lane < n_cg)
                            pend_u[j] = ld_co64(reinterpret_cast<const unsigned long long *>(
                                pbuf + (size_t)(q * Kw + w) * n_cg + lane));
                        if (lane == 0) {
                            S.pend_g[q] = jl[q];
                            S.pend_found[q] = found;
                            S.pend_m[q] = found ? S.row_m[q * Kw + w] : 0.0f;
                            apply(q, found, w);
                        }
                    }
                }
                if (tid == 0) { S.pend_n = n_need; S.pend_ncg = n_cg; }
            } else {
                // D2: walk each searching hypothesis through its window
                for (int q = wave; q < n_need; q += kWaves) {
                    int w;
                    const bool found = walk(q, w);
                    if (lane == 0) {
                        S.dec_w[q] = w;
                        S.dec_found[q] = found;
                    }
                }
                __syncthreads();
                // D3: softmax denominator of each chosen row, then the state update; a segment of
                // seg lanes serves one hypothesis
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
                        // log_softmax at the maximum = -log(sum exp(l - max))
                        if (found) S.score[jl[q]] -= logf(part);
                        apply(q, found, w);
                    }
                }
            }
            __syncthreads();
            build_two_lists(S, G, S.need, S.need_list, &S.n_need, S.active, S.act_list, &S.n_act);
            have_act = true;
            jl = S.need_list;
            n_need = uni(S.n_need);
            TR(5);
            lap(kTkD);
            if (FRAMELOOP) break;   // Alg. 2: the next step starts with the predictor again
        }
        if (!ok) break;
        pp ^= 1;
    }

    finish_scores();
    __syncthreads();

    // ---- what the next chunk takes up (every step that wrote these rows was followed by a
    // barrier of the cluster before its hypothesis could go inactive)
    if (chunked && ok) {
        if (lstm) {
            const int per = L * Hp;
            for (int idx = rank * kThreads + tid; idx < G * per; idx += C * kThreads) {
                const int g = idx / per, r = idx - g * per, l = r / Hp, u = r - l * Hp;
                if (S.took_part[g]) {
                    const size_t src = ((size_t)l * Bw + b0 + g) * Hp + u;
                    const size_t dst = ((size_t)l * B + S.gid[g]) * Hp + u;
                    p.st_h[dst] = ld_co(p.hbuf + (size_t)S.hpar[g] * L * Bw * Hp + src);
                    p.st_c[dst] = ld_co(p.cbuf + src);
                }
            }
        }
        if (rank == 0) {
            for (int g = tid; g < G; g += kThreads) {
                const int b = S.gid[g];
                p.st_started[b] = S.started[g];
                // frames of the next chunk already stepped over; a hypothesis stopped at its
                // label capacity gives up the rest of this chunk
                p.st_time[b] = max(S.time[g] - S.len[g], 0);
                p.st_last[b] = S.last[g];
                p.st_last2[b] = S.last2[g];
            }
        }
    }

    // ---- results of this cluster's hypotheses
    if (rank == 0) {
        for (int g = tid; g < G; g += kThreads) {
            p.out_len[S.gid[g]] = S.out_len[g];
            p.out_score[S.gid[g]] = S.score[g];
            // a wait of this cluster that ran out leaves its hypotheses incomplete: say so per row
            p.out_status[S.gid[g]] = S.status[g] | (ok ? 0 : TDT_HYP_ABORTED);
        }
        if (tid == 0 && p.out_stats) {
            auto add = [&](int slot, long long v) {
                atomicAdd((unsigned long long *)&p.out_stats[slot], (unsigned long long)v);
            };
            add(TDT_STAT_PRED_PASSES, st_pred_passes);
            add(TDT_STAT_PRED_ROWS, st_pred_rows);
            add(TDT_STAT_JOINT_PASSES, st_joint_passes);
            add(TDT_STAT_JOINT_ROWS, st_joint_rows);
            // every label-loop iteration takes one predictor pass
            atomicMax((unsigned long long *)&p.out_stats[TDT_STAT_OUTER_MAX], (unsigned long long)st_pred_passes);
            atomicMax((unsigned long long *)&p.out_stats[TDT_STAT_JOINT_PASSES_MAX],
                      (unsigned long long)st_joint_passes);
            if (!ok) add(TDT_STAT_ABORT, 1);
            if (TDT_PHASE_TIMERS && cl == TDT_TIMER_GROUP) {   // where one cluster's time went, in wall-clock ticks
                add(TDT_STAT_TICKS_PRED, S.tk[kTkP]);
                add(TDT_STAT_TICKS_PROJ, S.tk[kTkQ]);
                add(TDT_STAT_TICKS_JOINT, S.tk[kTkJ]);
                add(TDT_STAT_TICKS_DECIDE, S.tk[kTkD]);
                add(TDT_STAT_TICKS_BARRIER, S.tk[kTkBar]);
                add(TDT_STAT_TICKS_TOTAL, wall_clock64() - S.tk_start);
                for (int a = 0; a < 3; ++a)
                    for (int b = 0; b < 3; ++b) add(TDT_STAT_TICKS_FINE + a * 3 + b, S.tk_fine[a][b]);
            }
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

int kseg_max_for(const tdt_weights_t *w, bool on_the_fly)
{
    int kmax = w->h_joint;
    if (w->h_pred > kmax) kmax = w->h_pred;
    if (on_the_fly && w->d_enc > kmax) kmax = w->d_enc;   // the encoder output is staged too
    return kmax < KSEG ? kmax : KSEG;
}

size_t lds_bytes_for(const tdt_weights_t *w, bool on_the_fly)
{
    const int k = kseg_max_for(w, on_the_fly);
    const size_t tile = w->dtype == 1 ? (size_t)3 * RT * ActTile<uint16_t>::row_elems(k) * sizeof(uint16_t)
                                      : (size_t)RT * ActTile<float>::row_elems(k) * sizeof(float);
    // before the first tile is staged the same memory holds the batch's lengths while they are ranked
    const size_t lens = (size_t)kMaxRankedBatch * sizeof(int);
    return tile > lens ? tile : lens;
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

static const void *kernel_for(const tdt_weights_t *w, DecodeVariant v)
{
    const bool bf16 = w->dtype == 1;
    if (v.wide_joint)   // bfloat16, label-looping, precomputed projections (checked by the caller)
        return v.chunked ? (const void *)decode_kernel<uint16_t, true, false, false, true>
                         : (const void *)decode_kernel<uint16_t, false, false, false, true>;
    if (v.on_the_fly)
        return bf16 ? (const void *)decode_kernel<uint16_t, false, false, true>
                    : (const void *)decode_kernel<float, false, false, true>;
    if (v.frame_loop)
        return bf16 ? (const void *)decode_kernel<uint16_t, false, true, false>
                    : (const void *)decode_kernel<float, false, true, false>;
    if (bf16)
        return v.chunked ? (const void *)decode_kernel<uint16_t, true, false, false>
                         : (const void *)decode_kernel<uint16_t, false, false, false>;
    return v.chunked ? (const void *)decode_kernel<float, true, false, false>
                     : (const void *)decode_kernel<float, false, false, false>;
}

// The answer depends on the compiled form, the LDS it is launched with and the device only.  The
// attribute call and the occupancy query cost tens of microseconds of host time, so they are
// made once per (compiled form, device) and again only when a call needs more LDS than any
// before it (the attribute is only ever raised; less LDS cannot lower the occupancy).
namespace {
struct GridCacheEntry {
    const void *fn;
    size_t max_lds;
    int dev, grid;
};
constexpr int kGridCacheSize = 64;
GridCacheEntry g_grid_cache[kGridCacheSize];
int g_grid_cache_n = 0;
std::mutex g_grid_cache_mutex;
}  // namespace

int decode_max_grid(const tdt_weights_t *w, DecodeVariant v)
{
    const size_t lds = lds_bytes_for(w, v.on_the_fly);
    const void *fn = kernel_for(w, v);
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return 0;
    std::lock_guard<std::mutex> lock(g_grid_cache_mutex);
    GridCacheEntry *ent = nullptr;
    for (int i = 0; i < g_grid_cache_n; ++i)
        if (g_grid_cache[i].fn == fn && g_grid_cache[i].dev == dev) ent = &g_grid_cache[i];
    if (ent && lds <= ent->max_lds) return ent->grid;
    if (hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess) {
        (void)hipGetLastError();
        return 0;
    }
    int n_cu = 0, per_cu = 0;
    if (hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return 0;
    hipError_t e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, fn, kThreads, lds);
    if (e != hipSuccess || per_cu < 1) {
        (void)hipGetLastError();
        return 0;
    }
    int grid = n_cu;   // one workgroup per compute unit
    if (grid > kMaxGrid) grid = kMaxGrid;
    if (ent) {
        ent->max_lds = lds;
        ent->grid = grid;
    } else if (g_grid_cache_n < kGridCacheSize) {
        g_grid_cache[g_grid_cache_n++] = GridCacheEntry{fn, lds, dev, grid};
    }
    return grid;
}

// ticks per millisecond of the wall clock the kernels read (cached per device)
int wall_clock_khz()
{
    static int khz_of[64];
    int dev = 0, khz = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 100000;
    std::lock_guard<std::mutex> lock(g_grid_cache_mutex);
    if (khz_of[dev] > 0) return khz_of[dev];
    if (hipDeviceGetAttribute(&khz, hipDeviceAttributeWallClockRate, dev) != hipSuccess || khz <= 0) {
        (void)hipGetLastError();
        return 100000;
    }
    khz_of[dev] = khz;
    return khz;
}

hipError_t launch_decode(const DecodeParams &p, const tdt_weights_t *w, DecodeVariant v, int grid,
                         hipStream_t stream)
{
    const size_t lds = lds_bytes_for(w, v.on_the_fly);
    DecodeParams pc = p;
    pc.kseg_max = kseg_max_for(w, v.on_the_fly);
    pc.lds_bytes = (int)lds;
    void *args[] = {&pc};
    const void *fn = kernel_for(w, v);
    // cooperative launch: the runtime refuses a grid whose workgroups cannot all be
    // resident at once, which is what the cluster barriers rely on
    return hipLaunchCooperativeKernel(fn, dim3(grid), dim3(kThreads), args, (unsigned)lds, stream);
}

}  // namespace tdt
