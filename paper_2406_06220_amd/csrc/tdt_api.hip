// Host side of the C ABI: argument checks, workspace layout, launches.
#include <string.h>

#include <mutex>

#include "tdt_internal.h"

// Workspace of tdt_greedy_decode_static: device memory the library owns from the moment it is
// loaded until the process ends, one copy on every GPU the library runs on.  In host code this
// name is only a handle for hipGetSymbolAddress; the device address it yields (per device) is
// what kernels, and everything else on the host, use.
static __device__ __align__(256) unsigned char scratch[TDT_STATIC_SCRATCH_BYTES];

namespace tdt {

constexpr int kMaxDevices = 64;
static std::mutex g_scratch_mutex;
static void *g_scratch_ptr[kMaxDevices];   // device address of `scratch` on each device, once asked for

// the current device's copy of `scratch`, or null (with *err set) if it cannot be found
static void *static_scratch(hipError_t *err)
{
    int dev = -1;
    *err = hipGetDevice(&dev);
    if (*err != hipSuccess) return nullptr;
    if (dev < 0 || dev >= kMaxDevices) {
        *err = hipErrorInvalidDevice;
        return nullptr;
    }
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *ptr = nullptr;
        *err = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (*err != hipSuccess) {
            (void)hipGetLastError();
            return nullptr;
        }
        g_scratch_ptr[dev] = ptr;
    }
    return g_scratch_ptr[dev];
}

static size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

WorkspaceLayout workspace_layout(const tdt_weights_t *w, int B, int T)
{
    WorkspaceLayout L{};
    size_t off = 0;
    const size_t lstm_layers = w->pred_kind == TDT_PRED_LSTM ? (size_t)w->pred_layers : 0;
    // per-hypothesis arrays are addressed by (cluster, slot): n_clusters * ceil(B / n_clusters) rows
    const size_t rows = (size_t)B + kMaxGrid;
    L.packed = off;
    off = align_up(off + packed_layout(w).total, 256);
    L.enc_proj = off;
    off = align_up(off + (size_t)B * T * w->h_joint * sizeof(float), 256);
    L.pred_proj = off;
    off = align_up(off + rows * w->h_joint * sizeof(float), 256);
    L.emb_gates = off;
    if (lstm_layers > 0)
        off = align_up(off + (size_t)(w->vocab + 1) * 4 * w->h_pred * sizeof(float), 256);
    // stateless predictor: its projected output per label, one table per context position
    L.pred_tab = off;
    if (lstm_layers == 0)
        off = align_up(off + (size_t)w->pred_layers * (w->vocab + 1) * w->h_joint * sizeof(float), 256);
    L.partials = off;
    off = align_up(off + 2 * (size_t)kPartialEntries * sizeof(LsePartial), 256);
    // everything from here on is cleared by the init kernel of every call
    L.zero_begin = off;
    // per-row argmax cells: a cluster never scores more than min(kMaxRowsPerPass,
    // hyps * kMaxWindow) rows per pass, so (B + kMaxGrid) * kMaxWindow cells cover any split
    L.row_entries = (size_t)kRowBufs * ((size_t)B + kMaxGrid) * kMaxWindow;
    L.row_lab = off;
    off = align_up(off + L.row_entries * sizeof(unsigned long long), 256);
    L.row_dur = off;
    off = align_up(off + L.row_entries * sizeof(unsigned long long), 256);
    L.hbuf = off;
    off = align_up(off + 2 * lstm_layers * rows * w->h_pred * sizeof(float), 256);
    L.cbuf = off;
    off = align_up(off + lstm_layers * rows * w->h_pred * sizeof(float), 256);
    L.rgate = off;
    if (lstm_layers > 0) off = align_up(off + rows * 4 * w->h_pred * sizeof(float), 256);
    L.barrier = off;
    off = align_up(off + (size_t)(kMaxGrid + 1) * kBarrierStride * sizeof(unsigned), 256);   // + one spare word
    L.abort_flag = off;
    off = align_up(off + 256, 256);
    L.zero_end = off;
    L.total = off;
    return L;
}

StateLayout state_layout(const tdt_weights_t *w, int B)
{
    StateLayout L{};
    const size_t ints = align_up((size_t)B * sizeof(int32_t), 256);
    L.started = 0;
    L.time = ints;
    L.last = 2 * ints;
    L.last2 = 3 * ints;
    L.h = 4 * ints;
    const size_t fl = w->pred_kind == TDT_PRED_LSTM
                          ? align_up((size_t)w->pred_layers * B * w->h_pred * sizeof(float), 256) : 0;
    L.c = L.h + fl;
    L.total = L.c + fl;
    return L;
}

static int check_model(const tdt_weights_t *w)
{
    if (!w) return TDT_ERR_NULL;
    if (w->dtype != 0 && w->dtype != 1) return TDT_ERR_UNSUPPORTED;
    if (w->pred_kind != TDT_PRED_STATELESS && w->pred_kind != TDT_PRED_LSTM) return TDT_ERR_UNSUPPORTED;
    if (w->pred_layers < 1) return TDT_ERR_UNSUPPORTED;
    if (w->pred_kind == TDT_PRED_LSTM && w->pred_layers > TDT_MAX_LSTM_LAYERS) return TDT_ERR_UNSUPPORTED;
    if (w->pred_kind == TDT_PRED_STATELESS && w->pred_layers > TDT_MAX_CONTEXT) return TDT_ERR_UNSUPPORTED;
    const int dims[4] = {w->d_enc, w->h_joint, w->h_pred, w->emb_dim};
    for (int d : dims)
        if (d < 8 || d > TDT_MAX_DIM || d % 8 != 0) return TDT_ERR_SHAPE;
    if (w->vocab < 1 || w->vocab > (1 << 24)) return TDT_ERR_SHAPE;
    if (w->n_dur < 0 || w->n_dur > TDT_MAX_DURATIONS) return TDT_ERR_SHAPE;
    if (w->pred_kind == TDT_PRED_LSTM && w->emb_dim + w->h_pred > TDT_MAX_DIM) return TDT_ERR_SHAPE;
    if (w->pred_kind == TDT_PRED_LSTM && w->pred_layers > 1 && 2 * w->h_pred > TDT_MAX_DIM)
        return TDT_ERR_SHAPE;
    if (w->pred_kind == TDT_PRED_STATELESS && w->h_pred != w->pred_layers * w->emb_dim)
        return TDT_ERR_SHAPE;
    return TDT_OK;
}

// the kernels read rows of these arrays 16 bytes at a time
static bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

static int check_model_pointers(const tdt_weights_t *w, bool need_decoder)
{
    if (!w->w_enc || !w->b_enc) return TDT_ERR_NULL;
    if (!aligned16(w->w_enc) || !aligned16(w->b_enc)) return TDT_ERR_ALIGN;
    if (!need_decoder) return TDT_OK;
    if (!w->emb || !w->w_pred || !w->b_pred || !w->w_out || !w->b_out) return TDT_ERR_NULL;
    if (!aligned16(w->emb) || !aligned16(w->w_pred) || !aligned16(w->b_pred) || !aligned16(w->w_out) ||
        !aligned16(w->b_out))
        return TDT_ERR_ALIGN;
    if (w->pred_kind == TDT_PRED_LSTM)
        for (int l = 0; l < w->pred_layers; ++l) {
            if (!w->w_ih[l] || !w->w_hh[l] || !w->b_lstm[l]) return TDT_ERR_NULL;
            if (!aligned16(w->w_ih[l]) || !aligned16(w->w_hh[l]) || !aligned16(w->b_lstm[l])) return TDT_ERR_ALIGN;
        }
    return TDT_OK;
}

}  // namespace tdt

using namespace tdt;

extern "C" {

int tdt_workspace_bytes(const tdt_weights_t *weights, int B, int T, int u_cap, size_t *bytes)
{
    if (!weights || !bytes) return TDT_ERR_NULL;
    if (B < 1 || T < 1 || u_cap < 1) return TDT_ERR_SHAPE;
    const int st = check_model(weights);
    if (st != TDT_OK) return st;
    *bytes = workspace_layout(weights, B, T).total;
    return TDT_OK;
}

int tdt_encoder_projection(const void *enc, int64_t rows, const tdt_weights_t *weights, float *out,
                           void *stream)
{
    if (!weights) return TDT_ERR_NULL;
    const int st = check_model(weights);
    if (st != TDT_OK) return st;
    if (!enc || !out) return TDT_ERR_NULL;
    if (!aligned16(enc) || !aligned16(out)) return TDT_ERR_ALIGN;
    if (const int sp = check_model_pointers(weights, false); sp != TDT_OK) return sp;
    if (rows < 0 || rows > ((int64_t)1 << 31)) return TDT_ERR_SHAPE;
    if (launch_encoder_projection(enc, rows, weights, out, static_cast<hipStream_t>(stream)) != hipSuccess)
        return TDT_ERR_LAUNCH;
    return TDT_OK;
}

int tdt_encoder_projection_valid(const void *enc, const int32_t *enc_len, int B, int T,
                                 const tdt_weights_t *weights, float *out, void *stream)
{
    if (!weights) return TDT_ERR_NULL;
    const int st = check_model(weights);
    if (st != TDT_OK) return st;
    if (!enc || !enc_len || !out) return TDT_ERR_NULL;
    if (!aligned16(enc) || !aligned16(out)) return TDT_ERR_ALIGN;
    if (const int sp = check_model_pointers(weights, false); sp != TDT_OK) return sp;
    if (B < 1 || T < 1 || (int64_t)B * T > ((int64_t)1 << 31)) return TDT_ERR_SHAPE;
    if (launch_encoder_projection_valid(enc, enc_len, B, T, weights, out, static_cast<hipStream_t>(stream)) !=
        hipSuccess)
        return TDT_ERR_LAUNCH;
    return TDT_OK;
}

int tdt_state_bytes(const tdt_weights_t *weights, int B, size_t *bytes)
{
    if (!weights || !bytes) return TDT_ERR_NULL;
    if (B < 1) return TDT_ERR_SHAPE;
    const int st = check_model(weights);
    if (st != TDT_OK) return st;
    *bytes = state_layout(weights, B).total;
    return TDT_OK;
}

// the body of both decode entry points; `state` is null for whole utterances
static int decode_common(const void *enc, const int32_t *enc_len, int B, int T,
                         const tdt_weights_t *weights, const int32_t *durations, int max_symbols,
                         int u_cap, int32_t *out_labels, int32_t *out_frames, int32_t *out_len,
                         float *out_score, int32_t *out_status, int64_t *out_stats, void *state,
                         void *workspace, size_t workspace_bytes, const tdt_options_t *options,
                         void *stream)
{
    if (!weights) return TDT_ERR_NULL;
    int st = check_model(weights);
    if (st != TDT_OK) return st;
    if (!enc || !enc_len || !out_labels || !out_frames || !out_len || !out_score || !out_status)
        return TDT_ERR_NULL;
    if (!aligned16(enc)) return TDT_ERR_ALIGN;
    st = check_model_pointers(weights, true);
    if (st != TDT_OK) return st;
    if (B < 1 || T < 1 || u_cap < 1 || max_symbols < 1) return TDT_ERR_SHAPE;
    if ((int64_t)B * T > ((int64_t)1 << 31) || T > (1 << 30) || (int64_t)B * u_cap > ((int64_t)1 << 40)) return TDT_ERR_SHAPE;
    // durations (Sec. 3.3): one non-negative frame increment per class, at least one positive
    if ((weights->n_dur == 0) != (durations == nullptr)) return TDT_ERR_DURATIONS;
    bool any_pos = weights->n_dur == 0;
    const bool multi_blank = weights->multi_blank != 0;
    if (multi_blank && weights->n_dur < 1) return TDT_ERR_DURATIONS;
    for (int j = 0; j < weights->n_dur; ++j) {
        if (durations[j] < (multi_blank ? 1 : 0) || durations[j] > kMaxDuration) return TDT_ERR_DURATIONS;
        any_pos |= durations[j] > 0;
    }
    if (!any_pos) return TDT_ERR_DURATIONS;
    int window = 0, n_clusters = 0, joint_tiles = 0, algorithm = TDT_ALG_LABEL_LOOPING;
    int wait_timeout_us = 0, selftest_stall = 0, joint_kernel = TDT_JOINT_AUTO;
    bool reuse_enc_proj = false, on_the_fly = false;
    if (options) {
        window = options->window;
        n_clusters = options->n_clusters;
        reuse_enc_proj = options->reuse_enc_proj != 0;
        joint_tiles = options->joint_tiles;
        algorithm = options->algorithm;
        wait_timeout_us = options->wait_timeout_us;
        selftest_stall = options->selftest_stall;
        if (wait_timeout_us < 0) return TDT_ERR_UNSUPPORTED;
        if (selftest_stall && algorithm != TDT_ALG_FRAME_LOOPING) return TDT_ERR_UNSUPPORTED;
        if (algorithm != TDT_ALG_LABEL_LOOPING && algorithm != TDT_ALG_FRAME_LOOPING) return TDT_ERR_UNSUPPORTED;
        if (algorithm == TDT_ALG_FRAME_LOOPING && state) return TDT_ERR_UNSUPPORTED;
        if (options->projections != TDT_PROJ_PRECOMPUTED && options->projections != TDT_PROJ_ON_THE_FLY)
            return TDT_ERR_UNSUPPORTED;
        on_the_fly = options->projections == TDT_PROJ_ON_THE_FLY;
        if (on_the_fly && (state || reuse_enc_proj || algorithm != TDT_ALG_LABEL_LOOPING)) return TDT_ERR_UNSUPPORTED;
        if (window < 0 || window > kMaxWindow || n_clusters < 0 || joint_tiles < 0 || joint_tiles > 64)
            return TDT_ERR_UNSUPPORTED;
        joint_kernel = options->joint_kernel;
        if (joint_kernel < TDT_JOINT_AUTO || joint_kernel > TDT_JOINT_STREAMING) return TDT_ERR_UNSUPPORTED;
    }
    // the streaming joint pass: one stretch of the reduction, bfloat16, the default loops
    const bool can_stream = weights->dtype == 1 && weights->h_joint <= 1024 &&
                            algorithm == TDT_ALG_LABEL_LOOPING && !on_the_fly;
    if (joint_kernel == TDT_JOINT_STREAMING && !can_stream) return TDT_ERR_UNSUPPORTED;
    bool wide_joint = joint_kernel == TDT_JOINT_STREAMING ||
                      (joint_kernel == TDT_JOINT_AUTO && can_stream && weights->vocab + 1 + weights->n_dur >= 4096);
    const WorkspaceLayout L = workspace_layout(weights, B, T);
    if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255) != 0 || workspace_bytes < L.total)
        return TDT_ERR_WORKSPACE;

    DecodeVariant variant{state != nullptr, algorithm == TDT_ALG_FRAME_LOOPING, on_the_fly, wide_joint};
    int max_grid = decode_max_grid(weights, variant);
    if (max_grid < 1) return TDT_ERR_LAUNCH;
    // the streaming joint pass keeps one softmax partial per row and workgroup of a group, and the
    // decision step reads them with one lane each: at most 64 workgroups a group
    const int min_stream_clusters = (max_grid + 63) / 64;
    if (wide_joint && n_clusters != 0 && n_clusters < min_stream_clusters) {
        if (joint_kernel == TDT_JOINT_STREAMING) return TDT_ERR_UNSUPPORTED;
        wide_joint = false;
        variant.wide_joint = false;
        max_grid = decode_max_grid(weights, variant);
        if (max_grid < 1) return TDT_ERR_LAUNCH;
    }
    const int min_clusters = (B + kMaxHypsPerCluster - 1) / kMaxHypsPerCluster;
    if (n_clusters == 0) {
        // Measured on the paper-sized models (B = 1 ... 512, 2 ... 16 clusters).  A cluster runs
        // as long as its longest hypothesis and the fewer hypotheses it holds the shorter its
        // joint passes, so more clusters pay -- until a cluster has too few workgroups to give
        // each at most four column tiles of the predictor-side products (two weight batches per
        // wavefront); `fit` is the cluster count at which that holds.  Small batches: two
        // to four clusters.  An LSTM predictor: `fit`; from about 14 hypotheses per cluster of eight on,
        // where the row tiles are full either way, eight.  A stateless predictor: see below.
        const bool lstm = weights->pred_kind == TDT_PRED_LSTM;
        const int nt_a = (weights->h_joint + 15) / 16, nt_b = lstm ? (weights->h_pred + 3) / 4 : 0;
        const int q4 = (nt_a + 3) / 4 + (nt_b + 3) / 4;
        int fit = (2 * max_grid + q4) / (2 * q4);   // max_grid / q4, rounded
        if (fit < 1) fit = 1;
        if (B < 16 && lstm) {
            // two groups also for a single hypothesis (half the workgroups synchronise faster),
            // four from four hypotheses on (3 to 8 % faster than two at B = 4 ... 12)
            n_clusters = B < 4 ? 2 : (fit < 4 ? fit : 4);
            if (n_clusters < 2) n_clusters = 2;
        } else if (lstm) {
            n_clusters = fit;
            if (fit < 8 && B >= 14 * 8) n_clusters = 8;
        } else {
            // no predictor-side phase, no matrix but the output layer's: small groups.  Two
            // hypotheses a group up to 28 groups (nine workgroups a group: still one work item of
            // a joint pass each), from about 140 hypotheses on five a group, at most 64 groups
            // (measured on the stateless benchmark model, B = 16 ... 512)
            n_clusters = B / 2;
            if (n_clusters > 28) n_clusters = B / 5 > 28 ? B / 5 : 28;
            if (n_clusters > 64) n_clusters = 64;
            if (n_clusters < 2) n_clusters = 2;
        }
        if (n_clusters > B && B > 1) n_clusters = B;
        if (n_clusters < min_clusters) n_clusters = min_clusters;
        if (wide_joint) {
            // the streaming joint pass: a group's pass lasts as long as its workgroups need for the
            // output matrix, whatever the number of rows up to a full row tile -- groups of one
            // row tile (measured at B = 256: 16 groups 45 ms, 8 groups 51 ms, 4 groups 59 ms)
            const int full = (B + 15) / 16;   // row tiles of 16
            if (n_clusters < full) n_clusters = full < 16 ? full : 16;
            if (n_clusters < min_clusters) n_clusters = min_clusters;
            if (n_clusters < min_stream_clusters) n_clusters = min_stream_clusters;   // some may stay empty
        }
    }
    if (n_clusters < min_clusters || n_clusters > max_grid) return TDT_ERR_UNSUPPORTED;
    // every cluster gets max_grid / n_clusters workgroups; the launch is rounded up to whole
    // rounds of the dies (the kernel leaves the spare slots empty)
    int grid = max_grid / n_clusters * n_clusters;
    if ((grid + kXcds - 1) / kXcds * kXcds <= max_grid) grid = (grid + kXcds - 1) / kXcds * kXcds;

    hipStream_t s = static_cast<hipStream_t>(stream);
    char *ws = static_cast<char *>(workspace);
    float *enc_proj = reinterpret_cast<float *>(ws + L.enc_proj);

    float *emb_gates = reinterpret_cast<float *>(ws + L.emb_gates);
    // A stateless predictor's output depends on the last labels only, so its projection into the
    // joint space (Sec. 3.4) is tabulated per label once per call and the label loop has no
    // predictor-side product left.  (Not with projections on the fly, which is there to measure
    // the arrangement without any precomputation.)
    float *pred_tab = weights->pred_kind == TDT_PRED_STATELESS && !on_the_fly
                          ? reinterpret_cast<float *>(ws + L.pred_tab) : nullptr;
    const PackedLayout PL = packed_layout(weights);
    if (!reuse_enc_proj && weights->dtype == 1) {
        // one launch: the projection, the predictor side's per-label tables, the clearing
        // (projections on the fly: no rows for the projection here)
        if (launch_prepare_bf16(enc, enc_len, on_the_fly ? 0 : B, T, weights, enc_proj, emb_gates, pred_tab, PL,
                                on_the_fly, ws + L.packed, ws + L.zero_begin, L.zero_end - L.zero_begin,
                                reinterpret_cast<long long *>(out_stats), s) != hipSuccess)
            return TDT_ERR_LAUNCH;
    } else {
        // (a call that reuses the projections of an earlier one still gets its own copies of the
        // matrices: the caller vouches for the projections, not for what else the workspace holds)
        if (launch_pack_weights(weights, PL, on_the_fly, ws + L.packed, s) != hipSuccess) return TDT_ERR_LAUNCH;
        if (launch_init(ws + L.zero_begin, L.zero_end - L.zero_begin, reinterpret_cast<long long *>(out_stats),
                        s) != hipSuccess)
            return TDT_ERR_LAUNCH;
    }
    if (!reuse_enc_proj && weights->dtype != 1) {
        if (!on_the_fly && launch_encoder_projection_valid(enc, enc_len, B, T, weights, enc_proj, s) != hipSuccess)
            return TDT_ERR_LAUNCH;
        // first LSTM layer: its input product depends on the label only, so it is a table,
        // stored [label][unit][gate]
        if (weights->pred_kind == TDT_PRED_LSTM &&
            launch_linear(weights->emb, weights->vocab + 1, weights->emb_dim, weights->w_ih[0], weights->emb_dim,
                          4 * weights->h_pred, weights->b_lstm[0], weights->dtype, weights->h_pred, emb_gates,
                          s) != hipSuccess)
            return TDT_ERR_LAUNCH;
        if (pred_tab && launch_pred_tables(weights, pred_tab, s) != hipSuccess) return TDT_ERR_LAUNCH;
    }

    DecodeParams p{};
    p.B = B;
    p.T = T;
    p.d_enc = weights->d_enc;
    p.H = weights->h_joint;
    p.V = weights->vocab;
    p.D = multi_blank ? 0 : weights->n_dur;
    p.VL = multi_blank ? weights->vocab + weights->n_dur : weights->vocab;
    p.multi_blank = multi_blank;
    p.O = weights->vocab + 1 + weights->n_dur;
    p.pred_kind = weights->pred_kind;
    p.pred_layers = weights->pred_layers;
    p.h_pred = weights->h_pred;
    p.emb_dim = weights->emb_dim;
    p.max_symbols = max_symbols;
    p.u_cap = u_cap;
    p.window = window;
    p.joint_tiles = joint_tiles;
    p.n_clusters = n_clusters;
    p.frame_loop = algorithm == TDT_ALG_FRAME_LOOPING;
    p.selftest_stall = selftest_stall != 0;
    p.hyps_per_cluster = (B + n_clusters - 1) / n_clusters;
    for (int j = 0; j < TDT_MAX_DURATIONS; ++j) p.durations[j] = j < weights->n_dur ? durations[j] : 0;
    p.emb = weights->emb;
    for (int l = 0; l < TDT_MAX_LSTM_LAYERS; ++l) {
        p.w_ih[l] = weights->w_ih[l];
        p.w_hh[l] = weights->w_hh[l];
        p.b_lstm[l] = weights->b_lstm[l];
    }
    p.enc = enc;
    p.w_enc = weights->w_enc;
    p.b_enc = weights->b_enc;
    p.w_pred = weights->w_pred;
    p.b_pred = weights->b_pred;
    p.w_out = weights->w_out;
    p.b_out = weights->b_out;
    if (weights->dtype == 1) {   // the kernel multiplies by the fragment-major copies
        const char *pk = ws + L.packed;
        p.w_enc = pk + PL.w_enc.offset;
        p.w_pred = pk + PL.w_pred.offset;
        p.w_out = pk + PL.w_out.offset;
        for (int l = 0; l < TDT_MAX_LSTM_LAYERS; ++l) {
            p.w_ih[l] = pk + PL.w_ih[l].offset;   // (layer 0: not streamed, never read)
            p.w_hh[l] = pk + PL.w_hh[l].offset;
        }
    }
    p.enc_proj = enc_proj;
    p.emb_gates = emb_gates;
    p.pred_tab = pred_tab;
    p.enc_len = enc_len;
    p.out_labels = out_labels;
    p.out_frames = out_frames;
    p.out_len = out_len;
    p.out_status = out_status;
    p.out_score = out_score;
    p.out_stats = reinterpret_cast<long long *>(out_stats);
    if (state) {
        const StateLayout SL = state_layout(weights, B);
        char *sp = static_cast<char *>(state);
        p.st_started = reinterpret_cast<int32_t *>(sp + SL.started);
        p.st_time = reinterpret_cast<int32_t *>(sp + SL.time);
        p.st_last = reinterpret_cast<int32_t *>(sp + SL.last);
        p.st_last2 = reinterpret_cast<int32_t *>(sp + SL.last2);
        p.st_h = reinterpret_cast<float *>(sp + SL.h);
        p.st_c = reinterpret_cast<float *>(sp + SL.c);
    }
    p.hbuf = reinterpret_cast<float *>(ws + L.hbuf);
    p.cbuf = reinterpret_cast<float *>(ws + L.cbuf);
    p.rgate = reinterpret_cast<float *>(ws + L.rgate);
    p.pred_proj = reinterpret_cast<float *>(ws + L.pred_proj);
    p.partials = reinterpret_cast<LsePartial *>(ws + L.partials);
    p.row_lab = reinterpret_cast<unsigned long long *>(ws + L.row_lab);
    p.row_dur = reinterpret_cast<unsigned long long *>(ws + L.row_dur);
    p.rows_per_cluster = p.hyps_per_cluster * kMaxWindow < kMaxRowsPerPass
                             ? p.hyps_per_cluster * kMaxWindow : kMaxRowsPerPass;
    p.barrier = reinterpret_cast<unsigned *>(ws + L.barrier);
    p.abort_flag = reinterpret_cast<int *>(ws + L.abort_flag);
    {
        // bound on a single device-side wait: 4 s of the wall clock the kernel reads
        const int khz = wall_clock_khz();
        p.timeout_ticks = wait_timeout_us > 0 ? (long long)wait_timeout_us * khz / 1000 : 4000LL * khz;
        if (p.timeout_ticks < 1) p.timeout_ticks = 1;
    }
    if (launch_decode(p, weights, variant, grid, s) != hipSuccess) return TDT_ERR_LAUNCH;
    return TDT_OK;
}

int tdt_greedy_decode(const void *enc, const int32_t *enc_len, int B, int T,
                      const tdt_weights_t *weights, const int32_t *durations, int max_symbols,
                      int u_cap, int32_t *out_labels, int32_t *out_frames, int32_t *out_len,
                      float *out_score, int32_t *out_status, int64_t *out_stats, void *workspace,
                      size_t workspace_bytes, const tdt_options_t *options, void *stream)
{
    return decode_common(enc, enc_len, B, T, weights, durations, max_symbols, u_cap, out_labels,
                         out_frames, out_len, out_score, out_status, out_stats, nullptr, workspace,
                         workspace_bytes, options, stream);
}

int tdt_greedy_decode_static(const void *enc, const int32_t *enc_len, int B, int T,
                             const tdt_weights_t *weights, const int32_t *durations, int max_symbols,
                             int u_cap, int32_t *out_labels, int32_t *out_frames, int32_t *out_len,
                             float *out_score, int32_t *out_status, int64_t *out_stats,
                             const tdt_options_t *options, void *stream)
{
    if (!weights) return TDT_ERR_NULL;
    if (B < 1 || T < 1 || u_cap < 1) return TDT_ERR_SHAPE;
    const int st = check_model(weights);
    if (st != TDT_OK) return st;
    // the same layout as a caller's workspace; it has to fit the array the library holds
    const size_t need = workspace_layout(weights, B, T).total;
    if (need > (size_t)TDT_STATIC_SCRATCH_BYTES) return TDT_ERR_TOO_LARGE;
    hipError_t err = hipSuccess;
    void *ptr = static_scratch(&err);
    if (!ptr) return TDT_ERR_LAUNCH;
    // decode_common clears, with a kernel, every part of the workspace that has to start at zero
    return decode_common(enc, enc_len, B, T, weights, durations, max_symbols, u_cap, out_labels,
                         out_frames, out_len, out_score, out_status, out_stats, nullptr, ptr,
                         (size_t)TDT_STATIC_SCRATCH_BYTES, options, stream);
}

int tdt_greedy_decode_chunk(const void *enc, const int32_t *enc_len, int B, int T,
                            const tdt_weights_t *weights, const int32_t *durations, int max_symbols,
                            int u_cap, int32_t *out_labels, int32_t *out_frames, int32_t *out_len,
                            float *out_score, int32_t *out_status, int64_t *out_stats, void *state,
                            void *workspace, size_t workspace_bytes, const tdt_options_t *options,
                            void *stream)
{
    if (!state) return TDT_ERR_NULL;
    if ((reinterpret_cast<uintptr_t>(state) & 255) != 0) return TDT_ERR_WORKSPACE;
    return decode_common(enc, enc_len, B, T, weights, durations, max_symbols, u_cap, out_labels,
                         out_frames, out_len, out_score, out_status, out_stats, state, workspace,
                         workspace_bytes, options, stream);
}

const char *tdt_status_string(int status)
{
    switch (status) {
    case TDT_OK: return "ok";
    case TDT_ERR_NULL: return "a required pointer is NULL";
    case TDT_ERR_SHAPE: return "a size or model dimension is out of range";
    case TDT_ERR_UNSUPPORTED: return "unsupported dtype, predictor or option";
    case TDT_ERR_DURATIONS: return "bad duration list";
    case TDT_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case TDT_ERR_LAUNCH: return "HIP launch or query failed";
    case TDT_ERR_TOO_LARGE: return "sizes beyond the library's own scratch memory";
    case TDT_ERR_ALIGN: return "an input array is not 16-byte aligned";
    default: return "unknown status";
    }
}

}  // extern "C"
