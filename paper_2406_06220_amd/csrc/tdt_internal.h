// Internal declarations shared by the translation units of libtdt_decode.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "tdt_decode.h"

namespace tdt {

constexpr int kThreads = 512;                 // threads per workgroup of the decode kernel
constexpr int kWaves = kThreads / 64;         // 64-wide wavefronts per workgroup
constexpr int kMaxGrid = 256;                 // one workgroup per compute unit
constexpr int kMaxHypsPerCluster = 256;       // hypotheses one group of workgroups decodes
constexpr int kMaxRowsPerPass = 1024;         // (hypothesis, frame) rows of one joint pass
constexpr int kMaxColGroups = 64;             // output-column slices of one joint pass
constexpr int kMaxWindow = 64;                // frames of one hypothesis per joint pass
constexpr int kPartialEntries = kMaxRowsPerPass * kMaxGrid;  // per partial buffer
constexpr int kXcds = 8;                      // accelerator dies of an MI355X; workgroups are dealt to them in turn
constexpr int kBarrierStride = 32;            // uint32 slots between two workgroups' barrier flags
constexpr int kMaxRankedBatch = 1024;          // largest batch whose hypotheses are dealt to the clusters by length
constexpr int kMaxDuration = 1 << 20;          // largest frame increment of a duration class
constexpr int kRowBufs = 4;                   // rotating per-row argmax buffers

// Softmax-denominator share of one slice of label columns for one joint row.
struct __align__(8) LsePartial {
    float max_lab;   // largest label logit in the slice
    float sumexp;    // sum of exp(logit - max_lab) over the slice (0 if it has no label column)
};
static_assert(sizeof(LsePartial) == 8, "LsePartial must be 8 bytes");

struct DecodeParams {
    // sizes
    int B, T, d_enc, H, V, D, O;   // D: outputs of the duration head (0 for a multi-blank model)
    int VL;                // last output of the label head: V, or V + number of big blanks
    int multi_blank;       // the outputs V+1 .. VL are big blanks with the increments in durations[]
    int pred_kind, pred_layers, h_pred, emb_dim;
    int max_symbols, u_cap;
    int window;            // 0 = automatic
    int joint_tiles;       // column tiles per joint work item the automatic window aims at (0 = automatic: 4 to 8)
    int kseg_max;          // longest K segment staged at once (set by launch_decode)
    int lds_bytes;         // dynamic LDS of the launch, a multiple of 16 (set by launch_decode)
    int n_clusters, hyps_per_cluster;
    int frame_loop;        // non-zero: batched frame-looping (Algorithm 2) instead of label-looping
    int selftest_stall;    // non-zero: rank 0 of cluster 0 withholds its first barrier arrival
    int durations[TDT_MAX_DURATIONS];
    // weights
    const void *w_enc;       // [H][d_enc]   (read by the kernel only when it projects on the fly)
    const float *b_enc;
    const void *emb;
    const void *w_ih[TDT_MAX_LSTM_LAYERS], *w_hh[TDT_MAX_LSTM_LAYERS];
    const float *b_lstm[TDT_MAX_LSTM_LAYERS];
    const void *w_pred;
    const float *b_pred;
    const void *w_out;
    const float *b_out;
    // inputs
    const void *enc;         // [B][T][d_enc]   (read by the kernel only when it projects on the fly)
    float *enc_proj;         // [B][T][H]; on the fly: written row by row as joint passes need them
    const float *emb_gates;  // [V+1][h_pred][4 gates]: w_ih[0] * emb[label] + b_lstm[0] (LSTM only)
    const float *pred_tab;   // [ctx][V+1][H]: projected predictor output per label and context position
                             // (stateless predictor with precomputed projections only, else null)
    const int32_t *enc_len;  // [B]
    // outputs
    int32_t *out_labels, *out_frames, *out_len, *out_status;
    float *out_score;
    long long *out_stats;    // may be null
    // state carried between the chunks of longer utterances; all null for whole utterances
    int32_t *st_started, *st_time, *st_last, *st_last2;   // [B] each
    float *st_h, *st_c;      // [layers][B][h_pred] (LSTM only)
    // workspace
    float *hbuf;             // [2][layers][B][h_pred]  ping-pong hidden state
    float *cbuf;             // [layers][B][h_pred]
    float *rgate;            // [B][h_pred][4]: W_hh[0] . h of the first layer, for its next step
    float *pred_proj;        // [B][H]
    LsePartial *partials;    // [2][kPartialEntries]
    unsigned long long *row_lab;  // [n_clusters][kRowBufs][rows_per_cluster] packed (logit, ~label)
    unsigned long long *row_dur;  // same shape, packed (logit, ~duration class)
    int rows_per_cluster;
    unsigned *barrier;       // one flag word per workgroup, a cluster's flags side by side
    int *abort_flag;
    long long timeout_ticks; // bound on one wait, in wall-clock ticks
};

struct WorkspaceLayout {
    size_t packed;                 // the bfloat16 matrices the decode kernel streams, fragment by fragment
    size_t enc_proj, emb_gates, pred_tab, hbuf, cbuf, rgate, pred_proj, partials, row_lab, row_dur, barrier, abort_flag, total;
    size_t row_entries;            // uint64 entries in each of row_lab / row_dur
    size_t zero_begin, zero_end;   // byte range the init kernel clears
};

WorkspaceLayout workspace_layout(const tdt_weights_t *w, int B, int T);

// the caller-held state of tdt_greedy_decode_chunk: byte offsets of its arrays
struct StateLayout {
    size_t started, time, last, last2, h, c, total;
};
StateLayout state_layout(const tdt_weights_t *w, int B);

// launches (each returns a hipError_t)
hipError_t launch_encoder_projection(const void *enc, int64_t rows, const tdt_weights_t *w,
                                     float *out, hipStream_t stream);
// out[r][c(n)] = sum_k a[r][k] * w[n * ldw + k] + bias[n] (bias may be null); a and w in the
// model's dtype, out float32.  c(n) = n, or with group > 0 (N a multiple of group):
// c(n) = (n % group) * (N / group) + n / group, which puts the N / group outputs n, n + group,
// n + 2 group, ... side by side.
hipError_t launch_linear(const void *a, int64_t rows, int K, const void *w, int ldw, int N, const float *bias,
                         int dtype, int group, float *out, hipStream_t stream);
// bf16 models: encoder projection, the predictor side's per-label tables (first LSTM layer's
// input product into emb_gates; a stateless predictor's projected output into pred_tab, which may
// be null: then none) and the clearing of the zero region in one launch
// (the projection covers frames t < enc_len[b] of each of the B utterances only; B == 0: none)

// the encoder projection of the valid frames of B utterances (any dtype)
hipError_t launch_encoder_projection_valid(const void *enc, const int32_t *enc_len, int B, int T,
                                           const tdt_weights_t *w, float *out, hipStream_t stream);
// stateless predictor: pred_tab[c][label][:] = w_pred[:, c*E .. (c+1)*E) * emb_c[label] (+ b_pred
// in the last table), one launch per table
hipError_t launch_pred_tables(const tdt_weights_t *w, float *pred_tab, hipStream_t stream);
// Fragment-major copies of the bfloat16 weight matrices the decode kernel multiplies by.
// A matrix [N][K] (row-major) is cut into column tiles of 16 rows of it and steps of 32 inputs;
// fragment (tile, step) is 1 KiB, lane l's 16 bytes at l * 16: inputs step * 32 + (l / 16) * 8 .. + 7
// of the tile's row l % 16 -- what lane l feeds the matrix core -- zeros where the matrix ends.
// Fragments of a tile follow each other by step.  A wavefront's fragment load is then one
// contiguous KiB; from the row-major matrix it is 16 pieces of 64 bytes from 16 rows, which
// the texture addresser takes four times as long over.
// Row of a tile: plain tile*16 + j; for LSTM gate matrices (gate-major [4][h][K]) a tile is
// 4 hidden units x 4 gates: row (j % 4) * h + tile * 4 + j / 4.
struct PackedMatrix {
    size_t offset;   // bytes from the start of the packed region
    int tiles, steps;
};
struct PackedLayout {
    PackedMatrix w_enc, w_pred, w_out, w_ih[TDT_MAX_LSTM_LAYERS], w_hh[TDT_MAX_LSTM_LAYERS];
    size_t total;
};
PackedLayout packed_layout(const tdt_weights_t *w);
hipError_t launch_pack_weights(const tdt_weights_t *w, const PackedLayout &pl, bool on_the_fly, void *packed,
                               hipStream_t stream);
// (the same copies as part of the one launch that prepares a call)
hipError_t launch_prepare_bf16(const void *enc, const int32_t *enc_len, int B, int T, const tdt_weights_t *w,
                               float *enc_proj, float *emb_gates, float *pred_tab, const PackedLayout &pl,
                               bool on_the_fly, void *packed, void *zero_begin, size_t zero_bytes,
                               long long *out_stats, hipStream_t stream);
hipError_t launch_init(void *zero_begin, size_t zero_bytes, long long *out_stats,
                       hipStream_t stream);
// which compiled form of the decode kernel a call runs
struct DecodeVariant {
    bool chunked;      // tdt_greedy_decode_chunk
    bool frame_loop;   // TDT_ALG_FRAME_LOOPING
    bool on_the_fly;   // TDT_PROJ_ON_THE_FLY
    bool wide_joint;   // the joint pass streams the output matrix (TDT_JOINT_STREAMING)
};
hipError_t launch_decode(const DecodeParams &p, const tdt_weights_t *w, DecodeVariant v, int grid,
                         hipStream_t stream);
// largest grid the decode kernel can run with all workgroups resident, 0 on error
int decode_max_grid(const tdt_weights_t *w, DecodeVariant v);
// ticks per millisecond of the device wall clock the kernels read (100000 if the query fails)
int wall_clock_khz();

}  // namespace tdt
