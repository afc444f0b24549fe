/*
 * tdt_decode.h -- C ABI of the label-looping greedy decoder for Transducer and
 * Token-and-Duration Transducer (TDT) models on one AMD MI355X (gfx950).
 *
 * The library implements the paper's Algorithm 3 ("Label-looping Algorithm",
 * Sec. 3.2), its TDT variant (Sec. 3.3) and the precomputed encoder / predictor
 * projections (Sec. 3.4) as hand-written HIP kernels.  The label loop and the
 * frame loop are controlled on the device; a call enqueues work on the caller's
 * stream and returns without synchronising.
 *
 * Conventions
 *   - every pointer marked DEVICE is device memory owned by the caller; the
 *     library allocates nothing, keeps no state between calls, reads inputs and
 *     weights, and writes only outputs, the workspace and -- in the chunk-by-chunk
 *     call -- the state buffer the caller passes;
 *   - every matrix is [out_features][in_features], row-major; enc, the matrices, embedding
 *     tables and biases of the model and the output of the projection calls start at
 *     16-byte boundaries (rows are read and written 16 bytes at a time);
 *   - dtype 0: enc, embeddings and weight matrices are float32;
 *     dtype 1: they are bfloat16 (raw 16-bit patterns); biases are float32 in
 *     both cases, and every accumulation and intermediate value is float32;
 *   - labels are 0..V-1, the blank symbol is V, and V is also the start-of-
 *     sequence label fed to the predictor before the first emission;
 *   - functions return 0 on success or a negative tdt_status code; on a negative
 *     return nothing has been enqueued.
 */
#ifndef TDT_DECODE_H
#define TDT_DECODE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define TDT_MAX_LSTM_LAYERS 4
#define TDT_MAX_CONTEXT 2
#define TDT_MAX_DURATIONS 16
/* widest vector a kernel stages per row: d_enc, h_joint, h_pred and
   emb_dim + h_pred must not exceed it; all four dims must be multiples of 8 */
#define TDT_MAX_DIM 2048

enum tdt_status {
    TDT_OK = 0,
    TDT_ERR_NULL = -1,        /* a required pointer is NULL */
    TDT_ERR_SHAPE = -2,       /* B, T, u_cap or max_symbols < 1, or a model dim out of range */
    TDT_ERR_UNSUPPORTED = -3, /* dtype, predictor kind, layer count or option not supported */
    TDT_ERR_DURATIONS = -4,   /* n_dur / durations mismatch, entry outside [0, 2^20], or no positive entry */
    TDT_ERR_WORKSPACE = -5,   /* workspace NULL, misaligned or smaller than tdt_workspace_bytes */
    TDT_ERR_LAUNCH = -6,      /* the HIP runtime refused a launch or a query */
    TDT_ERR_TOO_LARGE = -7,   /* tdt_greedy_decode_static: the sizes need more than TDT_STATIC_SCRATCH_BYTES */
    TDT_ERR_ALIGN = -8        /* enc, a matrix, an embedding table, a bias or a projection output is not 16-byte aligned */
};

enum tdt_pred_kind {
    TDT_PRED_STATELESS = 0, /* dec = concatenated embeddings of the last `pred_layers` labels */
    TDT_PRED_LSTM = 1       /* dec = top hidden state of a `pred_layers`-layer LSTM */
};

/* per-hypothesis bits written to out_status */
#define TDT_HYP_TRUNCATED 1   /* stopped because it reached u_cap labels */
#define TDT_HYP_LEN_CLAMPED 2 /* enc_len[b] was outside [0, T] and was clamped */
#define TDT_HYP_ABORTED 4     /* a bounded device-side wait of this hypothesis' group ran out
                                 (see wait_timeout_us): its outputs are incomplete and, in the
                                 chunk-by-chunk call, its state was left as it was before the call */

/*
 * Model description (Sec. 2 "Background": encoder output, prediction network,
 * joiner; Sec. 3.4: the two projections into the joint space).
 *
 *   enc_proj[b,t] = w_enc * enc[b,t] + b_enc
 *   dec           = predictor(state, last label)
 *   pred_proj     = w_pred * dec + b_pred
 *   logits        = w_out * relu(enc_proj + pred_proj) + b_out
 *   logits[0..V]      label scores (index V = blank)
 *   logits[V+1..V+D]  TDT duration-class scores (n_dur = D; 0 for a Transducer)
 * Multi-blank Transducer (Sec. 1 of the paper, related work; `multi_blank` != 0): the D
 * extra outputs are big-blank symbols of the label head instead.  One argmax and one
 * softmax run over all V+1+D outputs; a label is emitted as in a Transducer (the frame
 * index stays), the blank moves on by one frame, big blank i (output V+1+i) by
 * durations[i] frames -- the advance rule of Sec. 3.3 with the increment read off the
 * chosen symbol.  The predictor sees labels only.
 *
 * LSTM gate order in w_ih / w_hh / b_lstm rows is i, f, g, o (four blocks of
 * h_pred rows); one bias vector per layer.  Layer 0 reads the embedding
 * (emb_dim), every further layer the hidden state of the layer below (h_pred).
 * Stateless predictor: `pred_layers` is the context size c (1 or 2); emb holds c
 * tables [c][V+1][emb_dim]; table c-1 embeds the newest label; h_pred must equal
 * c * emb_dim.  All pointers DEVICE; unused entries may be NULL.
 */
typedef struct {
    int32_t dtype;       /* 0 float32, 1 bfloat16 (see conventions) */
    int32_t d_enc;       /* encoder output width */
    int32_t h_joint;     /* joint hidden width H */
    int32_t vocab;       /* V, number of real labels */
    int32_t n_dur;       /* D, number of duration classes; 0 = plain Transducer */
    int32_t pred_kind;   /* enum tdt_pred_kind */
    int32_t pred_layers; /* LSTM layers (1..4) or stateless context size (1..2) */
    int32_t h_pred;      /* predictor output width */
    int32_t emb_dim;     /* embedding width (per table) */
    const void *w_enc;   /* [h_joint][d_enc] */
    const float *b_enc;  /* [h_joint] */
    const void *emb;     /* LSTM: [V+1][emb_dim]; stateless: [c][V+1][emb_dim] */
    const void *w_ih[TDT_MAX_LSTM_LAYERS];    /* [4*h_pred][emb_dim | h_pred] */
    const void *w_hh[TDT_MAX_LSTM_LAYERS];    /* [4*h_pred][h_pred] */
    const float *b_lstm[TDT_MAX_LSTM_LAYERS]; /* [4*h_pred] */
    const void *w_pred;  /* [h_joint][h_pred] */
    const float *b_pred; /* [h_joint] */
    const void *w_out;   /* [V+1+D][h_joint] */
    const float *b_out;  /* [V+1+D] */
    int32_t multi_blank; /* non-zero: the D extra outputs are big blanks of the label head
                            (needs n_dur >= 1 and every increment >= 1) */
} tdt_weights_t;

/*
 * Tuning knobs; pass NULL for defaults.  None of them changes the decoding rule; the
 * order in which a score's terms are summed, and with it the score's last bits, can
 * differ between settings.
 *   window      frames of one hypothesis scored per joint pass while it searches
 *               for its next non-blank label (the inner loop of Algorithm 3
 *               advances one frame per pass; since the predictor output is fixed
 *               during that loop, several upcoming frames can be scored at once
 *               and the first non-blank taken).  0 = automatic.
 *   n_clusters  the batch is split into this many groups of hypotheses that are
 *               decoded by disjoint sets of workgroups without waiting for each
 *               other.  0 = automatic (by batch size and model shape; see the design notes).
 *   reuse_enc_proj  non-zero: the workspace still holds the encoder projection (and the
 *               first LSTM layer's per-label input table) that an earlier call with the
 *               same enc, B, T and weights left there, and these steps are skipped
 *               (decoding one encoder output again with other settings; timing the
 *               decode kernel on its own).
 *   joint_tiles the automatic window is sized so that one joint pass gives every
 *               workgroup at most one work item of this many 16-column tiles of the
 *               output layer.  0 = automatic (4 in groups of fewer than five hypotheses,
 *               else 8).
 *               Ignored when window > 0.
 *   algorithm   TDT_ALG_LABEL_LOOPING (0, default): Algorithm 3.  TDT_ALG_FRAME_LOOPING:
 *               the conventional batched order the paper compares against (Algorithm 2)
 *               on the same kernels -- every step runs the predictor for every active
 *               hypothesis, scores one frame each, and keeps the new predictor state only
 *               where the step emitted a label.  Same hypotheses as label-looping; kept
 *               to measure what the re-ordering of the loops is worth.  `window` and
 *               `joint_tiles` are ignored; not available for tdt_greedy_decode_chunk.
 *   wait_timeout_us  bound on a single device-side wait of one workgroup for the others
 *               of its group, in microseconds; 0 = 4 seconds.  A wait that runs out sets
 *               TDT_STAT_ABORT and TDT_HYP_ABORTED in the out_status of every hypothesis of
 *               that group, every workgroup leaves the kernel, and those hypotheses are
 *               incomplete.  (A wait only runs out if workgroups of the kernel are
 *               not making progress, e.g. on a device shared with a debugger.)
 *   selftest_stall  non-zero: one workgroup of the first group never announces that it
 *               has arrived, so that the waits of its group run out -- a self-test of
 *               the path above (use a small wait_timeout_us); every workgroup still
 *               leaves the kernel normally.  Honoured with TDT_ALG_FRAME_LOOPING only
 *               (TDT_ERR_UNSUPPORTED otherwise), which keeps the hook out of the default kernels.
 *   projections TDT_PROJ_PRECOMPUTED (0, default): the encoder frames are projected into the
 *               joint space once, before the loops, and a predictor output once per label
 *               (Sec. 3.4).  TDT_PROJ_ON_THE_FLY: the arrangement that section compares
 *               against -- every joint pass first projects the encoder frames and the
 *               predictor outputs of exactly the rows it is about to score.  Same
 *               hypotheses; kept to measure what the precomputation is worth.  Needs
 *               TDT_ALG_LABEL_LOOPING and no reuse_enc_proj; not available for
 *               tdt_greedy_decode_chunk (TDT_ERR_UNSUPPORTED).
 *   joint_kernel  how the joint pass multiplies by the output matrix.  TDT_JOINT_AUTO (0): by the
 *               model's shape.  TDT_JOINT_TILED: work items of a few column tiles each, results
 *               exchanged through LDS per round (the form for output layers of about a thousand
 *               columns).  TDT_JOINT_STREAMING: every wavefront walks column tiles of its own with
 *               many weight fragments in flight and reduces its statistics once per work item
 *               (chosen automatically from 4096 outputs on, where a pass is bound by the rate at
 *               which a compute unit pulls its share of the matrix).  Same hypotheses either way.
 *               Streaming needs bfloat16 weights, h_joint <= 1024, TDT_ALG_LABEL_LOOPING,
 *               TDT_PROJ_PRECOMPUTED and, if n_clusters is given, at least 4 groups
 *               (TDT_ERR_UNSUPPORTED otherwise).
 */
enum tdt_algorithm { TDT_ALG_LABEL_LOOPING = 0, TDT_ALG_FRAME_LOOPING = 1 };
enum tdt_joint_kernel { TDT_JOINT_AUTO = 0, TDT_JOINT_TILED = 1, TDT_JOINT_STREAMING = 2 };
enum tdt_projections { TDT_PROJ_PRECOMPUTED = 0, TDT_PROJ_ON_THE_FLY = 1 };

typedef struct {
    int32_t window;
    int32_t n_clusters;
    int32_t reuse_enc_proj;
    int32_t joint_tiles;
    int32_t algorithm;   /* enum tdt_algorithm */
    int32_t wait_timeout_us;
    int32_t selftest_stall;
    int32_t projections; /* enum tdt_projections */
    int32_t joint_kernel; /* enum tdt_joint_kernel */
} tdt_options_t;

/* counters written to out_stats (int64 each); sums over all hypothesis groups */
enum tdt_stat {
    TDT_STAT_PRED_PASSES = 0, /* batched predictor steps executed (Alg. 3 line 6) */
    TDT_STAT_PRED_ROWS = 1,   /* hypothesis rows those steps updated */
    TDT_STAT_JOINT_PASSES = 2, /* batched joint passes executed (Alg. 3 lines 7 and 13) */
    TDT_STAT_JOINT_ROWS = 3,  /* (hypothesis, frame) rows those passes scored */
    TDT_STAT_OUTER_MAX = 4,   /* largest number of label-loop iterations of any group */
    TDT_STAT_JOINT_PASSES_MAX = 6, /* largest number of joint passes of any group */
    TDT_STAT_ABORT = 5,       /* non-zero if an internal wait timed out (the hypotheses of the groups
                                 concerned carry TDT_HYP_ABORTED in out_status) */
    /* library builds with phase timers only (-DTDT_PHASE_TIMERS=1; zero otherwise, because
       keeping them costs a microsecond or two per label): where the first hypothesis group's
       time went, in ticks of the device wall clock (hipDeviceAttributeWallClockRate):
       predictor, projection, joint, decision, waits, all */
    TDT_STAT_TICKS_PRED = 8,
    TDT_STAT_TICKS_PROJ = 9,
    TDT_STAT_TICKS_JOINT = 10,
    TDT_STAT_TICKS_DECIDE = 11,
    TDT_STAT_TICKS_BARRIER = 12,
    TDT_STAT_TICKS_TOTAL = 13,
    /* library builds with fine timers only (zero otherwise): 9 entries, for each of the
       predictor step, the predictor projection and the joint pass the ticks spent staging
       activations, multiplying, and in epilogues */
    TDT_STAT_TICKS_FINE = 14,
    TDT_STAT_COUNT = 24
};

/*
 * Bytes of DEVICE workspace tdt_greedy_decode needs for this model and these
 * sizes (projected encoder frames [B][T][h_joint] in float32 dominate; a bfloat16
 * model also gets copies of its matrices there, re-ordered for the matrix cores,
 * which every call writes anew: the caller's weights are only read).
 * Host-only computation.  Returns TDT_OK or TDT_ERR_NULL / _SHAPE / _UNSUPPORTED.
 */
int tdt_workspace_bytes(const tdt_weights_t *weights, int B, int T, int u_cap, size_t *bytes);

/*
 * Batched greedy decoding (Algorithm 3; Sec. 3.3 for TDT; Sec. 3.1 for the
 * batched hypothesis arrays the outputs mirror).
 *
 *   enc         DEVICE [B][T][d_enc], dtype per weights->dtype.  Frames at or
 *               beyond enc_len[b] are never read (nor projected: the encoder projection
 *               walks the valid frames only).
 *   enc_len     DEVICE [B] int32 valid frames per utterance; values outside
 *               [0, T] are clamped and flagged in out_status.
 *   durations   HOST [n_dur] frame increments of the duration classes
 *               (e.g. {0,1,2,3,4}), each in [0, 2^20], at least one positive; NULL
 *               iff n_dur == 0.  A blank with increment 0 advances one frame.
 *               Multi-blank models: the increments of the big blanks, each in [1, 2^20].
 *   max_symbols most labels a hypothesis may emit without its frame index moving;
 *               on the max_symbols-th the frame index is advanced by one.
 *   u_cap       label capacity per hypothesis; a hypothesis that reaches it stops
 *               and is flagged TDT_HYP_TRUNCATED.  len*max_symbols always suffices.
 *   out_labels  DEVICE [B][u_cap] int32 emitted labels      (first out_len[b] valid)
 *   out_frames  DEVICE [B][u_cap] int32 frame each label was emitted at
 *   out_len     DEVICE [B] int32
 *   out_score   DEVICE [B] float, sum over emitted labels of
 *               log_softmax(label logits)[label]
 *   out_status  DEVICE [B] int32 TDT_HYP_* bits
 *   out_stats   DEVICE [TDT_STAT_COUNT] int64, or NULL
 *   workspace   DEVICE, 256-byte aligned, >= tdt_workspace_bytes(); contents are
 *               scratch and may be reused by the caller after the stream drains
 *   stream      hipStream_t (NULL = default stream)
 *
 * Calls that share a workspace must not overlap.  Returns TDT_OK once
 * everything is enqueued; outputs are valid after the stream is synchronised.
 *
 * The call allocates nothing and enqueues only kernels (no memset or copy nodes), so it
 * may be recorded into a HIP graph by stream capture and replayed; `durations` and
 * `options` are read when the call is made, i.e. at capture time.
 */
int tdt_greedy_decode(const void *enc, const int32_t *enc_len, int B, int T,
                      const tdt_weights_t *weights, const int32_t *durations, int max_symbols,
                      int u_cap, int32_t *out_labels, int32_t *out_frames, int32_t *out_len,
                      float *out_score, int32_t *out_status, int64_t *out_stats,
                      void *workspace, size_t workspace_bytes, const tdt_options_t *options,
                      void *stream);

/*
 * tdt_greedy_decode for callers that cannot allocate device memory or have none to hand
 * over: code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  The workspace is an array of TDT_STATIC_SCRATCH_BYTES bytes that is part of
 * the library's device image: every GPU the library runs on holds its own copy from the
 * first call on that GPU until the process ends.  The call allocates nothing and frees
 * nothing; everything else -- arguments, outputs, options, error codes, asynchrony -- is
 * tdt_greedy_decode's.
 *
 * Limit: tdt_workspace_bytes(weights, B, T, u_cap) must not exceed
 * TDT_STATIC_SCRATCH_BYTES (64 MiB: e.g. B = 32 utterances of T = 250 frames with a joint
 * width of 640 and a 1024-label LSTM predictor need 37 MB); otherwise TDT_ERR_TOO_LARGE, and
 * nothing is enqueued.  All calls on one GPU share that GPU's array, which still holds what
 * the previous call left there; the call clears, with a kernel on `stream`, every part that
 * has to start at zero.  Calls that overlap on one GPU (different streams, or host threads
 * without ordering between them) race on the array and give undefined results; calls on
 * different GPUs are independent.
 */
#define TDT_STATIC_SCRATCH_BYTES (64u << 20)
int tdt_greedy_decode_static(const void *enc, const int32_t *enc_len, int B, int T,
                             const tdt_weights_t *weights, const int32_t *durations,
                             int max_symbols, int u_cap, int32_t *out_labels, int32_t *out_frames,
                             int32_t *out_len, float *out_score, int32_t *out_status,
                             int64_t *out_stats, const tdt_options_t *options, void *stream);

/*
 * Decoding utterances chunk by chunk (an extension beyond the paper, in the spirit of
 * its device-resident batched hypotheses, Sec. 3.1): the frames of each utterance
 * arrive in pieces, and every call decodes the next piece of all B utterances.  The
 * chunks of an utterance, decoded in order, give the labels of decoding their
 * concatenation with tdt_greedy_decode; out_frames count from the start of each
 * chunk and out_score is the sum over the labels emitted in the chunk.
 *
 * What an utterance carries from chunk to chunk sits in `state`, DEVICE memory of
 * tdt_state_bytes() bytes, 256-byte aligned, owned by the caller, read and
 * updated in place by every call:
 *
 *   int32 started[B]  the start-of-sequence predictor step has been taken (it is
 *                     taken in the first chunk in which the utterance has a frame to look at)
 *   int32 time[B]     frames of the NEXT chunk already stepped over (a TDT duration can
 *                     reach past the end of a chunk); >= 0
 *   int32 last[B]     newest label the predictor has seen, and
 *   int32 last2[B]    the one before (blank index V = none yet)
 *   float h[layers][B][h_pred], c[layers][B][h_pred]      LSTM predictor only
 *
 * each array starting at the next multiple of 256 bytes.  All bytes zero = nothing
 * decoded yet: the caller clears the state (or one utterance's entries in it) to
 * start a new stream.  Rows are independent, so a caller may move an utterance to
 * another batch slot by moving its entries.  The symbols-per-frame counter is not
 * carried: a chunk ends by stepping past its last frame, which resets it.  A
 * hypothesis that fills u_cap within a chunk is flagged TDT_HYP_TRUNCATED and
 * gives up the rest of that chunk; its state is that after its last kept label.
 *
 * All other arguments, the workspace and the error codes are those of
 * tdt_greedy_decode (T, enc_len and u_cap describe the chunk); TDT_ERR_NULL for a
 * NULL state, TDT_ERR_WORKSPACE for a misaligned one.  Calls that share a state
 * must not overlap.
 */
int tdt_state_bytes(const tdt_weights_t *weights, int B, size_t *bytes);
int tdt_greedy_decode_chunk(const void *enc, const int32_t *enc_len, int B, int T,
                            const tdt_weights_t *weights, const int32_t *durations,
                            int max_symbols, int u_cap, int32_t *out_labels, int32_t *out_frames,
                            int32_t *out_len, float *out_score, int32_t *out_status,
                            int64_t *out_stats, void *state, void *workspace,
                            size_t workspace_bytes, const tdt_options_t *options, void *stream);

/*
 * The encoder projection alone (Sec. 3.4, the precomputation at line 2 of
 * Algorithm 3): out[r][:] = w_enc * enc[r][:] + b_enc for r < rows.
 *   enc DEVICE [rows][d_enc] (dtype per weights), out DEVICE [rows][h_joint] float32.
 * Exposed so that the dense contraction can be checked and timed on its own.
 */
int tdt_encoder_projection(const void *enc, int64_t rows, const tdt_weights_t *weights,
                           float *out, void *stream);

/*
 * The same projection as the decode calls run it (Alg. 3 line 2 on utterances of different
 * lengths): enc DEVICE [B][T][d_enc], enc_len DEVICE [B]; out DEVICE [B][T][h_joint] float32, of
 * which only rows t < min(max(enc_len[b], 0), T) are written -- frames beyond an utterance's
 * length are neither read nor written.  B * T must not exceed 2^31.
 */
int tdt_encoder_projection_valid(const void *enc, const int32_t *enc_len, int B, int T,
                                 const tdt_weights_t *weights, float *out, void *stream);

/* Static, human-readable name of a status code. */
const char *tdt_status_string(int status);

#ifdef __cplusplus
}
#endif
#endif /* TDT_DECODE_H */
