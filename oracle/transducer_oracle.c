/*
 * TEST INFRASTRUCTURE -- not part of the product.
 *
 * Plain, slow, single-precision CPU definition of greedy Transducer / TDT
 * decoding, one utterance at a time, looping over FRAMES (the conventional
 * order of the paper's Algorithm 1).  The label-looping method of the paper
 * (Algorithm 3) is a re-ordering of these loops that must produce the same
 * hypotheses, so this file is "the definition written out": scalar loops, fp32
 * everywhere, no blocking, no batching, no code shared with the GPU library.
 * Only tests, the smoke check and the benchmark's cpu_baseline leg may use it.
 *
 * Model (Sec. 2 "Background" and Sec. 3.4 of the paper; layer shapes from the
 * benchmark configurations):
 *   enc_proj(t) = W_enc * enc[t] + b_enc                          (Sec. 3.4)
 *   dec, state' = predictor(state, last label)     LSTM or stateless embedding
 *   pred_proj   = W_pred * dec + b_pred                           (Sec. 3.4)
 *   logits      = W_out * relu(enc_proj(t) + pred_proj) + b_out
 *   logits[0..V]       label scores, index V = <blank>
 *   logits[V+1..V+D]   TDT duration scores (D = 0 for a plain Transducer)
 *
 * Multi-blank Transducer (related work the paper builds on, Sec. 1; multi_blank
 * != 0): the D extra outputs are "big blank" symbols of the LABEL head, each
 * with a fixed frame increment durations[i] >= 1.  One argmax and one softmax
 * over all V+1+D outputs; a label is emitted as in a plain Transducer (the
 * frame index stays), the standard blank moves on by one frame, big blank i by
 * durations[i] frames; the predictor is stepped on labels only.  Reading: the
 * paper only names the model; the advance rule is the one of Sec. 3.3 with the
 * increment read off the chosen blank symbol instead of a duration head.
 *
 * Readings of points the paper leaves open (each is a stated choice):
 *   - BOS is the blank index V; its embedding row is whatever the caller
 *     supplies (the generators zero it); the initial LSTM state is zero and the
 *     initial stateless context is [BOS, ..., BOS].
 *   - argmax returns the FIRST maximum; label and duration heads are argmaxed
 *     separately (TDT "decouples" token and duration, Sec. 1 / Sec. 3.3).
 *   - TDT: a decision at frame t advances t by the predicted duration whether or
 *     not the token is blank (Sec. 3.3); a blank with duration 0 advances by 1.
 *   - at most S labels may be emitted without the frame index moving; when the
 *     S-th is emitted the frame index is advanced by one.
 *   - score = sum over emitted labels of log_softmax(label logits)[label].
 *   - a hypothesis stops when it holds u_cap labels (status 1).
 *
 * Pins (tests/test_oracle_pins.py): the paper's Fig. 2 alignments and call
 * counts; a dense float64 lattice built from library matrix products; equality
 * with test-side label-looping (Algorithm 3) and batched frame-looping
 * (Algorithm 2) decoders; closed forms with the predictor switched off, with
 * durations {0} and {1}, with an extreme blank bias; row independence and
 * causality; for decoding in chunks, equality with the whole utterance under
 * random, even and frame-by-frame cuts, the figure's example cut in two, and the
 * carried predictor state against a replay of the emitted labels.  Parity unpinned: the score definition, the BOS convention and
 * the joiner's internal shape are readings of points the paper does not fix;
 * the pins check them only against an independent re-statement of the same
 * readings, not against a value the paper prints.
 *
 * All matrices are [out_features][in_features], row-major.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORC_MAX_LAYERS 4
#define ORC_MAX_CTX 2

typedef struct {
    int32_t d_enc, h_joint, vocab, n_dur;
    int32_t pred_kind;   /* 0 = stateless, 1 = LSTM */
    int32_t pred_layers; /* LSTM layers, or stateless context size */
    int32_t h_pred, emb_dim;
    const float *w_enc, *b_enc; /* [H][d_enc], [H] */
    const float *emb;           /* LSTM: [V+1][E]; stateless: [ctx][V+1][E] */
    const float *w_ih[ORC_MAX_LAYERS];   /* [4*Hp][in]  gate order i, f, g, o */
    const float *w_hh[ORC_MAX_LAYERS];   /* [4*Hp][Hp] */
    const float *b_lstm[ORC_MAX_LAYERS]; /* [4*Hp] */
    const float *w_pred, *b_pred;        /* [H][Hp], [H] */
    const float *w_out, *b_out;          /* [V+1+D][H], [V+1+D] */
    int32_t multi_blank;                 /* the D extra outputs are big blanks of the label head */
} orc_model_t;

/* predictor state: LSTM h and c per layer, or the last ctx labels */
typedef struct {
    float *h; /* [layers][Hp] */
    float *c; /* [layers][Hp] */
    int32_t ctx[ORC_MAX_CTX];
} orc_state_t;

/* ------------------------------------------------------------------------ */
/* primitives                                                                */
/* ------------------------------------------------------------------------ */

/* y = W x + b, every output a plain left-to-right sum */
static void linear(const float *W, const float *b, const float *x, int n_out, int n_in, float *y)
{
    for (int o = 0; o < n_out; ++o) {
        const float *w = W + (size_t)o * n_in;
        float acc = 0.0f;
        for (int k = 0; k < n_in; ++k) acc += w[k] * x[k];
        y[o] = b ? acc + b[o] : acc;
    }
}

static float sigmoidf_(float x) { return 1.0f / (1.0f + expf(-x)); }

int orc_state_floats(const orc_model_t *m)
{
    return m->pred_kind == 1 ? 2 * m->pred_layers * m->h_pred : 0;
}

static orc_state_t state_alloc(const orc_model_t *m)
{
    orc_state_t s;
    int n = m->pred_kind == 1 ? m->pred_layers * m->h_pred : 1;
    s.h = (float *)calloc((size_t)n, sizeof(float));
    s.c = (float *)calloc((size_t)n, sizeof(float));
    for (int i = 0; i < ORC_MAX_CTX; ++i) s.ctx[i] = m->vocab; /* BOS */
    return s;
}

static void state_free(orc_state_t *s)
{
    free(s->h);
    free(s->c);
}

/*
 * The predictor's output as a function of its state alone: the concatenated
 * embeddings of the context labels (stateless), or the top layer's h (LSTM).
 */
static void predictor_output(const orc_model_t *m, const orc_state_t *s, float *dec)
{
    const int Hp = m->h_pred, E = m->emb_dim, V1 = m->vocab + 1;
    if (m->pred_kind == 0) {
        for (int i = 0; i < m->pred_layers; ++i) {
            const float *row = m->emb + ((size_t)i * V1 + s->ctx[i]) * E;
            for (int k = 0; k < E; ++k) dec[i * E + k] = row[k];
        }
    } else {
        const float *top = s->h + (size_t)(m->pred_layers - 1) * Hp;
        for (int n = 0; n < Hp; ++n) dec[n] = top[n];
    }
}

/*
 * One predictor call (Algorithm 1, "dec, new_state = predictor(state, label)").
 * The state is updated in place: callers invoke it only when the new state is
 * to be kept (after BOS and after every non-blank label), which is the same
 * function as Algorithm 1's "compute always, commit on non-blank".
 */
static void predictor_step(const orc_model_t *m, orc_state_t *s, int label, float *dec,
                           float *scratch /* [4*Hp] */)
{
    const int Hp = m->h_pred, E = m->emb_dim;
    if (m->pred_kind == 0) {
        const int ctx = m->pred_layers;
        for (int i = 0; i + 1 < ctx; ++i) s->ctx[i] = s->ctx[i + 1];
        s->ctx[ctx - 1] = label;
        predictor_output(m, s, dec);
        return;
    }
    float *gates = scratch; /* [4*Hp] */
    const float *x = m->emb + (size_t)label * E;
    int in_dim = E;
    for (int l = 0; l < m->pred_layers; ++l) {
        float *h = s->h + (size_t)l * Hp, *c = s->c + (size_t)l * Hp;
        for (int r = 0; r < 4 * Hp; ++r) {
            const float *wi = m->w_ih[l] + (size_t)r * in_dim;
            const float *wh = m->w_hh[l] + (size_t)r * Hp;
            float a = 0.0f, q = 0.0f;
            for (int k = 0; k < in_dim; ++k) a += wi[k] * x[k];
            for (int k = 0; k < Hp; ++k) q += wh[k] * h[k];
            gates[r] = (a + q) + m->b_lstm[l][r];
        }
        for (int n = 0; n < Hp; ++n) {
            float ig = sigmoidf_(gates[n]);
            float fg = sigmoidf_(gates[Hp + n]);
            float gg = tanhf(gates[2 * Hp + n]);
            float og = sigmoidf_(gates[3 * Hp + n]);
            float cn = fg * c[n] + ig * gg;
            c[n] = cn;
            h[n] = og * tanhf(cn);
        }
        x = h;
        in_dim = Hp;
    }
    predictor_output(m, s, dec);
}

static void joint_logits(const orc_model_t *m, const float *enc_proj, const float *pred_proj,
                         float *hid, float *logits)
{
    const int H = m->h_joint;
    for (int k = 0; k < H; ++k) {
        float v = enc_proj[k] + pred_proj[k];
        hid[k] = v > 0.0f ? v : 0.0f;
    }
    linear(m->w_out, m->b_out, hid, m->vocab + 1 + m->n_dur, H, logits);
}

/* first maximum of x[0..n); *margin = max - second largest (INFINITY if n == 1) */
static int argmax_margin(const float *x, int n, float *margin)
{
    int best = 0;
    float vb = x[0], v2 = -INFINITY;
    for (int i = 1; i < n; ++i) {
        if (x[i] > vb) {
            v2 = vb;
            vb = x[i];
            best = i;
        } else if (x[i] > v2) {
            v2 = x[i];
        }
    }
    if (margin) *margin = (n > 1) ? vb - v2 : INFINITY;
    return best;
}

static float logsumexp(const float *x, int n)
{
    float mx = x[0];
    for (int i = 1; i < n; ++i)
        if (x[i] > mx) mx = x[i];
    float s = 0.0f;
    for (int i = 0; i < n; ++i) s += expf(x[i] - mx);
    return mx + logf(s);
}

/* ------------------------------------------------------------------------ */
/* primitives exported for the test-side re-orderings of the loops           */
/* ------------------------------------------------------------------------ */
void orc_enc_proj_frame(const orc_model_t *m, const float *enc_t, float *out)
{
    linear(m->w_enc, m->b_enc, enc_t, m->h_joint, m->d_enc, out);
}

/* state_buf: [2*layers*Hp] floats (h then c) for LSTM; ctx: [ORC_MAX_CTX] labels */
void orc_predictor_step(const orc_model_t *m, float *state_buf, int32_t *ctx, int label,
                        float *dec)
{
    orc_state_t s;
    const int n = m->pred_kind == 1 ? m->pred_layers * m->h_pred : 0;
    s.h = state_buf;
    s.c = state_buf ? state_buf + n : NULL;
    for (int i = 0; i < ORC_MAX_CTX; ++i) s.ctx[i] = ctx[i];
    float *scratch = (float *)malloc(sizeof(float) * (size_t)(5 * m->h_pred + 1));
    predictor_step(m, &s, label, dec, scratch);
    free(scratch);
    for (int i = 0; i < ORC_MAX_CTX; ++i) ctx[i] = s.ctx[i];
}

void orc_pred_proj(const orc_model_t *m, const float *dec, float *out)
{
    linear(m->w_pred, m->b_pred, dec, m->h_joint, m->h_pred, out);
}

void orc_joint(const orc_model_t *m, const float *enc_proj, const float *pred_proj, float *logits)
{
    float *hid = (float *)malloc(sizeof(float) * (size_t)m->h_joint);
    joint_logits(m, enc_proj, pred_proj, hid, logits);
    free(hid);
}

/* ------------------------------------------------------------------------ */
/* the definition: frame-looping greedy decoding of one utterance            */
/* ------------------------------------------------------------------------ */
typedef struct {
    int32_t cap;       /* capacity of the arrays below (0 = no trace) */
    int32_t n;         /* decisions recorded */
    int32_t *t, *u;    /* frame and number of labels already emitted */
    int32_t *k, *j;    /* label decision, duration-class decision (-1 if D == 0) */
    float *margin_lab; /* top-2 margin of the label head */
    float *margin_dur; /* top-2 margin of the duration head (INFINITY if D < 2) */
} orc_trace_t;

/*
 * What one utterance carries from one chunk of its frames to the next when it
 * is decoded piece by piece (an extension beyond the paper, defined by one
 * requirement: decoding the chunks in order gives the hypothesis of decoding
 * their concatenation, with frame indices counted from each chunk's start).
 * All zero = nothing decoded yet.
 */
typedef struct {
    int32_t started; /* the start-of-sequence predictor call has been made */
    int32_t time;    /* frames of the next chunk already stepped over (a TDT duration
                        can reach past the end of a chunk) */
    int32_t ctx[ORC_MAX_CTX]; /* stateless predictor: its context labels, oldest first */
    float *h, *c;    /* LSTM: [layers][Hp] each (unused for a stateless predictor) */
} orc_stream_t;

/*
 * Returns the status: 0 = complete, 1 = stopped at u_cap labels.
 * enc: [len or more][d_enc].  durations: [n_dur] frame increments, NULL if n_dur == 0.
 * out_durs may be NULL.  counts (may be NULL): [0] predictor calls, [1] joint calls.
 * stream == NULL: a whole utterance.  Otherwise the frames are the next chunk of
 * a longer utterance: decoding continues from *stream, which is updated.  The
 * start-of-sequence call is made in the first chunk that has a frame to look at.
 * The symbols-per-frame counter is never carried: a chunk ends by moving past
 * its last frame, which resets it.  A hypothesis stopped at u_cap loses the rest
 * of its chunk.
 */
static int decode_frames(const orc_model_t *m, const float *enc, int len, const int32_t *durations,
                         int max_symbols, int u_cap, int32_t *out_labels, int32_t *out_frames,
                         int32_t *out_durs, int32_t *out_len, float *out_score, orc_trace_t *trace,
                         int64_t *counts, orc_stream_t *stream)
{
    const int H = m->h_joint, V = m->vocab, D = m->n_dur, O = V + 1 + D;
    const int MB = m->multi_blank != 0;
    const int NL = MB ? O : V + 1; /* outputs of the label head */
    float *enc_proj = (float *)malloc(sizeof(float) * (size_t)H);
    float *pred_proj = (float *)malloc(sizeof(float) * (size_t)H);
    float *hid = (float *)malloc(sizeof(float) * (size_t)H);
    float *dec = (float *)malloc(sizeof(float) * (size_t)m->h_pred);
    float *logits = (float *)malloc(sizeof(float) * (size_t)O);
    float *scratch = (float *)malloc(sizeof(float) * (size_t)(5 * m->h_pred + 1));
    orc_state_t st = state_alloc(m);
    int64_t n_pred = 0, n_joint = 0;
    int status = 0, t = 0, sym = 0, n_hyp = 0, t_proj = -1;
    float score = 0.0f;
    if (trace) trace->n = 0;

    const int n_state = m->pred_kind == 1 ? m->pred_layers * m->h_pred : 0;
    int started = 1;
    if (stream) {
        t = stream->time;
        started = stream->started;
        if (started) { /* take up the predictor where the last chunk left it */
            memcpy(st.h, stream->h, sizeof(float) * (size_t)n_state);
            memcpy(st.c, stream->c, sizeof(float) * (size_t)n_state);
            for (int i = 0; i < ORC_MAX_CTX; ++i) st.ctx[i] = stream->ctx[i];
            predictor_output(m, &st, dec);
        } else if (t < len) {
            started = 1;
        }
    }
    if (!stream || (!stream->started && started)) {
        /* BOS call; its state is kept */
        predictor_step(m, &st, V, dec, scratch);
        ++n_pred;
    }
    if (started) linear(m->w_pred, m->b_pred, dec, H, m->h_pred, pred_proj);

    while (t < len && u_cap > 0) {
        if (t_proj != t) { /* same value for every visit of frame t */
            linear(m->w_enc, m->b_enc, enc + (size_t)t * m->d_enc, H, m->d_enc, enc_proj);
            t_proj = t;
        }
        joint_logits(m, enc_proj, pred_proj, hid, logits);
        ++n_joint;
        float mk = INFINITY, mj = INFINITY;
        const int k = argmax_margin(logits, NL, &mk);
        int j = -1, d;
        if (MB) { /* the chosen symbol says how far to move */
            d = (k < V) ? 0 : (k == V ? 1 : durations[k - V - 1]);
            if (k > V && d < 1) d = 1;
        } else if (D > 0) {
            j = argmax_margin(logits + V + 1, D, &mj);
            d = durations[j];
        } else {
            d = (k == V) ? 1 : 0;
        }
        if (trace && trace->n < trace->cap) {
            const int i = trace->n;
            trace->t[i] = t;
            trace->u[i] = n_hyp;
            trace->k[i] = k;
            trace->j[i] = j;
            trace->margin_lab[i] = mk;
            trace->margin_dur[i] = mj;
        }
        if (trace) ++trace->n;
        if (k >= V) { /* the blank, or a big blank */
            if (d == 0) d = 1;
            t += d;
            sym = 0;
        } else {
            out_labels[n_hyp] = k;
            out_frames[n_hyp] = t;
            score += logits[k] - logsumexp(logits, NL);
            ++sym;
            if (d == 0 && sym >= max_symbols) d = 1;
            if (out_durs) out_durs[n_hyp] = d;
            ++n_hyp;
            predictor_step(m, &st, k, dec, scratch);
            ++n_pred;
            linear(m->w_pred, m->b_pred, dec, H, m->h_pred, pred_proj);
            if (d > 0) {
                t += d;
                sym = 0;
            }
            if (n_hyp == u_cap) {
                status = 1;
                break;
            }
        }
    }
    *out_len = n_hyp;
    *out_score = score;
    if (counts) {
        counts[0] = n_pred;
        counts[1] = n_joint;
    }
    if (stream) {
        stream->time = t > len ? t - len : 0;
        if (started) {
            stream->started = 1;
            memcpy(stream->h, st.h, sizeof(float) * (size_t)n_state);
            memcpy(stream->c, st.c, sizeof(float) * (size_t)n_state);
            for (int i = 0; i < ORC_MAX_CTX; ++i) stream->ctx[i] = st.ctx[i];
        }
    }
    state_free(&st);
    free(enc_proj);
    free(pred_proj);
    free(hid);
    free(dec);
    free(logits);
    free(scratch);
    return status;
}

int orc_decode_utt(const orc_model_t *m, const float *enc, int len, const int32_t *durations,
                   int max_symbols, int u_cap, int32_t *out_labels, int32_t *out_frames,
                   int32_t *out_durs, int32_t *out_len, float *out_score, orc_trace_t *trace,
                   int64_t *counts)
{
    return decode_frames(m, enc, len, durations, max_symbols, u_cap, out_labels, out_frames,
                         out_durs, out_len, out_score, trace, counts, NULL);
}

/*
 * The next chunk of every utterance of a batch.  Per-utterance state in arrays:
 * started, time [B]; ctx [B][ORC_MAX_CTX]; h, c [B][layers*Hp] (LSTM only).
 */
int orc_decode_batch_chunk(const orc_model_t *m, const float *enc, const int32_t *enc_len, int B,
                           int T, const int32_t *durations, int max_symbols, int u_cap,
                           int32_t *out_labels, int32_t *out_frames, int32_t *out_len,
                           float *out_score, int32_t *out_status, int32_t *st_started,
                           int32_t *st_time, int32_t *st_ctx, float *st_h, float *st_c,
                           int n_threads)
{
    const size_t n_state = m->pred_kind == 1 ? (size_t)m->pred_layers * m->h_pred : 0;
    int used = 1;
#ifdef _OPENMP
    if (n_threads <= 0) n_threads = omp_get_max_threads();
    used = n_threads < B ? n_threads : B;
    if (used < 1) used = 1;
#pragma omp parallel for schedule(dynamic, 1) num_threads(used)
#endif
    for (int b = 0; b < B; ++b) {
        int len = enc_len[b];
        if (len < 0) len = 0;
        if (len > T) len = T;
        orc_stream_t s;
        s.started = st_started[b];
        s.time = st_time[b];
        for (int i = 0; i < ORC_MAX_CTX; ++i) s.ctx[i] = st_ctx[b * ORC_MAX_CTX + i];
        s.h = st_h + (size_t)b * n_state;
        s.c = st_c + (size_t)b * n_state;
        out_status[b] = decode_frames(
            m, enc + (size_t)b * T * m->d_enc, len, durations, max_symbols, u_cap,
            out_labels + (size_t)b * u_cap, out_frames + (size_t)b * u_cap, NULL, out_len + b,
            out_score + b, NULL, NULL, &s);
        st_started[b] = s.started;
        st_time[b] = s.time;
        for (int i = 0; i < ORC_MAX_CTX; ++i) st_ctx[b * ORC_MAX_CTX + i] = s.ctx[i];
    }
    return used;
}

/*
 * A batch is B independent utterances; threads only split the utterance loop.
 * enc: [B][T][d_enc]; outputs [B][u_cap].  n_threads <= 0: library default.
 * Returns the number of threads used.
 */
int orc_decode_batch(const orc_model_t *m, const float *enc, const int32_t *enc_len, int B, int T,
                     const int32_t *durations, int max_symbols, int u_cap, int32_t *out_labels,
                     int32_t *out_frames, int32_t *out_durs, int32_t *out_len, float *out_score,
                     int32_t *out_status, int64_t *counts /* [B][2] or NULL */, int n_threads)
{
    int used = 1;
#ifdef _OPENMP
    if (n_threads <= 0) n_threads = omp_get_max_threads();
    used = n_threads < B ? n_threads : B;
    if (used < 1) used = 1;
#pragma omp parallel for schedule(dynamic, 1) num_threads(used)
#endif
    for (int b = 0; b < B; ++b) {
        int len = enc_len[b];
        if (len < 0) len = 0;
        if (len > T) len = T;
        out_status[b] = orc_decode_utt(
            m, enc + (size_t)b * T * m->d_enc, len, durations, max_symbols, u_cap,
            out_labels + (size_t)b * u_cap, out_frames + (size_t)b * u_cap,
            out_durs ? out_durs + (size_t)b * u_cap : NULL, out_len + b, out_score + b, NULL,
            counts ? counts + 2 * (size_t)b : NULL);
    }
    return used;
}

/* ------------------------------------------------------------------------ */
/* tolerant validation of a candidate hypothesis                             */
/* ------------------------------------------------------------------------ */
/*
 * Accepts a candidate (labels, frames) for one utterance iff it is a greedy
 * decode under an argmax that may pick any entry within `tol` of the maximum
 * (label head and duration head independently).  The exact decode is the
 * special case where every choice is the first maximum.  Used only to judge
 * positions where another implementation's rounding order flips a near-tie.
 * Search: depth-first over admissible choices, exact argmax first, visited
 * (t, sym, u) states remembered.  *n_tie = choices on the accepted path that
 * were not the exact argmax; *score = score along the accepted path.
 */
#define ORC_MAX_ALT 8

typedef struct {
    const orc_model_t *m;
    const float *enc;
    int len, S, u_cap, cand_len;
    const int32_t *durations, *cand_labels, *cand_frames;
    float tol;
    float *enc_proj_cache; /* [len][H], filled lazily */
    uint8_t *enc_proj_have;
    float *pred_proj_all; /* [cand_len+1][H], teacher forced */
    uint8_t *dead;        /* [(len+1)][S+1][cand_len+1] */
    float *hid, *logits;
    int n_tie;
    float score;
} replay_t;

static size_t dead_index(const replay_t *r, int t, int sym, int u)
{
    return ((size_t)t * (size_t)(r->S + 1) + (size_t)sym) * (size_t)(r->cand_len + 1) + (size_t)u;
}

static int replay_rec(replay_t *r, int t, int sym, int u, float score, int n_tie)
{
    const orc_model_t *m = r->m;
    const int H = m->h_joint, V = m->vocab, D = m->n_dur;
    const int MB = m->multi_blank != 0;
    const int NL = MB ? V + 1 + D : V + 1;
    if (t >= r->len || u >= r->u_cap) {
        if (u == r->cand_len) {
            r->score = score;
            r->n_tie = n_tie;
            return 1;
        }
        return 0;
    }
    if (r->dead[dead_index(r, t, sym, u)]) return 0;
    if (!r->enc_proj_have[t]) {
        linear(m->w_enc, m->b_enc, r->enc + (size_t)t * m->d_enc, H, m->d_enc,
               r->enc_proj_cache + (size_t)t * H);
        r->enc_proj_have[t] = 1;
    }
    joint_logits(m, r->enc_proj_cache + (size_t)t * H, r->pred_proj_all + (size_t)u * H, r->hid,
                 r->logits);
    /* admissible label choices, exact argmax first */
    int ks[ORC_MAX_ALT], nk = 0, js[ORC_MAX_ALT], nj = 0;
    float lk[ORC_MAX_ALT];
    const int k0 = argmax_margin(r->logits, NL, NULL);
    const float lse = logsumexp(r->logits, NL);
    ks[nk] = k0;
    lk[nk++] = r->logits[k0];
    for (int i = 0; i < NL && nk < ORC_MAX_ALT; ++i)
        if (i != k0 && r->logits[i] >= r->logits[k0] - r->tol) {
            ks[nk] = i;
            lk[nk++] = r->logits[i];
        }
    if (D > 0 && !MB) {
        const float *dl = r->logits + V + 1;
        const int j0 = argmax_margin(dl, D, NULL);
        js[nj++] = j0;
        for (int i = 0; i < D && nj < ORC_MAX_ALT; ++i)
            if (i != j0 && dl[i] >= dl[j0] - r->tol) js[nj++] = i;
    } else {
        js[nj++] = -1;
    }
    for (int a = 0; a < nk; ++a) {
        for (int b = 0; b < nj; ++b) {
            const int k = ks[a];
            int d;
            if (MB) {
                d = (k < V) ? 0 : (k == V ? 1 : r->durations[k - V - 1]);
                if (k > V && d < 1) d = 1;
            } else {
                d = (D > 0) ? r->durations[js[b]] : (k == V ? 1 : 0);
            }
            const int tie = n_tie + (a != 0) + (b != 0);
            if (k >= V) {
                if (d == 0) d = 1;
                if (replay_rec(r, t + d, 0, u, score, tie)) return 1;
            } else {
                if (u >= r->cand_len || r->cand_labels[u] != k || r->cand_frames[u] != t)
                    continue;
                int s2 = sym + 1;
                if (d == 0 && s2 >= r->S) d = 1;
                const float sc = score + (lk[a] - lse);
                if (d > 0) {
                    if (replay_rec(r, t + d, 0, u + 1, sc, tie)) return 1;
                } else {
                    if (replay_rec(r, t, s2, u + 1, sc, tie)) return 1;
                }
            }
            /* the recursion overwrote the shared logits; nothing below needs them */
        }
    }
    r->dead[dead_index(r, t, sym, u)] = 1;
    return 0;
}

int orc_replay_utt(const orc_model_t *m, const float *enc, int len, const int32_t *durations,
                   int max_symbols, int u_cap, const int32_t *cand_labels,
                   const int32_t *cand_frames, int cand_len, float tol, int32_t *n_tie,
                   float *score)
{
    const int H = m->h_joint, V = m->vocab, O = V + 1 + m->n_dur;
    if (cand_len < 0 || cand_len > u_cap) return 0;
    for (int i = 0; i < cand_len; ++i)
        if (cand_labels[i] < 0 || cand_labels[i] >= V) return 0;
    replay_t r;
    memset(&r, 0, sizeof(r));
    r.m = m;
    r.enc = enc;
    r.len = len;
    r.S = max_symbols;
    r.u_cap = u_cap;
    r.cand_len = cand_len;
    r.durations = durations;
    r.cand_labels = cand_labels;
    r.cand_frames = cand_frames;
    r.tol = tol;
    r.enc_proj_cache = (float *)malloc(sizeof(float) * (size_t)(len > 0 ? len : 1) * H);
    r.enc_proj_have = (uint8_t *)calloc((size_t)(len > 0 ? len : 1), 1);
    r.pred_proj_all = (float *)malloc(sizeof(float) * (size_t)(cand_len + 1) * H);
    r.dead = (uint8_t *)calloc((size_t)(len + 1) * (size_t)(max_symbols + 1) * (size_t)(cand_len + 1), 1);
    r.hid = (float *)malloc(sizeof(float) * (size_t)H);
    r.logits = (float *)malloc(sizeof(float) * (size_t)O);
    /* teacher-forced predictor outputs: after BOS, after label 0, after label 1, ... */
    {
        orc_state_t st = state_alloc(m);
        float *dec = (float *)malloc(sizeof(float) * (size_t)m->h_pred);
        float *scratch = (float *)malloc(sizeof(float) * (size_t)(5 * m->h_pred + 1));
        for (int u = 0; u <= cand_len; ++u) {
            predictor_step(m, &st, u == 0 ? V : cand_labels[u - 1], dec, scratch);
            linear(m->w_pred, m->b_pred, dec, H, m->h_pred, r.pred_proj_all + (size_t)u * H);
        }
        free(dec);
        free(scratch);
        state_free(&st);
    }
    const int ok = replay_rec(&r, 0, 0, 0, 0.0f, 0);
    if (n_tie) *n_tie = ok ? r.n_tie : -1;
    if (score) *score = ok ? r.score : 0.0f;
    free(r.enc_proj_cache);
    free(r.enc_proj_have);
    free(r.pred_proj_all);
    free(r.dead);
    free(r.hid);
    free(r.logits);
    return ok;
}

/* all logits of one (frame, number-of-labels) lattice node, for dense checks */
void orc_lattice_logits(const orc_model_t *m, const float *enc_t, const int32_t *labels, int u,
                        float *logits)
{
    const int H = m->h_joint, V = m->vocab;
    orc_state_t st = state_alloc(m);
    float *dec = (float *)malloc(sizeof(float) * (size_t)m->h_pred);
    float *scratch = (float *)malloc(sizeof(float) * (size_t)(5 * m->h_pred + 1));
    float *ep = (float *)malloc(sizeof(float) * (size_t)H);
    float *pp = (float *)malloc(sizeof(float) * (size_t)H);
    float *hid = (float *)malloc(sizeof(float) * (size_t)H);
    for (int i = 0; i <= u; ++i) predictor_step(m, &st, i == 0 ? V : labels[i - 1], dec, scratch);
    linear(m->w_pred, m->b_pred, dec, H, m->h_pred, pp);
    linear(m->w_enc, m->b_enc, enc_t, H, m->d_enc, ep);
    joint_logits(m, ep, pp, hid, logits);
    free(dec);
    free(scratch);
    free(ep);
    free(pp);
    free(hid);
    state_free(&st);
}

int orc_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
