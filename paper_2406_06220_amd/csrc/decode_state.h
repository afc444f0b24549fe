// Shapes of the tile GEMMs and what a workgroup of the decode kernel keeps in LDS: its replica
// of the per-hypothesis control state (paper Sec. 3.1: the batched hypothesis arrays), the
// scratch of the current work item, and the descriptors a phase hands to the tile code.
// Included by decode.hip only.
#ifndef TDT_DECODE_STATE_H
#define TDT_DECODE_STATE_H

#include "tdt_internal.h"

// Profiling builds.  TDT_PHASE_TIMERS=1: thread 0 of the first hypothesis group books the device
// wall clock per phase (predictor, projection, joint, decision, waits) into the statistics; it
// costs one to two microseconds per label, so the default build leaves the entries at zero.
// TDT_FINE_TIMERS=1 (implies the former): also staging / multiply / epilogue inside each work item.
#ifndef TDT_FINE_TIMERS
#define TDT_FINE_TIMERS 0
#endif
#ifndef TDT_PHASE_TIMERS
#define TDT_PHASE_TIMERS TDT_FINE_TIMERS
#endif

// 1: profiling build.  Thread 0 of workgroup 0 records (event id, device wall clock) pairs of a
// few label-loop iterations into a device array that tdt_debug_trace() copies out -- a time line
// of one workgroup through the phases, their barriers and the steps of a work item.
#ifndef TDT_TRACE
#define TDT_TRACE 0
#endif

#if TDT_TRACE
__device__ long long g_trace[8192];   // [0]: events recorded; then (id << 48) | ticks
namespace tdt {
namespace {
__shared__ int g_tr_n, g_tr_on;
}
}
#define TR(id)                                                                                     \
    do {                                                                                           \
        if (blockIdx.x == 0 && threadIdx.x == 0 && tdt::g_tr_on && tdt::g_tr_n < 8190) {           \
            g_trace[1 + tdt::g_tr_n] = ((long long)(id) << 48) | (wall_clock64() & 0xffffffffffffll); \
            g_trace[0] = ++tdt::g_tr_n;                                                            \
        }                                                                                          \
    } while (0)
#else
#define TR(id) do { } while (0)
#endif

namespace tdt {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;

constexpr int RT = 16;       // activation rows per tile
constexpr int CT = 16;       // weight columns per tile
constexpr int KSEG = 1024;   // longest stretch of the reduction dimension staged at once
constexpr int CP_LD = CT + 1;
constexpr int kDeferPerWave = 4;                     // hypotheses per wavefront whose score term may be deferred
constexpr int kDeferred = kDeferPerWave * kWaves;
constexpr int kTabPerThread = kWaves * RT * CT / kThreads;

// How a joint pass with n searching hypotheses is cut: frames per hypothesis, row tiles, groups
// of column tiles and tiles per group, and the first work item of this workgroup.  A function
// of n only (for fixed options), so it is tabulated once when the kernel starts.
struct JointPlan {
    short Kw, n_tiles, n_cg, ti0;
    int tpg, cg0;
    int rcp_kw;   // ceil(2^20 / Kw)
    int w_lo, w_hi;   // streaming joint pass: this workgroup's range of its die's (row tile, column tile) pairs
};

struct HypShared {
    int gid[kMaxHypsPerCluster];     // the caller's index of the hypothesis in each slot
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
    unsigned char started[kMaxHypsPerCluster];   // the start-of-sequence predictor step is done (chunked decoding)
    unsigned char took_part[kMaxHypsPerCluster]; // was active in this call
    unsigned char hpar[kMaxHypsPerCluster];      // which half of hbuf holds the hypothesis's newest state
    unsigned char commit[kMaxHypsPerCluster];    // frame-looping: the last step emitted a label, so its predictor state is kept
    int act_list[kMaxHypsPerCluster];
    int need_list[kMaxHypsPerCluster];
    int n_act, n_need;
    int t_sync;                      // frame-looping: the frame index the batch is looking at
    int wave_cnt[kWaves], wave_cnt2[kWaves];
    int durations[TDT_MAX_DURATIONS];
    float cpart[kWaves][RT][CP_LD];  // per-wavefront 16x16 partial results of one round
    float bias[kWaves * CT];         // biases of the columns of the current round
    int row_a[kMaxRowsPerPass];      // per joint row: argmax label (V = blank)
    int row_d[kMaxRowsPerPass];      //                frame step of the argmax duration class
    float row_m[kMaxRowsPerPass];    //                largest label logit
    JointPlan jplan[kMaxHypsPerCluster + 1];   // by number of searching hypotheses
    int dec_w[kMaxHypsPerCluster];   // per searching hypothesis: window offset the walk stopped at
    unsigned char dec_found[kMaxHypsPerCluster];   // ... on a non-blank label
    int pend_n, pend_ncg;            // hypotheses whose score term is still in flight
    int pend_g[kDeferred];
    float pend_m[kDeferred];
    unsigned char pend_found[kDeferred];
    int aborted;
    // kept by thread 0 only: work counters and wall-clock ticks per phase
    long long tk[5];   // P, Q, J, D, barrier
    long long tk_last, tk_start;
    // thread 0 (profiling builds): ticks spent staging / multiplying / in epilogues, per phase P, Q, J
    long long tk_fine[3][3];
    int fine_phase;
};

// One stretch of the reduction dimension: `K` inputs, starting at offset k0 of input
// `part` of the phase, multiplied by columns [k0, k0 + K) of the rows of weight matrix
// `w` (row stride wld).  A phase has one or two inputs (the LSTM has the layer input and
// the hidden state); an input longer than KSEG is walked in KSEG pieces.
// One stretch of at most KSEG inputs of a weight matrix.  float32: w is the row-major matrix, wld
// its row length.  bfloat16: w is the fragment-major copy (1 KiB fragments, a tile's fragments in
// order of their step), nst the steps of a whole row.
struct Seg {
    const void *w;
    int wld, k0, K, part, nst;
};

// what the joint pass loads for two inputs of one row: projected encoder frame and
// projected predictor output
struct EncPred {
    float2 e, p;
};
// ... and with a stateless predictor of two labels of context, whose projected output is the sum
// of two table rows
struct EncPred2 {
    float2 e, p, p2;
};
// the same for four inputs (plain 16-byte loads from the per-label tables of a stateless predictor)
struct EncPred4 {
    float4 e, p;
};
struct EncPred4x2 {
    float4 e, p, p2;
};
// where one row of a joint pass reads them (valid false: past the end of the utterance)
struct JointRow {
    const float *enc, *pred, *pred2;
    int g;   // the hypothesis (slot in its group)
    bool valid;
};

// one row of encoder output that a pass projects on the fly
struct EncRow {
    const void *row;
    bool valid;
};

struct PhaseInputs {
    const void *w0, *w1;   // weight matrices of the two inputs (w1 null: one input)
    int K0, K1;
    __device__ int count() const
    {
        return (K0 + KSEG - 1) / KSEG + (w1 ? (K1 + KSEG - 1) / KSEG : 0);
    }
    __device__ Seg get(int i) const   // i < count(); branch-free enough to stay in registers
    {
        const int n0 = (K0 + KSEG - 1) / KSEG;
        const bool first = i < n0;
        Seg s;
        s.part = first ? 0 : 1;
        s.w = first ? w0 : w1;
        s.wld = first ? K0 : K1;
        s.k0 = (first ? i : i - n0) * KSEG;
        s.K = min(KSEG, s.wld - s.k0);
        s.nst = (s.wld + 31) >> 5;
        return s;
    }
};

}  // namespace
}  // namespace tdt

#endif
