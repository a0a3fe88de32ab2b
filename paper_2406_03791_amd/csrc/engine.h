// Internal declarations shared by the host API, the encoder-projection kernel
// and the persistent decode kernel.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "plan.h"

namespace rnnt {

enum Variant { kFrameLooping = 0, kLabelLooping = 1, kTdtLabelLooping = 2 };
// Kernel instance of Algorithm 1 for teams of one utterance (chosen by the launch, never a caller's variant).
constexpr int kFrameLoopingSingle = 3;

// Packed weights of one dense stage on the device.
struct StageDev {
    const float4 *w;       // [rank][wave][slot][step][lane], 16 bytes each: 4 fp32, 8 bf16 or 16 e4m3 weights
    int nks, nsteps, slots, kpad;
    long long rank_stride; // float4 elements per rank
};

// Slots of the per-team statistics record.
enum { kStatPred = 0, kStatJoint = 1, kStatSamples = 2, kStatPolls = 3, kStatCount = 8,
       kStatProf = 24, kStatStride = kStatCount + kStatProf };

struct DecodeParams {
    int F, E, H, L, J, V1, D, blank, NOUT;
    int VT;                 // output columns of the token distribution: V1, plus the big blanks of a multi-blank model
    int durations[kMaxDur]; // TDT: the durations; multi-blank: the spans of the big blanks (output columns V1 ...)
    int B, T, S, cap, variant;
    int wt;                 // WeightType of the packed stages
    int n_teams, team_size, lookahead;
    int search_steps;       // label looping: joint steps per search before the next prediction step (0: no limit)
    int groups, jteam_size; // joint groups per team and work-groups per joint group
    int plain_launch;       // ordinary instead of cooperative launch (engine flag)
    int spread;             // work-group i is rank i % team_size of team i / team_size (else team i % n_teams, rank i / n_teams)
    int serpentine;         // deal length-ranked utterances to teams 0..n-1, n-1..0, ... (else 0..n-1, 0..n-1)
    int xstride;            // floats per activation row in LDS
    int nu_max;             // most hidden units owned by a rank
    int gj_max;             // most joint output groups owned by a rank
    int gp_max;             // most prediction-projection output groups owned by a rank
    // dynamic LDS layout, offsets in floats
    int lds_xz, lds_red, lds_c, lds_part, lds_bias, lds_q;
    int lds_scale;          // scales of e4m3- or e2m1-stored weights (bfloat16 mode), see Lds::s_pred
    int sc_nb_in;           // scale blocks per row of the input stages' tables in LDS
    int rcap;               // rows the LDS state buffers are laid out for (>= rows of any team)
    int rg_planned;         // row groups the activation rows and partial sums in LDS are sized for
    int samples_cap;        // samples of a joint step the z rows and argmax candidates in LDS are sized for
    int fast_pred;          // teams of up to 4 rows: hidden vectors kept in LDS, tagged exchange (no barriers)
    int lds_hc;             // offset of the LDS copies of the hidden vectors [2][L][4][xstride]
    int n_tail;             // joint output columns nout_m .. nout_m + n_tail - 1 are computed by rank 0 .. n_tail - 1 with plain multiply-adds
    int nout_m;             // joint output columns covered by the MFMA stage (NOUT when n_tail == 0)
    int lds_tail;           // offset of a tail column's weight row [J rounded up to 4] and partial sums [waves][kMaxSamples]
    const float *w_tail;    // [n_tail][J rounded up to 4]
    int q_in_lds;           // q = W_pred h + b_pred of the team's rows is kept in LDS
    int qstride;            // floats per q row in LDS
    unsigned lds_bytes;
    unsigned spin_limit;
    const int *enc_len;     // [B]
    const float *P;         // [B, T, J] projected frames
    int *tokens; int *tok_len; int *frames; float *logits; int *durs;
    float *logps;           // [B, cap] log-softmax value of each emitted label, or NULL
    int *done;              // [B] set to 1 once an utterance's outputs are final, or NULL
    StageDev st0;                 // recurrent (h) parts of all layers
    StageDev stl[kMaxLayers];     // input parts of layers 1..L-1 (index = layer)
    StageDev spred;               // prediction-side joint projection
    StageDev sjoint;              // joint output projection
    const float *T0;        // [V1][H][4]: W_ih0 emb[v] + b_ih0 + b_hh0, gates of a unit adjacent
    const float *bias_l;    // [L][H][4]: b_ih + b_hh of layers >= 1 (layer 0 unused)
    const float *b_pred;    // [J]
    const float *b_out;     // [NOUT]
    // e4m3 / e2m1 storage in the bfloat16 mode: the power of two the codes of a weight row (e4m3)
    // or of each block of kScaleBlock weights of a row (e2m1) are multiplied by; nb = scale_blocks_of_matrix
    const float *sc_hh, *sc_ih;   // [L][H][4][nb], as bias_l (sc_ih of layer 0 unused)
    const float *sc_pred;   // [J][nb]
    const float *sc_out;    // [NOUT][nb]
    // team workspace
    float *hbuf;                  // [n_teams][2][L][kMaxRows][H]
    float *qbuf;                  // [n_teams][kMaxRows][J]
    unsigned long long *part;     // [n_teams * groups][2][kMaxSamples][jteam_size] token partial argmax
    unsigned long long *dpart;    // same for durations
    unsigned long long *lpart;    // same layout: a rank's sum of exp(logit - its maximum)
    unsigned long long *rowx;     // [n_teams][2][kMaxRows]: row state published by the owning joint group
    unsigned long long *xh;       // [n_teams][L][kMaxRows][H]: candidate hidden values as (step tag, float bits)
    unsigned long long *xq;       // [n_teams][kMaxRows][J]: q the same way
    unsigned *bar;                // [n_teams * 32]: one counter per team, 128 B apart
    unsigned *abort_flag;
    int *status;
    long long *stats;             // [n_teams][kStatStride]; phase timers after the counters
    int *xcc;                     // [n_teams * team_size]
};

// A call of many utterances takes several launches: the status word starts at zero in the call's
// first launch (zero_status) and the step counts in the first launch that uses their buffer
// (zero_stats); later launches add to them.
hipError_t launch_decode(const DecodeParams &p, bool zero_status, bool zero_stats, hipStream_t stream);

// Keeps the text of a failed HIP call for rnnt_status_string; returns RNNT_ERR_HIP.
int hip_fail(hipError_t e, const char *what);

hipError_t launch_encoder_projection(const float *enc_out, const int *enc_len, const float *w_enc,
                                     const float *b_enc, float *proj, int B, int T, int F, int J,
                                     bool round_x, hipStream_t stream);
// v[i] = nearest bfloat16 value of v[i] (ties to even), in place
hipError_t launch_round_bf16(float *v, long long n, hipStream_t stream);
// T0[v][u][g] = b_ih0[g*H+u] + b_hh0[g*H+u] + sum_e W_ih0[g*H+u][e] * emb[v][e]
hipError_t launch_fold_embedding(const float *emb, const float *w_ih0, const float *b_ih0,
                                 const float *b_hh0, float *T0, int V1, int E, int H,
                                 bool round_bf16, hipStream_t stream);

}  // namespace rnnt
