/*
 * CPU oracle for exact RNN-T / TDT greedy decoding.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain reference that the
 * HIP decoder is checked against.  It shares no code, header, table or helper
 * with the HIP path, and the product never calls it: only the tests, the
 * smoke check and the benchmark's cpu_baseline leg load this library.
 *
 * What it follows (paper = "Speed of Light Exact Greedy Decoding for RNN-T
 * Speech Recognition Models on GPU"):
 *   - decode_frame_looping : Algorithm 1 in its own order: lock-step frames, an
 *                            inner loop of at most max_symbols batched steps,
 *                            both networks run for the whole batch at every
 *                            step, sticky blank mask, masked state update.
 *   - decode_label_looping : the label-looping schedule described at the end of
 *                            the Related Work section (batch elements advance
 *                            their own frame index); with a duration head it is
 *                            the TDT label-looping decoder of the Results
 *                            section.
 *   - decode_sequential    : the per-utterance definition all schedules must
 *                            reproduce ("exact" in the Introduction: same
 *                            outputs as the baseline for the same inputs).
 *   - follow_sequential    : walks one utterance along a given token sequence
 *                            and reports where it departs from the argmax and
 *                            by how much (parity triage).
 * The paper leaves prediction() and joint() abstract.  Here prediction() is an
 * embedding plus L stacked LSTM cells (standard equations) whose top hidden
 * vector is g, and joint(f, g) = W_out relu(W_enc f + b_enc + W_pred g + b_pred)
 * + b_out.  The argmax is taken on the logits (a log-softmax would not change
 * it); each emission keeps the raw maximum logit (scores) and, when asked
 * for, its log-softmax value over the token columns (logps), which is the
 * score Algorithm 1 saves.
 *
 * A net can be switched to bfloat16 emulation (orc_lstm_net_emulate_bf16: weights
 * and every input of a dense product rounded to bfloat16, everything else as
 * before), the reference of the engine's bfloat16 mode.
 *
 * Arithmetic: every dot product is accumulated one term at a time in index
 * order, in the type REAL (float by default, double with -DREAL=double; build
 * with -ffp-contract=off so no fused multiply-add changes the rounding).
 * exp and tanh are evaluated in double and rounded to REAL.  Weights are
 * transposed once at set-up ([in][out]) so the inner loop runs across outputs;
 * each output still sums its terms in the same order.
 *
 * The encoder-side term W_enc f + b_enc depends only on (utterance, frame), so
 * the batched schedules compute it the first time a frame is used and keep it;
 * re-computing it at every inner step gives the same bits (the per-utterance
 * definition does recompute it per frame, and the schedules are tested to agree
 * with it bit for bit).
 *
 * Pins (tests/test_oracle_*.py): hand-traced lattices, brute force over all
 * tiny argmax tables against a pure-Python lattice walk, all-blank and
 * never-blank closed forms, the paper's B=2 alternating scenario step counts,
 * LSTM / linear numerics against torch CPU ops and a zero-weight closed form,
 * TDT reductions to RNN-T.  A full-size decode's logits have no external pin
 * (the paper prints none): "parity unpinned" for those values, pinned only by
 * the agreement of the independent schedules and the float64 build.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifndef REAL
#define REAL float
#endif
typedef REAL real;

#define ORC_STATUS_LEN_CLAMPED 1
#define ORC_STATUS_OVERFLOW 2
#define ORC_STATUS_REC_OVERFLOW 4

/* ------------------------------------------------------------------------ */
/* The two sub-networks behind a small interface, so that a table-driven net */
/* can stand in for the LSTM one in hand-traced tests.                       */
/* ------------------------------------------------------------------------ */
typedef struct net net_t;
struct net {
    int x_size;      /* reals per encoder frame as given by the caller       */
    int p_size;      /* reals per prepared frame (encoder-side joint term)    */
    int state_size;  /* reals of prediction-network state per utterance       */
    int g_size;      /* reals of prediction-network output                    */
    int V1;          /* vocabulary including blank                            */
    int D;           /* number of durations (0 = RNN-T)                       */
    int blank;       /* blank index, also the start-of-sequence label         */
    const int32_t *durations; /* [D] */
    int NB;          /* multi-blank transducer: number of "big blank" symbols  */
    const int32_t *spans;     /* [NB] frames each big blank advances by        */
    void (*prep)(const net_t *, const real *x_row, real *p_row);
    void (*pred)(const net_t *, int last_label, const real *state_in,
                 real *state_out, real *g);
    void (*joint)(const net_t *, const real *p_row, const real *g, real *logits);
    void *ctx;
};

/* ------------------------------- LSTM net -------------------------------- */
typedef struct {
    int F, E, H, L, J, V1, D;
    const real *emb;          /* [V1][E] as given                            */
    real **w_ih_t;            /* L x [in_l][4H]  transposed copies            */
    real **w_hh_t;            /* L x [H][4H]                                  */
    const real **b_ih;        /* L x [4H]                                     */
    const real **b_hh;        /* L x [4H]                                     */
    real *w_enc_t;            /* [F][J]                                       */
    const real *b_enc;
    real *w_pred_t;           /* [H][J]                                       */
    const real *b_pred;
    real *w_out_t;            /* [J][V1+D]                                    */
    const real *b_out;
    int bf16;                 /* bf16 emulation: see orc_lstm_net_emulate_bf16 */
    real *emb_rounded;        /* owned copy of emb with bf16 values, or NULL   */
} lstm_ctx;

/* Nearest bfloat16 value (8 exponent bits, 7 mantissa bits: the upper half of  */
/* an IEEE float32), ties to even, of a value taken as float32; NaN and         */
/* infinities pass through.                                                     */
static real round_bf16(real v)
{
    float f = (float)v;
    uint32_t u;
    memcpy(&u, &f, sizeof u);
    if ((u & 0x7f800000u) == 0x7f800000u) return (real)f;
    u += 0x7fffu + ((u >> 16) & 1u);
    u &= 0xffff0000u;
    memcpy(&f, &u, sizeof u);
    return (real)f;
}

static real *transpose_copy(const real *w, int n_out, int n_in)
{
    real *t = (real *)malloc(sizeof(real) * (size_t)n_out * (size_t)n_in);
    for (int o = 0; o < n_out; ++o)
        for (int i = 0; i < n_in; ++i)
            t[(size_t)i * n_out + o] = w[(size_t)o * n_in + i];
    return t;
}

/* y[o] = bias[o] + sum_i w[o][i] x[i], terms added in order i = 0, 1, ...    */
/* (two builds of the same loop, picked at load time by the CPU's vector     */
/* width; the per-output order of additions is the same in both)             */
__attribute__((target_clones("avx2", "default")))
static void affine(const real *w_t, const real *bias, const real *x, int n_in,
                   int n_out, real *y)
{
    for (int o = 0; o < n_out; ++o) y[o] = bias[o];
    for (int i = 0; i < n_in; ++i) {
        const real xi = x[i];
        const real *row = w_t + (size_t)i * n_out;
        for (int o = 0; o < n_out; ++o) y[o] += row[o] * xi;
    }
}

/* The same product with every input rounded to bfloat16 first (the weights    */
/* were rounded when the mode was switched on).  A product of two bfloat16      */
/* values is exact in float32, so only the additions round.                     */
static void affine_in(const lstm_ctx *c, const real *w_t, const real *bias, const real *x,
                      int n_in, int n_out, real *y)
{
    if (!c->bf16) { affine(w_t, bias, x, n_in, n_out, y); return; }
    real *xr = (real *)malloc(sizeof(real) * (size_t)(n_in > 0 ? n_in : 1));
    for (int i = 0; i < n_in; ++i) xr[i] = round_bf16(x[i]);
    affine(w_t, bias, xr, n_in, n_out, y);
    free(xr);
}

static real sigmoid_r(real v) { return (real)(1.0 / (1.0 + exp(-(double)v))); }
static real tanh_r(real v) { return (real)tanh((double)v); }

static void lstm_prep(const net_t *n, const real *x_row, real *p_row)
{
    const lstm_ctx *c = (const lstm_ctx *)n->ctx;
    affine_in(c, c->w_enc_t, c->b_enc, x_row, c->F, c->J, p_row);
}

/* state layout per utterance: for each layer l, h_l[H] then c_l[H].          */
static void lstm_pred(const net_t *n, int last_label, const real *state_in,
                      real *state_out, real *g)
{
    const lstm_ctx *c = (const lstm_ctx *)n->ctx;
    const int H = c->H;
    real *a = (real *)malloc(sizeof(real) * 8 * (size_t)H);
    real *b = a + 4 * H;
    const real *in = (c->emb_rounded ? c->emb_rounded : c->emb) + (size_t)last_label * c->E;
    int n_in = c->E;
    for (int l = 0; l < c->L; ++l) {
        const real *h = state_in + (size_t)l * 2 * H;
        const real *cc = h + H;
        real *h2 = state_out + (size_t)l * 2 * H;
        real *c2 = h2 + H;
        affine_in(c, c->w_ih_t[l], c->b_ih[l], in, n_in, 4 * H, a);
        affine_in(c, c->w_hh_t[l], c->b_hh[l], h, H, 4 * H, b);
        for (int j = 0; j < H; ++j) {
            const real gi = sigmoid_r(a[j] + b[j]);
            const real gf = sigmoid_r(a[H + j] + b[H + j]);
            const real gg = tanh_r(a[2 * H + j] + b[2 * H + j]);
            const real go = sigmoid_r(a[3 * H + j] + b[3 * H + j]);
            const real cn = gf * cc[j] + gi * gg;
            c2[j] = cn;
            h2[j] = go * tanh_r(cn);
        }
        in = h2;
        n_in = H;
    }
    memcpy(g, state_out + (size_t)(c->L - 1) * 2 * H, sizeof(real) * (size_t)H);
    free(a);
}

static void lstm_joint(const net_t *n, const real *p_row, const real *g,
                       real *logits)
{
    const lstm_ctx *c = (const lstm_ctx *)n->ctx;
    const int J = c->J;
    real *q = (real *)malloc(sizeof(real) * 2 * (size_t)J);
    real *z = q + J;
    affine_in(c, c->w_pred_t, c->b_pred, g, c->H, J, q);
    for (int j = 0; j < J; ++j) {
        const real s = p_row[j] + q[j];
        z[j] = s > (real)0 ? s : (real)0;
    }
    affine_in(c, c->w_out_t, c->b_out, z, J, c->V1 + c->D, logits);
    free(q);
}

net_t *orc_lstm_net_create(int F, int E, int H, int L, int J, int V1, int D,
                           int blank, const int32_t *durations, const real *emb,
                           const real *const *w_ih, const real *const *w_hh,
                           const real *const *b_ih, const real *const *b_hh,
                           const real *w_enc, const real *b_enc,
                           const real *w_pred, const real *b_pred,
                           const real *w_out, const real *b_out)
{
    net_t *n = (net_t *)calloc(1, sizeof(net_t));
    lstm_ctx *c = (lstm_ctx *)calloc(1, sizeof(lstm_ctx));
    c->F = F; c->E = E; c->H = H; c->L = L; c->J = J; c->V1 = V1; c->D = D;
    c->emb = emb;
    c->w_ih_t = (real **)calloc((size_t)L, sizeof(real *));
    c->w_hh_t = (real **)calloc((size_t)L, sizeof(real *));
    c->b_ih = (const real **)calloc((size_t)L, sizeof(real *));
    c->b_hh = (const real **)calloc((size_t)L, sizeof(real *));
    for (int l = 0; l < L; ++l) {
        c->w_ih_t[l] = transpose_copy(w_ih[l], 4 * H, l == 0 ? E : H);
        c->w_hh_t[l] = transpose_copy(w_hh[l], 4 * H, H);
        c->b_ih[l] = b_ih[l];
        c->b_hh[l] = b_hh[l];
    }
    c->w_enc_t = transpose_copy(w_enc, J, F);
    c->b_enc = b_enc;
    c->w_pred_t = transpose_copy(w_pred, J, H);
    c->b_pred = b_pred;
    c->w_out_t = transpose_copy(w_out, V1 + D, J);
    c->b_out = b_out;
    n->x_size = F; n->p_size = J; n->state_size = 2 * L * H; n->g_size = H;
    n->V1 = V1; n->D = D; n->blank = blank;
    int32_t *dur = (int32_t *)calloc((size_t)(D > 0 ? D : 1), sizeof(int32_t));
    for (int i = 0; i < D; ++i) dur[i] = durations[i];
    n->durations = dur;
    n->prep = lstm_prep; n->pred = lstm_pred; n->joint = lstm_joint;
    n->ctx = c;
    return n;
}

/* bfloat16 emulation (the paper's experiments run bfloat16 models, section on  */
/* the experimental set-up): every weight matrix of a dense product -- the      */
/* embedding table, W_ih and W_hh of every layer, W_enc, W_pred, W_out -- is     */
/* rounded to bfloat16 once, and every vector that enters such a product (an     */
/* encoder frame, an embedding row, a hidden vector, the joint's hidden vector)  */
/* is rounded to bfloat16 at that point.  Products are then exact; sums, biases, */
/* activations and the argmax stay in REAL as before.  This is what a decoder    */
/* with bfloat16 operands and float32 accumulation computes, up to the order of  */
/* the additions.  Not reversible.                                               */
void orc_lstm_net_emulate_bf16(net_t *n)
{
    if (n->prep != lstm_prep) return;
    lstm_ctx *c = (lstm_ctx *)n->ctx;
    if (c->bf16) return;
    c->bf16 = 1;
    for (int l = 0; l < c->L; ++l) {
        const size_t n_ih = (size_t)4 * c->H * (l == 0 ? c->E : c->H), n_hh = (size_t)4 * c->H * c->H;
        for (size_t i = 0; i < n_ih; ++i) c->w_ih_t[l][i] = round_bf16(c->w_ih_t[l][i]);
        for (size_t i = 0; i < n_hh; ++i) c->w_hh_t[l][i] = round_bf16(c->w_hh_t[l][i]);
    }
    for (size_t i = 0; i < (size_t)c->J * c->F; ++i) c->w_enc_t[i] = round_bf16(c->w_enc_t[i]);
    for (size_t i = 0; i < (size_t)c->J * c->H; ++i) c->w_pred_t[i] = round_bf16(c->w_pred_t[i]);
    for (size_t i = 0; i < (size_t)(c->V1 + c->D) * c->J; ++i) c->w_out_t[i] = round_bf16(c->w_out_t[i]);
    c->emb_rounded = (real *)malloc(sizeof(real) * (size_t)c->V1 * c->E);
    for (size_t i = 0; i < (size_t)c->V1 * c->E; ++i) c->emb_rounded[i] = round_bf16(c->emb[i]);
}
real orc_round_bf16(real v) { return round_bf16(v); }

/* Weight-only 8-bit quantisation of a matrix, one power-of-two scale per row    */
/* (the quantised products the paper's conclusion points to, here in the 8-bit    */
/* floating-point format OCP e4m3: 1 sign bit, 4 exponent bits with bias 7, 3      */
/* mantissa bits, subnormals m * 2^-9, no infinities, largest value 448).  For a   */
/* row with largest magnitude M > 0, k is the smallest integer with                 */
/* M * 2^-k <= 448 (kept within +-100; k = 0 for a row of zeros), and each weight   */
/* w becomes 2^k * e, e the e4m3 value nearest to w * 2^-k, a tie going to the      */
/* value with the even code.  Written as a search over the table of the 127         */
/* non-negative e4m3 values.  scales may be NULL.  The result holds bfloat16        */
/* values, so a net built on it and switched to bfloat16 emulation is the           */
/* reference of an engine that stores its weights this way.                         */
void orc_quantize_rows_e4m3(const real *w, long rows, long cols, real *out, real *scales)
{
    double table[127];
    int n = 0;
    for (int code = 0; code < 127; ++code) {        /* code 127 (all ones) is NaN */
        const int expo = code >> 3, mant = code & 7;
        table[n++] = expo == 0 ? ldexp((double)mant, -9) : ldexp(1.0 + mant / 8.0, expo - 7);
    }
    for (long r = 0; r < rows; ++r) {
        const real *row = w + r * cols;
        double M = 0.0;
        for (long i = 0; i < cols; ++i)
            if (fabs((double)row[i]) > M) M = fabs((double)row[i]);
        int k = 0;
        if (M > 0.0) {
            while (k < 100 && ldexp(M, -k) > 448.0) ++k;
            while (k > -100 && ldexp(M, -(k - 1)) <= 448.0) --k;
        }
        for (long i = 0; i < cols; ++i) {
            const double v = ldexp(fabs((double)row[i]), -k);
            int best = 0;
            for (int c = 1; c < 127; ++c) {
                const double d = fabs(v - table[c]), db = fabs(v - table[best]);
                if (d < db || (d == db && (c & 1) == 0)) best = c;
            }
            const double q = ldexp(table[best], k);
            out[r * cols + i] = (real)(row[i] < 0 ? -q : q);
        }
        if (scales) scales[r] = (real)ldexp(1.0, k);
    }
}

/* Weight-only 4-bit quantisation: the same with the 4-bit format OCP e2m1 (1      */
/* sign bit, 2 exponent bits with bias 1, 1 mantissa bit: magnitudes 0, 0.5, 1,    */
/* 1.5, 2, 3, 4, 6 for the codes 0..7) and one power-of-two scale per block of     */
/* `block` consecutive weights of a row (the last block of a row may be shorter):  */
/* k is the smallest integer with max|block| * 2^-k <= 6.  scales, if not NULL,    */
/* is [rows][ceil(cols / block)].                                                  */
void orc_quantize_blocks_e2m1(const real *w, long rows, long cols, long block, real *out,
                              real *scales)
{
    static const double table[8] = {0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0};
    const long nb = (cols + block - 1) / block;
    for (long r = 0; r < rows; ++r)
        for (long b = 0; b < nb; ++b) {
            const long lo = b * block, hi = lo + block < cols ? lo + block : cols;
            double M = 0.0;
            for (long i = lo; i < hi; ++i)
                if (fabs((double)w[r * cols + i]) > M) M = fabs((double)w[r * cols + i]);
            int k = 0;
            if (M > 0.0) {
                while (k < 100 && ldexp(M, -k) > 6.0) ++k;
                while (k > -100 && ldexp(M, -(k - 1)) <= 6.0) --k;
            }
            for (long i = lo; i < hi; ++i) {
                const double v = ldexp(fabs((double)w[r * cols + i]), -k);
                int best = 0;
                for (int c = 1; c < 8; ++c) {
                    const double d = fabs(v - table[c]), db = fabs(v - table[best]);
                    if (d < db || (d == db && (c & 1) == 0)) best = c;
                }
                const double q = ldexp(table[best], k);
                out[r * cols + i] = (real)(w[r * cols + i] < 0 ? -q : q);
            }
            if (scales) scales[r * nb + b] = (real)ldexp(1.0, k);
        }
}

/* ------------------------------ table net -------------------------------- */
/* x_row[0] carries the integer cell index (utterance * T + frame).  The      */
/* prediction state is the number of labels consumed so far; g = (tokens      */
/* emitted so far, last label).  logits = table[cell][u][last][:].            */
typedef struct {
    int U;            /* table extent along "tokens emitted so far"           */
    int V1, n_out;
    const real *table; /* [cells][U][V1][n_out] */
} table_ctx;

static void table_prep(const net_t *n, const real *x_row, real *p_row)
{
    (void)n;
    p_row[0] = x_row[0];
}

static void table_pred(const net_t *n, int last_label, const real *state_in,
                       real *state_out, real *g)
{
    (void)n;
    g[0] = state_in[0];          /* tokens emitted before this evaluation     */
    g[1] = (real)last_label;
    state_out[0] = state_in[0] + (real)1;
}

static void table_joint(const net_t *n, const real *p_row, const real *g,
                        real *logits)
{
    const table_ctx *c = (const table_ctx *)n->ctx;
    const long cell = (long)p_row[0];
    long u = (long)g[0];
    const long last = (long)g[1];
    if (u >= c->U) u = c->U - 1;
    const real *src = c->table + (((size_t)cell * c->U + (size_t)u) * c->V1 +
                                  (size_t)last) * c->n_out;
    memcpy(logits, src, sizeof(real) * (size_t)c->n_out);
}

net_t *orc_table_net_create(int V1, int D, int blank, const int32_t *durations,
                            int U, const real *table)
{
    net_t *n = (net_t *)calloc(1, sizeof(net_t));
    table_ctx *c = (table_ctx *)calloc(1, sizeof(table_ctx));
    c->U = U; c->V1 = V1; c->n_out = V1 + D; c->table = table;
    n->x_size = 1; n->p_size = 1; n->state_size = 1; n->g_size = 2;
    n->V1 = V1; n->D = D; n->blank = blank;
    int32_t *dur = (int32_t *)calloc((size_t)(D > 0 ? D : 1), sizeof(int32_t));
    for (int i = 0; i < D; ++i) dur[i] = durations[i];
    n->durations = dur;
    n->prep = table_prep; n->pred = table_pred; n->joint = table_joint;
    n->ctx = c;
    return n;
}

/* Multi-blank transducer (the paper's related work names it beside TDT as a  */
/* model that lets the decoder skip encoder frames): besides the labels and   */
/* the blank the output layer has NB "big blank" symbols, each with a span of  */
/* m_i frames.  All V1 + NB outputs form one distribution and one argmax.  A   */
/* blank advances the frame index by 1 and a big blank by its span; neither    */
/* is emitted, neither changes the prediction network's input, and both reset  */
/* the count of labels on the frame.  A label is handled as in an RNN-T.       */
/* This call re-reads a net created with D extra output columns: the columns   */
/* become the big blanks and their "durations" the spans; D becomes 0.         */
void orc_net_as_multi_blank(net_t *n)
{
    n->NB = n->D;
    n->spans = n->durations;
    n->D = 0;
}

void orc_net_destroy(net_t *n)
{
    if (!n) return;
    if (n->prep == lstm_prep) {
        lstm_ctx *c = (lstm_ctx *)n->ctx;
        for (int l = 0; l < c->L; ++l) { free(c->w_ih_t[l]); free(c->w_hh_t[l]); }
        free(c->w_ih_t); free(c->w_hh_t); free((void *)c->b_ih); free((void *)c->b_hh);
        free(c->w_enc_t); free(c->w_pred_t); free(c->w_out_t); free(c->emb_rounded);
    }
    free(n->ctx);
    free((void *)n->durations);
    free(n);
}

/* Direct access to the sub-networks for the numerics tests. */
void orc_net_prep(const net_t *n, const real *x_row, real *p_row) { n->prep(n, x_row, p_row); }
void orc_net_pred(const net_t *n, int last, const real *s_in, real *s_out, real *g) { n->pred(n, last, s_in, s_out, g); }
void orc_net_joint(const net_t *n, const real *p_row, const real *g, real *logits) { n->joint(n, p_row, g, logits); }
int orc_real_size(void) { return (int)sizeof(real); }

/* ------------------------------------------------------------------------ */
/* Decode I/O                                                                */
/* ------------------------------------------------------------------------ */
typedef struct {
    int32_t B, T, S, cap, rec_cap;
    int32_t skip_masked;   /* frame looping: 0 = every row runs both networks at  */
                           /* every inner step, as Algorithm 1 does; 1 = rows that */
                           /* are already masked are passed over (a shortcut whose */
                           /* equality with the literal form is pinned by tests)   */
    int32_t n_threads;     /* sequential decode: utterances in parallel        */
    int32_t status;        /* out: ORC_STATUS_* bits                           */
    const real *x;         /* [B][T][x_size]                                   */
    const int32_t *len;    /* [B]                                              */
    int32_t *tokens;       /* [B][cap]  emitted labels, -1 beyond tok_len      */
    int32_t *frames;       /* [B][cap]  frame index of each emission           */
    real *scores;          /* [B][cap]  maximum token logit of each emission   */
    int32_t *durs;         /* [B][cap]  TDT: duration value of each emission   */
    int32_t *tok_len;      /* [B]                                              */
    /* one record per joint evaluation whose result was used (may be NULL)    */
    int32_t *rec_t, *rec_u, *rec_k, *rec_d;   /* [B][rec_cap]                  */
    real *rec_top, *rec_margin, *rec_dmargin; /* [B][rec_cap]                  */
    int32_t *rec_len;                         /* [B]                           */
    /* counters of batched work                                               */
    int64_t stat_outer;      /* outer-loop iterations                          */
    int64_t stat_inner;      /* batched joint steps                            */
    int64_t stat_pred;       /* batched prediction-network calls               */
    int64_t stat_pred_rows;  /* utterance-level prediction evaluations         */
    int64_t stat_joint_rows; /* utterance-level joint evaluations              */
    real *logps;           /* [B][cap]  log-softmax value of each emitted label */
                           /* over the token columns: the score Algorithm 1     */
                           /* keeps beside the label (may be NULL)              */
} decode_io;

/* argmax over v[lo..hi) with the lowest index winning ties; *margin is the   */
/* gap to the runner-up (0 for a tie, +inf for a single element).            */
static int argmax_margin(const real *v, int lo, int hi, real *top, real *margin)
{
    int k = lo;
    real best = v[lo];
    real second = (real)-INFINITY;
    for (int j = lo + 1; j < hi; ++j) {
        if (v[j] > best) { second = best; best = v[j]; k = j; }
        else if (v[j] > second) second = v[j];
    }
    *top = best;
    *margin = best - second;
    return k;
}

/* log_softmax(v[0..n))[k] for the k holding the maximum `top`: the sum runs in  */
/* index order in double precision.                                           */
static real log_prob_of_top(const real *v, int n, real top)
{
    double s = 0.0;
    for (int j = 0; j < n; ++j) s += exp((double)v[j] - (double)top);
    return (real)(-log(s));
}

static int clamp_len(const decode_io *io, int b, int32_t *status)
{
    int n = io->len[b];
    if (n < 0) { n = 0; *status |= ORC_STATUS_LEN_CLAMPED; }
    if (n > io->T) { n = io->T; *status |= ORC_STATUS_LEN_CLAMPED; }
    return n;
}

static void emit(decode_io *io, int b, int k, int t, real v, real lp, int dval,
                 int32_t *status)
{
    const int n = io->tok_len[b];
    if (n < io->cap) {
        const size_t o = (size_t)b * io->cap + n;
        io->tokens[o] = k;
        if (io->frames) io->frames[o] = t;
        if (io->scores) io->scores[o] = v;
        if (io->logps) io->logps[o] = lp;
        if (io->durs) io->durs[o] = dval;
    } else {
        *status |= ORC_STATUS_OVERFLOW;
    }
    io->tok_len[b] = n + 1;
}

static void record(decode_io *io, int b, int t, int k, real top, real margin,
                   int dval, real dmargin, int32_t *status)
{
    if (!io->rec_len) return;
    const int n = io->rec_len[b];
    if (n < io->rec_cap) {
        const size_t o = (size_t)b * io->rec_cap + n;
        io->rec_t[o] = t; io->rec_u[o] = io->tok_len[b]; io->rec_k[o] = k;
        io->rec_d[o] = dval; io->rec_top[o] = top; io->rec_margin[o] = margin;
        io->rec_dmargin[o] = dmargin;
    } else {
        *status |= ORC_STATUS_REC_OVERFLOW;
    }
    io->rec_len[b] = n + 1;
}

static void clear_outputs(decode_io *io)
{
    for (int b = 0; b < io->B; ++b) {
        io->tok_len[b] = 0;
        if (io->rec_len) io->rec_len[b] = 0;
        for (int i = 0; i < io->cap; ++i) {
            const size_t o = (size_t)b * io->cap + i;
            io->tokens[o] = -1;
            if (io->frames) io->frames[o] = -1;
            if (io->scores) io->scores[o] = (real)0;
            if (io->logps) io->logps[o] = (real)0;
            if (io->durs) io->durs[o] = -1;
        }
    }
    io->status = 0;
    io->stat_outer = io->stat_inner = io->stat_pred = 0;
    io->stat_pred_rows = io->stat_joint_rows = 0;
}

/* Prepared frames, computed on first use. */
typedef struct {
    const net_t *net;
    const decode_io *io;
    real *p;           /* [B][T][p_size] */
    unsigned char *have;
} frame_cache;

static void cache_init(frame_cache *fc, const net_t *net, const decode_io *io)
{
    fc->net = net; fc->io = io;
    fc->p = (real *)malloc(sizeof(real) * (size_t)io->B * io->T * net->p_size + 16);
    fc->have = (unsigned char *)calloc((size_t)io->B * io->T + 1, 1);
}
static const real *cache_get(frame_cache *fc, int b, int t)
{
    const size_t cell = (size_t)b * fc->io->T + t;
    real *p = fc->p + cell * fc->net->p_size;
    if (!fc->have[cell]) {
        fc->net->prep(fc->net, fc->io->x + cell * fc->net->x_size, p);
        fc->have[cell] = 1;
    }
    return p;
}
static void cache_free(frame_cache *fc) { free(fc->p); free(fc->have); }

/* ------------------------------------------------------------------------ */
/* Algorithm 1: batched frame-looping greedy decoding.                       */
/* Variable names follow the algorithm.                                      */
/* ------------------------------------------------------------------------ */
int orc_decode_frame_looping(const net_t *net, decode_io *io)
{
    if (net->D != 0) return -1;   /* batched frame looping is not exact for TDT */
    if (net->NB != 0) return -1;  /* Algorithm 1 has one frame index for the whole batch */
    const int B = io->B, SS = net->state_size, GS = net->g_size;
    const int blank_index = net->blank;
    clear_outputs(io);
    int32_t status = 0;
    frame_cache fc; cache_init(&fc, net, io);
    real *hidden = (real *)calloc((size_t)B * SS, sizeof(real));       /* zeros */
    real *hidden_prime = (real *)calloc((size_t)B * SS, sizeof(real));
    real *g = (real *)calloc((size_t)B * GS, sizeof(real));
    real *logp = (real *)calloc((size_t)net->V1, sizeof(real));
    int *last_label = (int *)malloc(sizeof(int) * (size_t)B);
    int *out_len = (int *)malloc(sizeof(int) * (size_t)B);
    int *k = (int *)malloc(sizeof(int) * (size_t)B);
    real *v = (real *)malloc(sizeof(real) * (size_t)B);
    real *mg = (real *)malloc(sizeof(real) * (size_t)B);
    real *lp = (real *)calloc((size_t)B, sizeof(real));
    unsigned char *blank_mask = (unsigned char *)malloc((size_t)B);
    unsigned char *was_masked = (unsigned char *)malloc((size_t)B);
    int max_out_len = 0;
    for (int b = 0; b < B; ++b) {
        last_label[b] = blank_index;           /* start of sequence            */
        out_len[b] = clamp_len(io, b, &status);
        if (out_len[b] > max_out_len) max_out_len = out_len[b];
    }
    for (int time_idx = 0; time_idx < max_out_len; ++time_idx) {
        io->stat_outer++;
        int not_blank = 1;
        int symbols_added = 0;
        /* rows whose frames have run out take no further part in this frame  */
        for (int b = 0; b < B; ++b) blank_mask[b] = (time_idx >= out_len[b]);
        while (not_blank && symbols_added < io->S) {
            io->stat_inner++; io->stat_pred++;
            /* Both networks run for the whole batch, masked rows included     */
            /* (their frame may be padding; whatever they produce is dropped   */
            /* by the masked updates below).                                   */
            for (int b = 0; b < B; ++b) {
                was_masked[b] = blank_mask[b];
                if (blank_mask[b] && io->skip_masked) {
                    k[b] = blank_index; v[b] = 0; mg[b] = 0;
                    continue;
                }
                /* prediction network on (last label, state): output g and the */
                /* candidate state                                             */
                net->pred(net, last_label[b], hidden + (size_t)b * SS,
                          hidden_prime + (size_t)b * SS, g + (size_t)b * GS);
                /* joint network on this frame and g, then the best label and  */
                /* its score                                                   */
                net->joint(net, cache_get(&fc, b, time_idx), g + (size_t)b * GS, logp);
                k[b] = argmax_margin(logp, 0, net->V1, &v[b], &mg[b]);
                if (io->logps) lp[b] = log_prob_of_top(logp, net->V1, v[b]);
                io->stat_pred_rows++; io->stat_joint_rows++;
            }
            for (int b = 0; b < B; ++b) {
                if (!was_masked[b]) record(io, b, time_idx, k[b], v[b], mg[b], 0, 0, &status);
                /* a row that produced a blank is masked for the rest of the   */
                /* frame; the mask is sticky                                   */
                blank_mask[b] = blank_mask[b] || (k[b] == blank_index);
                if (!blank_mask[b]) {
                    /* unmasked rows keep their label and score, and take the  */
                    /* label and the candidate state as their new state        */
                    emit(io, b, k[b], time_idx, v[b], lp[b], 0, &status);
                    last_label[b] = k[b];
                    memcpy(hidden + (size_t)b * SS, hidden_prime + (size_t)b * SS,
                           sizeof(real) * (size_t)SS);
                }
            }
            /* the inner loop goes on while some row is unmasked               */
            not_blank = 0;
            for (int b = 0; b < B; ++b) if (!blank_mask[b]) not_blank = 1;
            symbols_added += 1;
        }
    }
    io->status = status;
    free(hidden); free(hidden_prime); free(g); free(logp); free(last_label);
    free(out_len); free(k); free(v); free(mg); free(lp); free(blank_mask); free(was_masked);
    cache_free(&fc);
    return 0;
}

/* ------------------------------------------------------------------------ */
/* Label looping (RNN-T when net->D == 0, TDT otherwise).                    */
/* Each utterance owns its frame index t[b]; the outer loop runs once per    */
/* label, the inner loop skips blanks.                                        */
/* ------------------------------------------------------------------------ */
int orc_decode_label_looping(const net_t *net, decode_io *io)
{
    const int B = io->B, SS = net->state_size, GS = net->g_size;
    const int V1 = net->V1, D = net->D, blank = net->blank, S = io->S;
    const int NB = net->NB, VT = V1 + NB;     /* VT: width of the token distribution */
    clear_outputs(io);
    int32_t status = 0;
    frame_cache fc; cache_init(&fc, net, io);
    real *state = (real *)calloc((size_t)B * SS, sizeof(real));
    real *state_prime = (real *)calloc((size_t)B * SS, sizeof(real));
    real *g = (real *)calloc((size_t)B * GS, sizeof(real));
    real *logits = (real *)calloc((size_t)(VT + D), sizeof(real));
    int *last = (int *)malloc(sizeof(int) * (size_t)B);
    int *len = (int *)malloc(sizeof(int) * (size_t)B);
    int *t = (int *)calloc((size_t)B, sizeof(int));
    int *n = (int *)calloc((size_t)B, sizeof(int));
    int *k = (int *)malloc(sizeof(int) * (size_t)B);
    int *d = (int *)calloc((size_t)B, sizeof(int));
    real *lp = (real *)calloc((size_t)B, sizeof(real));
    real *v = (real *)malloc(sizeof(real) * (size_t)B);
    unsigned char *active = (unsigned char *)malloc((size_t)B);
    unsigned char *searching = (unsigned char *)malloc((size_t)B);
    int any_active = 0;
    for (int b = 0; b < B; ++b) {
        last[b] = blank;
        len[b] = clamp_len(io, b, &status);
        active[b] = t[b] < len[b];
        any_active |= active[b];
    }
    while (any_active) {
        io->stat_outer++; io->stat_pred++;
        /* (i) one prediction-network step for the batch                      */
        for (int b = 0; b < B; ++b) {
            if (!active[b]) continue;
            net->pred(net, last[b], state + (size_t)b * SS,
                      state_prime + (size_t)b * SS, g + (size_t)b * GS);
            io->stat_pred_rows++;
        }
        /* (ii)+(iii) joint at each row's own frame until it holds a non-blank */
        int first = 1, any_searching = 1;
        for (int b = 0; b < B; ++b) searching[b] = active[b];
        while (any_searching) {
            io->stat_inner++;
            for (int b = 0; b < B; ++b) {
                if (!searching[b]) continue;
                if (!first) {
                    /* the previous evaluation of this row was a blank         */
                    /* (a TDT blank advances by its duration, at least 1; a big   */
                    /* blank by its span, kept in d[b] as well)                   */
                    int adv = 1;
                    if (D > 0 || NB > 0) adv = d[b] > 1 ? d[b] : 1;
                    t[b] += adv; n[b] = 0;
                    if (t[b] >= len[b]) { searching[b] = 0; active[b] = 0; continue; }
                }
                net->joint(net, cache_get(&fc, b, t[b]), g + (size_t)b * GS, logits);
                io->stat_joint_rows++;
                real mg, dmg = 0, dv;
                k[b] = argmax_margin(logits, 0, VT, &v[b], &mg);
                if (io->logps) lp[b] = log_prob_of_top(logits, VT, v[b]);
                int dval = 0;
                if (D > 0) {
                    const int di = argmax_margin(logits, V1, V1 + D, &dv, &dmg) - V1;
                    dval = net->durations[di];
                }
                if (k[b] >= V1) dval = net->spans[k[b] - V1];      /* a big blank */
                d[b] = dval;
                record(io, b, t[b], k[b], v[b], mg, dval, dmg, &status);
                if (k[b] != blank && k[b] < V1) searching[b] = 0;
            }
            first = 0;
            any_searching = 0;
            for (int b = 0; b < B; ++b) any_searching |= searching[b];
        }
        /* (iv) every active row holds a non-blank label at frame t[b]         */
        any_active = 0;
        for (int b = 0; b < B; ++b) {
            if (!active[b]) continue;
            emit(io, b, k[b], t[b], v[b], lp[b], d[b], &status);
            last[b] = k[b];
            memcpy(state + (size_t)b * SS, state_prime + (size_t)b * SS,
                   sizeof(real) * (size_t)SS);
            if (D > 0 && d[b] > 0) {
                t[b] += d[b]; n[b] = 0;
            } else {
                n[b] += 1;
                if (n[b] == S) { t[b] += 1; n[b] = 0; }
            }
            active[b] = t[b] < len[b];
            any_active |= active[b];
        }
    }
    io->status = status;
    free(state); free(state_prime); free(g); free(logits); free(last); free(len);
    free(t); free(n); free(k); free(d); free(v); free(lp); free(active); free(searching);
    cache_free(&fc);
    return 0;
}

/* ------------------------------------------------------------------------ */
/* The per-utterance definition.                                             */
/* ------------------------------------------------------------------------ */
static void decode_one(const net_t *net, decode_io *io, int b, int32_t *status,
                       int64_t *pred_rows, int64_t *joint_rows)
{
    const int SS = net->state_size, GS = net->g_size, V1 = net->V1, D = net->D;
    const int blank = net->blank, S = io->S;
    const int NB = net->NB, VT = V1 + NB;
    real *state = (real *)calloc((size_t)SS, sizeof(real));
    real *state_prime = (real *)calloc((size_t)SS, sizeof(real));
    real *g = (real *)calloc((size_t)GS, sizeof(real));
    real *p = (real *)calloc((size_t)net->p_size, sizeof(real));
    real *logits = (real *)calloc((size_t)(VT + D), sizeof(real));
    const int len = clamp_len(io, b, status);
    int t = 0, n = 0, last = blank, p_frame = -1;
    if (len > 0) { net->pred(net, last, state, state_prime, g); (*pred_rows)++; }
    while (t < len) {
        if (p_frame != t) {
            net->prep(net, io->x + ((size_t)b * io->T + t) * net->x_size, p);
            p_frame = t;
        }
        net->joint(net, p, g, logits);
        (*joint_rows)++;
        real v, mg, dv, dmg = 0;
        const int k = argmax_margin(logits, 0, VT, &v, &mg);
        int dval = 0;
        if (D > 0) dval = net->durations[argmax_margin(logits, V1, V1 + D, &dv, &dmg) - V1];
        if (k >= V1) dval = net->spans[k - V1];                    /* a big blank */
        record(io, b, t, k, v, mg, dval, dmg, status);
        if (k == blank || k >= V1) {
            t += ((D > 0 || NB > 0) && dval > 1) ? dval : 1;
            n = 0;
        } else {
            emit(io, b, k, t, v, io->logps ? log_prob_of_top(logits, VT, v) : (real)0, dval, status);
            last = k;
            memcpy(state, state_prime, sizeof(real) * (size_t)SS);
            if (D > 0 && dval > 0) { t += dval; n = 0; }
            else { n += 1; if (n == S) { t += 1; n = 0; } }
            if (t < len) { net->pred(net, last, state, state_prime, g); (*pred_rows)++; }
        }
    }
    free(state); free(state_prime); free(g); free(p); free(logits);
}

int orc_decode_sequential(const net_t *net, decode_io *io)
{
    clear_outputs(io);
    int32_t status = 0;
    int64_t pred_rows = 0, joint_rows = 0;
    int nt = io->n_threads > 0 ? io->n_threads : 1;
    (void)nt;
#pragma omp parallel for schedule(dynamic, 1) num_threads(nt) reduction(| : status) reduction(+ : pred_rows, joint_rows)
    for (int b = 0; b < io->B; ++b) decode_one(net, io, b, &status, &pred_rows, &joint_rows);
    io->status = status;
    io->stat_pred_rows = pred_rows;
    io->stat_joint_rows = joint_rows;
    return 0;
}

/* ------------------------------------------------------------------------ */
/* Follow one utterance along a given hypothesis.                            */
/* At every joint evaluation the given sequence implies a decision (emit its */
/* next token here, or blank).  The walk takes that decision and reports     */
/* each place where it is not the argmax together with how far below the     */
/* maximum the chosen logit lies.  Returns the number of such departures, or */
/* -1 when the sequence cannot be produced by any walk (tokens left over,    */
/* more than S labels on a frame, frames out of order).                      */
/* A multi-blank hypothesis does not say which of its blanks were big ones:  */
/* between labels the walk looks for a chain of blanks and big blanks that    */
/* lands on the next label's frame, each the maximum or less than tol below   */
/* it, and reports those that are not the maximum.                            */
/* For TDT the duration taken on a blank is not part of a hypothesis.  With  */
/* tol = 0 the walk takes its own argmax duration there.  With tol > 0 it    */
/* looks for the chain of blank evaluations that reaches the frame of the    */
/* hypothesis' next label (or the end of the utterance) with the smallest    */
/* worst gap, among chains whose blank and duration choices all lie less     */
/* than tol below their maxima; the non-argmax choices on that chain are     */
/* reported like any other departure.  If there is no such chain it falls    */
/* back to the argmax durations.                                             */
/* ------------------------------------------------------------------------ */
int orc_follow_sequential(const net_t *net, const real *x_b, int T, int len,
                          int S, const int32_t *tokens, const int32_t *frames,
                          const int32_t *durs, int n_tok, int max_report,
                          int32_t *rep_t, int32_t *rep_u, int32_t *rep_want,
                          int32_t *rep_got, real *rep_gap, real *worst_gap, real tol)
{
    const int SS = net->state_size, GS = net->g_size, V1 = net->V1, D = net->D;
    const int blank = net->blank;
    const int NB = net->NB, VT = V1 + NB;     /* multi-blank: one distribution over VT outputs */
    real *state = (real *)calloc((size_t)SS, sizeof(real));
    real *state_prime = (real *)calloc((size_t)SS, sizeof(real));
    real *g = (real *)calloc((size_t)GS, sizeof(real));
    real *p = (real *)calloc((size_t)net->p_size, sizeof(real));
    real *logits = (real *)calloc((size_t)(VT + D), sizeof(real));
    if (len > T) len = T;
    if (len < 0) len = 0;
    int t = 0, n = 0, u = 0, last = blank, departures = 0, bad = 0;
    *worst_gap = 0;
    if (len > 0) net->pred(net, last, state, state_prime, g);
    /* blank chains of TDT (tol > 0): best[t'] = smallest worst gap of a chain from the     */
    /* current frame to t', from_[t'] / how_[t'] = the step that achieves it                */
    real *best = (real *)malloc(sizeof(real) * (size_t)(len + 2));
    int *from_ = (int *)malloc(sizeof(int) * (size_t)(len + 2));
    int *how_ = (int *)malloc(sizeof(int) * (size_t)(len + 2));
    real *gap_b = (real *)malloc(sizeof(real) * (size_t)(len + 2));
    real *gap_d = (real *)malloc(sizeof(real) * (size_t)(len + 2));
    int *want_b = (int *)malloc(sizeof(int) * (size_t)(len + 2));
    int *want_d = (int *)malloc(sizeof(int) * (size_t)(len + 2));
    while (t < len) {
        if (NB > 0 && !(u < n_tok && frames[u] == t)) {
            /* Multi-blank, and the hypothesis has no label on this frame: it went on from   */
            /* here by blanks and big blanks, which it does not record.  Look for the chain   */
            /* of such symbols that lands exactly on the frame of its next label (or past     */
            /* the end) with the smallest worst gap, every symbol on it being the maximum or  */
            /* less than tol below it; the symbols that are not the maximum are reported.     */
            /* how_: -1 = the blank, i >= 0 = big blank i.                                     */
            const int target = (u < n_tok && frames[u] < len) ? frames[u] : len;
            if (u < n_tok && (frames[u] < t || frames[u] >= len)) { bad = 1; break; }
            for (int i = t; i <= len; ++i) { best[i] = (real)-1; from_[i] = -1; }
            best[t] = 0;
            for (int a = t; a < len && a < target; ++a) {
                if (best[a] < 0) continue;
                net->prep(net, x_b + (size_t)a * net->x_size, p);
                net->joint(net, p, g, logits);
                real v2, m2;
                const int k2 = argmax_margin(logits, 0, VT, &v2, &m2);
                want_b[a] = k2;
                for (int i = -1; i < NB; ++i) {
                    const int col = i < 0 ? blank : V1 + i;
                    const real gap = v2 - logits[col];
                    if (col != k2 && !(gap < tol)) continue;
                    int to = a + (i < 0 ? 1 : (net->spans[i] > 1 ? net->spans[i] : 1));
                    if (to > len) to = len;
                    if (to > target) continue;                /* would skip the next label's frame */
                    const real worst = best[a] > gap ? best[a] : gap;
                    if (best[to] < 0 || worst < best[to]) { best[to] = worst; from_[to] = a; how_[to] = i; }
                }
            }
            if (best[target] >= 0) {
                int chain[4096], nc = 0;
                for (int a = target; a != t && nc < 4096; a = from_[a]) chain[nc++] = a;
                for (int i = nc - 1; i >= 0; --i) {
                    const int to = chain[i], a = from_[to];
                    const int col = how_[to] < 0 ? blank : V1 + how_[to];
                    if (col == want_b[a]) continue;
                    net->prep(net, x_b + (size_t)a * net->x_size, p);
                    net->joint(net, p, g, logits);
                    real v2, m2;
                    (void)argmax_margin(logits, 0, VT, &v2, &m2);
                    const real gap = v2 - logits[col];
                    if (departures < max_report) {
                        rep_t[departures] = a; rep_u[departures] = u;
                        rep_want[departures] = want_b[a]; rep_got[departures] = col;
                        rep_gap[departures] = gap;
                    }
                    departures++;
                    if (gap > *worst_gap) *worst_gap = gap;
                }
                t = target; n = 0;
                continue;
            }
            /* no such chain: go on by the plain blank below, which reports its gap */
        }
        if (D > 0 && tol > (real)0 && !(u < n_tok && frames[u] == t)) {
            /* the hypothesis has a blank here: find the chain of blanks to its next label */
            const int target = (u < n_tok && frames[u] < len) ? frames[u] : len;   /* len = any frame >= len */
            if (u < n_tok && (frames[u] < t || frames[u] >= len)) { bad = 1; break; }
            for (int i = t; i <= len; ++i) { best[i] = (real)-1; from_[i] = -1; }
            best[t] = 0;
            for (int a = t; a < len && a < target; ++a) {
                if (best[a] < 0) continue;
                net->prep(net, x_b + (size_t)a * net->x_size, p);
                net->joint(net, p, g, logits);
                real v2, m2, dv2, dm2;
                const int k2 = argmax_margin(logits, 0, V1, &v2, &m2);
                const int d2 = argmax_margin(logits, V1, V1 + D, &dv2, &dm2) - V1;
                const real gb = v2 - logits[blank];
                gap_b[a] = gb; want_b[a] = k2; want_d[a] = d2;
                if (!(gb < tol)) continue;                    /* blank is no near-maximum here */
                for (int i = 0; i < D; ++i) {
                    const real gd = dv2 - logits[V1 + i];
                    if (!(gd < tol)) continue;
                    int to = a + (net->durations[i] > 1 ? net->durations[i] : 1);
                    if (to > len) to = len;
                    if (to > target) continue;                /* would skip the next label's frame */
                    real worst = best[a] > gb ? best[a] : gb;
                    if (gd > worst) worst = gd;
                    if (best[to] < 0 || worst < best[to]) { best[to] = worst; from_[to] = a; how_[to] = i; }
                }
            }
            if (best[target] >= 0) {
                /* report the non-argmax choices of the chain, in frame order */
                int chain[4096], nc = 0;
                for (int a = target; a != t && nc < 4096; a = from_[a]) chain[nc++] = a;
                for (int i = nc - 1; i >= 0; --i) {
                    const int to = chain[i], a = from_[to];
                    /* duration gap of the step a -> to: recompute from the stored choice */
                    net->prep(net, x_b + (size_t)a * net->x_size, p);
                    net->joint(net, p, g, logits);
                    real dv2, dm2;
                    (void)argmax_margin(logits, V1, V1 + D, &dv2, &dm2);
                    gap_d[a] = dv2 - logits[V1 + how_[to]];
                    if (gap_b[a] > 0) {
                        if (departures < max_report) {
                            rep_t[departures] = a; rep_u[departures] = u;
                            rep_want[departures] = want_b[a]; rep_got[departures] = blank;
                            rep_gap[departures] = gap_b[a];
                        }
                        departures++;
                        if (gap_b[a] > *worst_gap) *worst_gap = gap_b[a];
                    }
                    if (gap_d[a] > 0) {
                        if (departures < max_report) {
                            rep_t[departures] = a; rep_u[departures] = u;
                            rep_want[departures] = V1 + want_d[a]; rep_got[departures] = V1 + how_[to];
                            rep_gap[departures] = gap_d[a];
                        }
                        departures++;
                        if (gap_d[a] > *worst_gap) *worst_gap = gap_d[a];
                    }
                }
                t = target; n = 0;
                continue;
            }
            /* no chain within tol: take the argmax durations below and report what that gives */
        }
        net->prep(net, x_b + (size_t)t * net->x_size, p);
        net->joint(net, p, g, logits);
        real v, mg, dv = 0, dmg = 0;
        const int k = argmax_margin(logits, 0, VT, &v, &mg);
        int di = 0;
        if (D > 0) di = argmax_margin(logits, V1, V1 + D, &dv, &dmg) - V1;
        int choose = blank;
        if (u < n_tok && frames[u] == t) choose = tokens[u];
        if (choose < 0 || choose >= V1) { bad = 1; break; }
        if (choose != k) {
            const real gap = v - logits[choose];
            if (departures < max_report) {
                rep_t[departures] = t; rep_u[departures] = u;
                rep_want[departures] = k; rep_got[departures] = choose;
                rep_gap[departures] = gap;
            }
            departures++;
            if (gap > *worst_gap) *worst_gap = gap;
        }
        int dval = D > 0 ? net->durations[di] : 0;
        if (choose != blank && D > 0) {
            /* the hypothesis also fixes the duration of an emitted label;    */
            /* duration departures are reported as indices V1 + i             */
            int gi = -1;
            for (int i = 0; i < D; ++i) if (net->durations[i] == durs[u]) { gi = i; break; }
            if (gi < 0) { bad = 1; break; }
            if (gi != di) {
                const real gap = dv - logits[V1 + gi];
                if (departures < max_report) {
                    rep_t[departures] = t; rep_u[departures] = u;
                    rep_want[departures] = V1 + di; rep_got[departures] = V1 + gi;
                    rep_gap[departures] = gap;
                }
                departures++;
                if (gap > *worst_gap) *worst_gap = gap;
            }
            dval = durs[u];
        }
        if (choose == blank) {
            t += (D > 0 && dval > 1) ? dval : 1;
            n = 0;
        } else {
            u++;
            last = choose;
            memcpy(state, state_prime, sizeof(real) * (size_t)SS);
            if (D > 0 && dval > 0) { t += dval; n = 0; }
            else { n += 1; if (n == S) { t += 1; n = 0; } }
            if (t < len) net->pred(net, last, state, state_prime, g);
        }
    }
    if (u != n_tok) bad = 1;
    free(state); free(state_prime); free(g); free(p); free(logits);
    free(best); free(from_); free(how_); free(gap_b); free(gap_d); free(want_b); free(want_d);
    return bad ? -1 : departures;
}
