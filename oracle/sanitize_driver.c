/*
 * Sanitizer driver for the CPU oracle (TEST INFRASTRUCTURE ONLY, like the oracle itself).
 * Built by the CPU test suite with AddressSanitizer and UndefinedBehaviorSanitizer; includes
 * the oracle's source so that every function is instrumented.  Runs the three schedules, the
 * follow mode and the sub-network calls on small random LSTM nets (RNN-T and TDT) and a table
 * net, over the shapes where indexing mistakes would hide: empty and clamped lengths, a
 * capacity too small for the labels, a record buffer too small, one layer and three layers,
 * widths that are not multiples of the vector width.  Exit status 0 means no report; the
 * schedules are also required to agree, so a wild read that changes a result is seen too.
 */
#include "rnnt_oracle.c"

#include <stdio.h>

static uint64_t rng_state = 0x9e3779b97f4a7c15ull;
static real rnd(void)
{
    rng_state ^= rng_state << 13; rng_state ^= rng_state >> 7; rng_state ^= rng_state << 17;
    return (real)((double)(rng_state >> 11) / 9007199254740992.0 * 0.6 - 0.3);
}
static real *rnd_vec(size_t n)
{
    real *v = (real *)malloc(sizeof(real) * (n ? n : 1));
    for (size_t i = 0; i < n; ++i) v[i] = rnd();
    return v;
}

static int run_case(int F, int E, int H, int L, int J, int V1, int D, int B, int T, int S,
                    int cap, int rec_cap, const int32_t *len)
{
    const int32_t durations[4] = {0, 1, 2, 4};
    const real *w_ih[4], *w_hh[4], *b_ih[4], *b_hh[4];
    real *keep[32]; int nk = 0;
    real *emb = keep[nk++] = rnd_vec((size_t)V1 * E);
    for (int i = 0; i < E; ++i) emb[(size_t)(V1 - 1) * E + i] = 0;
    for (int l = 0; l < L; ++l) {
        w_ih[l] = keep[nk++] = rnd_vec((size_t)4 * H * (l == 0 ? E : H));
        w_hh[l] = keep[nk++] = rnd_vec((size_t)4 * H * H);
        b_ih[l] = keep[nk++] = rnd_vec((size_t)4 * H);
        b_hh[l] = keep[nk++] = rnd_vec((size_t)4 * H);
    }
    real *w_enc = keep[nk++] = rnd_vec((size_t)J * F), *b_enc = keep[nk++] = rnd_vec(J);
    real *w_pred = keep[nk++] = rnd_vec((size_t)J * H), *b_pred = keep[nk++] = rnd_vec(J);
    real *w_out = keep[nk++] = rnd_vec((size_t)(V1 + D) * J), *b_out = keep[nk++] = rnd_vec(V1 + D);
    b_out[V1 - 1] += (real)0.4;                       /* some blanks */
    net_t *net = orc_lstm_net_create(F, E, H, L, J, V1, D, V1 - 1, durations, emb, w_ih, w_hh, b_ih,
                                     b_hh, w_enc, b_enc, w_pred, b_pred, w_out, b_out);
    real *x = rnd_vec((size_t)B * T * F);
    int bad = 0;
    int32_t *tok[3]; int32_t *tl[3];
    for (int sched = 0; sched < 3; ++sched) {
        decode_io io; memset(&io, 0, sizeof io);
        io.B = B; io.T = T; io.S = S; io.cap = cap; io.rec_cap = rec_cap; io.n_threads = 2;
        io.x = x; io.len = len;
        io.tokens = tok[sched] = (int32_t *)malloc(sizeof(int32_t) * (size_t)B * cap);
        io.frames = (int32_t *)malloc(sizeof(int32_t) * (size_t)B * cap);
        io.scores = (real *)malloc(sizeof(real) * (size_t)B * cap);
        io.logps = (real *)malloc(sizeof(real) * (size_t)B * cap);
        io.durs = (int32_t *)malloc(sizeof(int32_t) * (size_t)B * cap);
        io.tok_len = tl[sched] = (int32_t *)malloc(sizeof(int32_t) * (size_t)B);
        if (rec_cap > 0) {
            const size_t n = (size_t)B * rec_cap;
            io.rec_t = (int32_t *)malloc(4 * n); io.rec_u = (int32_t *)malloc(4 * n);
            io.rec_k = (int32_t *)malloc(4 * n); io.rec_d = (int32_t *)malloc(4 * n);
            io.rec_top = (real *)malloc(sizeof(real) * n); io.rec_margin = (real *)malloc(sizeof(real) * n);
            io.rec_dmargin = (real *)malloc(sizeof(real) * n); io.rec_len = (int32_t *)malloc(4 * (size_t)B);
        }
        int rc = sched == 0 ? orc_decode_frame_looping(net, &io)
                            : (sched == 1 ? orc_decode_label_looping(net, &io) : orc_decode_sequential(net, &io));
        if (sched == 0 && D > 0) { if (rc != -1) bad = 1; }
        else if (rc != 0) bad = 1;
        if (sched == 2) {
            /* follow the per-utterance result: no departure, or overflowed capacity */
            for (int b = 0; b < B; ++b) {
                const int n = io.tok_len[b] < cap ? io.tok_len[b] : cap;
                int32_t rt[4], ru[4], rw[4], rg[4]; real gap[4], worst;
                int clamped = len[b] < 0 ? 0 : (len[b] > T ? T : len[b]);
                int dep = orc_follow_sequential(net, x + (size_t)b * T * F, T, clamped, S,
                                                io.tokens + (size_t)b * cap, io.frames + (size_t)b * cap,
                                                io.durs + (size_t)b * cap, n, 4, rt, ru, rw, rg, gap, &worst, (real)(b & 1 ? 0.05 : 0));
                if (io.tok_len[b] <= cap && dep != 0) bad = 1;
            }
        }
        free(io.frames); free(io.scores); free(io.logps); free(io.durs);
        free(io.rec_t); free(io.rec_u); free(io.rec_k); free(io.rec_d); free(io.rec_top);
        free(io.rec_margin); free(io.rec_dmargin); free(io.rec_len);
    }
    for (int sched = (D > 0 ? 2 : 1); sched < 3; ++sched) {
        const int ref = D > 0 ? 1 : 0;
        if (memcmp(tl[ref], tl[sched], sizeof(int32_t) * (size_t)B)) bad = 1;
        if (memcmp(tok[ref], tok[sched], sizeof(int32_t) * (size_t)B * cap)) bad = 1;
    }
    for (int i = 0; i < 3; ++i) { free(tok[i]); free(tl[i]); }
    free(x);
    orc_net_destroy(net);
    for (int i = 0; i < nk; ++i) free(keep[i]);
    return bad;
}

int main(void)
{
    int bad = 0;
    const int32_t len_a[5] = {7, 0, 3, 12, -2};         /* 12 > T and -2 are clamped */
    bad |= run_case(10, 6, 5, 1, 7, 6, 0, 5, 9, 3, 40, 50, len_a);
    bad |= run_case(10, 6, 5, 1, 7, 6, 0, 5, 9, 3, 4, 6, len_a);      /* capacity and records too small */
    bad |= run_case(13, 9, 9, 3, 11, 9, 0, 5, 9, 2, 30, 0, len_a);    /* three layers, no records */
    bad |= run_case(10, 6, 5, 2, 7, 6, 4, 5, 9, 3, 40, 50, len_a);    /* TDT */
    bad |= run_case(10, 6, 5, 2, 7, 6, 4, 5, 9, 1, 3, 2, len_a);      /* TDT, tight buffers */
    const int32_t len_b[1] = {1};
    bad |= run_case(3, 2, 2, 1, 2, 2, 0, 1, 1, 1, 1, 2, len_b);       /* the smallest shapes */
    /* table net */
    {
        const int V1 = 3, U = 4, T = 3, B = 2;
        real *table = rnd_vec((size_t)B * T * U * V1 * V1);
        net_t *net = orc_table_net_create(V1, 0, V1 - 1, NULL, U, table);
        real x[6] = {0, 1, 2, 3, 4, 5};
        const int32_t len[2] = {3, 2};
        for (int sched = 0; sched < 3; ++sched) {
            decode_io io; memset(&io, 0, sizeof io);
            int32_t tokens[2 * 8], tok_len[2];
            io.B = B; io.T = T; io.S = 2; io.cap = 8; io.n_threads = 1; io.x = x; io.len = len;
            io.tokens = tokens; io.tok_len = tok_len;
            int rc = sched == 0 ? orc_decode_frame_looping(net, &io)
                                : (sched == 1 ? orc_decode_label_looping(net, &io) : orc_decode_sequential(net, &io));
            if (rc != 0) bad = 1;
        }
        orc_net_destroy(net);
        free(table);
    }
    printf(bad ? "MISMATCH\n" : "ok\n");
    return bad;
}
