// Host side of the C ABI declared in include/rnnt_greedy.h: argument checks,
// weight repacking, workspace, launches.  Nothing here computes any part of the
// decode; every step of the path runs in the kernels.
#include "../../include/rnnt_greedy.h"

#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <functional>
#include <string>
#include <vector>

#include "engine.h"

using namespace rnnt;

namespace {

thread_local std::string g_hip_error;

int hip_fail(hipError_t e, const char *what)
{
    g_hip_error = std::string("HIP error in ") + what + ": " + hipGetErrorString(e);
    return RNNT_ERR_HIP;
}

#define HIP_TRY(expr)                                           \
    do {                                                        \
        hipError_t e_ = (expr);                                 \
        if (e_ != hipSuccess) return hip_fail(e_, #expr);       \
    } while (0)

constexpr int kLdsBytes = 160 * 1024;   // LDS of one gfx950 compute unit

struct DevBuf {
    void *p = nullptr;
    ~DevBuf() { if (p) (void)hipFree(p); }
    hipError_t alloc(size_t bytes) {
        if (p) { (void)hipFree(p); p = nullptr; }
        return hipMalloc(&p, bytes ? bytes : 16);
    }
    template <class T> T *as() const { return static_cast<T *>(p); }
};

struct PackedStage {
    StagePlan plan{};
    DevBuf w;
};

}  // namespace

struct rnnt_engine {
    rnnt_model_desc d{};
    int durations[kMaxDur] = {0};
    int NOUT = 0, max_B = 0, max_T = 0;
    int n_wg = 0;          // work-groups the device can keep resident (one per CU)
    int n_teams = 0, team_size = 0, lookahead = 0;
    // host copies of the weights that get repacked when the team size changes
    std::vector<std::vector<float>> w_ih, w_hh;
    std::vector<float> w_pred, w_out;
    // device: weights used as they are, derived tables, workspace
    DevBuf w_enc, b_enc, T0, bias_l, b_pred, b_out;
    DevBuf P, hbuf, qbuf, part, dpart, bar, abort_flag, status, stats, xcc;
    PackedStage st0, stl[kMaxLayers], spred, sjoint;
    // plan
    int xstride = 0, nu_max = 0, gj_max = 0, gp_max = 0;
    int lds_xz = 0, lds_red = 0, lds_c = 0, lds_part = 0, lds_bias = 0, lds_q = 0;
    int q_in_lds = 0, qstride = 0;
    unsigned lds_bytes = 0;
    int last_B = 0;
    hipEvent_t ev[3] = {nullptr, nullptr, nullptr};   // before projection, before decode, after
    bool timed = false;
    ~rnnt_engine() { for (auto &x : ev) if (x) (void)hipEventDestroy(x); }
};

namespace {

int upload_stage(PackedStage &ps, int ts, const std::function<int(int)> &ngroups,
                 const std::function<const float *(int, int, int)> &row_of)
{
    const StagePlan &pl = ps.plan;
    std::vector<float> host((size_t)ts * pl.rank_stride * 4, 0.f);
    for (int rank = 0; rank < ts; ++rank) {
        const int ntask = ngroups(rank) * pl.nks;
        for (int slot = 0; slot < pl.slots; ++slot)
            for (int wave = 0; wave < kWaves; ++wave)
                for (int lane = 0; lane < 64; ++lane) {
                    const int task = slot * kBlocksPerWg + wave * 16 + (lane >> 2);
                    if (task >= ntask) continue;
                    const int g = task / pl.nks, ks = task % pl.nks;
                    const float *row = row_of(rank, g, lane & 3);
                    if (!row) continue;
                    for (int step = 0; step < pl.nsteps; ++step) {
                        float *dst = host.data() +
                                     ((size_t)rank * pl.rank_stride +
                                      ((size_t)(slot * kWaves + wave) * pl.nsteps + step) * 64 + lane) * 4;
                        const int k0 = (ks * pl.nsteps + step) * 4;
                        for (int c = 0; c < 4; ++c)
                            if (k0 + c < pl.K) dst[c] = row[k0 + c];
                    }
                }
    }
    HIP_TRY(ps.w.alloc(host.size() * sizeof(float)));
    HIP_TRY(hipMemcpy(ps.w.p, host.data(), host.size() * sizeof(float), hipMemcpyHostToDevice));
    return RNNT_OK;
}

// Choose the stage plans and the LDS layout for `n_teams` teams and upload the
// repacked weights.  Synchronous.
int plan_and_pack(rnnt_engine *e, int n_teams)
{
    const rnnt_model_desc &d = e->d;
    if (n_teams < 1 || n_teams > e->n_wg) return RNNT_ERR_SHAPE;
    const int ts = e->n_wg / n_teams;
    if (ts < 1) return RNNT_ERR_SHAPE;
    const int rows_max = (e->max_B + n_teams - 1) / n_teams;
    if (rows_max > kMaxRows) return RNNT_ERR_SHAPE;
    const int H = d.H, L = d.L, J = d.J;
    auto nu_of = [&](int r) { return range_hi(r, ts, H) - range_lo(r, ts, H); };
    const int gp_all = (J + 3) / 4, gj_all = (e->NOUT + 3) / 4;
    auto gp_of = [&](int r) { return range_hi(r, ts, gp_all) - range_lo(r, ts, gp_all); };
    auto gj_of = [&](int r) { return range_hi(r, ts, gj_all) - range_lo(r, ts, gj_all); };
    int nu_max = 0, gp_max = 0, gj_max = 0;
    for (int r = 0; r < ts; ++r) {
        nu_max = std::max(nu_max, nu_of(r));
        gp_max = std::max(gp_max, gp_of(r));
        gj_max = std::max(gj_max, gj_of(r));
    }
    e->st0.plan = make_stage_plan(H, L * nu_max);
    for (int l = 1; l < L; ++l) e->stl[l].plan = make_stage_plan(H, nu_max);
    e->spred.plan = make_stage_plan(H, gp_max);
    e->sjoint.plan = make_stage_plan(J, gj_max);

    // LDS layout
    int kpad = std::max({e->st0.plan.kpad, e->spred.plan.kpad, e->sjoint.plan.kpad});
    for (int l = 1; l < L; ++l) kpad = std::max(kpad, e->stl[l].plan.kpad);
    const int xstride = kpad + 4;
    const int rgp = (rows_max + 3) / 4, rows_pad = rgp * 4;
    const int rgj = kMaxSamples / 4;
    auto red_need = [&](const StagePlan &pl, int groups, int rg) {
        return std::min(groups * pl.nks, kBlocksPerWg * pl.slots) * rg * 16;
    };
    int xz = std::max(L * rows_pad * xstride, kMaxSamples * xstride);
    int red = red_need(e->st0.plan, L * nu_max, rgp);
    for (int l = 1; l < L; ++l) red = std::max(red, red_need(e->stl[l].plan, nu_max, rgp));
    red = std::max(red, red_need(e->spred.plan, gp_max, rgp));
    if (e->sjoint.plan.slots == 1) xz = std::max(xz, red_need(e->sjoint.plan, gj_max, rgj));
    else red = std::max(red, red_need(e->sjoint.plan, gj_max, rgj));
    int off = 0;
    auto take = [&](int n) { int o = off; off += (n + 3) & ~3; return o; };
    e->lds_xz = take(xz);
    e->lds_red = take(red);
    e->lds_c = take(L * 2 * nu_max * kMaxRows);
    e->lds_part = take(L * nu_max * kMaxRows * 4);
    e->lds_bias = take(4 * (gp_max + gj_max + L * nu_max));
    if ((unsigned)off * 4u + 2048u > (unsigned)kLdsBytes) return RNNT_ERR_UNSUPPORTED;
    // q of the team's rows stays in LDS between joint steps when there is room
    e->qstride = (J + 3) & ~3;
    e->q_in_lds = ((unsigned)(off + rows_pad * e->qstride) * 4u + 2048u <= (unsigned)kLdsBytes);
    e->lds_q = e->q_in_lds ? take(rows_pad * e->qstride) : 0;
    e->lds_bytes = (unsigned)off * 4u;
    e->xstride = xstride; e->nu_max = nu_max; e->gj_max = gj_max; e->gp_max = gp_max;

    // weights
    int rc;
    rc = upload_stage(e->st0, ts, [&](int r) { return L * nu_of(r); },
                      [&](int r, int g, int j) -> const float * {
                          const int nu = nu_of(r);
                          const int layer = g / nu, u = range_lo(r, ts, H) + g % nu;
                          return e->w_hh[layer].data() + (size_t)(j * H + u) * H;
                      });
    if (rc) return rc;
    for (int l = 1; l < L; ++l) {
        rc = upload_stage(e->stl[l], ts, nu_of, [&](int r, int g, int j) -> const float * {
            return e->w_ih[l].data() + (size_t)(j * H + range_lo(r, ts, H) + g) * H;
        });
        if (rc) return rc;
    }
    rc = upload_stage(e->spred, ts, gp_of, [&](int r, int g, int j) -> const float * {
        const int col = (range_lo(r, ts, gp_all) + g) * 4 + j;
        return col < J ? e->w_pred.data() + (size_t)col * H : nullptr;
    });
    if (rc) return rc;
    rc = upload_stage(e->sjoint, ts, gj_of, [&](int r, int g, int j) -> const float * {
        const int col = (range_lo(r, ts, gj_all) + g) * 4 + j;
        return col < e->NOUT ? e->w_out.data() + (size_t)col * J : nullptr;
    });
    if (rc) return rc;

    // team workspace
    HIP_TRY(e->hbuf.alloc((size_t)n_teams * 2 * L * kMaxRows * H * sizeof(float)));
    HIP_TRY(e->qbuf.alloc((size_t)n_teams * kMaxRows * J * sizeof(float)));
    HIP_TRY(e->part.alloc((size_t)n_teams * 2 * kMaxSamples * ts * sizeof(unsigned long long)));
    HIP_TRY(e->dpart.alloc((size_t)n_teams * 2 * kMaxSamples * ts * sizeof(unsigned long long)));
    HIP_TRY(e->bar.alloc((size_t)n_teams * 32 * sizeof(unsigned)));
    HIP_TRY(e->stats.alloc((size_t)n_teams * kStatStride * sizeof(long long)));
    HIP_TRY(e->xcc.alloc((size_t)n_teams * ts * sizeof(int)));
    HIP_TRY(hipMemset(e->hbuf.p, 0, (size_t)n_teams * 2 * L * kMaxRows * H * sizeof(float)));
    HIP_TRY(hipMemset(e->qbuf.p, 0, (size_t)n_teams * kMaxRows * J * sizeof(float)));
    HIP_TRY(hipMemset(e->stats.p, 0, (size_t)n_teams * kStatStride * sizeof(long long)));
    HIP_TRY(hipMemset(e->xcc.p, 0, (size_t)n_teams * ts * sizeof(int)));
    HIP_TRY(hipDeviceSynchronize());
    e->n_teams = n_teams;
    e->team_size = ts;
    return RNNT_OK;
}

int fetch(std::vector<float> &dst, const float *dev, size_t n)
{
    dst.resize(n);
    HIP_TRY(hipMemcpy(dst.data(), dev, n * sizeof(float), hipMemcpyDeviceToHost));
    return RNNT_OK;
}

// Frames examined per utterance per joint step: the configured value, else 8,
// never more than the kMaxSamples samples a step can hold.
int effective_lookahead(const rnnt_engine *e, int rows)
{
    int la = e->lookahead > 0 ? e->lookahead : 8;
    if (la * rows > kMaxSamples) la = std::max(1, kMaxSamples / rows);
    return la;
}

StageDev dev_stage(const PackedStage &ps)
{
    StageDev s;
    s.w = ps.w.as<const float4>();
    s.nks = ps.plan.nks; s.nsteps = ps.plan.nsteps; s.slots = ps.plan.slots; s.kpad = ps.plan.kpad;
    s.rank_stride = ps.plan.rank_stride;
    return s;
}

int check_call(rnnt_engine *e, const float *enc_out, const int32_t *enc_len, int32_t B, int32_t T,
               int32_t max_symbols, int32_t *tokens_out, int32_t *tok_len_out, int32_t cap)
{
    if (!e || !enc_out || !enc_len || !tokens_out || !tok_len_out) return RNNT_ERR_NULL;
    if (B < 1 || B > e->max_B || T < 1 || T > e->max_T || max_symbols < 1 || cap < 1)
        return RNNT_ERR_SHAPE;
    if ((reinterpret_cast<uintptr_t>(enc_out) & 15u) != 0) return RNNT_ERR_SHAPE;
    return RNNT_OK;
}

int run_decode(rnnt_engine *e, int variant, const float *enc_out, const int32_t *enc_len, int32_t B,
               int32_t T, int32_t S, int32_t *tokens_out, int32_t *tok_len_out, int32_t cap,
               int32_t *frames_out, float *logit_out, int32_t *durs_out, hipStream_t stream)
{
    const rnnt_model_desc &d = e->d;
    HIP_TRY(hipEventRecord(e->ev[0], stream));
    HIP_TRY(launch_encoder_projection(enc_out, enc_len, e->w_enc.as<float>(), e->b_enc.as<float>(),
                                      e->P.as<float>(), B, T, d.F, d.J, stream));
    HIP_TRY(hipEventRecord(e->ev[1], stream));
    DecodeParams p{};
    p.F = d.F; p.E = d.E; p.H = d.H; p.L = d.L; p.J = d.J; p.V1 = d.V1; p.D = d.D;
    p.blank = d.blank; p.NOUT = e->NOUT;
    for (int i = 0; i < kMaxDur; ++i) p.durations[i] = e->durations[i];
    p.B = B; p.T = T; p.S = S; p.cap = cap; p.variant = variant;
    p.n_teams = e->n_teams; p.team_size = e->team_size;
    {
        const char *v = std::getenv("RNNT_SERPENTINE");
        p.serpentine = v ? (v[0] == '1') : 1;
    }
    const int rows = (B + e->n_teams - 1) / e->n_teams;
    p.lookahead = effective_lookahead(e, rows);
    p.xstride = e->xstride; p.nu_max = e->nu_max; p.gj_max = e->gj_max;
    p.lds_xz = e->lds_xz; p.lds_red = e->lds_red; p.lds_c = e->lds_c; p.lds_part = e->lds_part;
    p.lds_bias = e->lds_bias; p.lds_bytes = e->lds_bytes; p.gp_max = e->gp_max;
    p.lds_q = e->lds_q; p.q_in_lds = e->q_in_lds; p.qstride = e->qstride;
    p.spin_limit = 1u << 22;
    p.enc_len = enc_len; p.P = e->P.as<float>();
    p.tokens = tokens_out; p.tok_len = tok_len_out; p.frames = frames_out; p.logits = logit_out;
    p.durs = durs_out;
    p.st0 = dev_stage(e->st0);
    for (int l = 1; l < d.L; ++l) p.stl[l] = dev_stage(e->stl[l]);
    p.spred = dev_stage(e->spred);
    p.sjoint = dev_stage(e->sjoint);
    p.T0 = e->T0.as<float>(); p.bias_l = e->bias_l.as<float>();
    p.b_pred = e->b_pred.as<float>(); p.b_out = e->b_out.as<float>();
    p.hbuf = e->hbuf.as<float>(); p.qbuf = e->qbuf.as<float>();
    p.part = e->part.as<unsigned long long>(); p.dpart = e->dpart.as<unsigned long long>();
    p.bar = e->bar.as<unsigned>(); p.abort_flag = e->abort_flag.as<unsigned>();
    p.status = e->status.as<int>(); p.stats = e->stats.as<long long>(); p.xcc = e->xcc.as<int>();
    e->last_B = B;
    HIP_TRY(launch_decode(p, stream));
    HIP_TRY(hipEventRecord(e->ev[2], stream));
    e->timed = true;
    return RNNT_OK;
}

}  // namespace

extern "C" {

int rnnt_engine_create(const rnnt_model_desc *desc, int32_t max_B, int32_t max_T, int32_t flags,
                       rnnt_engine **out)
{
    (void)flags;
    if (!desc || !out) return RNNT_ERR_NULL;
    const rnnt_model_desc &d = *desc;
    if (!d.emb || !d.w_ih || !d.w_hh || !d.b_ih || !d.b_hh || !d.w_enc || !d.b_enc || !d.w_pred ||
        !d.b_pred || !d.w_out || !d.b_out)
        return RNNT_ERR_NULL;
    if (d.D > 0 && !d.durations) return RNNT_ERR_NULL;
    if (d.F < 1 || d.E < 1 || d.H < 1 || d.J < 1 || d.V1 < 2 || d.L < 1 || d.L > kMaxLayers ||
        d.D < 0 || d.D > kMaxDur || d.blank < 0 || d.blank >= d.V1 || max_B < 1 || max_T < 1)
        return RNNT_ERR_SHAPE;
    if (d.F % 16 != 0) return RNNT_ERR_UNSUPPORTED;   // K tile of the projection GEMM
    if (d.V1 > 65535) return RNNT_ERR_UNSUPPORTED;    // argmax partials carry a 16-bit column index
    for (int l = 0; l < d.L; ++l)
        if (!d.w_ih[l] || !d.w_hh[l] || !d.b_ih[l] || !d.b_hh[l]) return RNNT_ERR_NULL;
    for (int i = 0; i < d.D; ++i)
        if (d.durations[i] < 0) return RNNT_ERR_SHAPE;

    int dev = 0;
    HIP_TRY(hipGetDevice(&dev));
    hipDeviceProp_t prop;
    HIP_TRY(hipGetDeviceProperties(&prop, dev));
    int coop = 0;
    HIP_TRY(hipDeviceGetAttribute(&coop, hipDeviceAttributeCooperativeLaunch, dev));
    if (!coop) return RNNT_ERR_UNSUPPORTED;

    rnnt_engine *e = new rnnt_engine();
    struct Guard { rnnt_engine *e; ~Guard() { delete e; } } guard{e};
    e->d = d;
    e->d.durations = nullptr;
    for (int i = 0; i < d.D; ++i) e->durations[i] = d.durations[i];
    e->NOUT = d.V1 + d.D;
    e->max_B = max_B; e->max_T = max_T;
    // Teams per device, chosen from measurements on MI355X: small teams mean less lock-step
    // waiting between utterances and more independent step chains per XCD to hide the
    // exchange latency, large teams mean fewer copies of the weight stream.  8 teams of 32
    // work-groups (one XCD each) up to 16 utterances, 16 teams up to 48, 32 teams beyond.
    int n_teams = max_B <= 16 ? 8 : (max_B <= 48 ? 16 : 32);
    while ((max_B + n_teams - 1) / n_teams > kMaxRows) n_teams *= 2;
    e->n_wg = (prop.multiProcessorCount / n_teams) * n_teams;
    if (e->n_wg < n_teams) return RNNT_ERR_UNSUPPORTED;

    const size_t H = d.H, J = d.J;
    int rc;
    e->w_ih.resize(d.L); e->w_hh.resize(d.L);
    std::vector<float> b_ih, b_hh, bias_l((size_t)d.L * H * 4, 0.f);
    for (int l = 0; l < d.L; ++l) {
        const size_t n_in = l == 0 ? (size_t)d.E : H;
        if ((rc = fetch(e->w_ih[l], d.w_ih[l], 4 * H * n_in))) return rc;
        if ((rc = fetch(e->w_hh[l], d.w_hh[l], 4 * H * H))) return rc;
        if ((rc = fetch(b_ih, d.b_ih[l], 4 * H))) return rc;
        if ((rc = fetch(b_hh, d.b_hh[l], 4 * H))) return rc;
        for (size_t u = 0; u < H; ++u)
            for (size_t g = 0; g < 4; ++g)
                bias_l[((size_t)l * H + u) * 4 + g] = b_ih[g * H + u] + b_hh[g * H + u];
    }
    if ((rc = fetch(e->w_pred, d.w_pred, J * H))) return rc;
    if ((rc = fetch(e->w_out, d.w_out, (size_t)e->NOUT * J))) return rc;

    auto clone = [&](DevBuf &dst, const float *src, size_t n) -> int {
        HIP_TRY(dst.alloc(n * sizeof(float)));
        HIP_TRY(hipMemcpy(dst.p, src, n * sizeof(float), hipMemcpyDeviceToDevice));
        return RNNT_OK;
    };
    if ((rc = clone(e->w_enc, d.w_enc, J * d.F))) return rc;
    if ((rc = clone(e->b_enc, d.b_enc, J))) return rc;
    if ((rc = clone(e->b_pred, d.b_pred, J))) return rc;
    if ((rc = clone(e->b_out, d.b_out, (size_t)e->NOUT))) return rc;
    HIP_TRY(e->bias_l.alloc(bias_l.size() * sizeof(float)));
    HIP_TRY(hipMemcpy(e->bias_l.p, bias_l.data(), bias_l.size() * sizeof(float), hipMemcpyHostToDevice));
    HIP_TRY(e->T0.alloc((size_t)d.V1 * H * 4 * sizeof(float)));
    HIP_TRY(launch_fold_embedding(d.emb, d.w_ih[0], d.b_ih[0], d.b_hh[0], e->T0.as<float>(), d.V1,
                                  d.E, d.H, nullptr));
    HIP_TRY(e->P.alloc((size_t)max_B * max_T * J * sizeof(float)));
    HIP_TRY(e->abort_flag.alloc(sizeof(unsigned)));
    HIP_TRY(e->status.alloc(sizeof(int)));
    HIP_TRY(hipMemset(e->abort_flag.p, 0, sizeof(unsigned)));
    HIP_TRY(hipMemset(e->status.p, 0, sizeof(int)));
    if ((rc = plan_and_pack(e, n_teams))) return rc;
    for (auto &x : e->ev) HIP_TRY(hipEventCreate(&x));
    HIP_TRY(hipDeviceSynchronize());
    guard.e = nullptr;
    *out = e;
    return RNNT_OK;
}

int rnnt_engine_destroy(rnnt_engine *eng)
{
    if (!eng) return RNNT_ERR_NULL;
    hipError_t e = hipDeviceSynchronize();
    delete eng;
    if (e != hipSuccess) return hip_fail(e, "hipDeviceSynchronize");
    return RNNT_OK;
}

int rnnt_engine_configure(rnnt_engine *eng, int32_t n_teams, int32_t lookahead)
{
    if (!eng) return RNNT_ERR_NULL;
    if (lookahead < 0 || lookahead > kMaxSamples || n_teams < 0) return RNNT_ERR_SHAPE;
    HIP_TRY(hipDeviceSynchronize());
    if (n_teams > 0 && n_teams != eng->n_teams) {
        hipDeviceProp_t prop;
        int dev = 0;
        HIP_TRY(hipGetDevice(&dev));
        HIP_TRY(hipGetDeviceProperties(&prop, dev));
        const int old_wg = eng->n_wg, old_teams = eng->n_teams;
        eng->n_wg = (prop.multiProcessorCount / n_teams) * n_teams;
        int rc = eng->n_wg >= n_teams ? plan_and_pack(eng, n_teams) : RNNT_ERR_SHAPE;
        if (rc) {   // put the previous configuration back
            eng->n_wg = old_wg;
            (void)plan_and_pack(eng, old_teams);
            return rc;
        }
    }
    eng->lookahead = lookahead;
    return RNNT_OK;
}

int rnnt_greedy_decode(rnnt_engine *eng, const float *enc_out, const int32_t *enc_len, int32_t B,
                       int32_t T, int32_t max_symbols, int32_t *tokens_out, int32_t *tok_len_out,
                       int32_t cap, int32_t *frames_out, float *logit_out, rnnt_stream_t stream)
{
    int rc = check_call(eng, enc_out, enc_len, B, T, max_symbols, tokens_out, tok_len_out, cap);
    if (rc) return rc;
    if (eng->d.D != 0) return RNNT_ERR_VARIANT;
    return run_decode(eng, kFrameLooping, enc_out, enc_len, B, T, max_symbols, tokens_out,
                      tok_len_out, cap, frames_out, logit_out, nullptr,
                      static_cast<hipStream_t>(stream));
}

int rnnt_label_looping_decode(rnnt_engine *eng, const float *enc_out, const int32_t *enc_len,
                              int32_t B, int32_t T, int32_t max_symbols, int32_t *tokens_out,
                              int32_t *tok_len_out, int32_t cap, int32_t *frames_out,
                              float *logit_out, rnnt_stream_t stream)
{
    int rc = check_call(eng, enc_out, enc_len, B, T, max_symbols, tokens_out, tok_len_out, cap);
    if (rc) return rc;
    if (eng->d.D != 0) return RNNT_ERR_VARIANT;
    return run_decode(eng, kLabelLooping, enc_out, enc_len, B, T, max_symbols, tokens_out,
                      tok_len_out, cap, frames_out, logit_out, nullptr,
                      static_cast<hipStream_t>(stream));
}

int tdt_label_looping_decode(rnnt_engine *eng, const float *enc_out, const int32_t *enc_len,
                             int32_t B, int32_t T, int32_t max_symbols, int32_t *tokens_out,
                             int32_t *tok_len_out, int32_t cap, int32_t *frames_out,
                             float *logit_out, int32_t *durations_out, rnnt_stream_t stream)
{
    int rc = check_call(eng, enc_out, enc_len, B, T, max_symbols, tokens_out, tok_len_out, cap);
    if (rc) return rc;
    if (eng->d.D == 0) return RNNT_ERR_VARIANT;
    return run_decode(eng, kTdtLabelLooping, enc_out, enc_len, B, T, max_symbols, tokens_out,
                      tok_len_out, cap, frames_out, logit_out, durations_out,
                      static_cast<hipStream_t>(stream));
}

int rnnt_encoder_projection(rnnt_engine *eng, const float *enc_out, const int32_t *enc_len,
                            int32_t B, int32_t T, float *proj_out, rnnt_stream_t stream)
{
    if (!eng || !enc_out || !enc_len || !proj_out) return RNNT_ERR_NULL;
    if (B < 1 || T < 1) return RNNT_ERR_SHAPE;
    if ((reinterpret_cast<uintptr_t>(enc_out) & 15u) != 0) return RNNT_ERR_SHAPE;
    HIP_TRY(launch_encoder_projection(enc_out, enc_len, eng->w_enc.as<float>(),
                                      eng->b_enc.as<float>(), proj_out, B, T, eng->d.F, eng->d.J,
                                      static_cast<hipStream_t>(stream)));
    return RNNT_OK;
}

int rnnt_engine_status(rnnt_engine *eng, int32_t *status_out)
{
    if (!eng || !status_out) return RNNT_ERR_NULL;
    HIP_TRY(hipDeviceSynchronize());
    HIP_TRY(hipMemcpy(status_out, eng->status.p, sizeof(int), hipMemcpyDeviceToHost));
    return RNNT_OK;
}

int rnnt_engine_stats(rnnt_engine *eng, rnnt_stats *out)
{
    if (!eng || !out) return RNNT_ERR_NULL;
    HIP_TRY(hipDeviceSynchronize());
    std::vector<long long> st((size_t)eng->n_teams * kStatStride);
    std::vector<int> xcc((size_t)eng->n_teams * eng->team_size);
    HIP_TRY(hipMemcpy(st.data(), eng->stats.p, st.size() * sizeof(long long), hipMemcpyDeviceToHost));
    HIP_TRY(hipMemcpy(xcc.data(), eng->xcc.p, xcc.size() * sizeof(int), hipMemcpyDeviceToHost));
    std::memset(out, 0, sizeof(*out));
    for (int t = 0; t < eng->n_teams; ++t) {
        const long long *s = st.data() + (size_t)t * kStatStride;
        out->pred_steps += s[kStatPred];
        out->joint_steps += s[kStatJoint];
        out->joint_samples += s[kStatSamples];
        out->barrier_polls += s[kStatPolls];
        out->max_pred_steps = std::max<int64_t>(out->max_pred_steps, s[kStatPred]);
        out->max_joint_steps = std::max<int64_t>(out->max_joint_steps, s[kStatJoint]);
        // work-group i belongs to team i % n_teams
        int first = -1, mixed = 0;
        for (int r = 0; r < eng->team_size; ++r) {
            const int id = xcc[(size_t)r * eng->n_teams + t];
            if (first < 0) first = id;
            else if (id != first) mixed = 1;
        }
        if (t < std::min(eng->last_B, eng->n_teams)) out->xcd_mismatch += mixed;
    }
    if (const char *dump = std::getenv("RNNT_DUMP_PHASES")) {
        if (dump[0] == '1') {
            for (int t = 0; t < eng->n_teams; ++t) {
                const long long *s = st.data() + (size_t)t * kStatStride;
                std::fprintf(stderr, "team %d: %lld prediction steps, %lld joint steps; rank 0 phase timers (us):",
                             t, s[kStatPred], s[kStatJoint]);
                double tot = 0;
                for (int i = 0; i < 19; ++i) {
                    std::fprintf(stderr, " %d:%.0f", i, s[kStatCount + i] * 0.01);
                    tot += s[kStatCount + i] * 0.01;
                }
                std::fprintf(stderr, " total:%.0f\n", tot);
            }
        }
    }
    out->n_teams = eng->n_teams;
    out->team_size = eng->team_size;
    const int rows = (eng->last_B + eng->n_teams - 1) / std::max(1, eng->n_teams);
    out->lookahead = effective_lookahead(eng, std::max(1, rows));
    if (eng->timed) {
        HIP_TRY(hipEventElapsedTime(&out->projection_ms, eng->ev[0], eng->ev[1]));
        HIP_TRY(hipEventElapsedTime(&out->decode_ms, eng->ev[1], eng->ev[2]));
    }
    return RNNT_OK;
}

const char *rnnt_status_string(int code)
{
    switch (code) {
    case RNNT_OK: return "ok";
    case RNNT_ERR_NULL: return "a required pointer is NULL";
    case RNNT_ERR_SHAPE: return "a dimension, count or alignment is out of range";
    case RNNT_ERR_VARIANT: return "RNN-T call on a TDT engine or TDT call on an RNN-T engine";
    case RNNT_ERR_HIP: return g_hip_error.empty() ? "HIP runtime error" : g_hip_error.c_str();
    case RNNT_ERR_UNSUPPORTED: return "the device or the model shape is not supported";
    default: return "unknown status code";
    }
}

}  // extern "C"
