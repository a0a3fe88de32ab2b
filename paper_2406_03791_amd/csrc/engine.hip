// Host side of the C ABI declared in include/rnnt_greedy.h: argument checks,
// weight repacking, workspace, launches.  Every step of the decode runs in the kernels; the
// only arithmetic on the host is done once per engine, on weights: the two LSTM bias vectors
// of a layer are added (b_ih + b_hh, one fp32 addition per gate, the order the oracle adds
// them in) while the weights are repacked.
#include "../../include/rnnt_greedy.h"

#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdlib>
#include <cstring>
#include <functional>
#include <initializer_list>
#include <memory>
#include <string>
#include <vector>

#include "engine.h"
#include "pack.h"

using namespace rnnt;

namespace {

thread_local std::string g_hip_error;

}  // namespace

// Records the text rnnt_status_string(RNNT_ERR_HIP) returns; shared with the probes.
int rnnt::hip_fail(hipError_t e, const char *what)
{
    g_hip_error = std::string("HIP error in ") + what + ": " + hipGetErrorString(e);
    return RNNT_ERR_HIP;
}

namespace {

#define HIP_TRY(expr)                                           \
    do {                                                        \
        hipError_t e_ = (expr);                                 \
        if (e_ != hipSuccess) return hip_fail(e_, #expr);       \
    } while (0)

constexpr int kLdsBytes = 160 * 1024;   // LDS of one gfx950 compute unit
// Utterances one launch of the decode kernel takes.  A call with more is decoded in consecutive
// launches of up to this many (the projection runs once for the whole call): with more than 8
// rows per team the joint steps hold few frames per row and the prediction stages run on four
// row groups, and one launch of 256 utterances measured 29 ms against 2 x 10.8 ms for two of 128
// (label looping; Algorithm 1 52 against 2 x 19 ms, TDT 16.6 against 2 x 5.9 ms).
constexpr int kLaunchRows = 128;
// A wait on another work-group polls again about once a microsecond: a few seconds.
constexpr unsigned kDefaultSpinLimit = 1u << 22;
constexpr int kStaticLds = 3072;        // kept free for the kernel's static LDS (control block)

// Scratch of the entry point that allocates nothing (rnnt_label_looping_decode_noalloc): the
// projected frames and the team workspace of one call.  One copy per device, held until the
// process ends.  In host code this name is only a handle for hipGetSymbolAddress: the address
// kernels and copies use is the one that call returns (rnnt_engine::scratch).
static __device__ __align__(256) unsigned char scratch[RNNT_NOALLOC_SCRATCH_BYTES];

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

// One way of cutting the device into teams, with the weights packed for it and its workspace.
// A team of `team_size` work-groups runs the prediction network for all its utterances; it is
// made of `groups` joint groups of `jteam_size` work-groups, each of which owns a share of the
// team's utterances and searches for their next labels on its own.  groups == 1 is the plain
// arrangement (Algorithm 1 always uses it: its lock-step covers the whole team).
// Device memory a decode call works in besides its inputs, its outputs and the packed weights:
// the projected frames and what the teams exchange.  An engine owns one such set per team
// layout (allocated when the layout is planned); the entry point that allocates nothing carves
// the same set out of the library's static scratch array instead.
struct Workspace {
    float *P = nullptr;                 // [B, T, J] projected frames
    float *hbuf = nullptr, *qbuf = nullptr;
    unsigned long long *part = nullptr, *dpart = nullptr, *lpart = nullptr, *rowx = nullptr;
    unsigned long long *xh = nullptr, *xq = nullptr;
    unsigned *bar = nullptr, *abort_flag = nullptr;
    int *status = nullptr, *xcc = nullptr;
    long long *stats = nullptr;
};

// Bytes of each part of the team workspace for a layout (everything but P).
struct WorkspaceSizes {
    size_t hbuf, qbuf, part, rowx, bar, stats, xcc, xh, xq;
};

struct TeamConfig {
    int n_teams = 0, team_size = 0, groups = 1, jteam_size = 0;
    int for_B = 0;          // utterances per launch the layout was planned for (its rows per team follow)
    bool is_frame = false;  // a layout of Algorithm 1 (else of the label-looping decoders)
    PackedStage st0, stl[kMaxLayers], spred, sjoint;
    DevBuf hbuf, qbuf, part, dpart, lpart, rowx, bar, stats, xcc, xh, xq;
    Workspace ws;          // the buffers above plus the engine's P, abort flag and status word
    int xstride = 0, nu_max = 0, gj_max = 0, gp_max = 0;
    int lds_xz = 0, lds_red = 0, lds_c = 0, lds_part = 0, lds_bias = 0, lds_q = 0;
    int lds_scale = 0;     // scales of e4m3- or e2m1-stored weights in the bfloat16 mode, per stage [column][block]
    int sc_nb_in = 1;      // scale blocks per row the input stages of the layers above the first have in LDS
    int q_in_lds = 0, qstride = 0;
    int fast_pred = 0, lds_hc = 0;
    int n_tail = 0;        // joint output columns computed outside the MFMA stage, one per rank from rank 0 on
    int nout_m = 0;        // joint output columns of the MFMA stage (a whole number of groups per rank when n_tail > 0)
    int lds_tail = 0;
    DevBuf w_tail;         // [n_tail][J rounded up to 4]: the tail columns' weight rows
    int samples_cap = kMaxSamples;   // (utterance, frame) pairs of a joint step the LDS layout has room for
    int rcap = 0;
    int rg_planned = 0;
    unsigned lds_bytes = 0;
};

struct rnnt_engine {
    rnnt_model_desc d{};
    int durations[kMaxDur] = {0};
    int NOUT = 0, max_B = 0, max_T = 0;
    int plan_B = 0;        // utterances the team layouts are planned for: min(max_B, kLaunchRows)
    int n_wg = 0;          // work-groups the device can keep resident (one per CU)
    int lookahead = 0;
    int search_steps = 0;  // 0: chosen per call, -1: no limit, > 0: as given
    int wt = kWeightF32;   // storage of the packed (streamed) weights
    bool plain_launch = false;   // RNNT_FLAG_PLAIN_LAUNCH
    bool multi_blank = false;    // RNNT_FLAG_MULTI_BLANK: the D extra output columns are big blanks
    float *logp_out = nullptr;   // caller's [B, cap] buffer for log-probabilities, or none
    int32_t *done = nullptr;     // caller's [B] completion flags, or none
    unsigned spin_limit = kDefaultSpinLimit;   // polls a device-side wait may repeat before the call gives up
    // host copies of the weights that get repacked when the team layout changes
    std::vector<std::vector<float>> w_ih, w_hh;
    std::vector<float> w_pred, w_out;
    // device: weights used as they are, derived tables, workspace
    DevBuf w_enc, b_enc, T0, bias_l, b_pred, b_out;
    DevBuf sc_hh, sc_ih, sc_pred, sc_out;   // e4m3 storage in the bfloat16 mode: power-of-two scale of every weight row
    DevBuf P, abort_flag, status;
    // Team layouts, one per range of launch sizes in which the measured best arrangement (or
    // the rows per team, hence the prediction path) changes, in ascending order of for_B: a
    // launch of nb utterances runs in the first layout planned for at least nb.  An engine for
    // many utterances so decodes a small batch the way an engine made for that batch would.
    std::vector<std::unique_ptr<TeamConfig>> frame_cfgs;   // Algorithm 1
    std::vector<std::unique_ptr<TeamConfig>> label_cfgs;   // label looping, RNN-T and TDT
    // layouts (and workspaces) the launches of the last call ran in: where its statistics are
    struct Used { const TeamConfig *t; Workspace ws; int nb; };   // nb: utterances of its latest launch
    std::vector<Used> last_used;
    Workspace last_ws;      // where the last call kept its status word
    int last_B = 0;
    void *scratch = nullptr;   // device address of the library's static scratch array on the engine's device
    hipEvent_t ev[3] = {nullptr, nullptr, nullptr};   // before projection, before decode, after
    bool timed = false;
    ~rnnt_engine() { for (auto &x : ev) if (x) (void)hipEventDestroy(x); }
};

namespace {

int upload_stage(PackedStage &ps, int ts, const std::function<int(int)> &ngroups,
                 const std::function<const float *(int, int, int)> &row_of, bool row_scaled)
{
    std::vector<uint32_t> host = pack_stage(ps.plan, ts, ngroups, row_of, row_scaled);
    // the kernel's prefetch may run a few steps past the end of the last wave's run
    host.resize(host.size() + (size_t)kAheadSteps * 64 * 4, 0u);
    HIP_TRY(ps.w.alloc(host.size() * sizeof(uint32_t)));
    HIP_TRY(hipMemcpy(ps.w.p, host.data(), host.size() * sizeof(uint32_t), hipMemcpyHostToDevice));
    return RNNT_OK;
}

WorkspaceSizes workspace_sizes(int n_teams, int ts, int groups, int L, int H, int J)
{
    WorkspaceSizes z;
    const int tj = ts / groups;
    z.hbuf = (size_t)n_teams * 2 * L * kMaxRows * H * sizeof(float);
    z.qbuf = (size_t)n_teams * kMaxRows * J * sizeof(float);
    z.part = (size_t)n_teams * groups * 2 * kMaxSamples * tj * sizeof(unsigned long long);
    z.rowx = (size_t)n_teams * 2 * kMaxRows * sizeof(unsigned long long);
    z.bar = (size_t)n_teams * 32 * sizeof(unsigned);
    z.stats = (size_t)n_teams * kStatStride * sizeof(long long);
    z.xcc = (size_t)n_teams * ts * sizeof(int);
    z.xh = (size_t)n_teams * L * kMaxRows * H * sizeof(unsigned long long);
    z.xq = (size_t)n_teams * kMaxRows * J * sizeof(unsigned long long);
    return z;
}

// Choose the stage plans and the LDS layout for `n_teams` teams of `groups` joint groups and
// upload the repacked weights.  Synchronous.
int plan_and_pack(rnnt_engine *e, TeamConfig &t, int n_teams, int groups, int for_B)
{
    const rnnt_model_desc &d = e->d;
    if (n_teams < 1 || n_teams > e->n_wg || groups < 1) return RNNT_ERR_SHAPE;
    const int ts = e->n_wg / n_teams;
    if (ts < 1 || ts % groups != 0) return RNNT_ERR_SHAPE;
    const int tj = ts / groups;
    const int rows_max = (for_B + n_teams - 1) / n_teams;
    t.for_B = for_B;
    if (rows_max > kMaxRows) return RNNT_ERR_SHAPE;
    const int H = d.H, L = d.L, J = d.J;
    auto nu_of = [&](int r) { return range_hi(r, ts, H) - range_lo(r, ts, H); };
    const int gp_all = (J + 3) / 4;
    int gj_all = (e->NOUT + 3) / 4;          // output groups of the joint stage's MFMA part
    auto gp_of = [&](int r) { return range_hi(r, ts, gp_all) - range_lo(r, ts, gp_all); };
    auto gj_of = [&](int r) { return range_hi(r, tj, gj_all) - range_lo(r, tj, gj_all); };
    int nu_max = 0, gp_max = 0, gj_max = 0;
    for (int r = 0; r < ts; ++r) {
        nu_max = std::max(nu_max, nu_of(r));
        gp_max = std::max(gp_max, gp_of(r));
    }
    for (int r = 0; r < tj; ++r) gj_max = std::max(gj_max, gj_of(r));
    const int tail_k = (J + 3) & ~3;          // a tail column's weight row in LDS (see plan_joint_stage)
    const int gj_all_full = gj_all, gj_max_full = gj_max;
    // Stage plans and LDS layout.  Stages with more groups than blocks are first planned with K
    // slices over several passes (best use of the blocks); if the partial sums of such a plan do
    // not fit the LDS, they fall back to unsliced tasks.
    // the prediction kernels exist for 1, 2 and 4 row groups (pred_row_groups): the layout is
    // sized for the instance that will run, not for the rows alone
    const int rgp = pred_row_groups(rows_max), rows_pad = rgp * 4;
    // Samples a joint step may hold: rows of a joint group x frames examined per row (the
    // configured lookahead, else 8; 16 is always allowed for), at most kMaxSamples.  The z rows
    // and the argmax candidates in LDS are sized for it.
    const int rows_j_max = (rows_max + groups - 1) / groups;
    // The joint kernels exist for 1, 2, 4 and 8 row groups (joint_row_groups) and an instance
    // uses all of its rows and the partial-sum stride of its own group count: the capacity is
    // that of the instance that runs the largest step, not the largest step itself.
    // (Algorithm 1 examines as many frames per row as keep a step at 16 samples unless configured)
    const int la_plan = e->lookahead > 0 ? e->lookahead : (t.is_frame ? std::max(1, std::min(8, 16 / rows_j_max)) : 8);
    const int samples_want = std::min(kMaxSamples, std::max(16, rows_j_max * la_plan));
    const int rgj = joint_row_groups(samples_want);
    const int samples_cap = rgj * 4;
    int off = 0;
    auto take = [&](int n) { int o = off; off += (n + 3) & ~3; return o; };
    int xstride = 0;
    for (int attempt = 0; attempt < 2; ++attempt) {
        const bool single = attempt == 1;
        t.st0.plan = make_stage_plan(H, L * nu_max, e->wt, single);
        for (int l = 1; l < L; ++l) t.stl[l].plan = make_stage_plan(H, nu_max, e->wt, single);
        t.spred.plan = make_stage_plan(H, gp_max, e->wt, single);
        gj_all = gj_all_full; gj_max = gj_max_full;
        {
            const JointSplit js = plan_joint_stage(e->NOUT, J, tj, e->wt, single);
            t.sjoint.plan = js.plan; t.n_tail = js.n_tail; t.nout_m = js.nout_m;
            if (js.n_tail) { gj_all = js.nout_m / 4; gj_max = js.nout_m / (4 * tj); }
        }
        const int gjx = gj_max + (t.n_tail ? 1 : 0);    // candidates per sample: groups + the tail column
        int kpad = std::max({t.st0.plan.kpad, t.spred.plan.kpad, t.sjoint.plan.kpad});
        for (int l = 1; l < L; ++l) kpad = std::max(kpad, t.stl[l].plan.kpad);
        xstride = kpad + 4;
        auto red_need = [&](const StagePlan &pl, int grp, int rg) {
            return std::min(grp * pl.nks, kBlocksPerWg * pl.slots) * red_task_stride(rg);
        };
        int xz = std::max(L * rows_pad * xstride, samples_cap * xstride);
        int red = red_need(t.st0.plan, L * nu_max, rgp);
        for (int l = 1; l < L; ++l) red = std::max(red, red_need(t.stl[l].plan, nu_max, rgp));
        red = std::max(red, red_need(t.spred.plan, gp_max, rgp));
        // the joint step's argmax candidates (two 64-bit keys per sample and output group, the
        // per-sample maxima and the per-group exponential sums of the scores) go into the
        // partial-sum region when the joint sums sit in the z rows, else into the z rows
        const int cand_need = samples_cap * gjx * 4 + kMaxSamples + samples_cap * gjx + 8;
        if (t.sjoint.plan.slots == 1) {
            xz = std::max(xz, red_need(t.sjoint.plan, gj_max, rgj));
            red = std::max(red, cand_need);
        } else {
            red = std::max(red, red_need(t.sjoint.plan, gj_max, rgj));
            xz = std::max(xz, cand_need);
        }
        off = 0;
        t.lds_xz = take(xz);
        t.lds_red = take(red);
        t.rcap = rows_max;
        t.rg_planned = rgp;
        t.samples_cap = samples_cap;
        t.lds_c = take(L * 2 * nu_max * rows_max);
        t.lds_part = take(L * nu_max * rows_max * 4);
        t.lds_bias = take(4 * (gp_max + gj_max + L * nu_max));
        // row scales: projection, output, recurrent and input matrices of every layer
        {
            int nb_in = 1;
            for (int l = 1; l < L; ++l) nb_in = std::max(nb_in, scale_blocks(e->wt, t.stl[l].plan.kpad));
            t.sc_nb_in = nb_in;
            const bool scales = e->wt == kWeightFp8Bf16Arith || e->wt == kWeightFp4Bf16Arith;
            // one byte per scale (its exponent)
            t.lds_scale = scales ? take((gp_max * scale_blocks(e->wt, t.spred.plan.kpad) +
                                         gj_max * scale_blocks(e->wt, t.sjoint.plan.kpad) +
                                         L * nu_max * (scale_blocks(e->wt, t.st0.plan.kpad) + nb_in)))
                                 : 0;
        }
        // a tail column's weight row and its per-wave partial sums
        t.lds_tail = t.n_tail ? take(tail_k + kWaves * kMaxSamples) : 0;
        // room for a joint group's q rows as well (needed by joint groups, see below)
        const int q_need = groups > 1 ? ((rows_max + groups - 1) / groups) * ((J + 3) & ~3) : 0;
        if ((unsigned)(off + q_need) * 4u + (unsigned)kStaticLds <= (unsigned)kLdsBytes) break;
        if (single) return RNNT_ERR_UNSUPPORTED;
    }
    // q of the team's rows stays in LDS between joint steps when there is room
    t.qstride = (J + 3) & ~3;
    const int q_rows = (rows_max + groups - 1) / groups;   // a joint group keeps its own rows only
    t.q_in_lds = ((unsigned)(off + q_rows * t.qstride) * 4u + (unsigned)kStaticLds <= (unsigned)kLdsBytes);
    // joint groups that search on their own read q while the rest of the team may already be
    // rewriting the global copy: they need the LDS copy
    if (groups > 1 && !t.q_in_lds) return RNNT_ERR_UNSUPPORTED;
    t.lds_q = t.q_in_lds ? take(q_rows * t.qstride) : 0;
    // Teams of up to four utterances keep copies of all their hidden vectors in LDS and exchange
    // them as tagged words (prediction_step_fast), when there is room and the widths fit the
    // two words per row a thread polls.
    const int hc_need = 2 * L * 4 * xstride;
    t.fast_pred = rows_max <= 4 && t.q_in_lds && H <= 2 * kThreads && J <= 2 * kThreads &&
                  (unsigned)(off + hc_need) * 4u + (unsigned)kStaticLds <= (unsigned)kLdsBytes;
    t.lds_hc = t.fast_pred ? take(hc_need) : 0;
    t.lds_bytes = (unsigned)off * 4u;
    t.xstride = xstride; t.nu_max = nu_max; t.gj_max = gj_max; t.gp_max = gp_max;

    // weights
    int rc;
    const bool scaled = e->wt == kWeightFp8Bf16Arith;
    rc = upload_stage(t.st0, ts, [&](int r) { return L * nu_of(r); },
                      [&](int r, int g, int j) -> const float * {
                          const int nu = nu_of(r);
                          const int layer = g / nu, u = range_lo(r, ts, H) + g % nu;
                          return e->w_hh[layer].data() + (size_t)(j * H + u) * H;
                      }, scaled);
    if (rc) return rc;
    for (int l = 1; l < L; ++l) {
        rc = upload_stage(t.stl[l], ts, nu_of, [&](int r, int g, int j) -> const float * {
            return e->w_ih[l].data() + (size_t)(j * H + range_lo(r, ts, H) + g) * H;
        }, scaled);
        if (rc) return rc;
    }
    rc = upload_stage(t.spred, ts, gp_of, [&](int r, int g, int j) -> const float * {
        const int col = (range_lo(r, ts, gp_all) + g) * 4 + j;
        return col < J ? e->w_pred.data() + (size_t)col * H : nullptr;
    }, scaled);
    if (rc) return rc;
    rc = upload_stage(t.sjoint, tj, gj_of, [&](int r, int g, int j) -> const float * {
        const int col = (range_lo(r, tj, gj_all) + g) * 4 + j;
        return col < t.nout_m ? e->w_out.data() + (size_t)col * J : nullptr;
    }, scaled);
    if (rc) return rc;
    if (t.n_tail) {
        std::vector<float> rows((size_t)t.n_tail * tail_k, 0.f);
        for (int i = 0; i < t.n_tail; ++i)
            std::copy_n(e->w_out.data() + (size_t)(t.nout_m + i) * J, J, rows.data() + (size_t)i * tail_k);
        HIP_TRY(t.w_tail.alloc(rows.size() * sizeof(float)));
        HIP_TRY(hipMemcpy(t.w_tail.p, rows.data(), rows.size() * sizeof(float), hipMemcpyHostToDevice));
    }

    // team workspace
    const WorkspaceSizes z = workspace_sizes(n_teams, ts, groups, L, H, J);
    HIP_TRY(t.hbuf.alloc(z.hbuf));
    HIP_TRY(t.qbuf.alloc(z.qbuf));
    HIP_TRY(t.part.alloc(z.part));
    HIP_TRY(t.dpart.alloc(z.part));
    HIP_TRY(t.lpart.alloc(z.part));
    HIP_TRY(t.rowx.alloc(z.rowx));
    HIP_TRY(t.bar.alloc(z.bar));
    HIP_TRY(t.stats.alloc(z.stats));
    HIP_TRY(t.xcc.alloc(z.xcc));
    HIP_TRY(t.xh.alloc(z.xh));
    HIP_TRY(t.xq.alloc(z.xq));
    HIP_TRY(hipMemset(t.hbuf.p, 0, z.hbuf));
    HIP_TRY(hipMemset(t.qbuf.p, 0, z.qbuf));
    HIP_TRY(hipMemset(t.stats.p, 0, z.stats));
    HIP_TRY(hipMemset(t.xcc.p, 0, z.xcc));
    HIP_TRY(hipDeviceSynchronize());
    t.n_teams = n_teams;
    t.team_size = ts;
    t.groups = groups;
    t.jteam_size = tj;
    t.ws.P = e->P.as<float>();
    t.ws.abort_flag = e->abort_flag.as<unsigned>();
    t.ws.status = e->status.as<int>();
    t.ws.hbuf = t.hbuf.as<float>(); t.ws.qbuf = t.qbuf.as<float>();
    t.ws.part = t.part.as<unsigned long long>(); t.ws.dpart = t.dpart.as<unsigned long long>();
    t.ws.lpart = t.lpart.as<unsigned long long>(); t.ws.rowx = t.rowx.as<unsigned long long>();
    t.ws.bar = t.bar.as<unsigned>(); t.ws.stats = t.stats.as<long long>(); t.ws.xcc = t.xcc.as<int>();
    t.ws.xh = t.xh.as<unsigned long long>(); t.ws.xq = t.xq.as<unsigned long long>();
    return RNNT_OK;
}

// Default team layouts, chosen from measurements on MI355X (all with the rank-to-XCD mapping
// of spread_layout, so the size of a team does not change where its weights are read from).
//   Algorithm 1: one utterance per team while the teams keep at least 8 work-groups (no
//   lock-step waiting between utterances, and a prediction step per label of one utterance
//   only): 8, 16 or 32 teams; beyond 32 utterances the teams take several rows each.
//   Label looping: 8 teams of 32 up to 16 utterances, 16 teams of 16 beyond; two joint groups
//   per team from 9 utterances on, four for an RNN-T with five to eight utterances per team.
//   Engines for one or two utterances: 4 teams of 64 for either decoder (2-5 % faster than 8
//   teams of 32 there, equal from four utterances on; teams of 128 and 256 are slower).
int default_layouts(rnnt_engine *e)
{
    // A layout whose state does not fit the compute units' local memory (wide layers, many
    // layers, many rows per team) is followed by the others that divide the device, teams
    // with fewer rows first, before the engine is refused.
    auto with_fallbacks = [&](TeamConfig &cfg, int first, int groups_first, int for_B) {
        int rc = plan_and_pack(e, cfg, first, groups_first, for_B);
        for (int g = groups_first / 2; rc == RNNT_ERR_UNSUPPORTED && g >= 1; g /= 2)
            rc = plan_and_pack(e, cfg, first, g, for_B);
        for (int n = first * 2; rc == RNNT_ERR_UNSUPPORTED && n <= e->n_wg / 2; n *= 2)
            if (e->n_wg % n == 0) rc = plan_and_pack(e, cfg, n, 1, for_B);
        for (int n = first / 2; rc == RNNT_ERR_UNSUPPORTED && n >= 1; n /= 2)
            if (e->n_wg % n == 0 && (for_B + n - 1) / n <= kMaxRows) rc = plan_and_pack(e, cfg, n, 1, for_B);
        return rc;
    };
    // launch sizes up to which one arrangement is the measured best; the last layout is planned
    // for the largest launch the engine makes
    auto sizes = [&](std::initializer_list<int> upto) {
        std::vector<int> v;
        for (int b : upto)
            if (b < e->plan_B) v.push_back(b);
        v.push_back(e->plan_B);
        return v;
    };
    e->frame_cfgs.clear();
    e->label_cfgs.clear();
    e->last_used.clear();
    // (32 and 64: one and two rows per team of the 32-team arrangement, whose LDS plan keeps the
    // finer K slicing that the plan for four rows has no room for)
    for (int B : sizes({2, 8, 16, 32, 64})) {
        int nf = B <= 2 ? 4 : (B <= 8 ? 8 : (B <= 16 ? 16 : 32));
        while (nf > 1 && e->n_wg % nf != 0) nf /= 2;
        while ((B + nf - 1) / nf > kMaxRows) nf *= 2;
        e->frame_cfgs.emplace_back(new TeamConfig());
        e->frame_cfgs.back()->is_frame = true;
        const int rc = with_fallbacks(*e->frame_cfgs.back(), nf, 1, B);
        // a launch size whose state fits in no layout ends the list: larger calls are then
        // decoded in launches of the largest size that does fit
        if (rc == RNNT_ERR_UNSUPPORTED && e->frame_cfgs.size() > 1) { e->frame_cfgs.pop_back(); break; }
        if (rc) return rc;
    }
    // label looping: up to 64 utterances a team has at most four rows (the prediction step
    // that keeps the hidden vectors in LDS), beyond that four joint groups for an RNN-T
    for (int B : sizes({2, 8, 16, 64})) {
        int nl = B <= 2 ? 4 : (B <= 16 ? 8 : 16);
        while (nl > 1 && e->n_wg % nl != 0) nl /= 2;
        while ((B + nl - 1) / nl > kMaxRows) nl *= 2;
        const int rows = (B + nl - 1) / nl;
        const int ts = e->n_wg / nl;
        int groups = (B > 8 && rows >= 2 && ts % 2 == 0 && ts / 2 >= 8) ? 2 : 1;
        // five to eight rows per team: four groups of two rows keep a joint step at 16 samples
        // (2-3 % faster than two groups for an RNN-T at 72-128 utterances; slower for TDT)
        if (groups == 2 && rows >= 5 && rows <= 8 && ts % 4 == 0 && e->d.D == 0) groups = 4;
        e->label_cfgs.emplace_back(new TeamConfig());
        const int rc = with_fallbacks(*e->label_cfgs.back(), nl, groups, B);
        if (rc == RNNT_ERR_UNSUPPORTED && e->label_cfgs.size() > 1) { e->label_cfgs.pop_back(); break; }
        if (rc) return rc;
    }
    return RNNT_OK;
}

// The layout a launch of nb utterances runs in: the first one planned for at least nb.
const TeamConfig &pick_layout(const std::vector<std::unique_ptr<TeamConfig>> &cfgs, int nb)
{
    for (const auto &t : cfgs)
        if (t->for_B >= nb) return *t;
    return *cfgs.back();
}

int fetch(std::vector<float> &dst, const float *dev, size_t n)
{
    dst.resize(n);
    HIP_TRY(hipMemcpy(dst.data(), dev, n * sizeof(float), hipMemcpyDeviceToHost));
    return RNNT_OK;
}

// Frames examined per utterance per joint step: the configured value, else 8 (Algorithm 1:
// as many as keep a step at 16 samples, at most 8; 16 for calls of one or two utterances),
// never more than the kMaxSamples samples a joint group's step can hold.
int effective_lookahead(const rnnt_engine *e, const TeamConfig &t, int B)
{
    const int rows_team = (B + t.n_teams - 1) / t.n_teams;
    const int rows = std::max(1, (rows_team + t.groups - 1) / t.groups);
    int la = e->lookahead > 0 ? e->lookahead : 8;
    if (e->lookahead == 0 && t.is_frame) la = std::min(8, std::max(1, 16 / rows));
    // one or two utterances: most of the device idles, a joint step is cheap next to its fixed
    // cost, and 16 frames per step measured 2-5 % faster than 8 (slower from four utterances on)
    if (e->lookahead == 0 && B <= 2) la = 16;
    if (la * rows > t.samples_cap) la = std::max(1, t.samples_cap / rows);
    return la;
}

// Joint steps a label-looping search may take before the team's next prediction step (0: no
// limit): the configured value, else chosen from measurements.  A group with two or more rows
// stops after one step, so that a row in a long run of blanks does not hold up the rows that
// have their label; single-row groups of a team with four or more rows stop after two.
int effective_search_steps(const rnnt_engine *e, const TeamConfig &t, int B)
{
    if (t.is_frame) return 0;      // Algorithm 1 has no label search
    if (e->search_steps < 0) return 0;
    if (e->search_steps > 0) return e->search_steps;
    const int rows_team = (B + t.n_teams - 1) / t.n_teams;
    const int rows_group = (rows_team + t.groups - 1) / t.groups;
    if (rows_group >= 2) return 1;
    return rows_team >= 4 ? 2 : 0;
}

StageDev dev_stage(const PackedStage &ps)
{
    StageDev s;
    s.w = ps.w.as<const float4>();
    s.nks = ps.plan.nks; s.nsteps = ps.plan.nsteps; s.slots = ps.plan.slots; s.kpad = ps.plan.kpad;
    s.rank_stride = ps.plan.rank_stride;
    return s;
}

// Which work-group is which rank of which team.  Work-groups are dispatched to the 8 XCDs
// round-robin, and every XCD has its own 4 MB L2.  With rank = index % team_size the ranks
// r, r + 8, ... of every team share an XCD, so that XCD only ever reads its eighth of the
// packed weights (3 MB in fp32) and keeps it in its L2: the weight streams of all teams then
// come from L2 instead of the fabric.  The teams' exchanges cross XCDs, which costs little,
// because exchange data bypasses the L2s in any case.  Needs a team size that is a multiple
// of 8; otherwise team = index % n_teams, which keeps a team on as few XCDs as possible.
bool spread_layout(const TeamConfig &t) { return t.team_size % 8 == 0; }

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
               int32_t *frames_out, float *logit_out, int32_t *durs_out, hipStream_t stream,
               const Workspace *static_ws = nullptr)
{
    const rnnt_model_desc &d = e->d;
    const auto &cfgs = variant == kFrameLooping ? e->frame_cfgs : e->label_cfgs;
    // every launch reads the projected frames of the whole call from one buffer
    float *P = static_ws ? static_ws->P : e->P.as<float>();
    HIP_TRY(hipEventRecord(e->ev[0], stream));
    HIP_TRY(launch_encoder_projection(enc_out, enc_len, e->w_enc.as<float>(), e->b_enc.as<float>(),
                                      P, B, T, d.F, d.J, is_bf16_arith(e->wt), stream));
    HIP_TRY(hipEventRecord(e->ev[1], stream));
    e->last_B = B;
    e->last_used.clear();
    // the utterances [off, off + nb) per launch; status word and step counts add up over the launches
    const int launch_rows = cfgs.back()->for_B;      // at most kLaunchRows
    for (int off = 0; off < B; off += launch_rows) {
        const int nb = std::min(launch_rows, B - off);
        const TeamConfig &t = pick_layout(cfgs, nb);
        const Workspace &ws = static_ws ? *static_ws : t.ws;
        bool first_in_layout = true;
        for (auto &u : e->last_used)
            if (u.t == &t) { first_in_layout = false; u.nb = nb; }
        if (first_in_layout) e->last_used.push_back({&t, ws, nb});
        e->last_ws = ws;
        DecodeParams p{};
        p.F = d.F; p.E = d.E; p.H = d.H; p.L = d.L; p.J = d.J; p.V1 = d.V1; p.D = d.D;
        p.blank = d.blank; p.NOUT = e->NOUT;
        p.VT = d.V1;
        if (e->multi_blank) { p.VT = e->NOUT; p.D = 0; }   // one distribution over labels, blank and big blanks
        for (int i = 0; i < kMaxDur; ++i) p.durations[i] = e->durations[i];
        p.T = T; p.S = S; p.cap = cap; p.variant = variant;
        p.n_teams = t.n_teams; p.team_size = t.team_size;
        p.groups = t.groups; p.jteam_size = t.jteam_size;
        p.serpentine = 1;
        p.spread = spread_layout(t) ? 1 : 0;
        p.plain_launch = e->plain_launch ? 1 : 0;
        p.wt = e->wt;
        p.xstride = t.xstride; p.nu_max = t.nu_max; p.gj_max = t.gj_max;
        p.lds_xz = t.lds_xz; p.lds_red = t.lds_red; p.lds_c = t.lds_c; p.lds_part = t.lds_part;
        p.lds_scale = t.lds_scale; p.sc_nb_in = t.sc_nb_in;
        p.sc_hh = e->sc_hh.as<float>(); p.sc_ih = e->sc_ih.as<float>();
        p.sc_pred = e->sc_pred.as<float>(); p.sc_out = e->sc_out.as<float>();
        p.lds_bias = t.lds_bias; p.lds_bytes = t.lds_bytes; p.gp_max = t.gp_max;
        p.lds_q = t.lds_q; p.q_in_lds = t.q_in_lds; p.qstride = t.qstride;
        p.fast_pred = t.fast_pred; p.lds_hc = t.lds_hc;
        p.n_tail = t.n_tail; p.nout_m = t.nout_m; p.lds_tail = t.lds_tail;
        p.w_tail = t.n_tail ? t.w_tail.as<float>() : nullptr;
        p.rcap = t.rcap;
        p.rg_planned = t.rg_planned;
        p.samples_cap = t.samples_cap;
        p.spin_limit = e->spin_limit;
        p.st0 = dev_stage(t.st0);
        for (int l = 1; l < d.L; ++l) p.stl[l] = dev_stage(t.stl[l]);
        p.spred = dev_stage(t.spred);
        p.sjoint = dev_stage(t.sjoint);
        p.T0 = e->T0.as<float>(); p.bias_l = e->bias_l.as<float>();
        p.b_pred = e->b_pred.as<float>(); p.b_out = e->b_out.as<float>();
        p.hbuf = ws.hbuf; p.qbuf = ws.qbuf;
        p.part = ws.part; p.dpart = ws.dpart; p.lpart = ws.lpart; p.rowx = ws.rowx;
        p.bar = ws.bar; p.abort_flag = ws.abort_flag;
        p.status = ws.status; p.stats = ws.stats; p.xcc = ws.xcc;
        p.xh = ws.xh; p.xq = ws.xq;
        const long long oc = (long long)off * cap;
        p.B = nb;
        p.lookahead = effective_lookahead(e, t, nb);
        p.search_steps = effective_search_steps(e, t, nb);
        p.enc_len = enc_len + off; p.P = P + (long long)off * T * d.J;
        p.tokens = tokens_out + oc; p.tok_len = tok_len_out + off;
        p.frames = frames_out ? frames_out + oc : nullptr;
        p.logits = logit_out ? logit_out + oc : nullptr;
        p.durs = durs_out ? durs_out + oc : nullptr;
        p.logps = e->logp_out ? e->logp_out + oc : nullptr;
        p.done = e->done ? e->done + off : nullptr;
        // the status word is the engine's (or the static workspace's) for all layouts; the
        // step counts are kept per layout and start at zero in a layout's first launch
        HIP_TRY(launch_decode(p, off == 0, first_in_layout, stream));
    }
    HIP_TRY(hipEventRecord(e->ev[2], stream));
    e->timed = true;
    return RNNT_OK;
}

}  // namespace

extern "C" {

int rnnt_engine_create(const rnnt_model_desc *desc, int32_t max_B, int32_t max_T, int32_t flags,
                       rnnt_engine **out)
{
    if (!desc || !out) return RNNT_ERR_NULL;
    if (flags & ~(RNNT_FLAG_BF16_WEIGHTS | RNNT_FLAG_FP8_WEIGHTS | RNNT_FLAG_PLAIN_LAUNCH | RNNT_FLAG_BF16_ARITHMETIC |
                  RNNT_FLAG_MULTI_BLANK | RNNT_FLAG_FP4_WEIGHTS))
        return RNNT_ERR_SHAPE;
    {   // at most one of the three formats, or the bfloat16 mode with e4m3- or e2m1-stored weights
        const int fmt = flags & (RNNT_FLAG_BF16_WEIGHTS | RNNT_FLAG_FP8_WEIGHTS | RNNT_FLAG_BF16_ARITHMETIC |
                                 RNNT_FLAG_FP4_WEIGHTS);
        if ((fmt & (fmt - 1)) && fmt != (RNNT_FLAG_FP8_WEIGHTS | RNNT_FLAG_BF16_ARITHMETIC) &&
            fmt != (RNNT_FLAG_FP4_WEIGHTS | RNNT_FLAG_BF16_ARITHMETIC))
            return RNNT_ERR_SHAPE;
        if (fmt == RNNT_FLAG_FP4_WEIGHTS) return RNNT_ERR_SHAPE;   // 4-bit codes exist for the bfloat16 mode only
    }
    const rnnt_model_desc &d = *desc;
    if (!d.emb || !d.w_ih || !d.w_hh || !d.b_ih || !d.b_hh || !d.w_enc || !d.b_enc || !d.w_pred ||
        !d.b_pred || !d.w_out || !d.b_out)
        return RNNT_ERR_NULL;
    if (d.D > 0 && !d.durations) return RNNT_ERR_NULL;
    if (d.F < 1 || d.E < 1 || d.H < 1 || d.J < 1 || d.V1 < 2 || d.L < 1 || d.L > kMaxLayers ||
        d.D < 0 || d.D > kMaxDur || d.blank < 0 || d.blank >= d.V1 || max_B < 1 || max_T < 1)
        return RNNT_ERR_SHAPE;
    if (d.F % 16 != 0) return RNNT_ERR_UNSUPPORTED;   // K tile of the projection GEMM
    if ((long long)max_B * max_T > 0x7fffffffLL) return RNNT_ERR_UNSUPPORTED;   // frame numbers are 32-bit
    if (d.H % 4 != 0 || d.J % 4 != 0) return RNNT_ERR_UNSUPPORTED;   // rows are read 16 bytes at a time
    if (d.V1 + d.D > 65535) return RNNT_ERR_UNSUPPORTED;   // argmax partials carry a 16-bit column index
    for (int l = 0; l < d.L; ++l)
        if (!d.w_ih[l] || !d.w_hh[l] || !d.b_ih[l] || !d.b_hh[l]) return RNNT_ERR_NULL;
    const bool multi_blank = (flags & RNNT_FLAG_MULTI_BLANK) != 0;
    if (multi_blank && d.D < 1) return RNNT_ERR_SHAPE;
    for (int i = 0; i < d.D; ++i)
        if (d.durations[i] < (multi_blank ? 1 : 0)) return RNNT_ERR_SHAPE;   // a big blank moves on by at least one frame

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
    e->plan_B = std::min((int)max_B, kLaunchRows);
    e->wt = (flags & RNNT_FLAG_FP8_WEIGHTS) ? kWeightFp8
                                            : ((flags & RNNT_FLAG_BF16_WEIGHTS) ? kWeightBf16 : kWeightF32);
    if (flags & RNNT_FLAG_BF16_ARITHMETIC)
        e->wt = (flags & RNNT_FLAG_FP8_WEIGHTS) ? kWeightFp8Bf16Arith
                                                : ((flags & RNNT_FLAG_FP4_WEIGHTS) ? kWeightFp4Bf16Arith : kWeightBf16Arith);
    e->plain_launch = (flags & RNNT_FLAG_PLAIN_LAUNCH) != 0;
    e->multi_blank = multi_blank;
    e->n_wg = (prop.multiProcessorCount / 32) * 32;   // every layout divides it
    if (e->n_wg < 32) return RNNT_ERR_UNSUPPORTED;

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
    if (is_bf16_arith(e->wt)) {
        // bfloat16 mode: the matrices of the per-step products are rounded here (ties to even, the
        // same rounding the kernels apply to the vectors), then stored as bf16 without loss
        auto round_all = [](std::vector<float> &v) {
            for (float &x : v) {
                uint32_t u;
                std::memcpy(&u, &x, sizeof u);
                if ((u & 0x7f800000u) != 0x7f800000u) { u += 0x7fffu + ((u >> 16) & 1u); u &= 0xffff0000u; }
                std::memcpy(&x, &u, sizeof u);
            }
        };
        round_all(e->w_pred); round_all(e->w_out);
        for (int l = 0; l < d.L; ++l) { round_all(e->w_hh[l]); if (l > 0) round_all(e->w_ih[l]); }
    }
    if (e->wt == kWeightBf16) {
        // compact storage is lossless or refused: every streamed weight must be a bf16 value
        auto is_bf16 = [](const std::vector<float> &v) {
            for (float x : v) {
                uint32_t u;
                std::memcpy(&u, &x, sizeof u);
                if (u & 0xffffu) return false;
            }
            return true;
        };
        bool ok = is_bf16(e->w_pred) && is_bf16(e->w_out);
        for (int l = 0; l < d.L; ++l) ok = ok && is_bf16(e->w_hh[l]) && (l == 0 || is_bf16(e->w_ih[l]));
        if (!ok) return RNNT_ERR_SHAPE;
    }
    if (e->wt == kWeightFp8) {
        auto is_e4m3 = [](const std::vector<float> &v) {
            uint8_t code;
            for (float x : v)
                if (!e4m3_bits(x, &code)) return false;
            return true;
        };
        bool ok = is_e4m3(e->w_pred) && is_e4m3(e->w_out);
        for (int l = 0; l < d.L; ++l) ok = ok && is_e4m3(e->w_hh[l]) && (l == 0 || is_e4m3(e->w_ih[l]));
        if (!ok) return RNNT_ERR_SHAPE;
    }
    if (e->wt == kWeightFp8Bf16Arith || e->wt == kWeightFp4Bf16Arith) {
        // e4m3: every row is kept as codes times a power of two of its own, which the kernel's
        // widening instruction applies for free: lossless or refused, as above, but per row,
        // the scale 2^k with k = e4m3_row_exponent(row).  e2m1: the same per block of
        // kScaleBlock consecutive weights of a row, k = e2m1_block_exponent(block).
        // scales[row][block], nb blocks per row.
        const bool fp4 = e->wt == kWeightFp4Bf16Arith;
        const int wt = e->wt;
        auto scan = [fp4, wt](const std::vector<float> &m, size_t rows, size_t cols, std::vector<float> &scales) {
            const size_t nb = (size_t)scale_blocks_of_matrix(wt, (int)cols);
            scales.assign(rows * nb, 1.0f);
            uint8_t code;
            for (size_t r = 0; r < rows; ++r)
                for (size_t b = 0; b < nb; ++b) {
                    const size_t lo = fp4 ? b * kScaleBlock : 0, n = fp4 ? std::min((size_t)kScaleBlock, cols - lo) : cols;
                    const float *blk = m.data() + r * cols + lo;
                    const int k = fp4 ? e2m1_block_exponent(blk, (int)n) : e4m3_row_exponent(blk, (int)n);
                    for (size_t i = 0; i < n; ++i) {
                        const float v = std::ldexp(blk[i], -k);
                        if (!(fp4 ? e2m1_bits(v, &code) : e4m3_bits(v, &code))) return false;
                    }
                    scales[r * nb + b] = std::ldexp(1.0f, k);
                }
            return true;
        };
        const size_t nbh = (size_t)scale_blocks_of_matrix(wt, (int)H);
        std::vector<float> s_pred, s_out, rows_s;
        std::vector<float> s_hh((size_t)d.L * H * 4 * nbh, 1.0f), s_ih((size_t)d.L * H * 4 * nbh, 1.0f);
        bool ok = scan(e->w_pred, J, H, s_pred) && scan(e->w_out, (size_t)e->NOUT, J, s_out);
        for (int l = 0; ok && l < d.L; ++l) {
            // unit-major with the four gates together, as the biases of the layers are kept
            ok = scan(e->w_hh[l], 4 * H, H, rows_s);
            for (size_t u = 0; ok && u < H; ++u)
                for (size_t g = 0; g < 4; ++g)
                    for (size_t b = 0; b < nbh; ++b)
                        s_hh[(((size_t)l * H + u) * 4 + g) * nbh + b] = rows_s[(g * H + u) * nbh + b];
            if (l == 0 || !ok) continue;
            ok = scan(e->w_ih[l], 4 * H, H, rows_s);
            for (size_t u = 0; ok && u < H; ++u)
                for (size_t g = 0; g < 4; ++g)
                    for (size_t b = 0; b < nbh; ++b)
                        s_ih[(((size_t)l * H + u) * 4 + g) * nbh + b] = rows_s[(g * H + u) * nbh + b];
        }
        if (!ok) return RNNT_ERR_SHAPE;
        auto put = [&](DevBuf &dst, const std::vector<float> &v) -> int {
            HIP_TRY(dst.alloc(v.size() * sizeof(float)));
            HIP_TRY(hipMemcpy(dst.p, v.data(), v.size() * sizeof(float), hipMemcpyHostToDevice));
            return RNNT_OK;
        };
        if ((rc = put(e->sc_pred, s_pred)) || (rc = put(e->sc_out, s_out)) || (rc = put(e->sc_hh, s_hh)) ||
            (rc = put(e->sc_ih, s_ih)))
            return rc;
    }

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
    const bool bf16_mode = is_bf16_arith(e->wt);
    if (bf16_mode) HIP_TRY(launch_round_bf16(e->w_enc.as<float>(), (long long)J * d.F, nullptr));
    HIP_TRY(launch_fold_embedding(d.emb, d.w_ih[0], d.b_ih[0], d.b_hh[0], e->T0.as<float>(), d.V1,
                                  d.E, d.H, bf16_mode, nullptr));
    // this device's copy of the static scratch array (each device has its own, at its own address)
    HIP_TRY(hipGetSymbolAddress(&e->scratch, HIP_SYMBOL(scratch)));
    HIP_TRY(e->P.alloc((size_t)max_B * max_T * J * sizeof(float)));
    HIP_TRY(e->abort_flag.alloc(sizeof(unsigned)));
    HIP_TRY(e->status.alloc(sizeof(int)));
    HIP_TRY(hipMemset(e->abort_flag.p, 0, sizeof(unsigned)));
    HIP_TRY(hipMemset(e->status.p, 0, sizeof(int)));
    if ((rc = default_layouts(e))) return rc;
    for (auto &x : e->ev) HIP_TRY(hipEventCreate(&x));
    HIP_TRY(hipDeviceSynchronize());
    guard.e = nullptr;
    *out = e;
    return RNNT_OK;
}

int rnnt_quantize_rows_e4m3(const float *w, int64_t rows, int64_t cols, float *out, float *scales_out)
{
    if (!w || !out) return RNNT_ERR_NULL;
    if (rows < 0 || cols < 0 || cols > 0x7fffffff) return RNNT_ERR_SHAPE;
    for (int64_t r = 0; r < rows; ++r) {
        const float *row = w + r * cols;
        for (int64_t i = 0; i < cols; ++i)
            if (!std::isfinite(row[i])) return RNNT_ERR_SHAPE;
    }
    for (int64_t r = 0; r < rows; ++r) {
        const float *row = w + r * cols;
        float *dst = out + r * cols;
        const int k = e4m3_row_exponent(row, (int)cols);
        for (int64_t i = 0; i < cols; ++i) {
            const float v = std::ldexp(row[i], -k);
            dst[i] = std::ldexp(e4m3_round(std::fabs(v) > 448.0f ? std::copysign(448.0f, v) : v), k);
        }
        if (scales_out) scales_out[r] = std::ldexp(1.0f, k);
    }
    return RNNT_OK;
}

int rnnt_quantize_blocks_e2m1(const float *w, int64_t rows, int64_t cols, float *out, float *scales_out)
{
    static_assert(kScaleBlock == RNNT_FP4_BLOCK, "the header states the block length");
    if (!w || !out) return RNNT_ERR_NULL;
    if (rows < 0 || cols < 0 || cols > 0x7fffffff) return RNNT_ERR_SHAPE;
    for (int64_t i = 0; i < rows * cols; ++i)
        if (!std::isfinite(w[i])) return RNNT_ERR_SHAPE;
    const int64_t nb = (cols + kScaleBlock - 1) / kScaleBlock;
    for (int64_t r = 0; r < rows; ++r)
        for (int64_t b = 0; b < nb; ++b) {
            const int64_t lo = b * kScaleBlock, n = std::min<int64_t>(kScaleBlock, cols - lo);
            const float *blk = w + r * cols + lo;
            float *dst = out + r * cols + lo;
            const int k = e2m1_block_exponent(blk, (int)n);
            for (int64_t i = 0; i < n; ++i) {
                const float v = std::ldexp(blk[i], -k);
                dst[i] = std::ldexp(e2m1_round(std::fabs(v) > 6.0f ? std::copysign(6.0f, v) : v), k);
            }
            if (scales_out) scales_out[r * nb + b] = std::ldexp(1.0f, k);
        }
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

int rnnt_engine_configure(rnnt_engine *eng, int32_t n_teams, int32_t joint_groups, int32_t lookahead,
                          int32_t search_steps)
{
    if (!eng) return RNNT_ERR_NULL;
    if (lookahead < 0 || lookahead > kMaxSamples || n_teams < 0 || joint_groups < 0)
        return RNNT_ERR_SHAPE;
    if (n_teams == 0 && joint_groups != 0) return RNNT_ERR_SHAPE;
    if (search_steps < -1) return RNNT_ERR_SHAPE;
    HIP_TRY(hipDeviceSynchronize());
    if (n_teams > 0) {
        eng->last_used.clear();       // the workspaces the last call's statistics live in go away
        eng->last_ws = Workspace();
        eng->lookahead = lookahead;   // the layouts are sized for it
        // one layout for launches of every size: plain teams for Algorithm 1; the label-looping
        // decoders split each team further
        if (eng->n_wg % n_teams != 0) return RNNT_ERR_SHAPE;
        std::unique_ptr<TeamConfig> f(new TeamConfig()), l(new TeamConfig());
        f->is_frame = true;
        int rc = plan_and_pack(eng, *f, n_teams, 1, eng->plan_B);
        if (!rc) rc = plan_and_pack(eng, *l, n_teams, joint_groups ? joint_groups : 1, eng->plan_B);
        if (rc) return rc;            // the layouts in use stay as they were
        eng->frame_cfgs.clear(); eng->label_cfgs.clear();
        eng->frame_cfgs.push_back(std::move(f));
        eng->label_cfgs.push_back(std::move(l));
    }
    const bool replan = n_teams == 0 && lookahead != eng->lookahead;
    eng->lookahead = lookahead;
    eng->search_steps = search_steps;
    if (replan) {
        // the LDS layouts are sized for the samples of a joint step, which depend on the lookahead
        eng->last_used.clear();
        eng->last_ws = Workspace();
        int rc = RNNT_OK;
        for (auto &t : eng->frame_cfgs)
            if (!rc) rc = plan_and_pack(eng, *t, t->n_teams, 1, t->for_B);
        for (auto &t : eng->label_cfgs)
            if (!rc) rc = plan_and_pack(eng, *t, t->n_teams, t->groups, t->for_B);
        if (rc) {
            eng->lookahead = 0;
            (void)default_layouts(eng);
            return rc;
        }
    }
    return RNNT_OK;
}

int rnnt_engine_set_logp_output(rnnt_engine *eng, float *logp_out)
{
    if (!eng) return RNNT_ERR_NULL;
    eng->logp_out = logp_out;
    return RNNT_OK;
}

int rnnt_engine_set_done_flags(rnnt_engine *eng, int32_t *done)
{
    if (!eng) return RNNT_ERR_NULL;
    eng->done = done;
    return RNNT_OK;
}

int rnnt_engine_set_wait_limit(rnnt_engine *eng, int64_t polls)
{
    if (!eng) return RNNT_ERR_NULL;
    if (polls < -1 || polls > 0xffffffffll) return RNNT_ERR_SHAPE;
    eng->spin_limit = polls < 0 ? kDefaultSpinLimit : (unsigned)polls;
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
    if (eng->d.D != 0 && !eng->multi_blank) return RNNT_ERR_VARIANT;
    return run_decode(eng, kLabelLooping, enc_out, enc_len, B, T, max_symbols, tokens_out,
                      tok_len_out, cap, frames_out, logit_out, nullptr,
                      static_cast<hipStream_t>(stream));
}

int rnnt_label_looping_decode_noalloc(rnnt_engine *eng, const float *enc_out, const int32_t *enc_len,
                                      int32_t B, int32_t T, int32_t max_symbols, int32_t *tokens_out,
                                      int32_t *tok_len_out, int32_t cap, int32_t *frames_out,
                                      float *logit_out, rnnt_stream_t stream)
{
    int rc = check_call(eng, enc_out, enc_len, B, T, max_symbols, tokens_out, tok_len_out, cap);
    if (rc) return rc;
    if (eng->d.D != 0 && !eng->multi_blank) return RNNT_ERR_VARIANT;
    if (!eng->scratch) return RNNT_ERR_UNSUPPORTED;
    // one launch only: the workspace is that of one layout
    if (B > eng->label_cfgs.back()->for_B) return RNNT_ERR_SCRATCH;
    // carve the call's workspace out of the static array, every part 256-byte aligned
    const TeamConfig &t = pick_layout(eng->label_cfgs, B);
    const WorkspaceSizes z = workspace_sizes(t.n_teams, t.team_size, t.groups, eng->d.L, eng->d.H, eng->d.J);
    size_t off = 0;
    auto take = [&](size_t bytes) { const size_t o = off; off += (bytes + 255) & ~(size_t)255; return o; };
    const size_t o_P = take((size_t)B * T * eng->d.J * sizeof(float));
    const size_t o_h = take(z.hbuf), o_q = take(z.qbuf), o_p = take(z.part), o_d = take(z.part);
    const size_t o_l = take(z.part), o_r = take(z.rowx), o_b = take(z.bar), o_s = take(z.stats);
    const size_t o_x = take(z.xcc), o_a = take(sizeof(unsigned)), o_st = take(sizeof(int));
    const size_t o_xh = take(z.xh), o_xq = take(z.xq);
    if (off > (size_t)RNNT_NOALLOC_SCRATCH_BYTES) return RNNT_ERR_SCRATCH;
    unsigned char *base = static_cast<unsigned char *>(eng->scratch);
    Workspace ws;
    ws.P = reinterpret_cast<float *>(base + o_P);
    ws.hbuf = reinterpret_cast<float *>(base + o_h);
    ws.qbuf = reinterpret_cast<float *>(base + o_q);
    ws.part = reinterpret_cast<unsigned long long *>(base + o_p);
    ws.dpart = reinterpret_cast<unsigned long long *>(base + o_d);
    ws.lpart = reinterpret_cast<unsigned long long *>(base + o_l);
    ws.rowx = reinterpret_cast<unsigned long long *>(base + o_r);
    ws.bar = reinterpret_cast<unsigned *>(base + o_b);
    ws.stats = reinterpret_cast<long long *>(base + o_s);
    ws.xcc = reinterpret_cast<int *>(base + o_x);
    ws.abort_flag = reinterpret_cast<unsigned *>(base + o_a);
    ws.status = reinterpret_cast<int *>(base + o_st);
    ws.xh = reinterpret_cast<unsigned long long *>(base + o_xh);
    ws.xq = reinterpret_cast<unsigned long long *>(base + o_xq);
    // the reset kernel the decode launch starts with clears the counters, flags, tags and
    // statistics the previous call left; the decode kernel zeroes the state rows it reads
    return run_decode(eng, kLabelLooping, enc_out, enc_len, B, T, max_symbols, tokens_out,
                      tok_len_out, cap, frames_out, logit_out, nullptr,
                      static_cast<hipStream_t>(stream), &ws);
}

int tdt_label_looping_decode(rnnt_engine *eng, const float *enc_out, const int32_t *enc_len,
                             int32_t B, int32_t T, int32_t max_symbols, int32_t *tokens_out,
                             int32_t *tok_len_out, int32_t cap, int32_t *frames_out,
                             float *logit_out, int32_t *durations_out, rnnt_stream_t stream)
{
    int rc = check_call(eng, enc_out, enc_len, B, T, max_symbols, tokens_out, tok_len_out, cap);
    if (rc) return rc;
    if (eng->d.D == 0 || eng->multi_blank) return RNNT_ERR_VARIANT;
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
                                      is_bf16_arith(eng->wt), static_cast<hipStream_t>(stream)));
    return RNNT_OK;
}

int rnnt_engine_status(rnnt_engine *eng, int32_t *status_out)
{
    if (!eng || !status_out) return RNNT_ERR_NULL;
    HIP_TRY(hipDeviceSynchronize());
    const int *src = eng->last_ws.status ? eng->last_ws.status : eng->status.as<int>();
    HIP_TRY(hipMemcpy(status_out, src, sizeof(int), hipMemcpyDeviceToHost));
    return RNNT_OK;
}

int rnnt_engine_stats(rnnt_engine *eng, rnnt_stats *out)
{
    if (!eng || !out) return RNNT_ERR_NULL;
    HIP_TRY(hipDeviceSynchronize());
    std::memset(out, 0, sizeof(*out));
    if (eng->last_used.empty()) return RNNT_OK;
    // a call of more utterances than one launch takes may have run in more than one layout:
    // the counts are sums over them, the longest chains the largest per-team sums
    for (const auto &u : eng->last_used) {
        const TeamConfig *t = u.t;
        std::vector<long long> st((size_t)t->n_teams * kStatStride);
        std::vector<int> xcc((size_t)t->n_teams * t->team_size);
        HIP_TRY(hipMemcpy(st.data(), u.ws.stats, st.size() * sizeof(long long), hipMemcpyDeviceToHost));
        HIP_TRY(hipMemcpy(xcc.data(), u.ws.xcc, xcc.size() * sizeof(int), hipMemcpyDeviceToHost));
        for (int i = 0; i < t->n_teams; ++i) {
            const long long *s = st.data() + (size_t)i * kStatStride;
            out->pred_steps += s[kStatPred];
            out->joint_steps += s[kStatJoint];
            out->joint_samples += s[kStatSamples];
            out->barrier_polls += s[kStatPolls];
            out->max_pred_steps = std::max<int64_t>(out->max_pred_steps, s[kStatPred]);
            out->max_joint_steps = std::max<int64_t>(out->max_joint_steps, s[kStatJoint]);
            if (i >= std::min(u.nb, t->n_teams)) continue;   // the team had no utterance and left at once
            // Work-groups whose XCD is not the one their rank's weight slice is kept on: rank r of
            // every team is meant to sit on the XCD of rank r % 8 of the first team (layouts whose
            // teams are not multiples of 8 keep a team on one XCD instead).
            for (int r = 0; r < t->team_size; ++r) {
                const int id = xcc[(size_t)r * t->n_teams + i];
                const int want = spread_layout(*t) ? xcc[(size_t)(r % 8) * t->n_teams]
                                                   : xcc[(size_t)i];
                out->xcd_mismatch += id != want;
            }
        }
    }
    // the layout of the call's first launch
    const TeamConfig *t = eng->last_used.front().t;
    const int nb = std::max(1, std::min(eng->last_B, t->for_B));
    out->n_teams = t->n_teams;
    out->team_size = t->team_size;
    out->joint_groups = t->groups;
    out->lookahead = effective_lookahead(eng, *t, nb);
    out->search_steps = effective_search_steps(eng, *t, nb);
    if (eng->timed) {
        HIP_TRY(hipEventElapsedTime(&out->projection_ms, eng->ev[0], eng->ev[1]));
        HIP_TRY(hipEventElapsedTime(&out->decode_ms, eng->ev[1], eng->ev[2]));
    }
    return RNNT_OK;
}

int rnnt_engine_phase_timers(rnnt_engine *eng, int32_t team, double *us_out, int32_t n)
{
    if (!eng || !us_out) return RNNT_ERR_NULL;
#ifdef RNNT_PROFILE
    // (of the layout the call's first launch ran in)
    if (eng->last_used.empty()) return RNNT_ERR_SHAPE;
    const TeamConfig *t = eng->last_used.front().t;
    if (team < 0 || team >= t->n_teams || n < 0) return RNNT_ERR_SHAPE;
    HIP_TRY(hipDeviceSynchronize());
    long long raw[kStatProf];
    HIP_TRY(hipMemcpy(raw, eng->last_used.front().ws.stats + (size_t)team * kStatStride + kStatCount, sizeof raw,
                      hipMemcpyDeviceToHost));
    for (int i = 0; i < n; ++i) us_out[i] = i < kStatProf ? raw[i] * 0.01 : 0.0;   // 100 MHz clock
    return RNNT_OK;
#else
    (void)team; (void)n;
    return RNNT_ERR_UNSUPPORTED;
#endif
}

const char *rnnt_status_string(int code)
{
    switch (code) {
    case RNNT_OK: return "ok";
    case RNNT_ERR_NULL: return "a required pointer is NULL";
    case RNNT_ERR_SHAPE: return "a dimension, count or alignment is out of range";
    case RNNT_ERR_VARIANT: return "this decoder does not run this kind of model (RNN-T, TDT or multi-blank engine)";
    case RNNT_ERR_HIP: return g_hip_error.empty() ? "HIP runtime error" : g_hip_error.c_str();
    case RNNT_ERR_UNSUPPORTED: return "the device or the model shape is not supported";
    case RNNT_ERR_SCRATCH: return "the call needs more scratch than the static array holds (RNNT_NOALLOC_SCRATCH_BYTES)";
    default: return "unknown status code";
    }
}

}  // extern "C"
