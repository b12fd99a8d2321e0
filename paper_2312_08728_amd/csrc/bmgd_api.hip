// Host side of libbmgd: contexts, the two-slot buffer state machine, stream/event ordering between the
// buffering step and the computation step (Section 2.1), and the C ABI declared in include/bmgd.h.
#include "../../include/bmgd.h"
#include "bmgd_internal.h"

#include <math.h>
#include <stdio.h>
#include <string.h>

#include <algorithm>
#include <map>
#include <new>
#include <tuple>
#include <string>
#include <utility>
#include <vector>

using namespace bmgd;

namespace {

thread_local std::string g_create_error;

}  // namespace

void bmgd::set_create_error(const char* msg) { g_create_error = msg ? msg : ""; }

namespace {

constexpr size_t kAlign = 256;
constexpr int kMaxGroups = 256;                    // upper bound used to size the partial-sum scratch

size_t align_up(size_t v) { return (v + kAlign - 1) / kAlign * kAlign; }

struct Layout {
    size_t slot_x[2], slot_y[2], perm, theta, partial, ll_part, ll_theta, sync, sm_state, wbt, u, rt, xt, gram[2], prod[2], gram_perm, gram_cache, gram_cache_set, prod_cache, prod_cache_set, opt_m, opt_s, opt_len, eval, swa, total;
};

struct Slot {
    void* x = nullptr;
    void* y = nullptr;
    int64_t rows = 0;
    hipEvent_t copy_done = nullptr;                // the copy_end event of the slot's last load (owned by its RunRecord):
                                                   // one marker on the copy stream serves timing and ordering
    hipEvent_t compute_done = nullptr;             // recorded on the compute stream after the slot was read
    bool was_read = false;
};

struct RunRecord {                                 // events of one buffer, for the overlap statistics
    hipEvent_t copy_start = nullptr, copy_end = nullptr, start = nullptr, end = nullptr;
    bool has_copy = false;
    bool owns_end = true;                          // false: `end` is the stop event of the run's last chain launch
    int n_chain = 0, n_prep = 0;                   // launches of this run with an entry in open_chain / open_prep
};

constexpr size_t kMaxOpenRuns = 4096;              // runs whose events are held before the oldest half is folded

}  // namespace

struct bmgd_ctx {
    bmgd_config cfg{};
    int device = 0;
    int num_cus = 0;
    int64_t theta_len = 0;
    size_t x_itemsize = 4;
    void* ws = nullptr;
    bool owns_ws = false;
    Layout lay{};
    Slot slots[2];
    int next_slot = 0;                             // slot the next load goes to
    int pending = -1;                              // slot loaded but not yet run
    int32_t* perm = nullptr;
    float* theta = nullptr;
    float* partial = nullptr;
    unsigned long long* ll_part = nullptr;
    unsigned long long* ll_theta = nullptr;
    unsigned* sync = nullptr;
    SoftmaxState* sm_state = nullptr;              // softmax: learning rate and update counts of the pass being enqueued (device)
    // softmax, BMGD_CHAIN_GRAPH: the launches of one pass over one buffer, captured once per (buffer, rows, partition
    // slot) on a stream of the library's own and replayed on the caller's stream
    std::map<std::tuple<const void*, const void*, const int32_t*, int64_t>, hipGraphExec_t> pass_graphs;
    hipStream_t capture_stream = nullptr;
    void* wbt = nullptr;                           // softmax: bf16 copy of W, transposed
    float* u = nullptr;                            // softmax: logits scratch
    void* rt = nullptr;                            // softmax: residual scratch
    void* xt = nullptr;                            // softmax: transposed mini-batches of one pass
    // eq. (3.1) form.  The pre-pass over the buffer (partitions, moment matrices) runs on the caller's compute
    // stream and the one-workgroup chain on a stream of the library's own, so that the pre-pass of the next
    // buffer overlaps the chain of this one; two sets of partitions and matrices alternate.
    float* gram[2] = {nullptr, nullptr};
    bool products = false;                         // BMGD_CHAIN_PRODUCT: the steps of a launch multiplied together (gram_products.hip)
    float* prod[2] = {nullptr, nullptr};
    int psel = 0;
    bool prod_dense[2] = {false, false};           // the set last held dense matrices (the chain's layout needs its padding zero)
    int32_t* gram_perm[2] = {nullptr, nullptr};
    struct CachedMoments {                         // moment matrices of buffer index k under its fixed partition
        bool valid = false;
        // BMGD_CHAIN_PRODUCT: the product of the steps of a run over this buffer, kept as well while it stays the same
        // (made with this rate and this number of passes, no table of rates)
        bool prod_valid = false;
        float prod_alpha = 0.f;
        int prod_np = 0;
        int64_t rows = 0;
        hipEvent_t ready = nullptr;                // completes when the kernel that formed them has
    };
    std::vector<CachedMoments> mcache;             // [n_buffers] when cfg.cache_moments
    char* gram_cache = nullptr;
    char* prod_cache = nullptr;
    hipEvent_t cache_chain_done = nullptr;         // behind the latest chain that read the cache
    hipStream_t chain_stream = nullptr;
    hipEvent_t prep_done[2] = {nullptr, nullptr};  // stop event of the moment kernel that filled set i (owned by open_prep)
    hipEvent_t chain_done[2] = {nullptr, nullptr}; // stop event of the chain that read set i last (owned by open_chain)
    bool chain_pending[2] = {false, false};
    int gsel = 0;
    double busy_until = 0;                         // ms since `base` up to which run time has been accounted
    // learning rate per update (bmgd_set_lr_schedule): device copy for the kernels, host copy for the paths that
    // pass the rate per launch; lr_pos = updates enqueued since the schedule was set
    float* lr_tab_dev = nullptr;
    std::vector<float> lr_tab_host;
    int64_t lr_pos = 0;
    // optimizer state (kind != BMGD_OPT_SGD): arrays laid out like theta, update count for Adam's bias corrections
    const int32_t* subset = nullptr;               // rows the next run is restricted to (device; bmgd_set_row_subset)
    int64_t subset_count = 0;
    int64_t subset_limit = 0;                      // rows of the buffer those indices refer to (set when the run starts)
    float* swa = nullptr;                          // running average of theta, swa_count snapshots so far
    int64_t swa_count = 0;
    float* opt_m = nullptr;
    float* opt_s = nullptr;
    int64_t opt_k = 0;
    uint32_t tag_epoch = 0;                        // tags handed out so far for flagged-word exchanges
    GlmLaunchShape shape{};
    int chain = BMGD_CHAIN_PERSISTENT;
    int64_t buffer_counter = 0;
    int64_t steps = 0, sample_gradients = 0, h2d_bytes = 0;
    double copy_ms = 0, compute_ms = 0, wait_ms = 0, chain_ms = 0;
    int64_t chain_launches = 0;
    std::vector<std::pair<hipEvent_t, hipEvent_t>> open_chain;   // events around chain launches, unsettled
    std::vector<std::pair<hipEvent_t, hipEvent_t>> open_prep;    // events of the moment-matrix launches, unsettled
    double prep_ms = 0;
    int64_t prep_launches = 0;
    hipEvent_t base = nullptr;
    std::vector<RunRecord> open_records;
    std::vector<hipEvent_t> event_pool;
    RunRecord pending_copy;                        // copy events of the buffer that is loaded but not run
    hipStream_t last_copy = nullptr, last_compute = nullptr;
    bool used_copy = false, used_compute = false;
    bool poisoned = false;                         // a run failed or was abandoned: theta is not valid until it is set again
    std::string err;
};

namespace {

bool valid_config(const bmgd_config& c, std::string* why)
{
    auto bad = [&](const char* m) { *why = m; return false; };
    if (c.p <= 0) return bad("p must be positive");
    if (c.buffer_n <= 0 || c.buffer_n >= (int64_t(1) << 30)) return bad("buffer_n must be in [1, 2^30)");
    if (c.batch_n <= 0 || c.batch_n > c.buffer_n) return bad("batch_n must be in [1, buffer_n]");
    if (!(c.lr > 0.0) || !std::isfinite(c.lr)) return bad("lr must be finite and positive");
    if (c.passes < 1) return bad("passes must be at least 1");
    if (c.model != BMGD_LINEAR && c.model != BMGD_LOGISTIC && c.model != BMGD_SOFTMAX) return bad("unknown model");
    if (c.model == BMGD_SOFTMAX) {
        if (c.n_classes < 2 || c.n_classes > 2048) return bad("softmax needs 2 <= n_classes <= 2048");
        if (c.x_dtype != BMGD_BF16) return bad("softmax takes bf16 predictors");
        if (c.p % 8 != 0) return bad("softmax needs p to be a multiple of 8 (16-byte rows of bf16)");
        if ((double)c.p * 2048.0 * 4.0 > 8.0e9) return bad("p too large for softmax");
    } else if (c.x_dtype != BMGD_F32) {
        return bad("linear and logistic models take fp32 predictors");
    }
    if (c.reshuffle != BMGD_RESHUFFLE_PER_PASS && c.reshuffle != BMGD_RESHUFFLE_FIXED) return bad("unknown reshuffle mode");
    if (c.n_buffers < 0) return bad("n_buffers must be non-negative");
    if (c.chain != BMGD_CHAIN_AUTO && c.chain != BMGD_CHAIN_PERSISTENT && c.chain != BMGD_CHAIN_LAUNCH &&
        c.chain != BMGD_CHAIN_GRAM && c.chain != BMGD_CHAIN_GRAPH && c.chain != BMGD_CHAIN_PRODUCT)
        return bad("unknown chain mode");
    if (c.chain == BMGD_CHAIN_GRAPH && c.model != BMGD_SOFTMAX) return bad("BMGD_CHAIN_GRAPH is the softmax model's mode");
    if (c.model == BMGD_SOFTMAX && (c.chain == BMGD_CHAIN_PERSISTENT || c.chain == BMGD_CHAIN_GRAM || c.chain == BMGD_CHAIN_PRODUCT))
        return bad("softmax runs with BMGD_CHAIN_AUTO, BMGD_CHAIN_GRAPH or BMGD_CHAIN_LAUNCH");
    if ((c.chain == BMGD_CHAIN_GRAM || c.chain == BMGD_CHAIN_PRODUCT) && (c.model != BMGD_LINEAR || c.p > kGramMaxP))
        return bad("BMGD_CHAIN_GRAM and BMGD_CHAIN_PRODUCT need the linear model and p <= 128");
    if (c.chain == BMGD_CHAIN_PRODUCT) {
        // the steps of a launch are multiplied together: plain steps only, and the products' scratch has to stay reasonable
        if (c.optimizer != BMGD_OPT_SGD) return bad("BMGD_CHAIN_PRODUCT applies to plain steps only (BMGD_OPT_SGD)");
        const int64_t steps = (int64_t)kMaxPassesPerLaunch * ((c.buffer_n + c.batch_n - 1) / c.batch_n);
        if (gram_products_scratch_floats(c.p, steps) > (size_t(1) << 28))
            return bad("BMGD_CHAIN_PRODUCT: too many mini-batches per buffer (its scratch would exceed 1 GiB); use a larger batch_n");
    }
    if (c.n_workgroups < 0 || c.n_workgroups > kMaxGroups) return bad("n_workgroups must be in [0, 256]");
    if (c.barrier_timeout_us < 0) return bad("barrier_timeout_us must be non-negative");
    if (c.optimizer < BMGD_OPT_SGD || c.optimizer > BMGD_OPT_ADAM) return bad("unknown optimizer");
    if (c.cache_moments != 0 && c.cache_moments != 1) return bad("cache_moments must be 0 or 1");
    if (c.cache_moments) {
        if (c.reshuffle != BMGD_RESHUFFLE_FIXED || c.n_buffers < 1 || c.n_buffers > 65536)
            return bad("cache_moments needs BMGD_RESHUFFLE_FIXED and 1 <= n_buffers <= 65536");
        if (c.model != BMGD_LINEAR || c.p > kGramMaxP || (c.chain != BMGD_CHAIN_GRAM && c.chain != BMGD_CHAIN_PRODUCT && !(c.chain == BMGD_CHAIN_AUTO && c.batch_n >= 2 * c.p)))
            return bad("cache_moments needs the moment form (BMGD_CHAIN_GRAM, BMGD_CHAIN_PRODUCT, or BMGD_CHAIN_AUTO with batch_n >= 2 p)");
    }
    if (c.optimizer == BMGD_OPT_MOMENTUM || c.optimizer == BMGD_OPT_NAG) {
        if (!(c.momentum >= 0.0 && c.momentum < 1.0)) return bad("momentum must be in [0, 1)");
    }
    if (c.optimizer == BMGD_OPT_ADAM) {
        if (!(c.beta1 >= 0.0 && c.beta1 < 1.0) || !(c.beta2 >= 0.0 && c.beta2 < 1.0)) return bad("beta1 and beta2 must be in [0, 1)");
        if (!(c.eps >= 0.0) || !std::isfinite(c.eps)) return bad("eps must be finite and non-negative");
    }
    if (c.workspace != nullptr && (reinterpret_cast<uintptr_t>(c.workspace) % kAlign) != 0)
        return bad("workspace must be 256-byte aligned");
    if (c.model != BMGD_SOFTMAX) {
        GlmLaunchShape s;
        char msg[160];
        if (!glm_plan(c.p, c.batch_n, c.n_workgroups, kMaxGroups, &s, msg, sizeof msg)) {
            *why = msg;
            return false;
        }
    }
    if ((double)c.buffer_n * (double)c.p > 9.0e18 / 8) return bad("buffer too large");
    return true;
}

int resolve_chain(const bmgd_config& c);

// BMGD_CHAIN_PRODUCT, asked for or picked: BMGD_CHAIN_AUTO takes it for plain steps of least squares in the moment form
// when a launch has enough steps for the halved chain to matter (measured at 300 steps per launch: 0.151 against 0.175 ms
// per buffer) and nothing is cached (with cached matrices the caller chooses between the two forms).
bool wants_products(const bmgd_config& c)
{
    if (c.chain == BMGD_CHAIN_PRODUCT) return true;
    if (c.chain != BMGD_CHAIN_AUTO || !gram_eligible(c.model, c.p, c.batch_n) || c.optimizer != BMGD_OPT_SGD || c.cache_moments)
        return false;
    const int64_t M = (c.buffer_n + c.batch_n - 1) / c.batch_n;
    const int64_t steps = (int64_t)std::min<int64_t>(kMaxPassesPerLaunch, c.passes) * M;
    return steps >= 64 && gram_products_scratch_floats(c.p, (int64_t)kMaxPassesPerLaunch * M) <= (size_t(1) << 26);
}

Layout make_layout(const bmgd_config& c)
{
    Layout l{};
    const size_t item = c.x_dtype == BMGD_BF16 ? 2 : 4;
    const int64_t C = c.model == BMGD_SOFTMAX ? c.n_classes : 1;
    size_t off = 0;
    for (int s = 0; s < 2; ++s) {
        l.slot_x[s] = off; off += align_up((size_t)c.buffer_n * c.p * item);
        l.slot_y[s] = off; off += align_up((size_t)c.buffer_n * 4);
    }
    l.perm = off;    off += align_up((size_t)kMaxPassesPerLaunch * c.buffer_n * 4);   // passes may be raised later
    if (c.model == BMGD_SOFTMAX) {
        const SoftmaxDims d = softmax_dims(c.p, c.batch_n, C);
        const size_t m_max = (size_t)((c.buffer_n + c.batch_n - 1) / c.batch_n);
        l.theta = off;   off += align_up((size_t)c.p * d.c_pad * 4);             // fp32 master, [p][c_pad]
        l.partial = l.ll_part = l.ll_theta = off;
        l.sync = off;    off += align_up(64);
        l.sm_state = off; off += align_up(sizeof(SoftmaxState));
        l.wbt = off;     off += align_up((size_t)d.c_pad * d.p_pad * 2);
        l.u = off;       off += align_up((size_t)8 * d.m_pad * d.c_pad * 4);
        l.rt = off;      off += align_up((size_t)d.c_pad * d.n_pad * 2);
        l.xt = off;      off += align_up(m_max * (size_t)c.p * d.n_pad * 2);
    } else {
        l.theta = off;   off += align_up((size_t)c.p * 4);
        l.partial = off; off += align_up((size_t)2 * kMaxGroups * c.p * 4);
        const size_t pp = ((size_t)c.p + 15) & ~size_t(15);   // flagged-word rows are padded to whole 128-byte lines
        l.ll_part = off; off += align_up((size_t)2 * kMaxGroups * pp * 8);
        l.ll_theta = off; off += align_up((size_t)2 * kThetaCopies * pp * 8);
        l.sync = off;    off += align_up(64);
        l.sm_state = l.wbt = l.u = l.rt = l.xt = off;
    }
    l.gram[0] = l.gram[1] = l.gram_perm = off;
    if (resolve_chain(c) == BMGD_CHAIN_GRAM) {
        const size_t set = align_up((size_t)kMaxPassesPerLaunch * (size_t)((c.buffer_n + c.batch_n - 1) / c.batch_n) *
                                    (wants_products(c) ? gram_dense_bytes_per_batch(c.p) : gram_bytes_per_batch(c.p)));
        l.gram[0] = off; off += set;
        l.gram[1] = off; off += set;
        l.gram_perm = off; off += align_up((size_t)kMaxPassesPerLaunch * c.buffer_n * 4);   // second set of partitions
    }
    // BMGD_CHAIN_PRODUCT: two sets of scratch for the products of a launch's steps
    l.prod[0] = l.prod[1] = off;
    if (wants_products(c)) {
        const size_t set = align_up(4 * gram_products_scratch_floats(c.p, (int64_t)kMaxPassesPerLaunch * ((c.buffer_n + c.batch_n - 1) / c.batch_n)));
        l.prod[0] = off; off += set;
        l.prod[1] = off; off += set;
    }
    // moment matrices kept per buffer index (fixed partitions, cache_moments): n_buffers sets of one pass each
    l.gram_cache = off;
    l.gram_cache_set = 0;
    if (c.cache_moments) {
        l.gram_cache_set = align_up((size_t)((c.buffer_n + c.batch_n - 1) / c.batch_n) *
                                    (wants_products(c) ? gram_dense_bytes_per_batch(c.p) : gram_bytes_per_batch(c.p)));
        off += l.gram_cache_set * (size_t)c.n_buffers;
    }
    // BMGD_CHAIN_PRODUCT with cached moment matrices: per buffer index also the product of a run's steps
    l.prod_cache = off;
    l.prod_cache_set = 0;
    if (c.cache_moments && wants_products(c)) {
        l.prod_cache_set = align_up(gram_dense_bytes_per_batch(c.p));
        off += l.prod_cache_set * (size_t)c.n_buffers;
    }
    // optimizer state: like theta; with the redundant reduction every workgroup keeps a private copy (G * p <= 4096
    // words there, rows padded to 16)
    l.opt_m = l.opt_s = off;
    l.opt_len = 0;
    if (c.optimizer != BMGD_OPT_SGD) {
        const size_t pp16 = ((size_t)c.p + 15) & ~size_t(15);
        l.opt_len = c.model == BMGD_SOFTMAX ? (size_t)c.p * softmax_dims(c.p, c.batch_n, C).c_pad
                                            : std::max<size_t>(pp16, 4096 + 16 * (size_t)kMaxGroups);
        l.opt_m = off; off += align_up(l.opt_len * 4);
        l.opt_s = off;
        if (c.optimizer == BMGD_OPT_ADAM) off += align_up(l.opt_len * 4);
    }
    l.eval = off; off += align_up((size_t)kEvalBlocks * sizeof(double));   // partial sums of bmgd_eval_loss
    // running average of the estimate (bmgd_swa_update), laid out like theta
    l.swa = off; off += align_up(c.model == BMGD_SOFTMAX ? (size_t)c.p * softmax_dims(c.p, c.batch_n, C).c_pad * 4 : (size_t)c.p * 4);
    l.total = off;
    return l;
}

int resolve_chain(const bmgd_config& c)
{
    if (c.model == BMGD_SOFTMAX) return c.chain == BMGD_CHAIN_LAUNCH ? BMGD_CHAIN_LAUNCH : BMGD_CHAIN_GRAPH;
    if (wants_products(c)) return BMGD_CHAIN_GRAM;                  // the moment form with another way through the steps (ctx->products)
    if (c.chain != BMGD_CHAIN_AUTO) return c.chain;
    return gram_eligible(c.model, c.p, c.batch_n) ? BMGD_CHAIN_GRAM : BMGD_CHAIN_PERSISTENT;
}

int fail(bmgd_ctx* ctx, int code, const std::string& msg)
{
    if (ctx) ctx->err = msg; else g_create_error = msg;
    return code;
}

int hip_fail(bmgd_ctx* ctx, hipError_t e, const char* what)
{
    char buf[256];
    snprintf(buf, sizeof buf, "%s: %s", what, hipGetErrorString(e));
    (void)hipGetLastError();
    return fail(ctx, e == hipErrorOutOfMemory ? BMGD_ENOMEM : BMGD_EHIP, buf);
}

#define HIP_TRY(ctx, call)                                              \
    do {                                                                \
        hipError_t e_ = (call);                                         \
        if (e_ != hipSuccess) return hip_fail((ctx), e_, #call);        \
    } while (0)

hipEvent_t take_event(bmgd_ctx* ctx)
{
    if (!ctx->event_pool.empty()) {
        hipEvent_t e = ctx->event_pool.back();
        ctx->event_pool.pop_back();
        return e;
    }
    hipEvent_t e = nullptr;
    if (hipEventCreate(&e) != hipSuccess) return nullptr;
    return e;
}

void give_event(bmgd_ctx* ctx, hipEvent_t e) { if (e) ctx->event_pool.push_back(e); }

// Fold the oldest `count` finished runs into the running totals.  Their kernels and copies must have completed.
void settle_records(bmgd_ctx* ctx, size_t count)
{
    count = std::min(count, ctx->open_records.size());
    size_t n_chain = 0, n_prep = 0;
    for (size_t i = 0; i < count; ++i) {
        RunRecord& r = ctx->open_records[i];
        float t_start = 0.f, t_end = 0.f, c_start = 0.f, c_end = 0.f;
        // the part of this buffer's copy during which no earlier run was computing: copy time that was not hidden
        if (r.has_copy && hipEventElapsedTime(&c_start, ctx->base, r.copy_start) == hipSuccess &&
            hipEventElapsedTime(&c_end, ctx->base, r.copy_end) == hipSuccess && c_end > c_start) {
            ctx->copy_ms += c_end - c_start;
            const double from = std::max<double>(c_start, ctx->busy_until);
            if (c_end > from) ctx->wait_ms += c_end - from;
        }
        if (hipEventElapsedTime(&t_start, ctx->base, r.start) == hipSuccess &&
            hipEventElapsedTime(&t_end, ctx->base, r.end) == hipSuccess) {
            // runs may overlap (the pre-pass of one with the chain of the one before): count the union
            const double from = std::max<double>(t_start, ctx->busy_until);
            if (t_end > from) ctx->compute_ms += t_end - from;
            ctx->busy_until = std::max<double>(ctx->busy_until, t_end);
        }
        n_chain += (size_t)r.n_chain;
        n_prep += (size_t)r.n_prep;
    }
    // elapsed times first, hand-backs second: a run's `end` may be the stop event of its last chain launch
    const bool all = count == ctx->open_records.size();     // then also entries of a run that failed half-way
    n_chain = all ? ctx->open_chain.size() : std::min(n_chain, ctx->open_chain.size());
    n_prep = all ? ctx->open_prep.size() : std::min(n_prep, ctx->open_prep.size());
    for (size_t i = 0; i < n_chain; ++i) {
        auto& pr = ctx->open_chain[i];
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, pr.first, pr.second) == hipSuccess) { ctx->chain_ms += ms; ctx->chain_launches += 1; }
        give_event(ctx, pr.first); give_event(ctx, pr.second);
    }
    for (size_t i = 0; i < n_prep; ++i) {
        auto& pr = ctx->open_prep[i];
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, pr.first, pr.second) == hipSuccess) { ctx->prep_ms += ms; ctx->prep_launches += 1; }
        give_event(ctx, pr.first); give_event(ctx, pr.second);
    }
    for (size_t i = 0; i < count; ++i) {
        RunRecord& r = ctx->open_records[i];
        give_event(ctx, r.copy_start); give_event(ctx, r.copy_end);
        give_event(ctx, r.start);
        if (r.owns_end) give_event(ctx, r.end);
    }
    ctx->open_records.erase(ctx->open_records.begin(), ctx->open_records.begin() + (ptrdiff_t)count);
    ctx->open_chain.erase(ctx->open_chain.begin(), ctx->open_chain.begin() + (ptrdiff_t)n_chain);
    ctx->open_prep.erase(ctx->open_prep.begin(), ctx->open_prep.begin() + (ptrdiff_t)n_prep);
}

// A caller that never synchronises would otherwise pile up events without bound: once kMaxOpenRuns runs are open,
// wait for the older half (which also keeps the host from running arbitrarily far ahead of the device) and fold it.
// The events the next runs still wait on belong to the two latest runs, so none of them is handed back here.
int trim_records(bmgd_ctx* ctx)
{
    if (ctx->open_records.size() < kMaxOpenRuns) return BMGD_OK;
    const size_t count = ctx->open_records.size() / 2;
    HIP_TRY(ctx, hipEventSynchronize(ctx->open_records[count - 1].end));
    settle_records(ctx, count);
    return BMGD_OK;
}

int drain(bmgd_ctx* ctx)
{
    HIP_TRY(ctx, hipSetDevice(ctx->device));
    if (ctx->used_copy) HIP_TRY(ctx, hipStreamSynchronize(ctx->last_copy));
    if (ctx->used_compute) HIP_TRY(ctx, hipStreamSynchronize(ctx->last_compute));
    if (ctx->chain_stream) HIP_TRY(ctx, hipStreamSynchronize(ctx->chain_stream));
    ctx->chain_pending[0] = ctx->chain_pending[1] = false;
    settle_records(ctx, ctx->open_records.size());
    unsigned flag[2] = {0, 0};
    HIP_TRY(ctx, hipMemcpy(flag, ctx->sync + 1, sizeof flag, hipMemcpyDeviceToHost));
    if (flag[0] != 0 || flag[1] != 0) {
        HIP_TRY(ctx, hipMemset(ctx->sync, 0, 64));
        ctx->poisoned = true;
        if (flag[0] != 0)
            return fail(ctx, BMGD_EHIP, "a device-side wait exceeded barrier_timeout_us; the run was abandoned and theta is not valid (set it again with bmgd_set_theta before the next run)");
        return fail(ctx, BMGD_EINVAL, "a row subset held an index outside its buffer (row 0 was used in its place); theta is not valid (set it again with bmgd_set_theta before the next run)");
    }
    return BMGD_OK;
}

int64_t batches_of(int64_t rows, int64_t n) { return (rows + n - 1) / n; }

OptArgs opt_args(const bmgd_ctx* ctx, int64_t ahead)
{
    OptArgs o{};
    o.kind = ctx->cfg.optimizer;
    o.mu = (float)ctx->cfg.momentum;
    o.b1 = (float)ctx->cfg.beta1;
    o.b2 = (float)ctx->cfg.beta2;
    o.eps = (float)ctx->cfg.eps;
    o.m = ctx->opt_m;
    o.s = ctx->opt_s;
    o.k_base = (int)std::min<int64_t>(ctx->opt_k + ahead, 0x7FFFFFF0);
    return o;
}

// Learning rate of the update `ahead` updates after those already enqueued.
float rate_of(const bmgd_ctx* ctx, int64_t ahead)
{
    if (ctx->lr_tab_host.empty()) return (float)ctx->cfg.lr;
    const int64_t u = std::min<int64_t>(ctx->lr_pos + ahead, (int64_t)ctx->lr_tab_host.size() - 1);
    return ctx->lr_tab_host[(size_t)u];
}

// The steps of a launch in the moment form, on the library's chain stream: the chain of eq. (3.1) step by step, or
// (BMGD_CHAIN_PRODUCT) the steps multiplied together and applied once.
hipError_t launch_steps(bmgd_ctx* ctx, const float* set, int64_t rows, int64_t n, int np, int perm_stride, hipEvent_t ev0,
                        hipEvent_t ev1, bmgd_ctx::CachedMoments* keep = nullptr, uint32_t b = 0)
{
    const bmgd_config& c = ctx->cfg;
    const int lr_len = (int)ctx->lr_tab_host.size();
    const float* tab = lr_len ? ctx->lr_tab_dev : nullptr;
    const int lr_base = (int)std::min<int64_t>(ctx->lr_pos, std::max(lr_len - 1, 0));
    if (ctx->products) {
        // Fixed partitions with cached matrices (keep != null): as long as the rate and the number of passes stay what
        // they were, the product of a run over buffer index b is the same matrix every time; it is formed once and then
        // only applied.
        float* kept = keep && lr_len == 0 ? reinterpret_cast<float*>(ctx->prod_cache + (size_t)b * ctx->lay.prod_cache_set) : nullptr;
        if (kept && keep->prod_valid && keep->prod_alpha == (float)c.lr && keep->prod_np == np)
            return gram_launch_apply(kept, ctx->theta, (int)c.p, ctx->chain_stream, ev0, ev1);
        // (launches on one stream run in order, so the scratch of launch k - 2 is free; two sets alternate anyway, so that
        // nothing here depends on that)
        float* scratch = ctx->prod[ctx->psel];
        const bool pairs = kept == nullptr;
        if (pairs && ctx->prod_dense[ctx->psel]) {
            // the pairs go out in the chain's layout, whose padding is read (and multiplied by zeros): clear what a
            // round of dense matrices left there
            const size_t bytes = ctx->lay.prod[1] - ctx->lay.prod[0];
            hipError_t ce = hipMemsetAsync(scratch, 0, bytes, ctx->chain_stream);
            if (ce != hipSuccess) return ce;
        }
        ctx->prod_dense[ctx->psel] = !pairs;
        ctx->psel ^= 1;
        // Unless the product itself is wanted (to be kept), one round of products is made and the chain runs over the
        // pairs: every further round costs a kernel's start-up and fills the device, while the chain keeps to one unit.
        hipError_t e = gram_launch_products(set, ctx->theta, scratch, kept, (int)rows, (int)c.p, (int)n, np, perm_stride, (float)c.lr, tab,
                                            lr_base, lr_len, ctx->chain_stream, ev0, ev1, pairs);
        if (keep) {
            keep->prod_valid = kept != nullptr && e == hipSuccess;
            keep->prod_alpha = (float)c.lr;
            keep->prod_np = np;
        }
        return e;
    }
    return gram_launch_chain(set, ctx->theta, (int)rows, (int)c.p, (int)n, np, perm_stride, (float)c.lr, tab, lr_base, lr_len,
                             opt_args(ctx, 0), ctx->chain_stream, ev0, ev1);
}

// Enqueue passes t = first + 1 .. first + count over (x, y, rows) on `stream`, at most kMaxPassesPerLaunch per launch.
// *end_event receives the stop event of the last kernel if that kernel carries one (and then runs on the
// library's chain stream), else NULL: then the passes end with the last work enqueued on `stream`.
// *chunk_end (may be NULL) receives an event that completes when the last of these passes has: it stays valid until
// the run's records are settled.
int enqueue_passes(bmgd_ctx* ctx, const void* x, const void* y, int64_t rows, hipStream_t stream, int first, int count,
                   hipEvent_t* end_event, hipEvent_t* chunk_end)
{
    *end_event = nullptr;
    const bmgd_config& c = ctx->cfg;
    const int64_t n = std::min<int64_t>(c.batch_n, rows);
    const int64_t M = batches_of(rows, n);
    const bool fixed = c.reshuffle == BMGD_RESHUFFLE_FIXED;
    const uint32_t b = (uint32_t)(fixed && c.n_buffers > 0 ? ctx->buffer_counter % c.n_buffers : ctx->buffer_counter);
    const long long ticks = (c.barrier_timeout_us > 0 ? c.barrier_timeout_us : 2000000) * 100LL;
    const int lr_len = (int)ctx->lr_tab_host.size();
    // checked before anything is enqueued: step indices inside one launch stay below 2^23
    if (c.model != BMGD_SOFTMAX && ctx->chain != BMGD_CHAIN_GRAM &&
        (int64_t)std::min(kMaxPassesPerLaunch, count) * M >= (int64_t(1) << 23))
        return fail(ctx, BMGD_EINVAL, "passes per launch * batches per pass must stay below 2^23; use a larger batch_n");

    for (int t0 = first; t0 < first + count; t0 += kMaxPassesPerLaunch) {
        const int np = std::min(kMaxPassesPerLaunch, first + count - t0);
        PermKeys keys{};
        const int nperm = fixed ? 1 : np;
        for (int i = 0; i < nperm; ++i) perm_round_keys(c.seed, b, fixed ? 0u : (uint32_t)(t0 + i + 1), keys.key[i]);
        hipEvent_t ev0 = take_event(ctx), ev1 = take_event(ctx);
        if (!ev0 || !ev1) return fail(ctx, BMGD_EHIP, "could not create events");
        if (ctx->chain == BMGD_CHAIN_GRAM && c.cache_moments && !ctx->subset) {
            // Fixed partitions: the moment matrices of buffer index b are the same in every iteration (Section 3.1.1),
            // so they are formed once and every later run over that buffer is the chain alone.
            bmgd_ctx::CachedMoments& ce = ctx->mcache[b];
            float* set = reinterpret_cast<float*>(ctx->gram_cache + (size_t)b * ctx->lay.gram_cache_set);
            if (!ce.valid || ce.rows != rows) {
                if (!x || !y) return fail(ctx, BMGD_ESTATE, "the moment matrices of this buffer are not cached yet");
                if (!ce.ready) HIP_TRY(ctx, hipEventCreateWithFlags(&ce.ready, hipEventDisableTiming));
                hipEvent_t pv0 = take_event(ctx), pv1 = take_event(ctx);
                if (!pv0 || !pv1) return fail(ctx, BMGD_EHIP, "could not create events");
                ctx->open_prep.emplace_back(pv0, pv1);
                // a chain that still reads the old matrices of this index (another row count) must have finished
                if (ce.valid) HIP_TRY(ctx, hipStreamWaitEvent(stream, ctx->cache_chain_done, 0));
                HIP_TRY(ctx, launch_perm(ctx->gram_perm[0], rows, 1, keys, stream));
                HIP_TRY(ctx, gram_launch_moments(static_cast<const float*>(x), static_cast<const float*>(y), ctx->gram_perm[0], set,
                                                 (int)rows, (int)c.p, (int)n, np, 0, stream, pv0, pv1, ctx->products));
                HIP_TRY(ctx, hipEventRecord(ce.ready, stream));
                ce.valid = true;
                ce.prod_valid = false;
                ce.rows = rows;
            }
            HIP_TRY(ctx, hipStreamWaitEvent(ctx->chain_stream, ce.ready, 0));
            // (the product of a whole run can be kept: one launch must cover the run)
            HIP_TRY(ctx, launch_steps(ctx, set, rows, n, np, 0, ev0, ev1, count == np ? &ce : nullptr, b));
            if (!ctx->cache_chain_done) HIP_TRY(ctx, hipEventCreateWithFlags(&ctx->cache_chain_done, hipEventDisableTiming));
            HIP_TRY(ctx, hipEventRecord(ctx->cache_chain_done, ctx->chain_stream));
            ctx->lr_pos += (int64_t)np * M;
            ctx->opt_k += (int64_t)np * M;
            ctx->open_chain.emplace_back(ev0, ev1);
            *end_event = ev1;
            if (chunk_end) *chunk_end = ev1;
            continue;
        }
        if (ctx->chain == BMGD_CHAIN_GRAM) {
            const int i = ctx->gsel;
            ctx->gsel ^= 1;
            hipEvent_t pv0 = take_event(ctx), pv1 = take_event(ctx);
            if (!pv0 || !pv1) return fail(ctx, BMGD_EHIP, "could not create events");
            ctx->open_prep.emplace_back(pv0, pv1);
            // set i is free once the chain that read it last has finished
            if (ctx->chain_pending[i]) HIP_TRY(ctx, hipStreamWaitEvent(stream, ctx->chain_done[i], 0));
            HIP_TRY(ctx, launch_perm(ctx->gram_perm[i], rows, nperm, keys, stream, ctx->subset, ctx->subset_limit, ctx->sync + 2));
            // BMGD_CHAIN_PRODUCT (without cached matrices): the steps are multiplied in pairs right behind the moments
            // kernel, on the same stream (both fill the device; the chain, which keeps to one unit, overlaps the next
            // buffer's two), and the chain runs over the pairs.  Set i of the pairs is guarded like set i of the matrices.
            const bool pairs_here = ctx->products && !c.cache_moments;
            HIP_TRY(ctx, gram_launch_moments(static_cast<const float*>(x), static_cast<const float*>(y), ctx->gram_perm[i],
                                             ctx->gram[i], (int)rows, (int)c.p, (int)n, np, fixed ? 0 : (int)rows, stream,
                                             pv0, pairs_here ? nullptr : pv1, ctx->products));
            if (pairs_here) {
                HIP_TRY(ctx, gram_launch_pairs(ctx->gram[i], ctx->prod[i], (int)rows, (int)c.p, (int)n, np, fixed ? 0 : (int)rows,
                                               (float)c.lr, lr_len ? ctx->lr_tab_dev : nullptr,
                                               (int)std::min<int64_t>(ctx->lr_pos, std::max(lr_len - 1, 0)), lr_len, stream, nullptr, pv1));
            }
            ctx->prep_done[i] = pv1;
            HIP_TRY(ctx, hipStreamWaitEvent(ctx->chain_stream, ctx->prep_done[i], 0));
            // the timing events are completed by the chain's dispatch; the stop event also frees set i
            if (pairs_here) {
                const int half = (int)(((int64_t)np * M + 1) / 2);
                HIP_TRY(ctx, gram_launch_chain_steps(ctx->prod[i], ctx->theta, (int)c.p, half, half, 1.0f, nullptr, 0, 0, opt_args(ctx, 0),
                                                     ctx->chain_stream, ev0, ev1));
            } else {
                HIP_TRY(ctx, launch_steps(ctx, ctx->gram[i], rows, n, np, fixed ? 0 : (int)rows, ev0, ev1));
            }
            ctx->lr_pos += (int64_t)np * M;
            ctx->opt_k += (int64_t)np * M;
            ctx->chain_done[i] = ev1;                // stays valid until the records are settled, after a drain
            ctx->chain_pending[i] = true;
            ctx->open_chain.emplace_back(ev0, ev1);
            *end_event = ev1;
            if (chunk_end) *chunk_end = ev1;
            continue;
        }
        if (!fixed || t0 == 0)
            HIP_TRY(ctx, launch_perm(ctx->perm, rows, nperm, keys, stream, ctx->subset, ctx->subset_limit, ctx->sync + 2));
        if (c.model == BMGD_SOFTMAX) {
            HIP_TRY(ctx, hipEventRecord(ev0, stream));
            const SoftmaxDims d = softmax_dims(c.p, n, c.n_classes);
            const SoftmaxDims dmax = softmax_dims(c.p, c.batch_n, c.n_classes);
            // the launches of one pass (transpose of its mini-batches, then logits / residual / gradient + update per
            // mini-batch), onto `to`
            auto issue_pass = [&](const int32_t* pm, hipStream_t to) -> int {
                HIP_TRY(ctx, softmax_permute_transpose(x, pm, ctx->xt, (int)rows, (int)c.p, (int)n, d, to));
                for (int64_t m = 0; m < M; ++m) {
                    SoftmaxStep st{};
                    st.X = x;
                    st.y = static_cast<const int32_t*>(y);
                    st.idx = pm + m * n;
                    st.XT = static_cast<const char*>(ctx->xt) + (size_t)m * c.p * d.n_pad * 2;
                    st.W = ctx->theta;
                    st.WbT = ctx->wbt;
                    st.U = ctx->u;
                    st.Rt = ctx->rt;
                    st.nb = (int)std::min<int64_t>(n, rows - m * n);
                    st.p = (int)c.p;
                    st.C = c.n_classes;
                    st.opt = opt_args(ctx, 0);
                    st.state = ctx->sm_state;
                    st.u = (int)m;
                    st.lr_tab = lr_len ? ctx->lr_tab_dev : nullptr;
                    st.lr_len = lr_len;
                    SoftmaxDims ds = d;
                    ds.c_pad = dmax.c_pad;           // W and WbT keep the strides fixed at creation
                    ds.p_pad = dmax.p_pad;
                    HIP_TRY(ctx, softmax_step(st, ds, to));
                }
                return BMGD_OK;
            };
            for (int i = 0; i < np; ++i) {
                const int32_t* pm = ctx->perm + (fixed ? 0 : (size_t)i * rows);
                // what differs between two passes with the same launches: read by the kernels from device memory
                HIP_TRY(ctx, softmax_set_state(ctx->sm_state, (float)c.lr, (int)std::min<int64_t>(ctx->lr_pos, 0x7FFFFFF0),
                                               (int)std::min<int64_t>(ctx->opt_k, 0x7FFFFFF0), stream));
                if (ctx->chain == BMGD_CHAIN_GRAPH) {
                    const auto key = std::make_tuple(x, y, pm, rows);
                    auto it = ctx->pass_graphs.find(key);
                    if (it == ctx->pass_graphs.end()) {
                        if (ctx->pass_graphs.size() >= 64) {   // callers that keep bringing new buffers: start over
                            HIP_TRY(ctx, hipStreamSynchronize(stream));
                            for (auto& kv : ctx->pass_graphs) (void)hipGraphExecDestroy(kv.second);
                            ctx->pass_graphs.clear();
                        }
                        hipGraph_t graph = nullptr;
                        HIP_TRY(ctx, hipStreamBeginCapture(ctx->capture_stream, hipStreamCaptureModeThreadLocal));
                        const int rc = issue_pass(pm, ctx->capture_stream);
                        const hipError_t ce = hipStreamEndCapture(ctx->capture_stream, &graph);
                        if (rc != BMGD_OK) { if (graph) (void)hipGraphDestroy(graph); return rc; }
                        if (ce != hipSuccess) return hip_fail(ctx, ce, "hipStreamEndCapture");
                        hipGraphExec_t exec = nullptr;
                        const hipError_t ie = hipGraphInstantiate(&exec, graph, nullptr, nullptr, 0);
                        (void)hipGraphDestroy(graph);
                        if (ie != hipSuccess) return hip_fail(ctx, ie, "hipGraphInstantiate");
                        it = ctx->pass_graphs.emplace(key, exec).first;
                    }
                    HIP_TRY(ctx, hipGraphLaunch(it->second, stream));
                } else {
                    const int rc = issue_pass(pm, stream);
                    if (rc != BMGD_OK) return rc;
                }
                ctx->lr_pos += M;
                ctx->opt_k += M;
            }
            HIP_TRY(ctx, hipEventRecord(ev1, stream));
            ctx->open_chain.emplace_back(ev0, ev1);
            if (chunk_end) *chunk_end = ev1;
            continue;
        }
        GlmArgs a{};
        a.X = static_cast<const float*>(x);
        a.y = static_cast<const float*>(y);
        a.perm = ctx->perm;
        a.theta = ctx->theta;
        a.partial = ctx->partial;
        a.sync = ctx->sync;
        a.rows = (int)rows; a.p = (int)c.p; a.n = (int)n; a.npass = np;
        a.perm_stride = fixed ? 0 : (int)rows;
        a.model = c.model;
        a.L = ctx->shape.L;
        a.logL = 0;
        while ((1 << a.logL) < a.L) ++a.logL;
        a.reduce_mode = ctx->shape.reduce_mode;
        a.alpha = (float)c.lr;
        a.timeout_ticks = ticks;
        a.single_step = -1;
        a.ll_part = ctx->ll_part;
        a.ll_theta = ctx->ll_theta;
        a.lr_tab = lr_len ? ctx->lr_tab_dev : nullptr;
        a.lr_base = (int)std::min<int64_t>(ctx->lr_pos, std::max(lr_len - 1, 0));
        a.lr_len = lr_len;
        a.opt = opt_args(ctx, 0);
        HIP_TRY(ctx, hipEventRecord(ev0, stream));
        if (ctx->chain == BMGD_CHAIN_PERSISTENT) {
            const int64_t nsteps = (int64_t)np * M;
            if ((uint64_t)ctx->tag_epoch + (uint64_t)nsteps + 1 >= 0xFFFFFFFFull) {
                // tag space used up: clear the flagged words (stream-ordered) and start over
                HIP_TRY(ctx, launch_fill_zero(ctx->ll_part, ctx->lay.sync - ctx->lay.ll_part, stream));
                ctx->tag_epoch = 0;
            }
            a.tag_base = ctx->tag_epoch;
            a.s_begin = 0;
            a.s_end = (int)nsteps;
            ctx->tag_epoch += (uint32_t)nsteps;
            HIP_TRY(ctx, glm_launch_chain(ctx->shape, a, stream));
        } else {
            for (int64_t s = 0; s < (int64_t)np * M; ++s) {
                a.single_step = (int)s;
                a.alpha = rate_of(ctx, s);               // this mode passes the rate per launch
                a.lr_tab = nullptr;
                a.opt = opt_args(ctx, s);
                const int64_t m = s % M;
                const int nb = (int)std::min<int64_t>(n, rows - m * n);
                HIP_TRY(ctx, glm_launch_step(ctx->shape, a, nb, stream));
            }
        }
        HIP_TRY(ctx, hipEventRecord(ev1, stream));
        ctx->open_chain.emplace_back(ev0, ev1);
        if (chunk_end) *chunk_end = ev1;
        ctx->lr_pos += (int64_t)np * M;
        ctx->opt_k += (int64_t)np * M;
    }
    return BMGD_OK;
}

// Bookkeeping at the end of a run of `passes` passes over a buffer of `rows` rows.
void finish_run(bmgd_ctx* ctx, int64_t rows, int64_t passes)
{
    const int64_t n = std::min<int64_t>(ctx->cfg.batch_n, rows);
    ctx->steps += passes * batches_of(rows, n);
    ctx->sample_gradients += passes * rows;
    ctx->buffer_counter += 1;
}

// Rows the run over a buffer of `buffer_rows` rows works on: all of them, or the subset set for this run.
// Returns 0 (with the error set) if the subset does not fit the buffer.
int64_t rows_of_run(bmgd_ctx* ctx, int64_t buffer_rows)
{
    if (!ctx->subset) return buffer_rows;
    if (ctx->subset_count > buffer_rows) {
        fail(ctx, BMGD_EINVAL, "the row subset has more entries than the buffer has rows");
        return 0;
    }
    ctx->subset_limit = buffer_rows;
    return ctx->subset_count;
}

// A run call failed after it may have enqueued part of its work: the events it took go back to the pool, and theta
// counts as not valid (the kernels already enqueued have updated it for part of the run) until it is set again.
int abandon_run(bmgd_ctx* ctx, RunRecord& rec, int rc)
{
    give_event(ctx, rec.start);
    if (rec.owns_end) give_event(ctx, rec.end);
    rec.start = rec.end = nullptr;
    ctx->poisoned = true;
    return rc;
}

int refuse_if_poisoned(bmgd_ctx* ctx)
{
    if (!ctx->poisoned) return BMGD_OK;
    return fail(ctx, BMGD_ESTATE, "an earlier run failed or was abandoned and theta is not valid: call bmgd_set_theta first");
}

// Enqueue the T passes of Algorithm 1 over (x, y, rows).
int enqueue_compute(bmgd_ctx* ctx, const void* x, const void* y, int64_t rows, hipStream_t stream, hipEvent_t* end_event)
{
    const int rc = enqueue_passes(ctx, x, y, rows, stream, 0, ctx->cfg.passes, end_event, nullptr);
    if (rc == BMGD_OK) finish_run(ctx, rows, ctx->cfg.passes);
    return rc;
}

void destroy_ctx(bmgd_ctx* ctx)
{
    if (!ctx) return;
    (void)hipSetDevice(ctx->device);
    if (ctx->used_copy) (void)hipStreamSynchronize(ctx->last_copy);
    if (ctx->used_compute) (void)hipStreamSynchronize(ctx->last_compute);
    if (ctx->chain_stream) (void)hipStreamSynchronize(ctx->chain_stream);
    settle_records(ctx, ctx->open_records.size());
    if (ctx->chain_stream) (void)hipStreamDestroy(ctx->chain_stream);
    for (auto& kv : ctx->pass_graphs) (void)hipGraphExecDestroy(kv.second);
    if (ctx->capture_stream) (void)hipStreamDestroy(ctx->capture_stream);
    give_event(ctx, ctx->pending_copy.copy_start);
    give_event(ctx, ctx->pending_copy.copy_end);
    for (hipEvent_t e : ctx->event_pool) (void)hipEventDestroy(e);
    for (auto& ce : ctx->mcache)
        if (ce.ready) (void)hipEventDestroy(ce.ready);
    if (ctx->cache_chain_done) (void)hipEventDestroy(ctx->cache_chain_done);
    for (Slot& s : ctx->slots) {
        if (s.compute_done) (void)hipEventDestroy(s.compute_done);
    }
    if (ctx->base) (void)hipEventDestroy(ctx->base);
    if (ctx->lr_tab_dev) (void)hipFree(ctx->lr_tab_dev);
    if (ctx->owns_ws && ctx->ws) (void)hipFree(ctx->ws);
    delete ctx;
}

}  // namespace

#define BMGD_API __attribute__((visibility("default")))

extern "C" {

BMGD_API void bmgd_default_config(bmgd_config* cfg)
{
    if (!cfg) return;
    memset(cfg, 0, sizeof *cfg);
    cfg->model = BMGD_LINEAR;
    cfg->n_classes = 1;
    cfg->x_dtype = BMGD_F32;
    cfg->reshuffle = BMGD_RESHUFFLE_PER_PASS;
    cfg->chain = BMGD_CHAIN_AUTO;
    cfg->optimizer = BMGD_OPT_SGD;
    cfg->momentum = 0.9;
    cfg->beta1 = 0.9;
    cfg->beta2 = 0.999;
    cfg->eps = 1e-8;
}

BMGD_API size_t bmgd_workspace_bytes(const bmgd_config* cfg)
{
    std::string why;
    if (!cfg || !valid_config(*cfg, &why)) return 0;
    return make_layout(*cfg).total;
}

BMGD_API int bmgd_create_ex(const bmgd_config* cfg, bmgd_ctx** out)
{
    if (out) *out = nullptr;
    if (!cfg || !out) return fail(nullptr, BMGD_EINVAL, "cfg and out must not be NULL");
    std::string why;
    if (!valid_config(*cfg, &why)) return fail(nullptr, BMGD_EINVAL, why);

    int ndev = 0;
    hipError_t e = hipGetDeviceCount(&ndev);
    if (e != hipSuccess || ndev == 0) {
        (void)hipGetLastError();
        return fail(nullptr, BMGD_EHIP, "no HIP device available");
    }
    bmgd_ctx* ctx = new (std::nothrow) bmgd_ctx();
    if (!ctx) return fail(nullptr, BMGD_ENOMEM, "out of host memory");
    ctx->cfg = *cfg;
    if (ctx->cfg.model != BMGD_SOFTMAX) ctx->cfg.n_classes = 1;
    ctx->x_itemsize = cfg->x_dtype == BMGD_BF16 ? 2 : 4;
    ctx->theta_len = cfg->p * ctx->cfg.n_classes;
    ctx->lay = make_layout(ctx->cfg);

    auto bail = [&](int code) {
        g_create_error = ctx->err;
        destroy_ctx(ctx);
        return code;
    };
#define CREATE_TRY(call)                                                  \
    do {                                                                  \
        hipError_t e_ = (call);                                           \
        if (e_ != hipSuccess) return bail(hip_fail(ctx, e_, #call));      \
    } while (0)

    CREATE_TRY(hipGetDevice(&ctx->device));
    hipDeviceProp_t prop;
    CREATE_TRY(hipGetDeviceProperties(&prop, ctx->device));
    ctx->num_cus = prop.multiProcessorCount;
    if (cfg->workspace) {
        if (cfg->workspace_bytes < ctx->lay.total) {
            ctx->err = "workspace smaller than bmgd_workspace_bytes()";
            return bail(BMGD_ENOMEM);
        }
        ctx->ws = cfg->workspace;
    } else {
        CREATE_TRY(hipMalloc(&ctx->ws, ctx->lay.total));
        ctx->owns_ws = true;
    }
    char* base = static_cast<char*>(ctx->ws);
    for (int s = 0; s < 2; ++s) {
        ctx->slots[s].x = base + ctx->lay.slot_x[s];
        ctx->slots[s].y = base + ctx->lay.slot_y[s];
        CREATE_TRY(hipEventCreate(&ctx->slots[s].compute_done));
    }
    ctx->perm = reinterpret_cast<int32_t*>(base + ctx->lay.perm);
    ctx->theta = reinterpret_cast<float*>(base + ctx->lay.theta);
    ctx->partial = reinterpret_cast<float*>(base + ctx->lay.partial);
    ctx->ll_part = reinterpret_cast<unsigned long long*>(base + ctx->lay.ll_part);
    ctx->ll_theta = reinterpret_cast<unsigned long long*>(base + ctx->lay.ll_theta);
    ctx->sync = reinterpret_cast<unsigned*>(base + ctx->lay.sync);
    ctx->sm_state = reinterpret_cast<SoftmaxState*>(base + ctx->lay.sm_state);
    ctx->wbt = base + ctx->lay.wbt;
    ctx->u = reinterpret_cast<float*>(base + ctx->lay.u);
    ctx->rt = base + ctx->lay.rt;
    ctx->xt = base + ctx->lay.xt;
    ctx->gram[0] = reinterpret_cast<float*>(base + ctx->lay.gram[0]);
    ctx->gram[1] = reinterpret_cast<float*>(base + ctx->lay.gram[1]);
    ctx->prod[0] = reinterpret_cast<float*>(base + ctx->lay.prod[0]);
    ctx->prod[1] = reinterpret_cast<float*>(base + ctx->lay.prod[1]);
    ctx->products = wants_products(*cfg);
    if (ctx->products) CREATE_TRY(gram_products_prepare());
    ctx->gram_cache = base + ctx->lay.gram_cache;
    ctx->prod_cache = base + ctx->lay.prod_cache;
    if (cfg->cache_moments) ctx->mcache.resize((size_t)cfg->n_buffers);
    ctx->gram_perm[0] = ctx->perm;
    ctx->gram_perm[1] = reinterpret_cast<int32_t*>(base + ctx->lay.gram_perm);
    ctx->swa = reinterpret_cast<float*>(base + ctx->lay.swa);
    ctx->opt_m = reinterpret_cast<float*>(base + ctx->lay.opt_m);
    ctx->opt_s = reinterpret_cast<float*>(base + ctx->lay.opt_s);
    if (ctx->lay.total > ctx->lay.opt_m) CREATE_TRY(hipMemset(ctx->opt_m, 0, ctx->lay.total - ctx->lay.opt_m));
    CREATE_TRY(hipMemset(ctx->sync, 0, 64));
    if (cfg->model == BMGD_SOFTMAX) {
        // theta = 0 (padding classes included), bf16 copy = 0, residual scratch = 0
        CREATE_TRY(hipMemset(ctx->theta, 0, ctx->lay.sync - ctx->lay.theta));
        CREATE_TRY(hipMemset(ctx->wbt, 0, ctx->lay.xt - ctx->lay.wbt));
    } else {
        CREATE_TRY(hipMemset(ctx->theta, 0, (size_t)ctx->theta_len * 4));
        // flagged words start with tag 0, which no step ever waits for
        CREATE_TRY(hipMemset(ctx->partial, 0, ctx->lay.sync - ctx->lay.partial));   // (and the arrival flags kept in `partial`)
    }
    // moment matrices: the padding entries of their layout are read (and multiplied by zero) but never written
    // (also the cached ones)
    if (ctx->lay.opt_m > ctx->lay.gram[0]) CREATE_TRY(hipMemset(ctx->gram[0], 0, ctx->lay.opt_m - ctx->lay.gram[0]));
    CREATE_TRY(hipEventCreate(&ctx->base));
    CREATE_TRY(hipEventRecord(ctx->base, nullptr));

    if (cfg->model == BMGD_SOFTMAX) {
        CREATE_TRY(softmax_prepare(softmax_dims(cfg->p, cfg->batch_n, cfg->n_classes)));
        ctx->chain = resolve_chain(ctx->cfg);        // three launches per mini-batch update, replayed from a graph or issued one by one
        if (ctx->chain == BMGD_CHAIN_GRAPH) CREATE_TRY(hipStreamCreateWithFlags(&ctx->capture_stream, hipStreamNonBlocking));
    } else {
        char msg[160];
        if (!glm_plan(cfg->p, cfg->batch_n, cfg->n_workgroups, ctx->num_cus, &ctx->shape, msg, sizeof msg)) {
            ctx->err = msg;
            return bail(BMGD_EINVAL);
        }
        ctx->shape.with_optimizer = cfg->optimizer != BMGD_OPT_SGD;
        CREATE_TRY(glm_prepare(&ctx->shape));
        ctx->chain = resolve_chain(ctx->cfg);
        if (ctx->chain == BMGD_CHAIN_GRAM) {
            CREATE_TRY(hipStreamCreateWithFlags(&ctx->chain_stream, hipStreamNonBlocking));   // default priority
        }
    }
    CREATE_TRY(hipDeviceSynchronize());
#undef CREATE_TRY
    *out = ctx;
    return BMGD_OK;
}

BMGD_API bmgd_ctx* bmgd_create(int64_t p, int64_t buffer_n, int64_t batch_n, double lr, int passes)
{
    bmgd_config cfg;
    bmgd_default_config(&cfg);
    cfg.p = p; cfg.buffer_n = buffer_n; cfg.batch_n = batch_n; cfg.lr = lr; cfg.passes = passes;
    bmgd_ctx* ctx = nullptr;
    if (bmgd_create_ex(&cfg, &ctx) != BMGD_OK) return nullptr;
    return ctx;
}

// Copy (host_x, host_y) into the slot the next load goes to; `rec` receives the copy's events.
static int enqueue_load(bmgd_ctx* ctx, const void* host_x, const void* host_y, int64_t rows, hipStream_t cs, RunRecord& rec,
                        int* slot_out)
{
    Slot& slot = ctx->slots[ctx->next_slot];
    // the copy must not overwrite rows a run is still reading
    if (slot.was_read) HIP_TRY(ctx, hipStreamWaitEvent(cs, slot.compute_done, 0));
    if (!rec.copy_start) rec.copy_start = take_event(ctx);
    if (!rec.copy_end) rec.copy_end = take_event(ctx);
    if (!rec.copy_start || !rec.copy_end) return fail(ctx, BMGD_EHIP, "could not create events");
    const size_t xbytes = (size_t)rows * ctx->cfg.p * ctx->x_itemsize, ybytes = (size_t)rows * 4;
    HIP_TRY(ctx, hipEventRecord(rec.copy_start, cs));
    HIP_TRY(ctx, hipMemcpyAsync(slot.x, host_x, xbytes, hipMemcpyHostToDevice, cs));
    HIP_TRY(ctx, hipMemcpyAsync(slot.y, host_y, ybytes, hipMemcpyHostToDevice, cs));
    HIP_TRY(ctx, hipEventRecord(rec.copy_end, cs));
    slot.copy_done = rec.copy_end;
    rec.has_copy = true;
    slot.rows = rows;
    ctx->h2d_bytes += (int64_t)(xbytes + ybytes);
    *slot_out = ctx->next_slot;
    ctx->next_slot ^= 1;
    ctx->last_copy = cs;
    ctx->used_copy = true;
    return BMGD_OK;
}

BMGD_API int bmgd_load_buffer_async(bmgd_ctx* ctx, const void* host_x, const void* host_y, int64_t rows, void* copy_stream)
{
    if (!ctx) return BMGD_EINVAL;
    if (!host_x || !host_y) return fail(ctx, BMGD_EINVAL, "host_x and host_y must not be NULL");
    if (rows < 1 || rows > ctx->cfg.buffer_n) return fail(ctx, BMGD_EINVAL, "rows must be in [1, buffer_n]");
    if (ctx->pending >= 0) return fail(ctx, BMGD_ESTATE, "a buffer is already loaded and has not been run");
    HIP_TRY(ctx, hipSetDevice(ctx->device));
    int slot = -1;
    const int rc = enqueue_load(ctx, host_x, host_y, rows, static_cast<hipStream_t>(copy_stream), ctx->pending_copy, &slot);
    if (rc != BMGD_OK) return rc;
    ctx->pending = slot;
    return BMGD_OK;
}

BMGD_API int bmgd_run_buffer(bmgd_ctx* ctx, void* compute_stream)
{
    if (!ctx) return BMGD_EINVAL;
    if (ctx->pending < 0) return fail(ctx, BMGD_ESTATE, "no buffer is loaded");
    if (refuse_if_poisoned(ctx) != BMGD_OK) return BMGD_ESTATE;
    HIP_TRY(ctx, hipSetDevice(ctx->device));
    hipStream_t s = static_cast<hipStream_t>(compute_stream);
    Slot& slot = ctx->slots[ctx->pending];
    const int64_t run_rows = rows_of_run(ctx, slot.rows);
    if (run_rows == 0) return BMGD_EINVAL;
    RunRecord rec = ctx->pending_copy;
    rec.start = take_event(ctx); rec.end = take_event(ctx);
    if (!rec.start || !rec.end) return fail(ctx, BMGD_EHIP, "could not create events");
    HIP_TRY(ctx, hipStreamWaitEvent(s, slot.copy_done, 0));       // never read a slot that is still filling
    HIP_TRY(ctx, hipEventRecord(rec.start, s));
    hipEvent_t last = nullptr;
    const size_t chain0 = ctx->open_chain.size(), prep0 = ctx->open_prep.size();
    const int rc = enqueue_compute(ctx, slot.x, slot.y, run_rows, s, &last);
    ctx->subset = nullptr;                                        // a subset holds for one run
    ctx->last_compute = s;
    ctx->used_compute = true;
    if (rc != BMGD_OK) return abandon_run(ctx, rec, rc);
    if (last) { give_event(ctx, rec.end); rec.end = last; rec.owns_end = false; }
    else HIP_TRY(ctx, hipEventRecord(rec.end, s));
    HIP_TRY(ctx, hipEventRecord(slot.compute_done, s));           // every kernel that reads the slot runs on s
    slot.was_read = true;
    rec.n_chain = (int)(ctx->open_chain.size() - chain0);
    rec.n_prep = (int)(ctx->open_prep.size() - prep0);
    ctx->open_records.push_back(rec);
    ctx->pending_copy = RunRecord();
    ctx->pending = -1;
    return trim_records(ctx);
}

// The adaptive run behind both entry points: passes over the loaded buffer until the buffer that follows has
// arrived on the device.  That buffer is either given (next_x, next_y, next_rows) or comes from `reader`, which is
// polled before every pass and whose buffer is copied as soon as it is in host memory.
static int run_adaptive(bmgd_ctx* ctx, hipStream_t s, hipStream_t cs, const void* next_x, const void* next_y, int64_t next_rows,
                        bmgd_reader* reader, int min_passes, int max_passes, int* passes_done, int64_t* next_rows_out)
{
    if (passes_done) *passes_done = 0;
    if (next_rows_out) *next_rows_out = 0;
    if (ctx->pending < 0) return fail(ctx, BMGD_ESTATE, "no buffer is loaded");
    if (refuse_if_poisoned(ctx) != BMGD_OK) return BMGD_ESTATE;
    if (min_passes < 1 || max_passes < min_passes || max_passes > (1 << 20))
        return fail(ctx, BMGD_EINVAL, "need 1 <= min_passes <= max_passes <= 2^20");
    HIP_TRY(ctx, hipSetDevice(ctx->device));
    Slot& slot = ctx->slots[ctx->pending];
    const int64_t run_rows = rows_of_run(ctx, slot.rows);
    if (run_rows == 0) return BMGD_EINVAL;
    RunRecord rec = ctx->pending_copy;
    ctx->pending_copy = RunRecord();
    rec.start = take_event(ctx); rec.end = take_event(ctx);
    if (!rec.start || !rec.end) return fail(ctx, BMGD_EHIP, "could not create events");
    HIP_TRY(ctx, hipStreamWaitEvent(s, slot.copy_done, 0));
    HIP_TRY(ctx, hipEventRecord(rec.start, s));
    const size_t chain0 = ctx->open_chain.size(), prep0 = ctx->open_prep.size();
    ctx->last_compute = s;
    ctx->used_compute = true;

    // the buffering step for the next buffer, into the other slot (Section 2.1: both steps at the same time)
    enum { kAwaitingHost, kCopying, kNone } next = next_x ? kAwaitingHost : (reader ? kAwaitingHost : kNone);
    RunRecord next_rec;
    int next_slot = -1;
    auto start_copy = [&](bool block) -> int {
        const void *x = next_x, *y = next_y;
        int64_t rows = next_rows;
        if (reader) {
            int end = 0;
            const int rc = reader_take(reader, block, &x, &y, &rows, &end);
            if (rc != BMGD_OK) return fail(ctx, rc, std::string("reader: ") + bmgd_reader_last_error(reader));
            if (end) { next = kNone; return BMGD_OK; }
            if (!x) return BMGD_OK;                      // not in host memory yet
            if (rows > ctx->cfg.buffer_n) {
                (void)bmgd_reader_release(reader, nullptr, 0);
                return fail(ctx, BMGD_EINVAL, "the reader's buffers are larger than buffer_n");
            }
        }
        const int rc = enqueue_load(ctx, x, y, rows, cs, next_rec, &next_slot);
        if (reader) (void)bmgd_reader_release(reader, cs, rc == BMGD_OK);
        if (rc != BMGD_OK) return rc;
        if (next_rows_out) *next_rows_out = rows;
        next = kCopying;
        return BMGD_OK;
    };

    // One pass per launch; at most two passes enqueued and unfinished, so that the decision to stop lags the arrival
    // of the next buffer by at most two passes and the device still never runs dry.
    int passes = 0;
    hipEvent_t last = nullptr, in_flight[2] = {nullptr, nullptr};
    for (;;) {
        if (next == kAwaitingHost) {
            const int rc = start_copy(false);
            if (rc != BMGD_OK) return rc;
        }
        if (passes >= max_passes) break;
        if (passes >= min_passes) {
            if (next == kNone) break;
            if (next == kCopying) {
                const hipError_t q = hipEventQuery(next_rec.copy_end);
                if (q == hipSuccess) break;
                if (q != hipErrorNotReady) return hip_fail(ctx, q, "hipEventQuery(copy of the next buffer)");
            }
        }
        if (in_flight[0]) HIP_TRY(ctx, hipEventSynchronize(in_flight[0]));
        hipEvent_t chunk = nullptr;
        const int rc = enqueue_passes(ctx, slot.x, slot.y, run_rows, s, passes, 1, &last, &chunk);
        if (rc != BMGD_OK) {
            if (next_slot >= 0) {
                // the copy of the next buffer has been started: that buffer is the loaded one now, and the events of
                // this buffer's copy (which every kernel enqueued so far already waits for) go back to the pool
                give_event(ctx, rec.copy_start); give_event(ctx, rec.copy_end);
                ctx->pending_copy = next_rec;
                ctx->pending = next_slot;
            } else {
                ctx->pending_copy = rec;                 // still the loaded buffer, with its copy events
                ctx->pending_copy.start = ctx->pending_copy.end = nullptr;
            }
            return abandon_run(ctx, rec, rc);
        }
        in_flight[0] = in_flight[1];
        in_flight[1] = chunk;
        passes += 1;
    }
    finish_run(ctx, run_rows, passes);
    ctx->subset = nullptr;
    if (last) { give_event(ctx, rec.end); rec.end = last; rec.owns_end = false; }
    else HIP_TRY(ctx, hipEventRecord(rec.end, s));
    HIP_TRY(ctx, hipEventRecord(slot.compute_done, s));
    slot.was_read = true;
    rec.n_chain = (int)(ctx->open_chain.size() - chain0);
    rec.n_prep = (int)(ctx->open_prep.size() - prep0);
    ctx->open_records.push_back(rec);
    ctx->pending = -1;
    if (passes_done) *passes_done = passes;
    // max_passes reached before the reader had the next buffer: wait for it now, so that the call ends as promised
    if (next == kAwaitingHost) {
        const int rc = start_copy(true);
        if (rc != BMGD_OK) return rc;
    }
    ctx->pending = next_slot;
    ctx->pending_copy = next_rec;
    return trim_records(ctx);
}

BMGD_API int bmgd_run_buffer_adaptive(bmgd_ctx* ctx, void* compute_stream, const void* next_host_x, const void* next_host_y,
                                      int64_t next_rows, void* copy_stream, int min_passes, int max_passes, int* passes_done)
{
    if (!ctx) return BMGD_EINVAL;
    const bool have_next = next_host_x != nullptr || next_host_y != nullptr;
    if (have_next && (!next_host_x || !next_host_y)) return fail(ctx, BMGD_EINVAL, "next_host_x and next_host_y go together");
    if (have_next && (next_rows < 1 || next_rows > ctx->cfg.buffer_n))
        return fail(ctx, BMGD_EINVAL, "next_rows must be in [1, buffer_n]");
    return run_adaptive(ctx, static_cast<hipStream_t>(compute_stream), static_cast<hipStream_t>(copy_stream), next_host_x,
                        next_host_y, next_rows, nullptr, min_passes, max_passes, passes_done, nullptr);
}

BMGD_API int bmgd_run_buffer_adaptive_reader(bmgd_ctx* ctx, void* compute_stream, bmgd_reader* reader, void* copy_stream,
                                             int min_passes, int max_passes, int* passes_done, int64_t* next_rows)
{
    if (!ctx) return BMGD_EINVAL;
    if (!reader) return fail(ctx, BMGD_EINVAL, "reader must not be NULL");
    return run_adaptive(ctx, static_cast<hipStream_t>(compute_stream), static_cast<hipStream_t>(copy_stream), nullptr, nullptr,
                        0, reader, min_passes, max_passes, passes_done, next_rows);
}

// A run over rows that are already on the device (or, with dev_x = dev_y = NULL, over a buffer whose moment matrices
// are cached: then no row is read).
static int run_resident(bmgd_ctx* ctx, const void* dev_x, const void* dev_y, int64_t rows, hipStream_t s)
{
    if (refuse_if_poisoned(ctx) != BMGD_OK) return BMGD_ESTATE;
    HIP_TRY(ctx, hipSetDevice(ctx->device));
    const int64_t run_rows = rows_of_run(ctx, rows);
    if (run_rows == 0) return BMGD_EINVAL;
    RunRecord rec;
    rec.start = take_event(ctx); rec.end = take_event(ctx);
    if (!rec.start || !rec.end) return fail(ctx, BMGD_EHIP, "could not create events");
    HIP_TRY(ctx, hipEventRecord(rec.start, s));
    hipEvent_t last = nullptr;
    const size_t chain0 = ctx->open_chain.size(), prep0 = ctx->open_prep.size();
    const int rc = enqueue_compute(ctx, dev_x, dev_y, run_rows, s, &last);
    ctx->subset = nullptr;
    ctx->last_compute = s;
    ctx->used_compute = true;
    if (rc != BMGD_OK) return abandon_run(ctx, rec, rc);
    if (last) { give_event(ctx, rec.end); rec.end = last; rec.owns_end = false; }
    else HIP_TRY(ctx, hipEventRecord(rec.end, s));
    rec.n_chain = (int)(ctx->open_chain.size() - chain0);
    rec.n_prep = (int)(ctx->open_prep.size() - prep0);
    ctx->open_records.push_back(rec);
    return trim_records(ctx);
}

BMGD_API int bmgd_run_device_buffer(bmgd_ctx* ctx, const void* dev_x, const void* dev_y, int64_t rows, void* compute_stream)
{
    if (!ctx) return BMGD_EINVAL;
    if (!dev_x || !dev_y) return fail(ctx, BMGD_EINVAL, "dev_x and dev_y must not be NULL");
    if (rows < 1 || rows >= (int64_t(1) << 30)) return fail(ctx, BMGD_EINVAL, "rows must be in [1, 2^30)");
    if (rows > ctx->cfg.buffer_n) return fail(ctx, BMGD_EINVAL, "rows must not exceed buffer_n");
    if ((reinterpret_cast<uintptr_t>(dev_x) % 16) != 0 || (reinterpret_cast<uintptr_t>(dev_y) % 4) != 0)
        return fail(ctx, BMGD_EINVAL, "device buffers must be at least 16-byte aligned");
    return run_resident(ctx, dev_x, dev_y, rows, static_cast<hipStream_t>(compute_stream));
}

BMGD_API int bmgd_run_cached_buffer(bmgd_ctx* ctx, void* compute_stream)
{
    if (!ctx) return BMGD_EINVAL;
    if (!ctx->cfg.cache_moments) return fail(ctx, BMGD_ESTATE, "the context was created without cache_moments");
    if (ctx->subset) return fail(ctx, BMGD_ESTATE, "a row subset is set: cached moment matrices cover whole buffers");
    const bmgd_ctx::CachedMoments& ce = ctx->mcache[(size_t)(ctx->buffer_counter % ctx->cfg.n_buffers)];
    if (!ce.valid) return fail(ctx, BMGD_ESTATE, "the moment matrices of this buffer are not cached yet");
    return run_resident(ctx, nullptr, nullptr, ce.rows, static_cast<hipStream_t>(compute_stream));
}

BMGD_API int bmgd_clear_moment_cache(bmgd_ctx* ctx)
{
    if (!ctx) return BMGD_EINVAL;
    const int rc = drain(ctx);                           // no chain may still be reading them
    if (rc != BMGD_OK) return rc;
    for (auto& ce : ctx->mcache) ce.valid = ce.prod_valid = false;
    return BMGD_OK;
}

BMGD_API int bmgd_eval_loss(bmgd_ctx* ctx, const void* dev_x, const void* dev_y, int64_t rows, void* stream, double* host_out)
{
    if (!ctx) return BMGD_EINVAL;
    if (!dev_x || !dev_y || !host_out) return fail(ctx, BMGD_EINVAL, "dev_x, dev_y and host_out must not be NULL");
    if (rows < 1 || rows >= (int64_t(1) << 30)) return fail(ctx, BMGD_EINVAL, "rows must be in [1, 2^30)");
    if ((reinterpret_cast<uintptr_t>(dev_x) % 16) != 0 || (reinterpret_cast<uintptr_t>(dev_y) % 4) != 0)
        return fail(ctx, BMGD_EINVAL, "device buffers must be at least 16-byte aligned");
    const int rc = drain(ctx);
    if (rc != BMGD_OK) return rc;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const bmgd_config& c = ctx->cfg;
    double* partial = reinterpret_cast<double*>(static_cast<char*>(ctx->ws) + ctx->lay.eval);
    std::vector<double> host(kEvalBlocks);
    double total = 0.0;
    if (c.model == BMGD_SOFTMAX) {
        const SoftmaxDims d = softmax_dims(c.p, c.batch_n, c.n_classes);
        const int64_t chunk = std::min<int64_t>(c.batch_n, (int64_t)kEvalBlocks * 8);
        for (int64_t r0 = 0; r0 < rows; r0 += chunk) {
            const int nb = (int)std::min<int64_t>(chunk, rows - r0);
            HIP_TRY(ctx, softmax_launch_loss(static_cast<const char*>(dev_x) + (size_t)r0 * c.p * 2,
                                             static_cast<const int32_t*>(dev_y) + r0, nb, (int)c.p, c.n_classes, ctx->wbt, ctx->u,
                                             d, partial, s));
            const int nblocks = (nb + 7) / 8;
            HIP_TRY(ctx, hipMemcpyAsync(host.data(), partial, (size_t)nblocks * sizeof(double), hipMemcpyDeviceToHost, s));
            HIP_TRY(ctx, hipStreamSynchronize(s));
            for (int b = 0; b < nblocks; ++b) total += host[(size_t)b];
        }
    } else {
        const int nblocks = (int)std::min<int64_t>(kEvalBlocks, (rows + 3) / 4);
        HIP_TRY(ctx, glm_launch_loss(static_cast<const float*>(dev_x), static_cast<const float*>(dev_y), ctx->theta, (int)rows,
                                     (int)c.p, c.model, partial, nblocks, s));
        HIP_TRY(ctx, hipMemcpyAsync(host.data(), partial, (size_t)nblocks * sizeof(double), hipMemcpyDeviceToHost, s));
        HIP_TRY(ctx, hipStreamSynchronize(s));
        for (int b = 0; b < nblocks; ++b) total += host[(size_t)b];
    }
    *host_out = total / (double)rows;
    return BMGD_OK;
}

BMGD_API int bmgd_sync(bmgd_ctx* ctx)
{
    if (!ctx) return BMGD_EINVAL;
    return drain(ctx);
}

BMGD_API int bmgd_get_theta(bmgd_ctx* ctx, float* host_out, int64_t len)
{
    if (!ctx) return BMGD_EINVAL;
    if (!host_out) return fail(ctx, BMGD_EINVAL, "host_out must not be NULL");
    if (len != ctx->theta_len) return fail(ctx, BMGD_EINVAL, "len must equal p (p * n_classes for softmax)");
    const int rc = drain(ctx);
    if (rc != BMGD_OK) return rc;
    if (ctx->cfg.model == BMGD_SOFTMAX) {
        const SoftmaxDims d = softmax_dims(ctx->cfg.p, ctx->cfg.batch_n, ctx->cfg.n_classes);
        const size_t C = (size_t)ctx->cfg.n_classes;
        HIP_TRY(ctx, hipMemcpy2D(host_out, C * 4, ctx->theta, (size_t)d.c_pad * 4, C * 4, (size_t)ctx->cfg.p, hipMemcpyDeviceToHost));
        return BMGD_OK;
    }
    HIP_TRY(ctx, hipMemcpy(host_out, ctx->theta, (size_t)len * 4, hipMemcpyDeviceToHost));
    return BMGD_OK;
}

BMGD_API int bmgd_set_theta(bmgd_ctx* ctx, const float* host_in, int64_t len)
{
    if (!ctx) return BMGD_EINVAL;
    if (!host_in) return fail(ctx, BMGD_EINVAL, "host_in must not be NULL");
    if (len != ctx->theta_len) return fail(ctx, BMGD_EINVAL, "len must equal p (p * n_classes for softmax)");
    const int rc = drain(ctx);                           // (an abandoned run found only now is what this call is the remedy for)
    if (rc != BMGD_OK && !ctx->poisoned) return rc;
    ctx->poisoned = false;
    if (ctx->cfg.model == BMGD_SOFTMAX) {
        const SoftmaxDims d = softmax_dims(ctx->cfg.p, ctx->cfg.batch_n, ctx->cfg.n_classes);
        const size_t C = (size_t)ctx->cfg.n_classes;
        HIP_TRY(ctx, hipMemcpy2D(ctx->theta, (size_t)d.c_pad * 4, host_in, C * 4, C * 4, (size_t)ctx->cfg.p, hipMemcpyHostToDevice));
        HIP_TRY(ctx, softmax_refresh_shadow(ctx->theta, ctx->wbt, (int)ctx->cfg.p, d, nullptr));
        HIP_TRY(ctx, hipDeviceSynchronize());
        return BMGD_OK;
    }
    HIP_TRY(ctx, hipMemcpy(ctx->theta, host_in, (size_t)len * 4, hipMemcpyHostToDevice));
    return BMGD_OK;
}

BMGD_API int bmgd_set_lr(bmgd_ctx* ctx, double lr)
{
    if (!ctx) return BMGD_EINVAL;
    if (!(lr > 0.0) || !std::isfinite(lr)) return fail(ctx, BMGD_EINVAL, "lr must be finite and positive");
    ctx->cfg.lr = lr;
    return BMGD_OK;
}

BMGD_API int bmgd_reset_optimizer(bmgd_ctx* ctx)
{
    if (!ctx) return BMGD_EINVAL;
    const int rc = drain(ctx);
    if (rc != BMGD_OK) return rc;
    if (ctx->lay.eval > ctx->lay.opt_m) HIP_TRY(ctx, hipMemset(ctx->opt_m, 0, ctx->lay.eval - ctx->lay.opt_m));
    ctx->opt_k = 0;
    return BMGD_OK;
}

BMGD_API int bmgd_set_row_subset(bmgd_ctx* ctx, const int32_t* dev_idx, int64_t count)
{
    if (!ctx) return BMGD_EINVAL;
    if (!dev_idx && count != 0) return fail(ctx, BMGD_EINVAL, "dev_idx must not be NULL unless count is 0");
    if (count < 0 || count > ctx->cfg.buffer_n) return fail(ctx, BMGD_EINVAL, "count must be in [0, buffer_n]");
    if ((reinterpret_cast<uintptr_t>(dev_idx) % 4) != 0) return fail(ctx, BMGD_EINVAL, "dev_idx must be 4-byte aligned");
    ctx->subset = count > 0 ? dev_idx : nullptr;
    ctx->subset_count = count;
    return BMGD_OK;
}

BMGD_API int bmgd_swa_update(bmgd_ctx* ctx, void* compute_stream)
{
    if (!ctx) return BMGD_EINVAL;
    HIP_TRY(ctx, hipSetDevice(ctx->device));
    // behind the last update of theta: in the moment form those run on the library's stream
    hipStream_t s = ctx->chain == BMGD_CHAIN_GRAM ? ctx->chain_stream : static_cast<hipStream_t>(compute_stream);
    const size_t n = (ctx->lay.total - ctx->lay.swa) / 4;           // whole array, padding included (stays 0)
    HIP_TRY(ctx, launch_running_mean(ctx->swa, ctx->theta, n, 1.0f / (float)(ctx->swa_count + 1), ctx->swa_count == 0, s));
    ctx->swa_count += 1;
    if (ctx->chain != BMGD_CHAIN_GRAM) {
        ctx->last_compute = s;
        ctx->used_compute = true;
    }
    return BMGD_OK;
}

BMGD_API int bmgd_get_swa(bmgd_ctx* ctx, float* host_out, int64_t len, int64_t* count)
{
    if (!ctx) return BMGD_EINVAL;
    if (count) *count = ctx->swa_count;
    if (!host_out) return fail(ctx, BMGD_EINVAL, "host_out must not be NULL");
    if (len != ctx->theta_len) return fail(ctx, BMGD_EINVAL, "len must equal p (p * n_classes for softmax)");
    if (ctx->swa_count == 0) return fail(ctx, BMGD_ESTATE, "no estimate has been averaged yet");
    const int rc = drain(ctx);
    if (rc != BMGD_OK) return rc;
    if (ctx->cfg.model == BMGD_SOFTMAX) {
        const SoftmaxDims d = softmax_dims(ctx->cfg.p, ctx->cfg.batch_n, ctx->cfg.n_classes);
        const size_t C = (size_t)ctx->cfg.n_classes;
        HIP_TRY(ctx, hipMemcpy2D(host_out, C * 4, ctx->swa, (size_t)d.c_pad * 4, C * 4, (size_t)ctx->cfg.p, hipMemcpyDeviceToHost));
        return BMGD_OK;
    }
    HIP_TRY(ctx, hipMemcpy(host_out, ctx->swa, (size_t)len * 4, hipMemcpyDeviceToHost));
    return BMGD_OK;
}

BMGD_API int bmgd_swa_reset(bmgd_ctx* ctx)
{
    if (!ctx) return BMGD_EINVAL;
    ctx->swa_count = 0;                                  // the next bmgd_swa_update starts over from its snapshot
    return BMGD_OK;
}

BMGD_API int bmgd_set_lr_schedule(bmgd_ctx* ctx, const float* host_alphas, int64_t len)
{
    if (!ctx) return BMGD_EINVAL;
    if (len < 0 || len >= (int64_t(1) << 30) || (len > 0 && !host_alphas))
        return fail(ctx, BMGD_EINVAL, "host_alphas must hold len values, 0 <= len < 2^30");
    for (int64_t i = 0; i < len; ++i)
        if (!(host_alphas[i] > 0.f) || !std::isfinite(host_alphas[i]))
            return fail(ctx, BMGD_EINVAL, "every learning rate must be finite and positive");
    const int rc = drain(ctx);
    if (rc != BMGD_OK) return rc;
    // captured passes hold the table's address and length among their kernels' arguments: captured again when next used
    for (auto& kv : ctx->pass_graphs) (void)hipGraphExecDestroy(kv.second);
    ctx->pass_graphs.clear();
    if (ctx->lr_tab_dev) { HIP_TRY(ctx, hipFree(ctx->lr_tab_dev)); ctx->lr_tab_dev = nullptr; }
    ctx->lr_tab_host.clear();
    ctx->lr_pos = 0;
    if (len == 0) return BMGD_OK;
    HIP_TRY(ctx, hipMalloc(reinterpret_cast<void**>(&ctx->lr_tab_dev), (size_t)len * sizeof(float)));
    HIP_TRY(ctx, hipMemcpy(ctx->lr_tab_dev, host_alphas, (size_t)len * sizeof(float), hipMemcpyHostToDevice));
    ctx->lr_tab_host.assign(host_alphas, host_alphas + len);
    return BMGD_OK;
}

BMGD_API int bmgd_set_passes(bmgd_ctx* ctx, int passes)
{
    if (!ctx) return BMGD_EINVAL;
    if (passes < 1) return fail(ctx, BMGD_EINVAL, "passes must be at least 1");
    ctx->cfg.passes = passes;
    return BMGD_OK;
}

BMGD_API int bmgd_set_position(bmgd_ctx* ctx, int64_t buffer_counter)
{
    if (!ctx) return BMGD_EINVAL;
    if (buffer_counter < 0 || buffer_counter > 0xFFFFFFFFLL) return fail(ctx, BMGD_EINVAL, "buffer_counter out of range");
    ctx->buffer_counter = buffer_counter;
    return BMGD_OK;
}

BMGD_API int bmgd_get_perm(bmgd_ctx* ctx, int64_t buffer_counter, int pass, int32_t* host_out, int64_t len)
{
    if (!ctx) return BMGD_EINVAL;
    if (!host_out) return fail(ctx, BMGD_EINVAL, "host_out must not be NULL");
    if (len < 1 || len > ctx->cfg.buffer_n) return fail(ctx, BMGD_EINVAL, "len must be in [1, buffer_n]");
    if (pass < 0 || buffer_counter < 0 || buffer_counter > 0xFFFFFFFFLL) return fail(ctx, BMGD_EINVAL, "bad pass or buffer_counter");
    const int rc = drain(ctx);
    if (rc != BMGD_OK) return rc;
    PermKeys keys{};
    perm_round_keys(ctx->cfg.seed, (uint32_t)buffer_counter, (uint32_t)pass, keys.key[0]);
    HIP_TRY(ctx, launch_perm(ctx->perm, len, 1, keys, nullptr));
    HIP_TRY(ctx, hipMemcpy(host_out, ctx->perm, (size_t)len * 4, hipMemcpyDeviceToHost));
    return BMGD_OK;
}

BMGD_API int bmgd_get_stats(bmgd_ctx* ctx, bmgd_stats* out)
{
    if (!ctx) return BMGD_EINVAL;
    if (!out) return fail(ctx, BMGD_EINVAL, "out must not be NULL");
    const int rc = drain(ctx);
    memset(out, 0, sizeof *out);
    out->buffers_run = ctx->buffer_counter;
    out->steps = ctx->steps;
    out->sample_gradients = ctx->sample_gradients;
    out->h2d_bytes = ctx->h2d_bytes;
    out->copy_ms = ctx->copy_ms;
    out->compute_ms = ctx->compute_ms;
    out->wait_ms = ctx->wait_ms;
    const bool one_group = ctx->chain == BMGD_CHAIN_GRAM;       // the chain itself runs in a single workgroup
    out->n_workgroups = one_group ? 1 : ctx->shape.G;
    out->threads_per_group = one_group ? gram_chain_threads(ctx->cfg.p)
                             : ctx->chain == BMGD_CHAIN_PERSISTENT ? ctx->shape.chain_block : ctx->shape.block;
    out->chain = ctx->products ? BMGD_CHAIN_PRODUCT : ctx->chain;
    out->chain_ms = ctx->chain_ms;
    out->chain_launches = ctx->chain_launches;
    out->prep_ms = ctx->prep_ms;
    out->prep_launches = ctx->prep_launches;
    return rc;
}

BMGD_API const char* bmgd_last_error(const bmgd_ctx* ctx)
{
    return ctx ? ctx->err.c_str() : g_create_error.c_str();
}

BMGD_API void bmgd_destroy(bmgd_ctx* ctx) { destroy_ctx(ctx); }

}  // extern "C"
