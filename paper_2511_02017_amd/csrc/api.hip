// C ABI of libtapout: argument validation, scratch ownership, launch sequencing.
// Every entry point validates on the host, then only enqueues kernels.
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>
#include <limits>
#include <vector>

#include "common.h"

using namespace tapout;

struct tapout_ctx {
    tapout_config cfg;
    Partial *part = nullptr;      size_t part_cap = 0;       // slice partials of the draft pass (and of a shard pass)
    Partial *part_t = nullptr;                                 // slice partials of the target pass (same capacity)
    double *part1 = nullptr, *part2 = nullptr;                // residual sampler slice sums
    JobRecord *jobs = nullptr;                                 // per final-token job: what to draw from, and its band list
    uint32_t *flags_ws = nullptr;
    int32_t *arm_played = nullptr;                             // [max_batch]: the arms a round was drafted under (see draft_stats_impl)
    double *exp_table = nullptr;                               // 2^(k/256), k = 0..255, for the final-token passes
    int nsl_max = 0;                                           // final-token slices per row at cfg.vocab
    double *sum_r = nullptr, *sum_r2 = nullptr; int64_t *count = nullptr;   // bandit state [n_bandits, n_arms]
    // state of the stateful stop rules (allocated only when an arm needs it)
    bool stateful = false;
    float *prev_entropy = nullptr;                             // [max_batch]
    double *accept_rate = nullptr, *lambda = nullptr;          // [max_batch], [max_batch, n_arms]
    float *round_entropy = nullptr;                            // [max_batch, max_k] entropies of the last draft_stats call
    int round_K = 0;                                           // its K (0: no draft_stats call yet)
    int positions = 1;                                         // bandits per slot: 1, or max_k for token-level bandits
    int wgs_target = 4096;        // workgroups a streaming launch aims for
    int min_slice = 4096;         // smallest slice (elements) a row is cut into
    int slice_bytes = 65536;      // slice size aimed for when the rows alone give enough workgroups
    int fuse_head = -1;           // tapout_verify: accept decisions inside the slice kernel (1), in a launch of their own (0), by size (-1)
    int exp_lookup = 1;           // final token: exponentials of bfloat16 row pairs from the table (1) or computed (0)
    int defer_epilogue = 1;       // tapout_round: the draft epilogue may run beside the final-token locate kernel (1) or keeps its own launch (0)
    // optional kernel timing (tapout_profile_*): event pairs around the launches of selected kernels
    uint32_t prof_mask = 0;
    int prof_cap = 0;
    std::vector<hipEvent_t> prof_start[TAPOUT_PROFILE_KINDS], prof_stop[TAPOUT_PROFILE_KINDS];
    int prof_used[TAPOUT_PROFILE_KINDS] = {0};
    int prof_stride = 1;                                   // "profile_stride": events on every n-th launch of a kernel only
    unsigned prof_tick[TAPOUT_PROFILE_KINDS] = {0};
    char err[256] = {0};
};

// Scratch of tapout_draft_stats_static, the entry point that allocates nothing: its slice partials live here instead
// of in context memory.  Every GPU the library runs on holds its own copy at its own address until the process ends.
// In host code the name is only a handle for the symbol: the device address is looked up once per device
// (static_scratch below) and that pointer is what kernels get.
static __device__ __align__(256) unsigned char scratch[(size_t)TAPOUT_STATIC_MAX_PARTIALS * sizeof(Partial)];

namespace {

constexpr int kMaxWgsTarget = 1 << 16;
// "fuse_head" = -1: fuse while the slice kernel's workgroups are all resident at once: a second round of workgroups
// would pay the prologue a second time (measured at V = 128256 with five workgroups per CU: fused wins by 1.5-2.5 us
// up to 1280 workgroups and loses by 1-2 us from 1536 on).  Four per CU when a row is bfloat16: the table of
// exponentials takes 36 KB of LDS per workgroup.
constexpr int kFuseHeadMaxWgs = 1280, kFuseHeadMaxWgsBf16 = 1024;
constexpr int kMinSliceBytes = 16384;            // lower limit of the "slice_bytes" option (sizes the partial buffer)
thread_local char g_create_err[256] = {0};

tapout_status fail(tapout_ctx *ctx, tapout_status st, const char *fmt, ...)
{
    char *dst = ctx ? ctx->err : g_create_err;
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(dst, 256, fmt, ap);
    va_end(ap);
    return st;
}

tapout_status hip_fail(tapout_ctx *ctx, hipError_t e, const char *what)
{
    return fail(ctx, TAPOUT_EHIP, "%s: %s", what, hipGetErrorString(e));
}

struct DeviceGuard {
    int prev = -1; bool changed = false;
    explicit DeviceGuard(int dev) {
        if (hipGetDevice(&prev) == hipSuccess && prev != dev) changed = hipSetDevice(dev) == hipSuccess;
    }
    ~DeviceGuard() { if (changed) (void)hipSetDevice(prev); }
};

// Vectors per slice: a multiple of 64 (whole 1 KB wavefront loads) such that nsplit slices cover a row
// whatever its alignment (an unaligned row has at most one vector more than an aligned one).
int slice_vectors(int V, int dtype, int nsplit)
{
    const int vec = dtype == TAPOUT_F32 ? 4 : 8;
    const int nvec = (V + vec - 1) / vec + 1;
    return (((nvec + nsplit - 1) / nsplit) + 63) & ~63;
}

// Slices per row: enough for about wgs_target workgroups per launch when rows are few, and slices of about
// slice_bytes when rows are many (a launch ends ragged by about half the duration of one workgroup, so
// workgroups that stream a whole long row cost several percent of the launch); never below min_slice
// elements per slice, which no longer amortises a workgroup's fixed cost.  slice_bytes is the size for 2-byte
// elements; slices of 4-byte elements hold as many elements, twice the bytes (a workgroup's arithmetic goes by the
// element, and a launch of many short workgroups is held up by their dispatch: V = 256000, 512 sequences, binary32
// target rows in 128 KB slices 828 us, in 64 KB slices 840 us; bfloat16 draft rows the other way round, 401 / 385 us).
int choose_nsplit_for(int wgs_target, int min_slice, int slice_bytes, int64_t rows, int V, int dtype)
{
    const int64_t row_bytes = (int64_t)V * (dtype == TAPOUT_F32 ? 4 : 2);
    int64_t want = (wgs_target + rows - 1) / rows;
    const int64_t by_bytes = row_bytes / ((int64_t)slice_bytes * (dtype == TAPOUT_F32 ? 2 : 1));
    if (want < by_bytes) want = by_bytes;
    int64_t by_size = V / min_slice;
    if (by_size < 1) by_size = 1;
    if (want > by_size) want = by_size;
    if (want > kStageCap) want = kStageCap;      // an epilogue stages whole rows of partials in LDS
    if (want < 1) want = 1;
    return (int)want;
}

int choose_nsplit(const tapout_ctx *ctx, int64_t rows, int V, int dtype)
{
    return choose_nsplit_for(ctx->wgs_target, ctx->min_slice, ctx->slice_bytes, rows, V, dtype);
}

// ---- device address of the static scratch, per device ------------------------------------------------
constexpr size_t kStaticPartials = TAPOUT_STATIC_MAX_PARTIALS;
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void *g_scratch_ptr[kMaxDevices] = {nullptr};

// Device address of `scratch` on the current device `dev`, or NULL (the HIP error is left in *err).
Partial *static_scratch(int dev, hipError_t *err)
{
    *err = hipSuccess;
    if (dev < 0 || dev >= kMaxDevices) { *err = hipErrorInvalidDevice; return nullptr; }
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        *err = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (*err != hipSuccess || !p) { if (*err == hipSuccess) *err = hipErrorInvalidSymbol; return nullptr; }
        g_scratch_ptr[dev] = p;
    }
    return (Partial *)g_scratch_ptr[dev];
}

const char *check_logits(const tapout_logits *l, const char *name, int V, int rows_k, char *buf)
{
    if (!l || !l->ptr) { snprintf(buf, 128, "%s logits pointer is NULL", name); return buf; }
    if (l->dtype != TAPOUT_F32 && l->dtype != TAPOUT_BF16) { snprintf(buf, 128, "%s logits: unknown dtype %d", name, l->dtype); return buf; }
    int esz = l->dtype == TAPOUT_F32 ? 4 : 2;
    if ((uintptr_t)l->ptr % esz) { snprintf(buf, 128, "%s logits pointer is not element-aligned", name); return buf; }
    if (l->stride_b < 0 || l->stride_k < 0) { snprintf(buf, 128, "%s logits: negative stride", name); return buf; }
    (void)V; (void)rows_k;
    return nullptr;
}

// Enqueue one kernel; when timing of `kind` is on, hand the launcher an event pair that the
// runtime stamps with the begin and end of the kernel's execution.
template <class F>
hipError_t timed(tapout_ctx *ctx, int kind, F launch)
{
    bool on = (ctx->prof_mask >> kind) & 1u && ctx->prof_used[kind] < ctx->prof_cap;
    if (on && ctx->prof_stride > 1) on = ctx->prof_tick[kind]++ % ctx->prof_stride == 0;     // time one launch in prof_stride
    if (!on) return launch(Timing{});
    const int i = ctx->prof_used[kind];
    hipError_t e = launch(Timing{ctx->prof_start[kind][i], ctx->prof_stop[kind][i]});
    if (e == hipSuccess) ctx->prof_used[kind] = i + 1;
    return e;
}

void profile_release(tapout_ctx *ctx)
{
    for (int k = 0; k < TAPOUT_PROFILE_KINDS; ++k) {
        for (hipEvent_t ev : ctx->prof_start[k]) (void)hipEventDestroy(ev);
        for (hipEvent_t ev : ctx->prof_stop[k]) (void)hipEventDestroy(ev);
        ctx->prof_start[k].clear(); ctx->prof_stop[k].clear(); ctx->prof_used[k] = 0; ctx->prof_tick[k] = 0;
    }
    ctx->prof_mask = 0; ctx->prof_cap = 0;
}

BanditArgs bandit_args(const tapout_ctx *ctx, int B)
{
    BanditArgs a{};
    a.policy = ctx->cfg.policy; a.n_bandits = ctx->cfg.n_bandits; a.n_arms = ctx->cfg.n_arms; a.B = B;
    a.positions = ctx->positions;
    a.reward = ctx->cfg.reward; a.alpha = ctx->cfg.alpha;
    a.sum_r = ctx->sum_r; a.sum_r2 = ctx->sum_r2; a.count = ctx->count;
    for (int j = 0; j < TAPOUT_MAX_ARMS; ++j) a.rule[j] = ctx->cfg.rule[j];
    if (ctx->stateful) {
        a.prev_entropy = ctx->prev_entropy; a.accept_rate = ctx->accept_rate; a.lambda = ctx->lambda;
        a.round_entropy = ctx->round_entropy; a.round_K = ctx->round_K;
        a.ad_alpha = ctx->cfg.adaedl_alpha; a.ad_beta1 = ctx->cfg.adaedl_beta1; a.ad_beta2 = ctx->cfg.adaedl_beta2;
        a.ad_eps = ctx->cfg.adaedl_eps; a.ad_steer = ctx->cfg.adaedl_steer;
    }
    return a;
}

tapout_status check_shape(tapout_ctx *ctx, int B, int K, int V)
{
    if (B < 0 || B > ctx->cfg.max_batch) return fail(ctx, TAPOUT_EINVAL, "B = %d outside [0, max_batch = %d]", B, ctx->cfg.max_batch);
    if (K < 1 || K > ctx->cfg.max_k) return fail(ctx, TAPOUT_EINVAL, "K = %d outside [1, max_k = %d]", K, ctx->cfg.max_k);
    if (V < 1 || V > ctx->cfg.vocab) return fail(ctx, TAPOUT_EINVAL, "V = %d outside [1, vocab = %d]", V, ctx->cfg.vocab);
    return TAPOUT_OK;
}

}  // namespace

extern "C" {

void tapout_default_config(tapout_config *cfg, int32_t max_batch, int32_t max_k, int32_t vocab)
{
    if (!cfg) return;
    memset(cfg, 0, sizeof *cfg);
    cfg->device = 0;
    cfg->max_batch = max_batch; cfg->max_k = max_k; cfg->vocab = vocab;
    cfg->n_arms = 3;
    cfg->rule[0] = TAPOUT_RULE_SVIP;    cfg->threshold[0] = 0.6f;
    cfg->rule[1] = TAPOUT_RULE_MAXCONF; cfg->threshold[1] = 0.8f;
    cfg->rule[2] = TAPOUT_RULE_MARGIN;  cfg->threshold[2] = 0.2f;
    cfg->policy = TAPOUT_UCB1;
    cfg->n_bandits = max_batch;
    cfg->alpha = 0.5;
    cfg->reward = TAPOUT_REWARD_BLEND;
    cfg->granularity = TAPOUT_SEQUENCE_LEVEL;
    cfg->adaedl_gamma = 0.5; cfg->adaedl_alpha = 0.9; cfg->adaedl_beta1 = 0.5; cfg->adaedl_beta2 = 0.9;
    cfg->adaedl_eps = 0.01; cfg->adaedl_rate0 = 0.9;
}

tapout_status tapout_create(tapout_ctx **out, const tapout_config *cfg)
{
    if (!out) return fail(nullptr, TAPOUT_EINVAL, "out is NULL");
    *out = nullptr;
    if (!cfg) return fail(nullptr, TAPOUT_EINVAL, "cfg is NULL");
    if (cfg->max_batch < 1 || cfg->max_k < 1 || cfg->vocab < 1)
        return fail(nullptr, TAPOUT_EINVAL, "max_batch, max_k and vocab must be positive");
    if (cfg->max_k > 4096) return fail(nullptr, TAPOUT_EINVAL, "max_k = %d exceeds 4096", cfg->max_k);
    if (cfg->max_batch > 65535) return fail(nullptr, TAPOUT_EINVAL, "max_batch = %d exceeds 65535", cfg->max_batch);
    if ((int64_t)cfg->max_batch * (cfg->max_k + 1) > (int64_t)1 << 26)
        return fail(nullptr, TAPOUT_EINVAL, "max_batch * (max_k + 1) exceeds 2^26 rows");
    if (cfg->n_arms < 1 || cfg->n_arms > TAPOUT_MAX_ARMS) return fail(nullptr, TAPOUT_EINVAL, "n_arms = %d outside [1, %d]", cfg->n_arms, TAPOUT_MAX_ARMS);
    bool stateful = false, adaedl = false;
    for (int a = 0; a < cfg->n_arms; ++a) {
        if (cfg->rule[a] < TAPOUT_RULE_SVIP || cfg->rule[a] > TAPOUT_RULE_ADAEDL)
            return fail(nullptr, TAPOUT_EUNSUPPORTED, "arm %d: rule %d is not implemented", a, cfg->rule[a]);
        if (!(cfg->threshold[a] == cfg->threshold[a])) return fail(nullptr, TAPOUT_EINVAL, "arm %d: threshold is NaN", a);
        if (cfg->rule[a] == TAPOUT_RULE_SVIP_DIFF || cfg->rule[a] == TAPOUT_RULE_ADAEDL) stateful = true;
        if (cfg->rule[a] == TAPOUT_RULE_ADAEDL) adaedl = true;
    }
    if (cfg->policy < TAPOUT_UCB1 || cfg->policy > TAPOUT_TS_GAUSS) return fail(nullptr, TAPOUT_EUNSUPPORTED, "policy %d is not implemented", cfg->policy);
    if (cfg->granularity != TAPOUT_SEQUENCE_LEVEL && cfg->granularity != TAPOUT_TOKEN_LEVEL)
        return fail(nullptr, TAPOUT_EUNSUPPORTED, "granularity %d is not implemented", cfg->granularity);
    if (cfg->draft_sampling != 0 && cfg->draft_sampling != 1) return fail(nullptr, TAPOUT_EINVAL, "draft_sampling must be 0 or 1");
    if (cfg->reward != TAPOUT_REWARD_BLEND && cfg->reward != TAPOUT_REWARD_SIMPLE) return fail(nullptr, TAPOUT_EUNSUPPORTED, "reward %d is not implemented", cfg->reward);
    if (cfg->adaedl_steer != 0 && cfg->adaedl_steer != 1) return fail(nullptr, TAPOUT_EINVAL, "adaedl_steer must be 0 or 1");
    if (adaedl) {
        if (!(cfg->adaedl_gamma >= 0.0) || !(cfg->adaedl_gamma < INFINITY)) return fail(nullptr, TAPOUT_EINVAL, "adaedl_gamma must be finite and >= 0");
        if (!(cfg->adaedl_beta1 >= 0.0 && cfg->adaedl_beta1 <= 1.0) || !(cfg->adaedl_beta2 >= 0.0 && cfg->adaedl_beta2 <= 1.0))
            return fail(nullptr, TAPOUT_EINVAL, "adaedl_beta1 and adaedl_beta2 must lie in [0, 1]");
        if (!(cfg->adaedl_alpha == cfg->adaedl_alpha) || !(cfg->adaedl_eps == cfg->adaedl_eps) || !(cfg->adaedl_rate0 == cfg->adaedl_rate0))
            return fail(nullptr, TAPOUT_EINVAL, "adaedl_alpha, adaedl_eps and adaedl_rate0 must not be NaN");
    }
    if (cfg->n_bandits != 1 && cfg->n_bandits != cfg->max_batch) return fail(nullptr, TAPOUT_EINVAL, "n_bandits must be 1 or max_batch");
    if (!(cfg->alpha >= 0.0 && cfg->alpha <= 1.0)) return fail(nullptr, TAPOUT_EINVAL, "alpha outside [0, 1]");
    int ndev = 0;
    if (hipGetDeviceCount(&ndev) != hipSuccess || cfg->device < 0 || cfg->device >= ndev)
        return fail(nullptr, TAPOUT_EHIP, "device %d not available (%d HIP devices)", cfg->device, ndev);

    tapout_ctx *c = new (std::nothrow) tapout_ctx;
    if (!c) return fail(nullptr, TAPOUT_ENOMEM, "host allocation failed");
    c->cfg = *cfg;
    DeviceGuard guard(cfg->device);
    const size_t rows = (size_t)cfg->max_batch * (cfg->max_k + 1);
    int64_t by_bytes_max = (int64_t)cfg->vocab * 4 / kMinSliceBytes;
    by_bytes_max = by_bytes_max < 1 ? 1 : (by_bytes_max > kStageCap ? kStageCap : by_bytes_max);
    c->part_cap = rows * (size_t)by_bytes_max + kMaxWgsTarget;   // rows * nsplit under either rule of choose_nsplit
    c->positions = cfg->granularity == TAPOUT_TOKEN_LEVEL ? cfg->max_k : 1;
    const size_t nstate = (size_t)cfg->n_bandits * c->positions * cfg->n_arms;
    c->nsl_max = (cfg->vocab + kSampleSlice - 1) / kSampleSlice;
    // final-token jobs: one per sequence (verification) or one per draft row (draft-token sampling)
    const size_t njobs = (size_t)cfg->max_batch * (cfg->draft_sampling ? cfg->max_k : 1);
    // 2^(k/256), then exp(x) of every bfloat16 x with 2^-12 <= |x| < 63.5: entry idx (x > 0) or pairs + idx (x < 0),
    // idx = 1 + (magnitude bits - (115 << 7)); idx 0 stands for all smaller magnitudes and holds NaN (the kernels
    // notice and compute), the last idx for all larger ones and holds zeros
    std::vector<double> table(256 + kExpBf16Doubles);
    for (int k = 0; k < 256; ++k) table[k] = std::exp2((double)k / 256.0);
    const int pairs = kExpBf16Doubles / 2;
    for (int idx = 0; idx < pairs; ++idx) {
        double pos, neg;
        if (idx == 0) pos = neg = std::numeric_limits<double>::quiet_NaN();
        else if (idx == pairs - 1) pos = neg = 0.0;
        else {
            const uint32_t bits = (uint32_t)((115 << 7) + idx - 1) << 16;
            float x;
            memcpy(&x, &bits, sizeof x);
            pos = std::exp((double)x);
            neg = std::exp(-(double)x);
        }
        table[256 + idx] = pos;
        table[256 + pairs + idx] = neg;
    }
    bool ok = hipMalloc(&c->part, c->part_cap * sizeof(Partial)) == hipSuccess
           && hipMalloc(&c->part_t, c->part_cap * sizeof(Partial)) == hipSuccess
           && hipMalloc(&c->part1, njobs * c->nsl_max * 5 * sizeof(double)) == hipSuccess
           && hipMalloc(&c->part2, njobs * c->nsl_max * sizeof(double)) == hipSuccess
           && hipMalloc(&c->exp_table, table.size() * sizeof(double)) == hipSuccess
           && hipMemcpy(c->exp_table, table.data(), table.size() * sizeof(double), hipMemcpyHostToDevice) == hipSuccess
           && hipMalloc(&c->jobs, njobs * sizeof(JobRecord)) == hipSuccess
           && hipMalloc(&c->flags_ws, (size_t)cfg->max_batch * sizeof(uint32_t)) == hipSuccess
           && hipMalloc(&c->arm_played, (size_t)cfg->max_batch * sizeof(int32_t)) == hipSuccess
           && hipMalloc(&c->sum_r, nstate * sizeof(double)) == hipSuccess
           && hipMalloc(&c->sum_r2, nstate * sizeof(double)) == hipSuccess
           && hipMalloc(&c->count, nstate * sizeof(int64_t)) == hipSuccess
           && hipMemset(c->sum_r, 0, nstate * sizeof(double)) == hipSuccess
           && hipMemset(c->sum_r2, 0, nstate * sizeof(double)) == hipSuccess
           && hipMemset(c->count, 0, nstate * sizeof(int64_t)) == hipSuccess;
    c->stateful = stateful;
    if (ok && stateful) {
        const size_t nb = (size_t)cfg->max_batch;
        std::vector<float> pe(nb, NAN);
        std::vector<double> ar(nb, cfg->adaedl_rate0), lam(nb * cfg->n_arms);
        for (size_t b = 0; b < nb; ++b)
            for (int a = 0; a < cfg->n_arms; ++a) lam[b * cfg->n_arms + a] = (double)cfg->threshold[a];
        ok = hipMalloc(&c->prev_entropy, nb * sizeof(float)) == hipSuccess
          && hipMalloc(&c->accept_rate, nb * sizeof(double)) == hipSuccess
          && hipMalloc(&c->lambda, nb * cfg->n_arms * sizeof(double)) == hipSuccess
          && hipMalloc(&c->round_entropy, nb * cfg->max_k * sizeof(float)) == hipSuccess
          && hipMemcpy(c->prev_entropy, pe.data(), nb * sizeof(float), hipMemcpyHostToDevice) == hipSuccess
          && hipMemcpy(c->accept_rate, ar.data(), nb * sizeof(double), hipMemcpyHostToDevice) == hipSuccess
          && hipMemcpy(c->lambda, lam.data(), nb * cfg->n_arms * sizeof(double), hipMemcpyHostToDevice) == hipSuccess;
    }
    if (!ok) {
        (void)hipGetLastError();
        tapout_destroy(c);
        return fail(nullptr, TAPOUT_ENOMEM, "device allocation failed");
    }
    *out = c;
    return TAPOUT_OK;
}

tapout_status tapout_destroy(tapout_ctx *ctx)
{
    if (!ctx) return TAPOUT_OK;
    DeviceGuard guard(ctx->cfg.device);
    profile_release(ctx);
    (void)hipFree(ctx->part); (void)hipFree(ctx->part_t); (void)hipFree(ctx->part1); (void)hipFree(ctx->part2);
    (void)hipFree(ctx->jobs); (void)hipFree(ctx->flags_ws); (void)hipFree(ctx->arm_played);
    (void)hipFree(ctx->exp_table);
    (void)hipFree(ctx->sum_r); (void)hipFree(ctx->sum_r2); (void)hipFree(ctx->count);
    (void)hipFree(ctx->prev_entropy); (void)hipFree(ctx->accept_rate); (void)hipFree(ctx->lambda); (void)hipFree(ctx->round_entropy);
    delete ctx;
    return TAPOUT_OK;
}

const char *tapout_last_error(const tapout_ctx *ctx) { return ctx ? ctx->err : g_create_err; }

tapout_status tapout_set_option(tapout_ctx *ctx, const char *name, int32_t value)
{
    if (!ctx || !name) return TAPOUT_EINVAL;
    if (!strcmp(name, "wgs_target")) {
        if (value < 1 || value > kMaxWgsTarget) return fail(ctx, TAPOUT_EINVAL, "wgs_target outside [1, %d]", kMaxWgsTarget);
        ctx->wgs_target = value;
    } else if (!strcmp(name, "slice_bytes")) {
        if (value < kMinSliceBytes) return fail(ctx, TAPOUT_EINVAL, "slice_bytes below %d", kMinSliceBytes);
        ctx->slice_bytes = value;
    } else if (!strcmp(name, "min_slice")) {
        if (value < 256) return fail(ctx, TAPOUT_EINVAL, "min_slice below 256 elements");
        ctx->min_slice = value;
    } else if (!strcmp(name, "profile_stride")) {
        if (value < 1) return fail(ctx, TAPOUT_EINVAL, "profile_stride below 1");
        ctx->prof_stride = value;
    } else if (!strcmp(name, "fuse_head")) {
        if (value < -1 || value > 1) return fail(ctx, TAPOUT_EINVAL, "fuse_head outside {-1, 0, 1}");
        ctx->fuse_head = value;
    } else if (!strcmp(name, "exp_lookup")) {
        if (value < 0 || value > 1) return fail(ctx, TAPOUT_EINVAL, "exp_lookup outside {0, 1}");
        ctx->exp_lookup = value;
    } else if (!strcmp(name, "defer_epilogue")) {
        if (value < 0 || value > 1) return fail(ctx, TAPOUT_EINVAL, "defer_epilogue outside {0, 1}");
        ctx->defer_epilogue = value;
    } else return fail(ctx, TAPOUT_EINVAL, "unknown option '%s'", name);
    return TAPOUT_OK;
}

tapout_status tapout_bandit_select(tapout_ctx *ctx, int32_t B, const float *u_ts,
                                   int32_t *arm_out, uint32_t *flags, void *stream)
{
    if (!ctx) return TAPOUT_EINVAL;
    if (B < 0 || B > ctx->cfg.max_batch) return fail(ctx, TAPOUT_EINVAL, "B = %d outside [0, max_batch = %d]", B, ctx->cfg.max_batch);
    if (B == 0) return TAPOUT_OK;
    if (!arm_out) return fail(ctx, TAPOUT_EINVAL, "arm_out is NULL");
    if ((ctx->cfg.policy == TAPOUT_TS_BETA || ctx->cfg.policy == TAPOUT_TS_GAUSS) && !u_ts) return fail(ctx, TAPOUT_EINVAL, "Thompson Sampling needs u_ts");
    DeviceGuard guard(ctx->cfg.device);
    BanditArgs a = bandit_args(ctx, B);
    hipStream_t st = (hipStream_t)stream;
    hipError_t e = timed(ctx, TAPOUT_PROFILE_SELECT, [&](Timing tm) { return launch_bandit_select(a, u_ts, arm_out, flags, st, tm); });
    return e == hipSuccess ? TAPOUT_OK : hip_fail(ctx, e, "bandit_select launch");
}

tapout_status tapout_bandit_update(tapout_ctx *ctx, int32_t B, const int32_t *arm,
                                   const int32_t *accept_len, const int32_t *n_draft,
                                   const int32_t *gamma, const uint8_t *active, void *stream)
{
    if (!ctx) return TAPOUT_EINVAL;
    if (B < 0 || B > ctx->cfg.max_batch) return fail(ctx, TAPOUT_EINVAL, "B = %d outside [0, max_batch = %d]", B, ctx->cfg.max_batch);
    if (B == 0) return TAPOUT_OK;
    if (!arm || !accept_len || !n_draft || !gamma) return fail(ctx, TAPOUT_EINVAL, "arm, accept_len, n_draft and gamma are required");
    DeviceGuard guard(ctx->cfg.device);
    BanditArgs a = bandit_args(ctx, B);
    hipStream_t st = (hipStream_t)stream;
    hipError_t e = timed(ctx, TAPOUT_PROFILE_UPDATE, [&](Timing tm) { return launch_bandit_update(a, arm, accept_len, n_draft, gamma, active, st, tm); });
    return e == hipSuccess ? TAPOUT_OK : hip_fail(ctx, e, "bandit_update launch");
}

tapout_status tapout_bandit_update_select(tapout_ctx *ctx, int32_t B, const int32_t *arm,
                                          const int32_t *accept_len, const int32_t *n_draft,
                                          const int32_t *gamma, const uint8_t *active,
                                          const float *u_ts, int32_t *arm_out, uint32_t *flags, void *stream)
{
    if (!ctx) return TAPOUT_EINVAL;
    if (B < 0 || B > ctx->cfg.max_batch) return fail(ctx, TAPOUT_EINVAL, "B = %d outside [0, max_batch = %d]", B, ctx->cfg.max_batch);
    if (B == 0) return TAPOUT_OK;
    if (!arm || !accept_len || !n_draft || !gamma) return fail(ctx, TAPOUT_EINVAL, "arm, accept_len, n_draft and gamma are required");
    if (!arm_out) return fail(ctx, TAPOUT_EINVAL, "arm_out is NULL");
    if ((ctx->cfg.policy == TAPOUT_TS_BETA || ctx->cfg.policy == TAPOUT_TS_GAUSS) && !u_ts) return fail(ctx, TAPOUT_EINVAL, "Thompson Sampling needs u_ts");
    DeviceGuard guard(ctx->cfg.device);
    BanditArgs a = bandit_args(ctx, B);
    hipStream_t st = (hipStream_t)stream;
    hipError_t e = timed(ctx, TAPOUT_PROFILE_UPDATE, [&](Timing tm) { return launch_bandit_update_select(a, arm, accept_len, n_draft, gamma, active, u_ts, arm_out, flags, st, tm); });
    return e == hipSuccess ? TAPOUT_OK : hip_fail(ctx, e, "bandit_update_select launch");
}

namespace {
struct VerifyCall;
hipError_t stream_pair(tapout_ctx *ctx, const RowReduceArgs &d, int d_dtype, const VerifyCall &c, hipStream_t st);
RowReduceArgs target_pass_args(tapout_ctx *ctx, const VerifyCall &c);

// tapout_draft_stats.  pair != NULL (tapout_round): the streaming pass is one launch over the draft rows and the target
// rows of *pair, with pair_nsplit slices per row for both.  defer != NULL (tapout_round): the epilogue is not launched;
// its arguments go to *defer for the caller to run later, the slice count to *defer_nsplit, and the streaming pass
// leaves the logits of the drafted tokens in its partials.
tapout_status draft_stats_impl(tapout_ctx *ctx, const tapout_logits *draft,
                                 int32_t B, int32_t K, int32_t V,
                                 const int32_t *draft_tok, const int32_t *k_len, const int32_t *arm,
                                 const float *u_draft,
                                 float *lse, float *entropy, float *p_top1, float *p_top2, float *margin,
                                 int32_t *top1_id, float *logq_tok, int32_t *sampled_tok,
                                 int32_t *n_stop, uint8_t *stop_fired, uint32_t *flags, void *stream,
                                 const VerifyCall *pair, int pair_nsplit, DraftFinalArgs *defer = nullptr, int *defer_nsplit = nullptr)
{
    if (!ctx) return TAPOUT_EINVAL;
    tapout_status s = check_shape(ctx, B, K, V);
    if (s != TAPOUT_OK) return s;
    if (B == 0) return TAPOUT_OK;
    char buf[128];
    if (const char *m = check_logits(draft, "draft", V, K, buf)) return fail(ctx, TAPOUT_EINVAL, "%s", m);
    if (arm && !n_stop && !stop_fired) return fail(ctx, TAPOUT_EINVAL, "arm given but neither n_stop nor stop_fired");
    if (u_draft && draft_tok) return fail(ctx, TAPOUT_EINVAL, "draft_tok and u_draft exclude each other");
    if (u_draft && !sampled_tok) return fail(ctx, TAPOUT_EINVAL, "u_draft given but sampled_tok is NULL");
    if (u_draft && !ctx->cfg.draft_sampling) return fail(ctx, TAPOUT_EINVAL, "u_draft needs a context created with draft_sampling = 1");
    DeviceGuard guard(ctx->cfg.device);
    hipStream_t st = (hipStream_t)stream;
    const int64_t rows = (int64_t)B * K;
    const int nsplit = pair ? pair_nsplit : choose_nsplit(ctx, rows, V, draft->dtype);
    if ((size_t)(rows * nsplit) > ctx->part_cap) return fail(ctx, TAPOUT_EINVAL, "internal: partial buffer too small");

    RowReduceArgs r{draft->ptr, draft->stride_b, draft->stride_k, V, K, nsplit, slice_vectors(V, draft->dtype, nsplit), (int32_t)rows, k_len, 0, ctx->part};
    if (defer) {
        if (u_draft || !draft_tok) return fail(ctx, TAPOUT_EINVAL, "internal: a deferred epilogue needs the caller's draft tokens");
        r.tok = draft_tok; r.tok_rows = K;
        // The deferred epilogue runs in the launch whose other workgroups may end the round and write the next
        // round's arms over the caller's array (sequence-level bandits: arm is [B], in and out): it reads the arms
        // the round was drafted under from a copy that the streaming pass, two launches earlier, leaves here.
        if (arm && ctx->positions == 1) { r.arm_src = arm; r.arm_dst = ctx->arm_played; }
    }
    hipError_t e = pair ? stream_pair(ctx, r, draft->dtype, *pair, st)
                        : timed(ctx, TAPOUT_PROFILE_DRAFT_PASS, [&](Timing tm) { return launch_row_reduce(r, draft->dtype, true, st, tm); });
    if (e != hipSuccess) return hip_fail(ctx, e, "draft pass launch");
    if (u_draft) {
        // draw the tokens first (one final-token job per draft row), so that the finaliser can form log q(tok)
        VerifyArgs va{};
        va.tbase = draft->ptr; va.t_dtype = draft->dtype; va.t_stride_b = draft->stride_b; va.t_stride_k = draft->stride_k;
        va.dbase = draft->ptr; va.d_dtype = draft->dtype; va.d_stride_b = draft->stride_b; va.d_stride_k = draft->stride_k;
        va.B = B; va.K = K; va.V = V; va.nsplit = nsplit; va.nsl = (V + kSampleSlice - 1) / kSampleSlice;
        va.jps = K; va.n_jobs = (int32_t)rows;
        va.part = ctx->part; va.n_draft = k_len; va.u_sample = u_draft; va.tok_direct = sampled_tok;
        va.flags_ws = ctx->flags_ws; va.jobs = ctx->jobs;
        va.part1 = ctx->part1; va.part2 = ctx->part2; va.exp_table = ctx->exp_table;
        if (!ctx->exp_lookup) va.vflags |= kVerifyNoExpTable;
        e = timed(ctx, TAPOUT_PROFILE_SAMPLE_HEAD, [&](Timing tm) { return launch_sample_head(va, st, tm); });
        for (int pass = 1; pass <= 2 && e == hipSuccess; ++pass)
            e = timed(ctx, TAPOUT_PROFILE_SAMPLE_SLICES + pass - 1, [&](Timing tm) { return launch_verify(va, pass, st, tm); });
        if (e != hipSuccess) return hip_fail(ctx, e, "draft sampling launch");
        draft_tok = sampled_tok;
    }
    DraftFinalArgs f{};
    f.base = draft->ptr; f.dtype = draft->dtype; f.stride_b = draft->stride_b; f.stride_k = draft->stride_k;
    f.B = B; f.K = K; f.V = V; f.nsplit = nsplit; f.per = r.per; f.part = ctx->part;
    f.draft_tok = draft_tok; f.k_len = k_len; f.arm = r.arm_dst ? r.arm_dst : arm;
    f.arm_stride = ctx->positions > 1 ? ctx->cfg.max_k : 0;
    f.n_arms = ctx->cfg.n_arms;
    for (int a = 0; a < TAPOUT_MAX_ARMS; ++a) { f.rule[a] = ctx->cfg.rule[a]; f.threshold[a] = ctx->cfg.threshold[a]; }
    f.lse = lse; f.entropy = entropy; f.p_top1 = p_top1; f.p_top2 = p_top2; f.margin = margin; f.logq_tok = logq_tok;
    f.top1_id = top1_id; f.n_stop = n_stop; f.stop_fired = stop_fired; f.flags = flags;
    if (ctx->stateful) {
        f.prev_entropy = ctx->prev_entropy; f.lambda = ctx->lambda; f.adaedl_gamma = ctx->cfg.adaedl_gamma;
        f.round_entropy = ctx->round_entropy;
        ctx->round_K = K;
    }
    if (defer) { *defer = f; *defer_nsplit = nsplit; return TAPOUT_OK; }
    e = timed(ctx, TAPOUT_PROFILE_DRAFT_FINALIZE, [&](Timing tm) { return launch_draft_finalize(f, st, tm); });
    return e == hipSuccess ? TAPOUT_OK : hip_fail(ctx, e, "draft finalize launch");
}
}  // namespace

tapout_status tapout_draft_stats(tapout_ctx *ctx, const tapout_logits *draft,
                                 int32_t B, int32_t K, int32_t V,
                                 const int32_t *draft_tok, const int32_t *k_len, const int32_t *arm,
                                 const float *u_draft,
                                 float *lse, float *entropy, float *p_top1, float *p_top2, float *margin,
                                 int32_t *top1_id, float *logq_tok, int32_t *sampled_tok,
                                 int32_t *n_stop, uint8_t *stop_fired, uint32_t *flags, void *stream)
{
    return draft_stats_impl(ctx, draft, B, K, V, draft_tok, k_len, arm, u_draft, lse, entropy, p_top1, p_top2, margin,
                            top1_id, logq_tok, sampled_tok, n_stop, stop_fired, flags, stream, nullptr, 0);
}

tapout_status tapout_draft_stats_static(const tapout_logits *draft, int32_t B, int32_t K, int32_t V,
                                 const int32_t *draft_tok, const int32_t *k_len, const int32_t *arm,
                                 int32_t n_arms, const int32_t *rule, const float *threshold,
                                 float *lse, float *entropy, float *p_top1, float *p_top2, float *margin,
                                 int32_t *top1_id, float *logq_tok,
                                 int32_t *n_stop, uint8_t *stop_fired, uint32_t *flags, void *stream)
{
    if (B < 0 || B > 65535) return fail(nullptr, TAPOUT_EINVAL, "B = %d outside [0, 65535]", B);
    if (K < 1 || K > kScanCap) return fail(nullptr, TAPOUT_EINVAL, "K = %d outside [1, %d]", K, kScanCap);
    if (V < 1) return fail(nullptr, TAPOUT_EINVAL, "V = %d must be positive", V);
    if (B == 0) return TAPOUT_OK;
    char buf[128];
    if (const char *m = check_logits(draft, "draft", V, K, buf)) return fail(nullptr, TAPOUT_EINVAL, "%s", m);
    if (arm) {
        if (!n_stop && !stop_fired) return fail(nullptr, TAPOUT_EINVAL, "arm given but neither n_stop nor stop_fired");
        if (n_arms < 1 || n_arms > TAPOUT_MAX_ARMS || !rule || !threshold)
            return fail(nullptr, TAPOUT_EINVAL, "arm given: need 1 <= n_arms <= %d, rule and threshold", TAPOUT_MAX_ARMS);
        for (int a = 0; a < n_arms; ++a) {
            if (rule[a] != TAPOUT_RULE_SVIP && rule[a] != TAPOUT_RULE_MAXCONF && rule[a] != TAPOUT_RULE_MARGIN)
                return fail(nullptr, TAPOUT_EUNSUPPORTED, "arm %d: rule %d carries state between drafts and needs a context", a, rule[a]);
            if (!(threshold[a] == threshold[a])) return fail(nullptr, TAPOUT_EINVAL, "arm %d: threshold is NaN", a);
        }
    }
    const int64_t rows = (int64_t)B * K;
    const int nsplit = choose_nsplit_for(4096, 4096, 65536, rows, V, draft->dtype);       // the defaults of a context
    if ((uint64_t)rows * (uint64_t)nsplit > kStaticPartials)
        return fail(nullptr, TAPOUT_EINVAL, "B * K * slices = %lld x %d exceeds the static scratch of %zu slice partials",
                    (long long)rows, nsplit, kStaticPartials);
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return hip_fail(nullptr, e, "hipGetDevice");
    Partial *part = static_scratch(dev, &e);
    if (!part) return hip_fail(nullptr, e, "hipGetSymbolAddress(scratch)");
    hipStream_t st = (hipStream_t)stream;
    RowReduceArgs r{draft->ptr, draft->stride_b, draft->stride_k, V, K, nsplit, slice_vectors(V, draft->dtype, nsplit), (int32_t)rows, k_len, 0, part};
    e = launch_row_reduce(r, draft->dtype, true, st, Timing{});
    if (e != hipSuccess) return hip_fail(nullptr, e, "draft pass launch");
    DraftFinalArgs f{};
    f.base = draft->ptr; f.dtype = draft->dtype; f.stride_b = draft->stride_b; f.stride_k = draft->stride_k;
    f.B = B; f.K = K; f.V = V; f.nsplit = nsplit; f.per = r.per; f.part = part;
    f.draft_tok = draft_tok; f.k_len = k_len; f.arm = arm;
    f.n_arms = arm ? n_arms : 0;
    for (int a = 0; a < TAPOUT_MAX_ARMS; ++a) {
        f.rule[a] = (arm && a < n_arms) ? rule[a] : TAPOUT_RULE_SVIP;
        f.threshold[a] = (arm && a < n_arms) ? threshold[a] : 0.0f;
    }
    f.lse = lse; f.entropy = entropy; f.p_top1 = p_top1; f.p_top2 = p_top2; f.margin = margin; f.logq_tok = logq_tok;
    f.top1_id = top1_id; f.n_stop = n_stop; f.stop_fired = stop_fired; f.flags = flags;
    e = launch_draft_finalize(f, st, Timing{});
    return e == hipSuccess ? TAPOUT_OK : hip_fail(nullptr, e, "draft finalize launch");
}

tapout_status tapout_shard_stats(tapout_ctx *ctx, const tapout_logits *shard,
                                 int32_t B, int32_t KK, int32_t Vs, int32_t vocab_offset,
                                 const int32_t *len, int32_t rows_mode, const int32_t *tok,
                                 tapout_shard_stat *out, void *stream)
{
    if (!ctx) return TAPOUT_EINVAL;
    if (rows_mode != 0 && rows_mode != 1) return fail(ctx, TAPOUT_EINVAL, "rows_mode must be 0 (draft rows) or 1 (target rows)");
    if (B < 0 || B > ctx->cfg.max_batch) return fail(ctx, TAPOUT_EINVAL, "B = %d outside [0, max_batch = %d]", B, ctx->cfg.max_batch);
    if (KK < 1 + rows_mode || KK > ctx->cfg.max_k + rows_mode) return fail(ctx, TAPOUT_EINVAL, "KK = %d outside [%d, %d]", KK, 1 + rows_mode, ctx->cfg.max_k + rows_mode);
    if (Vs < 1 || Vs > ctx->cfg.vocab) return fail(ctx, TAPOUT_EINVAL, "Vs = %d outside [1, vocab = %d]", Vs, ctx->cfg.vocab);
    if (vocab_offset < 0 || (int64_t)vocab_offset + Vs > INT32_MAX) return fail(ctx, TAPOUT_EINVAL, "vocab_offset out of range");
    if (B == 0) return TAPOUT_OK;
    char buf[128];
    if (const char *m = check_logits(shard, "shard", Vs, KK, buf)) return fail(ctx, TAPOUT_EINVAL, "%s", m);
    if (!out) return fail(ctx, TAPOUT_EINVAL, "out is NULL");
    if (rows_mode == 1 && !len) return fail(ctx, TAPOUT_EINVAL, "rows_mode 1 needs len (n_draft)");
    DeviceGuard guard(ctx->cfg.device);
    hipStream_t st = (hipStream_t)stream;
    const int64_t rows = (int64_t)B * KK;
    const int nsplit = choose_nsplit(ctx, rows, Vs, shard->dtype);
    if ((size_t)(rows * nsplit) > ctx->part_cap) return fail(ctx, TAPOUT_EINVAL, "internal: partial buffer too small");
    RowReduceArgs r{shard->ptr, shard->stride_b, shard->stride_k, Vs, KK, nsplit, slice_vectors(Vs, shard->dtype, nsplit), (int32_t)rows, len, rows_mode, ctx->part};
    // the draft pass also tracks the second maximum and the entropy sum; target rows need neither, but a record has one layout
    hipError_t e = timed(ctx, rows_mode ? TAPOUT_PROFILE_TARGET_PASS : TAPOUT_PROFILE_DRAFT_PASS,
                         [&](Timing tm) { return launch_row_reduce(r, shard->dtype, true, st, tm); });
    if (e != hipSuccess) return hip_fail(ctx, e, "shard pass launch");
    ShardMergeArgs m{shard->ptr, shard->dtype, shard->stride_b, shard->stride_k, B, KK, Vs, nsplit, r.per, vocab_offset, rows_mode,
                     ctx->part, len, tok, (Partial *)out};
    e = launch_shard_merge(m, st, Timing{});
    return e == hipSuccess ? TAPOUT_OK : hip_fail(ctx, e, "shard merge launch");
}

tapout_status tapout_draft_stats_sharded(tapout_ctx *ctx, const tapout_shard_stat *stats, int32_t G,
                                 int32_t B, int32_t K, int32_t V,
                                 const int32_t *draft_tok, const int32_t *k_len, const int32_t *arm,
                                 float *lse, float *entropy, float *p_top1, float *p_top2, float *margin,
                                 int32_t *top1_id, float *logq_tok,
                                 int32_t *n_stop, uint8_t *stop_fired, uint32_t *flags, void *stream)
{
    if (!ctx) return TAPOUT_EINVAL;
    if (B < 0 || B > ctx->cfg.max_batch) return fail(ctx, TAPOUT_EINVAL, "B = %d outside [0, max_batch = %d]", B, ctx->cfg.max_batch);
    if (K < 1 || K > ctx->cfg.max_k) return fail(ctx, TAPOUT_EINVAL, "K = %d outside [1, max_k = %d]", K, ctx->cfg.max_k);
    if (V < 1) return fail(ctx, TAPOUT_EINVAL, "V = %d must be positive", V);
    if (G < 1 || G > kStageCap) return fail(ctx, TAPOUT_EINVAL, "G = %d outside [1, %d]", G, kStageCap);
    if (B == 0) return TAPOUT_OK;
    if (!stats) return fail(ctx, TAPOUT_EINVAL, "stats is NULL");
    if (arm && !n_stop && !stop_fired) return fail(ctx, TAPOUT_EINVAL, "arm given but neither n_stop nor stop_fired");
    DeviceGuard guard(ctx->cfg.device);
    hipStream_t st = (hipStream_t)stream;
    DraftFinalArgs f{};
    f.base = nullptr; f.dtype = TAPOUT_F32;
    f.B = B; f.K = K; f.V = V; f.nsplit = G; f.shards = G; f.part = (const Partial *)stats;
    f.draft_tok = draft_tok; f.k_len = k_len; f.arm = arm;
    f.arm_stride = ctx->positions > 1 ? ctx->cfg.max_k : 0;
    f.n_arms = ctx->cfg.n_arms;
    for (int a = 0; a < TAPOUT_MAX_ARMS; ++a) { f.rule[a] = ctx->cfg.rule[a]; f.threshold[a] = ctx->cfg.threshold[a]; }
    f.lse = lse; f.entropy = entropy; f.p_top1 = p_top1; f.p_top2 = p_top2; f.margin = margin; f.logq_tok = logq_tok;
    f.top1_id = top1_id; f.n_stop = n_stop; f.stop_fired = stop_fired; f.flags = flags;
    if (ctx->stateful) {
        f.prev_entropy = ctx->prev_entropy; f.lambda = ctx->lambda; f.adaedl_gamma = ctx->cfg.adaedl_gamma;
        f.round_entropy = ctx->round_entropy;
        ctx->round_K = K;
    }
    hipError_t e = timed(ctx, TAPOUT_PROFILE_DRAFT_FINALIZE, [&](Timing tm) { return launch_draft_finalize(f, st, tm); });
    return e == hipSuccess ? TAPOUT_OK : hip_fail(ctx, e, "sharded draft finalize launch");
}

tapout_status tapout_verify_accept_sharded(tapout_ctx *ctx, const tapout_shard_stat *stats, int32_t G,
                                 int32_t B, int32_t K, int32_t V,
                                 const float *logq_tok, const int32_t *draft_tok, const int32_t *n_draft,
                                 const uint8_t *greedy, const float *u_accept, const float *draft_lse,
                                 int32_t *accept_len, int32_t *out_tok, int32_t *n_out,
                                 float *target_lse, float *logp_tok, int32_t *target_top1,
                                 tapout_final_job *final_jobs, uint32_t *flags, void *stream)
{
    if (!ctx) return TAPOUT_EINVAL;
    if (B < 0 || B > ctx->cfg.max_batch) return fail(ctx, TAPOUT_EINVAL, "B = %d outside [0, max_batch = %d]", B, ctx->cfg.max_batch);
    if (K < 1 || K > ctx->cfg.max_k) return fail(ctx, TAPOUT_EINVAL, "K = %d outside [1, max_k = %d]", K, ctx->cfg.max_k);
    if (V < 1) return fail(ctx, TAPOUT_EINVAL, "V = %d must be positive", V);
    if (G < 1 || G > kStageCap) return fail(ctx, TAPOUT_EINVAL, "G = %d outside [1, %d]", G, kStageCap);
    if (B == 0) return TAPOUT_OK;
    if (!stats || !logq_tok || !draft_tok || !n_draft || !u_accept) return fail(ctx, TAPOUT_EINVAL, "stats, logq_tok, draft_tok, n_draft and u_accept are required");
    if (final_jobs && !draft_lse) return fail(ctx, TAPOUT_EINVAL, "final_jobs needs draft_lse");
    if (!accept_len || !out_tok || !n_out) return fail(ctx, TAPOUT_EINVAL, "accept_len, out_tok and n_out are required");
    DeviceGuard guard(ctx->cfg.device);
    hipStream_t st = (hipStream_t)stream;
    VerifyArgs va{};
    va.B = B; va.K = K; va.V = V; va.nsplit = G; va.shards = G; va.jps = 1; va.n_jobs = B;
    va.part = (const Partial *)stats;
    va.logq_tok = logq_tok; va.draft_tok = draft_tok; va.n_draft = n_draft; va.greedy = greedy; va.u_accept = u_accept;
    va.draft_lse = draft_lse; va.final_jobs = (SampleJob *)final_jobs;
    va.accept_len = accept_len; va.out_tok = out_tok; va.n_out = n_out;
    va.target_lse = target_lse; va.logp_tok = logp_tok; va.target_top1 = target_top1; va.flags = flags;
    va.exp_table = ctx->exp_table;                  // the accept decisions' exponentials
    hipError_t e = timed(ctx, TAPOUT_PROFILE_VERIFY_HEAD, [&](Timing tm) { return launch_verify(va, 0, st, tm); });
    return e == hipSuccess ? TAPOUT_OK : hip_fail(ctx, e, "sharded verify head launch");
}

namespace {
tapout_status shard_final_args(tapout_ctx *ctx, const tapout_logits *target_shard, const tapout_logits *draft_shard,
                               int32_t B, int32_t K, int32_t Vs, const tapout_final_job *jobs, ShardFinalArgs *out)
{
    if (B < 0 || B > ctx->cfg.max_batch) return fail(ctx, TAPOUT_EINVAL, "B = %d outside [0, max_batch = %d]", B, ctx->cfg.max_batch);
    if (K < 1 || K > ctx->cfg.max_k) return fail(ctx, TAPOUT_EINVAL, "K = %d outside [1, max_k = %d]", K, ctx->cfg.max_k);
    if (Vs < 1 || Vs > ctx->cfg.vocab) return fail(ctx, TAPOUT_EINVAL, "Vs = %d outside [1, vocab = %d]", Vs, ctx->cfg.vocab);
    if (B == 0) return TAPOUT_OK;
    char buf[128];
    if (const char *m = check_logits(target_shard, "target shard", Vs, K + 1, buf)) return fail(ctx, TAPOUT_EINVAL, "%s", m);
    if (const char *m = check_logits(draft_shard, "draft shard", Vs, K, buf)) return fail(ctx, TAPOUT_EINVAL, "%s", m);
    if (!jobs) return fail(ctx, TAPOUT_EINVAL, "jobs is NULL");
    ShardFinalArgs a{};
    VerifyArgs &va = a.v;
    va.tbase = target_shard->ptr; va.t_dtype = target_shard->dtype; va.t_stride_b = target_shard->stride_b; va.t_stride_k = target_shard->stride_k;
    va.dbase = draft_shard->ptr; va.d_dtype = draft_shard->dtype; va.d_stride_b = draft_shard->stride_b; va.d_stride_k = draft_shard->stride_k;
    va.B = B; va.K = K; va.V = Vs; va.nsl = (Vs + kSampleSlice - 1) / kSampleSlice;
    va.jps = 1; va.n_jobs = B;
    va.jobs = ctx->jobs; va.part1 = ctx->part1; va.part2 = ctx->part2; va.exp_table = ctx->exp_table;
    if (!ctx->exp_lookup) va.vflags |= kVerifyNoExpTable;
    a.jobs_in = (const SampleJob *)jobs;
    *out = a;
    return TAPOUT_OK;
}
}  // namespace

tapout_status tapout_shard_final_sums(tapout_ctx *ctx, const tapout_logits *target_shard, const tapout_logits *draft_shard,
                                 int32_t B, int32_t K, int32_t Vs, const tapout_final_job *jobs,
                                 double *sums, void *stream)
{
    if (!ctx) return TAPOUT_EINVAL;
    ShardFinalArgs a{};
    tapout_status s = shard_final_args(ctx, target_shard, draft_shard, B, K, Vs, jobs, &a);
    if (s != TAPOUT_OK || B == 0) return s;
    if (!sums) return fail(ctx, TAPOUT_EINVAL, "sums is NULL");
    DeviceGuard guard(ctx->cfg.device);
    a.sums_out = sums;
    hipError_t e = launch_shard_final_sums(a, (hipStream_t)stream);
    return e == hipSuccess ? TAPOUT_OK : hip_fail(ctx, e, "shard final sums launch");
}

tapout_status tapout_shard_final_token(tapout_ctx *ctx, const tapout_logits *target_shard, const tapout_logits *draft_shard,
                                 int32_t B, int32_t K, int32_t Vs, int32_t vocab_offset, int32_t G, int32_t g,
                                 const tapout_final_job *jobs, const double *sums_all, const double *exact_all,
                                 const float *u_sample, int32_t *tok_out, double *exact_mass, uint8_t *need_exact,
                                 void *stream)
{
    if (!ctx) return TAPOUT_EINVAL;
    ShardFinalArgs a{};
    tapout_status s = shard_final_args(ctx, target_shard, draft_shard, B, K, Vs, jobs, &a);
    if (s != TAPOUT_OK || B == 0) return s;
    if (G < 1 || g < 0 || g >= G) return fail(ctx, TAPOUT_EINVAL, "need 0 <= g < G, got g = %d, G = %d", g, G);
    if (vocab_offset < 0 || (int64_t)vocab_offset + Vs > INT32_MAX) return fail(ctx, TAPOUT_EINVAL, "vocab_offset out of range");
    if (!sums_all || !u_sample || !tok_out || !exact_mass || !need_exact)
        return fail(ctx, TAPOUT_EINVAL, "sums_all, u_sample, tok_out, exact_mass and need_exact are required");
    DeviceGuard guard(ctx->cfg.device);
    a.v.u_sample = u_sample;
    a.sums_all = sums_all; a.exact_all = exact_all; a.G = G; a.g = g; a.vocab_offset = vocab_offset;
    a.tok_out = tok_out; a.exact_mass = exact_mass; a.need_exact = need_exact;
    hipError_t e = launch_shard_final_token(a, (hipStream_t)stream);
    return e == hipSuccess ? TAPOUT_OK : hip_fail(ctx, e, "shard final token launch");
}

namespace {

struct VerifyCall {
    const tapout_logits *target, *draft;
    int32_t B, K, V;
    const float *draft_lse, *logq_tok; const int32_t *draft_tok, *n_draft; const uint8_t *greedy;
    const float *u_accept, *u_sample;
    int32_t *accept_len, *out_tok, *n_out; float *target_lse, *logp_tok; int32_t *target_top1; uint32_t *flags;
    // derived by verify_check
    int nsplit, nsl; bool fused;
};

tapout_status verify_check(tapout_ctx *ctx, VerifyCall &c)
{
    tapout_status s = check_shape(ctx, c.B, c.K, c.V);
    if (s != TAPOUT_OK || c.B == 0) return s;
    char buf[128];
    if (const char *m = check_logits(c.target, "target", c.V, c.K + 1, buf)) return fail(ctx, TAPOUT_EINVAL, "%s", m);
    if (const char *m = check_logits(c.draft, "draft", c.V, c.K, buf)) return fail(ctx, TAPOUT_EINVAL, "%s", m);
    if (!c.draft_lse || !c.logq_tok || !c.draft_tok || !c.n_draft || !c.u_accept || !c.u_sample)
        return fail(ctx, TAPOUT_EINVAL, "draft_lse, logq_tok, draft_tok, n_draft, u_accept and u_sample are required");
    if (!c.accept_len || !c.out_tok || !c.n_out) return fail(ctx, TAPOUT_EINVAL, "accept_len, out_tok and n_out are required");
    const int64_t rows = (int64_t)c.B * (c.K + 1);
    c.nsplit = choose_nsplit(ctx, rows, c.V, c.target->dtype);
    if ((size_t)(rows * c.nsplit) > ctx->part_cap) return fail(ctx, TAPOUT_EINVAL, "internal: partial buffer too small");
    // With few sequences the final-token slice kernel is a handful of workgroups per compute unit and its launch
    // is latency: then the accept decisions are taken inside it (by every workgroup of a sequence again) and the
    // head launch with its hand-over through memory goes away.  With many sequences that kernel is bound by
    // arithmetic and the repeated head would add to it: separate launch.
    c.nsl = (c.V + kSampleSlice - 1) / kSampleSlice;
    const int64_t slice_wgs = (int64_t)c.B * ((c.nsl + 3) / 4);
    const bool any_bf16 = c.target->dtype == TAPOUT_BF16 || c.draft->dtype == TAPOUT_BF16;
    c.fused = ctx->fuse_head < 0 ? slice_wgs <= (any_bf16 ? kFuseHeadMaxWgsBf16 : kFuseHeadMaxWgs) : ctx->fuse_head == 1;
    return TAPOUT_OK;
}

// The streaming pass over the target rows (it needs n_draft and the drafted tokens, nothing the draft pass computes).
RowReduceArgs target_pass_args(tapout_ctx *ctx, const VerifyCall &c)
{
    const int64_t rows = (int64_t)c.B * (c.K + 1);
    return RowReduceArgs{c.target->ptr, c.target->stride_b, c.target->stride_k, c.V, c.K + 1, c.nsplit, slice_vectors(c.V, c.target->dtype, c.nsplit),
                         (int32_t)rows, c.n_draft, 1, ctx->part_t,
                         c.fused ? ctx->jobs : nullptr, c.draft_tok, c.K};     // the pass also picks up the logits of the drafted tokens
}

hipError_t verify_target_pass(tapout_ctx *ctx, const VerifyCall &c, hipStream_t st)
{
    const RowReduceArgs r = target_pass_args(ctx, c);
    return timed(ctx, TAPOUT_PROFILE_TARGET_PASS, [&](Timing tm) { return launch_row_reduce(r, c.target->dtype, false, st, tm); });
}

// Draft rows and target rows in one launch (tapout_round).
hipError_t stream_pair(tapout_ctx *ctx, const RowReduceArgs &d, int d_dtype, const VerifyCall &c, hipStream_t st)
{
    const RowReduceArgs t = target_pass_args(ctx, c);
    return timed(ctx, TAPOUT_PROFILE_STREAM_PAIR, [&](Timing tm) { return launch_row_reduce_pair(d, d_dtype, t, c.target->dtype, st, tm); });
}

// Accept decisions, first rejection, final token.
// tail (tapout_round): what the locate kernel needs to end each sequence's round, or NULL.
struct RoundTail { const int32_t *arm_in, *gamma; const uint8_t *active; const float *u_ts; int32_t *arm_out; uint32_t *flags; };

// fin (tapout_round): the draft epilogue has not run: the accept decisions take log q(tok) from the draft partials
// (fin_nsplit slices per draft row) and the epilogue runs in the locate kernel's launch.
hipError_t verify_rest(tapout_ctx *ctx, const VerifyCall &c, hipStream_t st, const RoundTail *tail = nullptr,
                       const DraftFinalArgs *fin = nullptr, int fin_nsplit = 0, int tail_kind = 1)
{
    VerifyArgs va{};
    if (fin) { va.vflags |= kVerifyOwnQ; va.d_nsplit = fin_nsplit; va.dpart = fin->part; }
    if (!ctx->exp_lookup) va.vflags |= kVerifyNoExpTable;
    if (tail) {
        va.bandit_tail = tail_kind;                 // 1: in the locate workgroups (UCB), 2: workgroups of their own (Thompson Sampling)
        va.bandit = bandit_args(ctx, c.B);
        va.b_arm_in = tail->arm_in; va.b_gamma = tail->gamma; va.b_active = tail->active; va.b_u_ts = tail->u_ts;
        va.b_arm_out = tail->arm_out; va.b_flags = tail->flags;
    }
    va.tbase = c.target->ptr; va.t_dtype = c.target->dtype; va.t_stride_b = c.target->stride_b; va.t_stride_k = c.target->stride_k;
    va.dbase = c.draft->ptr; va.d_dtype = c.draft->dtype; va.d_stride_b = c.draft->stride_b; va.d_stride_k = c.draft->stride_k;
    va.B = c.B; va.K = c.K; va.V = c.V; va.nsplit = c.nsplit; va.nsl = c.nsl;
    va.jps = 1; va.n_jobs = c.B; va.fused_head = c.fused ? 1 : 0;
    va.part = ctx->part_t;
    va.draft_lse = c.draft_lse; va.logq_tok = c.logq_tok; va.draft_tok = c.draft_tok; va.n_draft = c.n_draft; va.greedy = c.greedy;
    va.u_accept = c.u_accept; va.u_sample = c.u_sample;
    va.accept_len = c.accept_len; va.out_tok = c.out_tok; va.n_out = c.n_out;
    va.target_lse = c.target_lse; va.logp_tok = c.logp_tok; va.target_top1 = c.target_top1; va.flags = c.flags;
    va.flags_ws = ctx->flags_ws; va.jobs = ctx->jobs;
    va.part1 = ctx->part1; va.part2 = ctx->part2; va.exp_table = ctx->exp_table;
    hipError_t e = hipSuccess;
    for (int pass = c.fused ? 1 : 0; pass <= 2 && e == hipSuccess; ++pass)
        e = timed(ctx, TAPOUT_PROFILE_VERIFY_HEAD + pass, [&](Timing tm) { return launch_verify(va, pass, st, tm, fin); });
    return e;
}

}  // namespace

tapout_status tapout_verify(tapout_ctx *ctx, const tapout_logits *target, const tapout_logits *draft,
                            int32_t B, int32_t K, int32_t V,
                            const float *draft_lse, const float *logq_tok,
                            const int32_t *draft_tok, const int32_t *n_draft, const uint8_t *greedy,
                            const float *u_accept, const float *u_sample,
                            int32_t *accept_len, int32_t *out_tok, int32_t *n_out,
                            float *target_lse, float *logp_tok, int32_t *target_top1,
                            uint32_t *flags, void *stream)
{
    if (!ctx) return TAPOUT_EINVAL;
    VerifyCall c{target, draft, B, K, V, draft_lse, logq_tok, draft_tok, n_draft, greedy, u_accept, u_sample,
                 accept_len, out_tok, n_out, target_lse, logp_tok, target_top1, flags, 0, 0, false};
    tapout_status s = verify_check(ctx, c);
    if (s != TAPOUT_OK || B == 0) return s;
    DeviceGuard guard(ctx->cfg.device);
    hipStream_t st = (hipStream_t)stream;
    hipError_t e = verify_target_pass(ctx, c, st);
    if (e != hipSuccess) return hip_fail(ctx, e, "target pass launch");
    e = verify_rest(ctx, c, st);
    return e == hipSuccess ? TAPOUT_OK : hip_fail(ctx, e, "verify launch");
}

tapout_status tapout_round(tapout_ctx *ctx, const tapout_round_args *a, void *stream)
{
    if (!ctx) return TAPOUT_EINVAL;
    if (!a) return fail(ctx, TAPOUT_EINVAL, "args is NULL");
    if (!a->arm) return fail(ctx, TAPOUT_EINVAL, "arm is required");
    if (!a->lse || !a->logq_tok || !a->draft_tok) return fail(ctx, TAPOUT_EINVAL, "draft_tok, lse and logq_tok are required (verification reads them)");
    if (!a->n_draft && !a->n_stop) return fail(ctx, TAPOUT_EINVAL, "n_draft is NULL (verify up to the stop position) but n_stop is NULL too");
    if (!a->gamma) return fail(ctx, TAPOUT_EINVAL, "gamma is required");
    if ((ctx->cfg.policy == TAPOUT_TS_BETA || ctx->cfg.policy == TAPOUT_TS_GAUSS) && !a->u_ts_next) return fail(ctx, TAPOUT_EINVAL, "Thompson Sampling needs u_ts_next");
    const int32_t *n_draft = a->n_draft ? a->n_draft : a->n_stop;
    VerifyCall c{a->target, a->draft, a->B, a->K, a->V, a->lse, a->logq_tok, a->draft_tok, n_draft, a->greedy, a->u_accept, a->u_sample,
                 a->accept_len, a->out_tok, a->n_out, a->target_lse, a->logp_tok, a->target_top1, a->verify_flags, 0, 0, false};
    tapout_status s = verify_check(ctx, c);
    if (s != TAPOUT_OK || a->B == 0) return s;
    DeviceGuard guard(ctx->cfg.device);
    hipStream_t st = (hipStream_t)stream;
    // The target pass reads nothing the draft side writes unless n_draft is this round's stop position: then one launch
    // streams the draft rows and the target rows together, both cut into the same number of slices.
    // (Tensors of different element sizes too: slices go by the element, so both halves want the same number of them.
    // V = 256000, 512 sequences, bfloat16 draft and binary32 target rows: 1213 us against 388 + 828 us.)
    const bool pair = a->n_draft != nullptr && a->n_draft != a->n_stop && 2 * a->B <= 65535;
    if (pair) {
        // slices for the rows of both tensors together: half as many, twice as long, as either pass would take alone
        // (the slice count of the tensor with the larger elements: never more slices than the other would take)
        const int wide = (a->target->dtype == TAPOUT_F32 || a->draft->dtype == TAPOUT_F32) ? TAPOUT_F32 : TAPOUT_BF16;
        c.nsplit = choose_nsplit(ctx, (int64_t)a->B * (2 * a->K + 1), a->V, wide);
        if ((size_t)((int64_t)a->B * (a->K + 1) * c.nsplit) > ctx->part_cap) return fail(ctx, TAPOUT_EINVAL, "internal: partial buffer too small");
    }
    // With n_draft from the caller nothing of the verification waits for the draft epilogue's outputs if the accept
    // decisions form log q(tok) from the draft partials themselves (shapes whose partials one workgroup merges across
    // lanes; the stateful rules' epilogue hands entropies to the end of the round, so it keeps its place): then the
    // epilogue, a latency-bound kernel of B workgroups, runs beside the final-token locate kernel, another one, in
    // one launch.
    const int d_nsplit = pair ? c.nsplit : choose_nsplit(ctx, (int64_t)a->B * a->K, a->V, a->draft->dtype);
    const bool defer = a->n_draft != nullptr && a->n_draft != a->n_stop && !ctx->stateful && ctx->defer_epilogue &&
                       own_q_shape(a->K, c.nsplit, d_nsplit);
    DraftFinalArgs fin{};
    int fin_nsplit = 0;
    s = draft_stats_impl(ctx, a->draft, a->B, a->K, a->V, a->draft_tok, a->k_len, a->arm, nullptr,
                         a->lse, a->entropy, a->p_top1, a->p_top2, a->margin, a->top1_id, a->logq_tok, nullptr,
                         a->n_stop, a->stop_fired, a->draft_flags, stream, pair ? &c : nullptr, c.nsplit,
                         defer ? &fin : nullptr, &fin_nsplit);
    if (s != TAPOUT_OK) return s;
    hipError_t e = hipSuccess;
    if (!pair) {
        e = verify_target_pass(ctx, c, st);
        if (e != hipSuccess) return hip_fail(ctx, e, "target pass launch");
    }
    // Sequence-level UCB bandits, one per sequence: the final-token locate kernel, one workgroup per sequence, also
    // applies the reward and picks the next arm.  Gaussian Thompson Sampling, shared and token-level bandits take a
    // launch of their own.
    const bool own = ctx->positions == 1 && ctx->cfg.n_bandits != 1;
    const bool tail = own && (ctx->cfg.policy == TAPOUT_UCB1 || ctx->cfg.policy == TAPOUT_UCB_TUNED);
    // Thompson Sampling with Beta posteriors: the same launch carries the end of the round as workgroups of its own
    const bool ts_tail = own && ctx->cfg.policy == TAPOUT_TS_BETA && a->u_ts_next != nullptr;
    const RoundTail rt{a->arm, a->gamma, a->active, a->u_ts_next, a->arm, a->select_flags};
    e = verify_rest(ctx, c, st, (tail || ts_tail) ? &rt : nullptr, defer ? &fin : nullptr, fin_nsplit, ts_tail ? 2 : 1);
    if (e != hipSuccess) return hip_fail(ctx, e, "verify launch");
    if (tail || ts_tail) return TAPOUT_OK;
    return tapout_bandit_update_select(ctx, a->B, a->arm, a->accept_len, n_draft, a->gamma, a->active, a->u_ts_next, a->arm, a->select_flags, stream);
}

tapout_status tapout_profile_enable(tapout_ctx *ctx, uint32_t kind_mask, int32_t max_records)
{
    if (!ctx) return TAPOUT_EINVAL;
    if (max_records < 0 || max_records > (1 << 20)) return fail(ctx, TAPOUT_EINVAL, "max_records outside [0, 2^20]");
    if (kind_mask >> TAPOUT_PROFILE_KINDS) return fail(ctx, TAPOUT_EINVAL, "kind_mask names an unknown kernel");
    DeviceGuard guard(ctx->cfg.device);
    profile_release(ctx);
    if (!kind_mask || !max_records) return TAPOUT_OK;
    for (int k = 0; k < TAPOUT_PROFILE_KINDS; ++k) {
        if (!((kind_mask >> k) & 1u)) continue;
        for (int i = 0; i < max_records; ++i) {
            hipEvent_t a = nullptr, b = nullptr;
            if (hipEventCreate(&a) != hipSuccess || hipEventCreate(&b) != hipSuccess) {
                if (a) (void)hipEventDestroy(a);
                profile_release(ctx);
                return fail(ctx, TAPOUT_EHIP, "hipEventCreate failed");
            }
            ctx->prof_start[k].push_back(a); ctx->prof_stop[k].push_back(b);
        }
    }
    ctx->prof_mask = kind_mask; ctx->prof_cap = max_records;
    return TAPOUT_OK;
}

tapout_status tapout_profile_read(tapout_ctx *ctx, int32_t kind, double *total_ms, int32_t *launches, void *stream)
{
    if (!ctx) return TAPOUT_EINVAL;
    if (kind < 0 || kind >= TAPOUT_PROFILE_KINDS || !total_ms || !launches) return fail(ctx, TAPOUT_EINVAL, "bad kind or NULL output");
    DeviceGuard guard(ctx->cfg.device);
    hipError_t e = hipStreamSynchronize((hipStream_t)stream);
    if (e != hipSuccess) return hip_fail(ctx, e, "profile_read sync");
    double sum = 0.0;
    for (int i = 0; i < ctx->prof_used[kind]; ++i) {
        float ms = 0.0f;
        e = hipEventElapsedTime(&ms, ctx->prof_start[kind][i], ctx->prof_stop[kind][i]);
        if (e != hipSuccess) return hip_fail(ctx, e, "hipEventElapsedTime");
        sum += ms;
    }
    *total_ms = sum; *launches = ctx->prof_used[kind];
    ctx->prof_used[kind] = 0;
    ctx->prof_tick[kind] = 0;
    return TAPOUT_OK;
}

tapout_status tapout_bandit_get_state(tapout_ctx *ctx, double *sum_r, double *sum_r2, int64_t *count, void *stream)
{
    if (!ctx) return TAPOUT_EINVAL;
    if (!sum_r || !count) return fail(ctx, TAPOUT_EINVAL, "sum_r and count are required");
    DeviceGuard guard(ctx->cfg.device);
    const size_t n = (size_t)ctx->cfg.n_bandits * ctx->positions * ctx->cfg.n_arms;
    hipStream_t st = (hipStream_t)stream;
    hipError_t e = hipMemcpyAsync(sum_r, ctx->sum_r, n * sizeof(double), hipMemcpyDeviceToHost, st);
    if (e == hipSuccess && sum_r2) e = hipMemcpyAsync(sum_r2, ctx->sum_r2, n * sizeof(double), hipMemcpyDeviceToHost, st);
    if (e == hipSuccess) e = hipMemcpyAsync(count, ctx->count, n * sizeof(int64_t), hipMemcpyDeviceToHost, st);
    if (e == hipSuccess) e = hipStreamSynchronize(st);
    return e == hipSuccess ? TAPOUT_OK : hip_fail(ctx, e, "bandit_get_state");
}

tapout_status tapout_bandit_set_state(tapout_ctx *ctx, const double *sum_r, const double *sum_r2, const int64_t *count, void *stream)
{
    if (!ctx) return TAPOUT_EINVAL;
    if (!sum_r || !count) return fail(ctx, TAPOUT_EINVAL, "sum_r and count are required");
    const size_t n = (size_t)ctx->cfg.n_bandits * ctx->positions * ctx->cfg.n_arms;
    for (size_t i = 0; i < n; ++i) {
        if (count[i] < 0 || !(sum_r[i] >= 0.0) || sum_r[i] > (double)count[i])
            return fail(ctx, TAPOUT_EINVAL, "state entry %zu: need count >= 0 and 0 <= sum_r <= count", i);
        if (sum_r2 && (!(sum_r2[i] >= 0.0) || sum_r2[i] > (double)count[i]))
            return fail(ctx, TAPOUT_EINVAL, "state entry %zu: need 0 <= sum_r2 <= count", i);
    }
    std::vector<double> q;
    if (!sum_r2) {                                   // all plays of an arm taken to have had its mean reward
        q.resize(n);
        for (size_t i = 0; i < n; ++i) q[i] = count[i] > 0 ? sum_r[i] * sum_r[i] / (double)count[i] : 0.0;
        sum_r2 = q.data();
    }
    DeviceGuard guard(ctx->cfg.device);
    hipStream_t st = (hipStream_t)stream;
    hipError_t e = hipMemcpyAsync(ctx->sum_r, sum_r, n * sizeof(double), hipMemcpyHostToDevice, st);
    if (e == hipSuccess) e = hipMemcpyAsync(ctx->sum_r2, sum_r2, n * sizeof(double), hipMemcpyHostToDevice, st);
    if (e == hipSuccess) e = hipMemcpyAsync(ctx->count, count, n * sizeof(int64_t), hipMemcpyHostToDevice, st);
    if (e == hipSuccess) e = hipStreamSynchronize(st);
    return e == hipSuccess ? TAPOUT_OK : hip_fail(ctx, e, "bandit_set_state");
}

tapout_status tapout_rule_state_get(tapout_ctx *ctx, float *prev_entropy, double *accept_rate, double *lambda, void *stream)
{
    if (!ctx) return TAPOUT_EINVAL;
    if (!ctx->stateful) return fail(ctx, TAPOUT_EINVAL, "the configuration has no SVIP_DIFF or ADAEDL arm: no rule state");
    DeviceGuard guard(ctx->cfg.device);
    const size_t nb = (size_t)ctx->cfg.max_batch;
    hipStream_t st = (hipStream_t)stream;
    hipError_t e = hipSuccess;
    if (prev_entropy) e = hipMemcpyAsync(prev_entropy, ctx->prev_entropy, nb * sizeof(float), hipMemcpyDeviceToHost, st);
    if (e == hipSuccess && accept_rate) e = hipMemcpyAsync(accept_rate, ctx->accept_rate, nb * sizeof(double), hipMemcpyDeviceToHost, st);
    if (e == hipSuccess && lambda) e = hipMemcpyAsync(lambda, ctx->lambda, nb * ctx->cfg.n_arms * sizeof(double), hipMemcpyDeviceToHost, st);
    if (e == hipSuccess) e = hipStreamSynchronize(st);
    return e == hipSuccess ? TAPOUT_OK : hip_fail(ctx, e, "rule_state_get");
}

tapout_status tapout_rule_state_set(tapout_ctx *ctx, const float *prev_entropy, const double *accept_rate, const double *lambda, void *stream)
{
    if (!ctx) return TAPOUT_EINVAL;
    if (!ctx->stateful) return fail(ctx, TAPOUT_EINVAL, "the configuration has no SVIP_DIFF or ADAEDL arm: no rule state");
    const size_t nb = (size_t)ctx->cfg.max_batch;
    if (accept_rate)
        for (size_t i = 0; i < nb; ++i)
            if (!(accept_rate[i] == accept_rate[i])) return fail(ctx, TAPOUT_EINVAL, "accept_rate[%zu] is NaN", i);
    if (lambda)
        for (size_t i = 0; i < nb * ctx->cfg.n_arms; ++i)
            if (!(lambda[i] == lambda[i])) return fail(ctx, TAPOUT_EINVAL, "lambda[%zu] is NaN", i);
    DeviceGuard guard(ctx->cfg.device);
    hipStream_t st = (hipStream_t)stream;
    hipError_t e = hipSuccess;
    if (prev_entropy) e = hipMemcpyAsync(ctx->prev_entropy, prev_entropy, nb * sizeof(float), hipMemcpyHostToDevice, st);
    if (e == hipSuccess && accept_rate) e = hipMemcpyAsync(ctx->accept_rate, accept_rate, nb * sizeof(double), hipMemcpyHostToDevice, st);
    if (e == hipSuccess && lambda) e = hipMemcpyAsync(ctx->lambda, lambda, nb * ctx->cfg.n_arms * sizeof(double), hipMemcpyHostToDevice, st);
    if (e == hipSuccess) e = hipStreamSynchronize(st);
    return e == hipSuccess ? TAPOUT_OK : hip_fail(ctx, e, "rule_state_set");
}

}  // extern "C"
