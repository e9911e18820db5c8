// C-ABI entry points of libhadfl.so: argument validation, the host-side context, and the fixed launch
// sequence of one aggregation cycle.  Every step of the cycle itself runs in HIP kernels.
#include <cstdio>
#include <cstring>
#include <cmath>
#include <numeric>
#include <algorithm>
#include <new>

#include "kernels.h"
#include "train.h"

using namespace hadfl;

struct hadfl_ctx {
    hadfl_config cfg{};
    std::vector<hadfl_op> custom;
    NetPlan plan;
    hipStream_t stream = nullptr;
    int device = 0;
    // caller-owned device memory
    float* replicas = nullptr;
    char* scratch = nullptr;
    // carved out of scratch
    float* agg = nullptr;
    TrainBuffers tb;
    int32_t *steps_d = nullptr, *selected = nullptr, *sel_sorted = nullptr;
    float *sel_weight = nullptr, *weights = nullptr;
    double* f = nullptr;
    double* pred = nullptr;          // [3][N]: smoothing states s1, s2 and the forecast (Sec. 3.2)
    int32_t* bcast_d = nullptr;      // [N]: rows that receive a group's aggregate
    uint8_t *flag = nullptr, *avail_d = nullptr;
    // host state
    std::vector<int32_t> steps, order, bcast_h;
    int last_n_select = 0;           // size of the last selection (cfg.n_select, or a group's)
    // availability masks cross the boundary through two pinned slots used in turn; ev_slot[i] marks the end of the
    // copy out of slot i, so refilling a slot waits for that copy alone, not for the stream
    uint8_t* avail_pinned = nullptr;         // [2][N]
    hipEvent_t ev_slot[2] = {nullptr, nullptr};
    bool slot_used[2] = {false, false};
    int next_slot = 0;
    bool have_selection = false, have_agg = false, have_forecast = false;
    TrainEngine* engine = nullptr;
    Profiler prof;
    std::string err;
};

namespace {

thread_local std::string g_init_error;

struct Carver {
    size_t off = 0;
    template <typename T> size_t take(size_t count) {
        off = (off + 255) / 256 * 256;
        const size_t at = off;
        off += count * sizeof(T);
        return at;
    }
};

struct Carved {
    size_t agg, mom, grad, work, order, versions, cursor, loss, steps, selected, sel_sorted, sel_weight, weights, f,
        pred, bcast, flag, avail, total;
};

hadfl_status validate(const hadfl_config* cfg, std::string& err)
{
    if (!cfg) { err = "cfg is null"; return HADFL_EINVAL; }
    if (cfg->n_replicas < 1 || cfg->n_replicas > kMaxReplicas) { err = "n_replicas must be in [1, 1024]"; return HADFL_EINVAL; }
    if (cfg->n_select < 1 || cfg->n_select > cfg->n_replicas) { err = "n_select must be in [1, n_replicas]"; return HADFL_EINVAL; }
    if (cfg->weight_mode != 0 && cfg->weight_mode != 1) { err = "weight_mode must be 0 or 1"; return HADFL_EINVAL; }
    if (cfg->t_sync < 1 || cfg->steps_per_unit < 1) { err = "t_sync and steps_per_unit must be positive"; return HADFL_EINVAL; }
    if (cfg->net != HADFL_NET_NONE) {
        if (cfg->batch < 1 || cfg->n_samples < 1 || cfg->n_samples % cfg->batch != 0) {
            err = "n_samples must be a positive multiple of batch"; return HADFL_EINVAL;
        }
        if (cfg->batch > 1024) { err = "batch above 1024 is not supported"; return HADFL_EUNSUPPORTED; }
        if (!(cfg->lr > 0.f) || !(cfg->momentum >= 0.f) || !(cfg->momentum < 1.f)) {
            err = "lr must be positive and momentum in [0, 1)"; return HADFL_EINVAL;
        }
        if (cfg->n_classes < 2 || cfg->n_classes > 1024) { err = "n_classes must be in [2, 1024]"; return HADFL_EINVAL; }
    }
    return HADFL_OK;
}

Carved carve(const hadfl_config& cfg, const NetPlan& plan)
{
    Carver c;
    Carved o{};
    const size_t N = (size_t)cfg.n_replicas, rs = (size_t)plan.row_stride;
    const bool train = cfg.net != HADFL_NET_NONE;
    o.agg = c.take<float>(rs);
    o.mom = c.take<float>((train && cfg.momentum != 0.f) ? N * rs : 0);
    o.grad = c.take<float>(train ? N * rs : 0);
    o.work = c.take<float>(train ? (size_t)train_work_floats(cfg, plan) : 0);
    o.order = c.take<int32_t>(N);
    o.versions = c.take<int32_t>(N);
    o.cursor = c.take<int64_t>(N);
    o.loss = c.take<float>(N);
    o.steps = c.take<int32_t>(N);
    o.selected = c.take<int32_t>((size_t)cfg.n_select);
    o.sel_sorted = c.take<int32_t>((size_t)cfg.n_select);
    o.sel_weight = c.take<float>((size_t)cfg.n_select);
    o.weights = c.take<float>(N);
    o.f = c.take<double>(N);
    o.pred = c.take<double>(3 * N);
    o.bcast = c.take<int32_t>(N);
    o.flag = c.take<uint8_t>(N);
    o.avail = c.take<uint8_t>(N);
    o.total = (c.off + 255) / 256 * 256;
    return o;
}

hadfl_status fail(hadfl_ctx* ctx, hadfl_status st, const std::string& msg)
{
    if (ctx) ctx->err = msg; else g_init_error = msg;
    return st;
}

hadfl_status hip_fail(hadfl_ctx* ctx, hipError_t e, const char* what)
{
    return fail(ctx, HADFL_EDEVICE, std::string(what) + ": " + hipGetErrorString(e));
}

// Nothing may propagate out of a C entry point: a failed host allocation becomes HADFL_ENOMEM.
template <typename F> hadfl_status guard(hadfl_ctx* ctx, F&& body) noexcept
{
    try { return body(); }
    catch (const std::bad_alloc&) {
        try { return fail(ctx, HADFL_ENOMEM, "out of host memory"); } catch (...) { return HADFL_ENOMEM; }
    }
    catch (...) {
        try { return fail(ctx, HADFL_ENOMEM, "unexpected host exception"); } catch (...) { return HADFL_ENOMEM; }
    }
}

#define HIP_TRY(ctx, expr) do { hipError_t e_ = (expr); if (e_ != hipSuccess) return hip_fail((ctx), e_, #expr); } while (0)

// one replica's row <-> a dense host vector, segment by segment (the row pads every layer's slice to 256 bytes)
hadfl_status copy_row(hadfl_ctx* ctx, float* row, float* host, size_t n, bool to_device)
{
    for (const NetPlan::Seg& sg : ctx->plan.segs) {
        if ((size_t)sg.if_off >= n) break;
        const size_t cnt = std::min<size_t>((size_t)sg.count, n - (size_t)sg.if_off);
        if (to_device) HIP_TRY(ctx, hipMemcpyAsync(row + sg.row_off, host + sg.if_off, cnt * sizeof(float), hipMemcpyHostToDevice, ctx->stream));
        else HIP_TRY(ctx, hipMemcpyAsync(host + sg.if_off, row + sg.row_off, cnt * sizeof(float), hipMemcpyDeviceToHost, ctx->stream));
    }
    HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
    return HADFL_OK;
}

// E_k = t_sync * steps_per_unit * r_k / gcd(r)  (Sec. 2.3, Sec. 3.3)
hadfl_status step_counts(const int32_t* ratio, int n, int t_sync, int steps_per_unit, std::vector<int32_t>& steps, std::string& err)
{
    if (n < 1 || t_sync < 1 || steps_per_unit < 1) { err = "n, t_sync and steps_per_unit must be positive"; return HADFL_EINVAL; }
    int64_t g = 0;
    for (int k = 0; k < n; ++k) {
        if (ratio[k] <= 0) { err = "computing-power ratios must be positive"; return HADFL_EINVAL; }
        g = std::gcd<int64_t, int64_t>(g, ratio[k]);
    }
    steps.resize((size_t)n);
    for (int k = 0; k < n; ++k) {
        const int64_t e = (int64_t)t_sync * steps_per_unit * (ratio[k] / g);
        if (e > (1 << 20)) { err = "step count above 2^20"; return HADFL_EINVAL; }
        steps[k] = (int32_t)e;
    }
    return HADFL_OK;
}

hadfl_status momentum_args(hadfl_ctx* ctx, int32_t replica, const void* p, size_t n)
{
    if (!ctx || !p) return fail(ctx, HADFL_EINVAL, "null argument");
    if (!ctx->engine || !ctx->tb.mom) return fail(ctx, HADFL_ESTATE, "this context keeps no momentum buffers");
    if (replica < 0 || replica >= ctx->cfg.n_replicas) return fail(ctx, HADFL_EINVAL, "replica out of range");
    if (n > (size_t)ctx->plan.m_train) return fail(ctx, HADFL_EINVAL, "n exceeds m_train");
    return HADFL_OK;
}

}  // namespace

// ---------------------------------------------------------------------------------------------------------
namespace hadfl {

hipEvent_t Profiler::get()
{
    if (!pool.empty()) { hipEvent_t e = pool.back(); pool.pop_back(); return e; }
    hipEvent_t e = nullptr;
    if (hipEventCreate(&e) != hipSuccess) return nullptr;
    return e;
}
void Profiler::begin(const char* name, hipStream_t s, double flops, double bytes)
{
    if (!on) return;
    Rec r{name, get(), get(), flops, bytes};
    if (r.a) (void)hipEventRecord(r.a, s);
    recs.push_back(r);
}
void Profiler::end(hipStream_t s)
{
    if (!on || recs.empty()) return;
    if (recs.back().b) (void)hipEventRecord(recs.back().b, s);
}
void Profiler::clear()
{
    for (Rec& r : recs) { if (r.a) pool.push_back(r.a); if (r.b) pool.push_back(r.b); }
    recs.clear();
}
Profiler::~Profiler()
{
    clear();
    for (hipEvent_t e : pool) (void)hipEventDestroy(e);
}

}  // namespace hadfl

// ---------------------------------------------------------------------------------------------------------
extern "C" {

hadfl_status hadfl_param_count(const hadfl_config* cfg, int64_t* m_train, int64_t* m_total, int64_t* row_stride)
{
    return guard(nullptr, [&]() -> hadfl_status {
    std::string err;
    hadfl_status st = validate(cfg, err);
    if (st != HADFL_OK) return fail(nullptr, st, err);
    NetPlan plan;
    st = build_plan(*cfg, plan, err);
    if (st != HADFL_OK) return fail(nullptr, st, err);
    if (m_train) *m_train = plan.m_train;
    if (m_total) *m_total = plan.m_total;
    if (row_stride) *row_stride = plan.row_stride;
    return HADFL_OK;
    });
}

hadfl_status hadfl_param_layout(const hadfl_config* cfg, hadfl_tensor_info* out, int32_t cap, int32_t* n)
{
    return guard(nullptr, [&]() -> hadfl_status {
    std::string err;
    hadfl_status st = validate(cfg, err);
    if (st != HADFL_OK) return fail(nullptr, st, err);
    NetPlan plan;
    st = build_plan(*cfg, plan, err);
    if (st != HADFL_OK) return fail(nullptr, st, err);
    if (!n) return fail(nullptr, HADFL_EINVAL, "n is null");
    std::vector<hadfl_tensor_info> rows;
    if (cfg->net == HADFL_NET_NONE) {
        rows.push_back({0, plan.m_total, 0, 1});
    } else {
        for (const Layer& l : plan.layers) {
            const TensorShape a = plan.tensors[l.in0];
            if (l.type == HADFL_OP_CONV || l.type == HADFL_OP_DENSE) {
                const int64_t fan = l.type == HADFL_OP_CONV ? (int64_t)l.k * l.k * a.c : a.numel();
                rows.push_back({l.if_w_off, l.w_count, 0, (int32_t)fan});
                if (l.bias) rows.push_back({l.if_b_off, l.cout, 1, (int32_t)fan});
            } else if (l.type == HADFL_OP_BN) {
                rows.push_back({l.if_w_off, a.c, 2, a.c});
                rows.push_back({l.if_b_off, a.c, 3, a.c});
            }
        }
        for (const Layer& l : plan.layers)
            if (l.type == HADFL_OP_BN) {
                const int c = plan.tensors[l.in0].c;
                rows.push_back({l.if_stat_off, c, 4, c});
                rows.push_back({l.if_stat_off + c, c, 5, c});
            }
    }
    if (out) for (int32_t i = 0; i < cap && i < (int32_t)rows.size(); ++i) out[i] = rows[i];
    *n = (int32_t)rows.size();
    return HADFL_OK;
    });
}

hadfl_status hadfl_workspace_bytes(const hadfl_config* cfg, size_t* params_bytes, size_t* scratch_bytes)
{
    return guard(nullptr, [&]() -> hadfl_status {
    std::string err;
    hadfl_status st = validate(cfg, err);
    if (st != HADFL_OK) return fail(nullptr, st, err);
    NetPlan plan;
    st = build_plan(*cfg, plan, err);
    if (st != HADFL_OK) return fail(nullptr, st, err);
    if (params_bytes) *params_bytes = (size_t)cfg->n_replicas * (size_t)plan.row_stride * sizeof(float);
    if (scratch_bytes) *scratch_bytes = carve(*cfg, plan).total;
    return HADFL_OK;
    });
}

hadfl_status hadfl_init_replicas(const hadfl_config* cfg, const void* w0_dev, void* replicas_dev, void* scratch_dev,
                                 const void* x_dev, const int32_t* y_dev, const int32_t* ratio_host, void* stream,
                                 hadfl_ctx** out)
{
    return guard(nullptr, [&]() -> hadfl_status {
    std::string err;
    hadfl_status st = validate(cfg, err);
    if (st != HADFL_OK) return fail(nullptr, st, err);
    if (!out) return fail(nullptr, HADFL_EINVAL, "out is null");
    if (!replicas_dev || !scratch_dev) return fail(nullptr, HADFL_EINVAL, "replicas_dev and scratch_dev must not be null");
    if (((uintptr_t)replicas_dev | (uintptr_t)scratch_dev) & 255) return fail(nullptr, HADFL_EINVAL, "replicas_dev and scratch_dev must be 256-byte aligned");
    if (w0_dev && ((uintptr_t)w0_dev & 3)) return fail(nullptr, HADFL_EINVAL, "w0_dev must be 4-byte aligned");
    const bool train = cfg->net != HADFL_NET_NONE;
    if (train && (!x_dev || !y_dev)) return fail(nullptr, HADFL_EINVAL, "x_dev and y_dev are required for a trainable network");
    if (train && !w0_dev) return fail(nullptr, HADFL_EINVAL, "w0_dev is required for a trainable network");
    if (train && ((uintptr_t)x_dev & 15)) return fail(nullptr, HADFL_EINVAL, "x_dev must be 16-byte aligned");
    if (!ratio_host) return fail(nullptr, HADFL_EINVAL, "ratio_host is null");

    hadfl_ctx* ctx = new (std::nothrow) hadfl_ctx();
    if (!ctx) return fail(nullptr, HADFL_ENOMEM, "out of host memory");
    struct Holder { hadfl_ctx* p; ~Holder() { if (p) hadfl_destroy(p); } } holder{ctx};   // freed on every early return
    ctx->cfg = *cfg;
    if (cfg->net == HADFL_NET_CUSTOM && cfg->custom_ops && cfg->n_custom_ops > 0) {
        ctx->custom.assign(cfg->custom_ops, cfg->custom_ops + cfg->n_custom_ops);
        ctx->cfg.custom_ops = ctx->custom.data();
    }
    auto bail = [&](hadfl_status s, const std::string& m) { return fail(nullptr, s, m); };
    st = build_plan(ctx->cfg, ctx->plan, err);
    if (st != HADFL_OK) return bail(st, err);

    const int N = cfg->n_replicas;
    st = step_counts(ratio_host, N, cfg->t_sync, cfg->steps_per_unit, ctx->steps, err);
    if (st != HADFL_OK) return bail(st, err);
    ctx->order.resize(N);
    std::iota(ctx->order.begin(), ctx->order.end(), 0);
    std::stable_sort(ctx->order.begin(), ctx->order.end(), [&](int a, int b) { return ctx->steps[a] > ctx->steps[b]; });

    ctx->stream = (hipStream_t)stream;
    if (hipGetDevice(&ctx->device) != hipSuccess) return bail(HADFL_EDEVICE, "no HIP device");
    ctx->replicas = (float*)replicas_dev;
    ctx->scratch = (char*)scratch_dev;
    const Carved c = carve(ctx->cfg, ctx->plan);
    char* b = ctx->scratch;
    ctx->agg = (float*)(b + c.agg);
    ctx->tb.replicas = ctx->replicas;
    ctx->tb.mom = (train && cfg->momentum != 0.f) ? (float*)(b + c.mom) : nullptr;
    ctx->tb.grad = train ? (float*)(b + c.grad) : nullptr;
    ctx->tb.work = train ? (float*)(b + c.work) : nullptr;
    ctx->tb.x = (const float*)x_dev; ctx->tb.y = y_dev;
    ctx->tb.order = (int32_t*)(b + c.order);
    ctx->tb.versions = (int32_t*)(b + c.versions);
    ctx->tb.cursor = (long long*)(b + c.cursor);
    ctx->tb.loss = (float*)(b + c.loss);
    ctx->steps_d = (int32_t*)(b + c.steps);
    ctx->selected = (int32_t*)(b + c.selected);
    ctx->sel_sorted = (int32_t*)(b + c.sel_sorted);
    ctx->sel_weight = (float*)(b + c.sel_weight);
    ctx->weights = (float*)(b + c.weights);
    ctx->f = (double*)(b + c.f);
    ctx->pred = (double*)(b + c.pred);
    ctx->bcast_d = (int32_t*)(b + c.bcast);
    ctx->flag = (uint8_t*)(b + c.flag);
    ctx->avail_d = (uint8_t*)(b + c.avail);

    hipStream_t s = ctx->stream;
    auto dev = [&](hipError_t e, const char* what) -> bool {
        if (e == hipSuccess) return true;
        err = std::string(what) + ": " + hipGetErrorString(e);
        return false;
    };
    if (!dev(hipHostMalloc((void**)&ctx->avail_pinned, 2 * (size_t)N, hipHostMallocDefault), "hipHostMalloc")) return bail(HADFL_EDEVICE, err);
    for (int i = 0; i < 2; ++i)
        if (!dev(hipEventCreateWithFlags(&ctx->ev_slot[i], hipEventDisableTiming), "hipEventCreate")) return bail(HADFL_EDEVICE, err);
    // small state: everything after the work area starts at zero (versions, cursors, flags, losses)
    {
        const size_t small_bytes = c.total - c.order;
        if (!dev(launch_fill_u32((uint32_t*)(b + c.order), 0u, (int64_t)(small_bytes / 4), s), "fill")) return bail(HADFL_EDEVICE, err);
    }
    if (!dev(hipMemcpyAsync(ctx->steps_d, ctx->steps.data(), sizeof(int32_t) * N, hipMemcpyHostToDevice, s), "copy steps")) return bail(HADFL_EDEVICE, err);
    if (!dev(hipMemcpyAsync(ctx->tb.order, ctx->order.data(), sizeof(int32_t) * N, hipMemcpyHostToDevice, s), "copy order")) return bail(HADFL_EDEVICE, err);
    if (!dev(hipStreamSynchronize(s), "synchronize")) return bail(HADFL_EDEVICE, err);   // host vectors may move after this

    // Algorithm 1, first line: w_k <- w0 for every replica (padding of each row stays zero)
    if (w0_dev) {
        const int64_t rs = ctx->plan.row_stride;
        if (!dev(launch_fill_u32((uint32_t*)ctx->replicas, 0u, (int64_t)N * rs, s), "zero rows")) return bail(HADFL_EDEVICE, err);
        for (const NetPlan::Seg& sg : ctx->plan.segs)
            if (!dev(launch_bcast_rows((const float*)w0_dev + sg.if_off, ctx->replicas + sg.row_off, rs, sg.count, N, s), "broadcast w0"))
                return bail(HADFL_EDEVICE, err);
    }
    if (ctx->tb.mom && !dev(launch_fill_u32((uint32_t*)ctx->tb.mom, 0u, (int64_t)N * ctx->plan.row_stride, s), "zero momentum"))
        return bail(HADFL_EDEVICE, err);
    if (ctx->tb.grad && !dev(launch_fill_u32((uint32_t*)ctx->tb.grad, 0u, (int64_t)N * ctx->plan.row_stride, s), "zero gradients"))
        return bail(HADFL_EDEVICE, err);
    if (train) {
        st = train_create(ctx->cfg, ctx->plan, ctx->tb, ctx->steps, ctx->order, &ctx->engine, err);
        if (st != HADFL_OK) return bail(st, err);
    }
    holder.p = nullptr;
    *out = ctx;
    return HADFL_OK;
    });
}

hadfl_status hadfl_local_steps(hadfl_ctx* ctx)
{
    return guard(ctx, [&]() -> hadfl_status {
    if (!ctx) return fail(nullptr, HADFL_EINVAL, "ctx is null");
    if (!ctx->engine) return fail(ctx, HADFL_ESTATE, "this context has no trainable network");
    std::string err;
    hadfl_status st = train_run(ctx->engine, ctx->stream, &ctx->prof, err);
    if (st != HADFL_OK) return fail(ctx, st, err);
    return HADFL_OK;
    });
}

static hadfl_status select_common(hadfl_ctx* ctx, const int32_t* versions_i32, const double* versions_f64,
                                  const uint8_t* avail_host, uint64_t cycle, int n_select)
{
    const int N = ctx->cfg.n_replicas;
    const uint8_t* avail_d = nullptr;
    if (avail_host) {
        int na = 0;
        for (int k = 0; k < N; ++k) na += avail_host[k] ? 1 : 0;
        if (na < n_select) return fail(ctx, HADFL_EINVAL, "fewer available replicas than n_select");
        // two pinned staging slots used in turn: before refilling one, wait for the copy that last read it
        const int slot = ctx->next_slot;
        ctx->next_slot ^= 1;
        if (ctx->slot_used[slot]) HIP_TRY(ctx, hipEventSynchronize(ctx->ev_slot[slot]));
        uint8_t* stage = ctx->avail_pinned + (size_t)slot * N;
        for (int k = 0; k < N; ++k) stage[k] = avail_host[k] ? 1 : 0;
        // the device copy of the mask is read by the selection kernel of this call and rewritten by the next call's copy,
        // both on the context's stream, in order
        HIP_TRY(ctx, hipMemcpyAsync(ctx->avail_d, stage, (size_t)N, hipMemcpyHostToDevice, ctx->stream));
        HIP_TRY(ctx, hipEventRecord(ctx->ev_slot[slot], ctx->stream));
        ctx->slot_used[slot] = true;
        avail_d = ctx->avail_d;
    }
    SelectArgs a{};
    a.versions = versions_i32;
    a.versions_f64 = versions_f64;
    a.avail = avail_d;
    a.n = N; a.n_select = n_select; a.weight_mode = ctx->cfg.weight_mode;
    a.seed = ctx->cfg.seed; a.cycle = cycle;
    a.selected = ctx->selected; a.sel_sorted = ctx->sel_sorted; a.sel_weight = ctx->sel_weight;
    a.flag = ctx->flag; a.weights = ctx->weights; a.f = ctx->f;
    ctx->prof.begin("select", ctx->stream, 0.0, 13.0 * N);
    hipError_t e = launch_select(a, ctx->stream);
    ctx->prof.end(ctx->stream);
    if (e != hipSuccess) return hip_fail(ctx, e, "select kernel");
    ctx->have_selection = true;
    ctx->last_n_select = n_select;
    return HADFL_OK;
}

hadfl_status hadfl_select(hadfl_ctx* ctx, const int32_t* versions_dev, const uint8_t* avail_host, uint64_t cycle)
{
    return guard(ctx, [&]() -> hadfl_status {
    if (!ctx) return fail(nullptr, HADFL_EINVAL, "ctx is null");
    return select_common(ctx, versions_dev ? versions_dev : ctx->tb.versions, nullptr, avail_host, cycle, ctx->cfg.n_select);
    });
}

hadfl_status hadfl_select_static(const int32_t* versions_dev, const uint8_t* avail_dev, int32_t n_replicas, int32_t n_select,
                                 int32_t weight_mode, uint64_t seed, uint64_t cycle, int32_t* selected_dev, uint8_t* flag_dev,
                                 float* weights_dev, void* stream)
{
    return guard(nullptr, [&]() -> hadfl_status {
    if (!versions_dev || !selected_dev || !flag_dev || !weights_dev) return fail(nullptr, HADFL_EINVAL, "null argument");
    if (((uintptr_t)versions_dev | (uintptr_t)selected_dev | (uintptr_t)weights_dev) & 3)
        return fail(nullptr, HADFL_EINVAL, "versions_dev, selected_dev and weights_dev must be 4-byte aligned");
    if (n_replicas < 1 || n_replicas > kMaxReplicas)
        return fail(nullptr, HADFL_EINVAL, "n_replicas must be in [1, 1024]: the static working memory holds 1024 replicas");
    if (n_select < 1 || n_select > n_replicas) return fail(nullptr, HADFL_EINVAL, "n_select must be in [1, n_replicas]");
    if (weight_mode != 0 && weight_mode != 1) return fail(nullptr, HADFL_EINVAL, "weight_mode must be 0 or 1");
    SelectArgs a{};
    a.versions = versions_dev; a.avail = avail_dev;
    a.n = n_replicas; a.n_select = n_select; a.weight_mode = weight_mode; a.seed = seed; a.cycle = cycle;
    a.selected = selected_dev; a.flag = flag_dev; a.weights = weights_dev;
    const hipError_t e = launch_select_static(a, (hipStream_t)stream);
    if (e != hipSuccess) return hip_fail(nullptr, e, "static selection");
    return HADFL_OK;
    });
}

hadfl_status hadfl_select_real(hadfl_ctx* ctx, const double* versions_dev, const uint8_t* avail_host, uint64_t cycle)
{
    return guard(ctx, [&]() -> hadfl_status {
    if (!ctx) return fail(nullptr, HADFL_EINVAL, "ctx is null");
    if (!versions_dev && !ctx->have_forecast)
        return fail(ctx, HADFL_ESTATE, "hadfl_select_real without versions needs a preceding hadfl_predict_versions");
    if (versions_dev && ((uintptr_t)versions_dev & 7)) return fail(ctx, HADFL_EINVAL, "versions_dev must be 8-byte aligned");
    return select_common(ctx, nullptr, versions_dev ? versions_dev : ctx->pred + 2 * (size_t)ctx->cfg.n_replicas, avail_host, cycle,
                         ctx->cfg.n_select);
    });
}

hadfl_status hadfl_predict_versions(hadfl_ctx* ctx, const int32_t* versions_dev, double alpha, int32_t horizon)
{
    return guard(ctx, [&]() -> hadfl_status {
    if (!ctx) return fail(nullptr, HADFL_EINVAL, "ctx is null");
    if (!(alpha > 0.0) || !(alpha < 1.0)) return fail(ctx, HADFL_EINVAL, "alpha must be in (0, 1)");
    if (horizon < 0 || horizon > (1 << 20)) return fail(ctx, HADFL_EINVAL, "horizon must be in [0, 2^20]");
    const size_t N = (size_t)ctx->cfg.n_replicas;
    const hipError_t e = launch_predict(versions_dev ? versions_dev : ctx->tb.versions, ctx->pred, ctx->pred + N, ctx->pred + 2 * N,
                                        (int)N, alpha, horizon, ctx->have_forecast ? 0 : 1, ctx->stream);
    if (e != hipSuccess) return hip_fail(ctx, e, "predict kernel");
    ctx->have_forecast = true;
    return HADFL_OK;
    });
}

hadfl_status hadfl_get_predicted(hadfl_ctx* ctx, double* predicted)
{
    return guard(ctx, [&]() -> hadfl_status {
    if (!ctx || !predicted) return fail(ctx, HADFL_EINVAL, "null argument");
    if (!ctx->have_forecast) return fail(ctx, HADFL_ESTATE, "no forecast yet");
    const size_t N = (size_t)ctx->cfg.n_replicas;
    HIP_TRY(ctx, hipMemcpyAsync(predicted, ctx->pred + 2 * N, sizeof(double) * N, hipMemcpyDeviceToHost, ctx->stream));
    HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
    return HADFL_OK;
    });
}

hadfl_status hadfl_step_counts(const int32_t* ratio_host, int32_t n, int32_t t_sync, int32_t steps_per_unit, int32_t* steps_host)
{
    return guard(nullptr, [&]() -> hadfl_status {
    if (!ratio_host || !steps_host) return fail(nullptr, HADFL_EINVAL, "null argument");
    std::vector<int32_t> st;
    std::string err;
    const hadfl_status rc = step_counts(ratio_host, n, t_sync, steps_per_unit, st, err);
    if (rc != HADFL_OK) return fail(nullptr, rc, err);
    for (int32_t k = 0; k < n; ++k) steps_host[k] = st[k];
    return HADFL_OK;
    });
}

hadfl_status hadfl_steps_from_times(const double* times_host, int32_t n, int32_t e_warmup, double quantum, int32_t t_sync,
                                    int32_t steps_per_unit, int32_t* steps_host)
{
    return guard(nullptr, [&]() -> hadfl_status {
    if (!times_host || !steps_host) return fail(nullptr, HADFL_EINVAL, "null argument");
    if (n < 1 || e_warmup < 1 || t_sync < 1 || steps_per_unit < 1 || !(quantum > 0.0))
        return fail(nullptr, HADFL_EINVAL, "n, e_warmup, quantum, t_sync and steps_per_unit must be positive");
    const int64_t cap = 1 << 20;
    std::vector<int64_t> q((size_t)n);
    int64_t H = 1;
    for (int32_t k = 0; k < n; ++k) {
        if (!(times_host[k] > 0.0)) return fail(nullptr, HADFL_EINVAL, "calculation times must be positive");
        const double units = std::nearbyint(times_host[k] / (double)e_warmup / quantum);
        if (!(units < (double)cap)) return fail(nullptr, HADFL_EINVAL, "quantum too fine for these times");
        q[k] = units < 1.0 ? 1 : (int64_t)units;
        H = H / std::gcd<int64_t, int64_t>(H, q[k]) * q[k];
        if (H > cap * cap) return fail(nullptr, HADFL_EINVAL, "quantum too fine for these times");
    }
    std::vector<int32_t> st((size_t)n);
    for (int32_t k = 0; k < n; ++k) {
        const int64_t e = (int64_t)t_sync * steps_per_unit * (H / q[k]);
        if (e > cap) return fail(nullptr, HADFL_EINVAL, "step count above 2^20: quantum too fine for these times");
        st[k] = (int32_t)e;
    }
    for (int32_t k = 0; k < n; ++k) steps_host[k] = st[k];
    return HADFL_OK;
    });
}

hadfl_status hadfl_set_lr(hadfl_ctx* ctx, float lr)
{
    return guard(ctx, [&]() -> hadfl_status {
    if (!ctx) return fail(nullptr, HADFL_EINVAL, "ctx is null");
    if (!ctx->engine) return fail(ctx, HADFL_ESTATE, "this context has no trainable network");
    if (!(lr > 0.f)) return fail(ctx, HADFL_EINVAL, "lr must be positive");
    ctx->cfg.lr = lr;
    train_set_lr(ctx->engine, lr);
    return HADFL_OK;
    });
}

hadfl_status hadfl_set_steps(hadfl_ctx* ctx, const int32_t* steps_host)
{
    return guard(ctx, [&]() -> hadfl_status {
    if (!ctx || !steps_host) return fail(ctx, HADFL_EINVAL, "null argument");
    const int N = ctx->cfg.n_replicas;
    for (int k = 0; k < N; ++k)
        if (steps_host[k] < 0 || steps_host[k] > (1 << 20)) return fail(ctx, HADFL_EINVAL, "step counts must be in [0, 2^20]");
    // the copies below read host vectors that are about to change: let earlier copies out of them finish
    HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
    ctx->steps.assign(steps_host, steps_host + N);
    std::iota(ctx->order.begin(), ctx->order.end(), 0);
    std::stable_sort(ctx->order.begin(), ctx->order.end(), [&](int a, int b) { return ctx->steps[a] > ctx->steps[b]; });
    HIP_TRY(ctx, hipMemcpyAsync(ctx->steps_d, ctx->steps.data(), sizeof(int32_t) * N, hipMemcpyHostToDevice, ctx->stream));
    HIP_TRY(ctx, hipMemcpyAsync(ctx->tb.order, ctx->order.data(), sizeof(int32_t) * N, hipMemcpyHostToDevice, ctx->stream));
    HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
    if (ctx->engine) train_set_steps(ctx->engine, ctx->steps);
    return HADFL_OK;
    });
}

hadfl_status hadfl_aggregate(hadfl_ctx* ctx, int32_t resync)
{
    return guard(ctx, [&]() -> hadfl_status {
    if (!ctx) return fail(nullptr, HADFL_EINVAL, "ctx is null");
    if (!ctx->have_selection) return fail(ctx, HADFL_ESTATE, "hadfl_aggregate needs a preceding hadfl_select");
    // algorithmic traffic: n_select rows read, the aggregate written (+ every replica row written when broadcasting)
    const double agg_bytes = 4.0 * (double)ctx->plan.m_total * (ctx->last_n_select + 1 + (resync ? ctx->cfg.n_replicas : 0));
    ctx->prof.begin(resync ? "aggregate_bcast" : "aggregate", ctx->stream, 0.0, agg_bytes);
    hipError_t e = launch_aggregate(ctx->replicas, ctx->plan.row_stride, ctx->plan.row_stride, ctx->sel_sorted,
                                    ctx->sel_weight, ctx->last_n_select, ctx->agg, resync ? ctx->cfg.n_replicas : 0,
                                    ctx->replicas, nullptr, ctx->stream);
    ctx->prof.end(ctx->stream);
    if (e != hipSuccess) return hip_fail(ctx, e, "aggregate kernel");
    ctx->have_agg = true;
    return HADFL_OK;
    });
}

hadfl_status hadfl_select_group(hadfl_ctx* ctx, const int32_t* versions_dev, const uint8_t* member_host, int32_t n_select,
                                uint64_t cycle)
{
    return guard(ctx, [&]() -> hadfl_status {
    if (!ctx || !member_host) return fail(ctx, HADFL_EINVAL, "null argument");
    if (n_select < 1 || n_select > ctx->cfg.n_select) return fail(ctx, HADFL_EINVAL, "n_select must be in [1, cfg.n_select]");
    return select_common(ctx, versions_dev ? versions_dev : ctx->tb.versions, nullptr, member_host, cycle, n_select);
    });
}

hadfl_status hadfl_aggregate_group(hadfl_ctx* ctx, const uint8_t* member_host)
{
    return guard(ctx, [&]() -> hadfl_status {
    if (!ctx || !member_host) return fail(ctx, HADFL_EINVAL, "null argument");
    if (!ctx->have_selection) return fail(ctx, HADFL_ESTATE, "hadfl_aggregate_group needs a preceding selection");
    const int N = ctx->cfg.n_replicas;
    // the list below is copied from a host vector that is about to change: let an earlier copy out of it finish
    HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
    ctx->bcast_h.clear();
    for (int k = 0; k < N; ++k) if (member_host[k]) ctx->bcast_h.push_back(k);
    const int nb = (int)ctx->bcast_h.size();
    if (nb > 0)
        HIP_TRY(ctx, hipMemcpyAsync(ctx->bcast_d, ctx->bcast_h.data(), sizeof(int32_t) * nb, hipMemcpyHostToDevice, ctx->stream));
    const double agg_bytes = 4.0 * (double)ctx->plan.m_total * (ctx->last_n_select + 1 + nb);
    ctx->prof.begin("aggregate_group", ctx->stream, 0.0, agg_bytes);
    hipError_t e = launch_aggregate(ctx->replicas, ctx->plan.row_stride, ctx->plan.row_stride, ctx->sel_sorted,
                                    ctx->sel_weight, ctx->last_n_select, ctx->agg, nb, ctx->replicas, ctx->bcast_d, ctx->stream);
    ctx->prof.end(ctx->stream);
    if (e != hipSuccess) return hip_fail(ctx, e, "aggregate kernel");
    ctx->have_agg = true;
    return HADFL_OK;
    });
}

hadfl_status hadfl_get_steps(hadfl_ctx* ctx, int32_t* steps)
{
    return guard(ctx, [&]() -> hadfl_status {
    if (!ctx || !steps) return fail(ctx, HADFL_EINVAL, "null argument");
    HIP_TRY(ctx, hipMemcpyAsync(steps, ctx->steps_d, sizeof(int32_t) * ctx->cfg.n_replicas, hipMemcpyDeviceToHost, ctx->stream));
    HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
    return HADFL_OK;
    });
}

hadfl_status hadfl_get_versions(hadfl_ctx* ctx, int32_t* versions, int64_t* cursors)
{
    return guard(ctx, [&]() -> hadfl_status {
    if (!ctx || !versions) return fail(ctx, HADFL_EINVAL, "null argument");
    const size_t N = (size_t)ctx->cfg.n_replicas;
    HIP_TRY(ctx, hipMemcpyAsync(versions, ctx->tb.versions, sizeof(int32_t) * N, hipMemcpyDeviceToHost, ctx->stream));
    if (cursors) HIP_TRY(ctx, hipMemcpyAsync(cursors, ctx->tb.cursor, sizeof(int64_t) * N, hipMemcpyDeviceToHost, ctx->stream));
    HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
    return HADFL_OK;
    });
}

hadfl_status hadfl_get_selected(hadfl_ctx* ctx, int32_t* selected, int32_t* count, uint8_t* flag, float* weights)
{
    return guard(ctx, [&]() -> hadfl_status {
    if (!ctx || !selected) return fail(ctx, HADFL_EINVAL, "null argument");
    if (!ctx->have_selection) return fail(ctx, HADFL_ESTATE, "no selection yet");
    const size_t N = (size_t)ctx->cfg.n_replicas;
    HIP_TRY(ctx, hipMemcpyAsync(selected, ctx->selected, sizeof(int32_t) * ctx->last_n_select, hipMemcpyDeviceToHost, ctx->stream));
    if (count) *count = ctx->last_n_select;
    if (flag) HIP_TRY(ctx, hipMemcpyAsync(flag, ctx->flag, N, hipMemcpyDeviceToHost, ctx->stream));
    if (weights) HIP_TRY(ctx, hipMemcpyAsync(weights, ctx->weights, sizeof(float) * N, hipMemcpyDeviceToHost, ctx->stream));
    HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
    return HADFL_OK;
    });
}

hadfl_status hadfl_get_params(hadfl_ctx* ctx, int32_t replica, float* out, size_t n)
{
    return guard(ctx, [&]() -> hadfl_status {
    if (!ctx || !out) return fail(ctx, HADFL_EINVAL, "null argument");
    if (replica < -1 || replica >= ctx->cfg.n_replicas) return fail(ctx, HADFL_EINVAL, "replica out of range");
    if (n > (size_t)ctx->plan.m_total) return fail(ctx, HADFL_EINVAL, "n exceeds m_total");
    if (replica == -1 && !ctx->have_agg) return fail(ctx, HADFL_ESTATE, "no aggregate yet");
    float* row = replica < 0 ? ctx->agg : ctx->replicas + (size_t)replica * ctx->plan.row_stride;
    return copy_row(ctx, row, out, n, false);
    });
}

hadfl_status hadfl_set_params(hadfl_ctx* ctx, int32_t replica, const float* in, size_t n)
{
    return guard(ctx, [&]() -> hadfl_status {
    if (!ctx || !in) return fail(ctx, HADFL_EINVAL, "null argument");
    if (replica < 0 || replica >= ctx->cfg.n_replicas) return fail(ctx, HADFL_EINVAL, "replica out of range");
    if (n > (size_t)ctx->plan.m_total) return fail(ctx, HADFL_EINVAL, "n exceeds m_total");
    return copy_row(ctx, ctx->replicas + (size_t)replica * ctx->plan.row_stride, const_cast<float*>(in), n, true);
    });
}

hadfl_status hadfl_get_momentum(hadfl_ctx* ctx, int32_t replica, float* out, size_t n)
{
    return guard(ctx, [&]() -> hadfl_status {
    const hadfl_status st = momentum_args(ctx, replica, out, n);
    if (st != HADFL_OK) return st;
    return copy_row(ctx, ctx->tb.mom + (size_t)replica * ctx->plan.row_stride, out, n, false);
    });
}

hadfl_status hadfl_set_momentum(hadfl_ctx* ctx, int32_t replica, const float* in, size_t n)
{
    return guard(ctx, [&]() -> hadfl_status {
    const hadfl_status st = momentum_args(ctx, replica, in, n);
    if (st != HADFL_OK) return st;
    return copy_row(ctx, ctx->tb.mom + (size_t)replica * ctx->plan.row_stride, const_cast<float*>(in), n, true);
    });
}

hadfl_status hadfl_set_option(hadfl_ctx* ctx, int32_t option, int32_t value)
{
    return guard(ctx, [&]() -> hadfl_status {
    if (!ctx) return fail(nullptr, HADFL_EINVAL, "ctx is null");
    if (!ctx->engine) return fail(ctx, HADFL_ESTATE, "this context has no trainable network");
    switch (option) {
    case HADFL_OPT_SIDE_STREAM:
        if (value != 0 && value != 1) return fail(ctx, HADFL_EINVAL, "HADFL_OPT_SIDE_STREAM takes 0 or 1");
        train_set_side_stream(ctx->engine, value != 0);
        return HADFL_OK;
    case HADFL_OPT_TILE_HINT:
        if (value < 0 || value > 2) return fail(ctx, HADFL_EINVAL, "HADFL_OPT_TILE_HINT takes 0, 1 or 2");
        train_set_tile_hint(ctx->engine, value);
        return HADFL_OK;
    default:
        return fail(ctx, HADFL_EINVAL, "unknown option");
    }
    });
}

hadfl_status hadfl_get_losses(hadfl_ctx* ctx, float* loss)
{
    return guard(ctx, [&]() -> hadfl_status {
    if (!ctx || !loss) return fail(ctx, HADFL_EINVAL, "null argument");
    HIP_TRY(ctx, hipMemcpyAsync(loss, ctx->tb.loss, sizeof(float) * ctx->cfg.n_replicas, hipMemcpyDeviceToHost, ctx->stream));
    HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
    return HADFL_OK;
    });
}

hadfl_status hadfl_profile_enable(hadfl_ctx* ctx, int32_t on)
{
    return guard(ctx, [&]() -> hadfl_status {
    if (!ctx) return fail(nullptr, HADFL_EINVAL, "ctx is null");
    HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
    ctx->prof.clear();
    ctx->prof.on = on != 0;
    ctx->prof.detail = on == 2;
    return HADFL_OK;
    });
}

hadfl_status hadfl_profile_read(hadfl_ctx* ctx, hadfl_kernel_time* out, int32_t cap, int32_t* n)
{
    return guard(ctx, [&]() -> hadfl_status {
    if (!ctx || !n) return fail(ctx, HADFL_EINVAL, "null argument");
    HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
    std::vector<hadfl_kernel_time> rows;
    for (const Profiler::Rec& r : ctx->prof.recs) {
        float ms = 0.f;
        if (!r.a || !r.b || hipEventElapsedTime(&ms, r.a, r.b) != hipSuccess) continue;
        size_t i = 0;
        for (; i < rows.size(); ++i) if (r.name == rows[i].name) break;
        if (i == rows.size()) {
            hadfl_kernel_time t{};
            std::snprintf(t.name, sizeof(t.name), "%s", r.name.c_str());
            rows.push_back(t);
        }
        rows[i].launches += 1;
        rows[i].total_ms += ms;
        rows[i].flops += r.flops;
        rows[i].bytes += r.bytes;
    }
    if (out) for (int32_t i = 0; i < cap && i < (int32_t)rows.size(); ++i) out[i] = rows[i];
    *n = (int32_t)rows.size();
    ctx->prof.clear();
    return HADFL_OK;
    });
}

const char* hadfl_last_error(const hadfl_ctx* ctx) { return ctx ? ctx->err.c_str() : g_init_error.c_str(); }

void hadfl_destroy(hadfl_ctx* ctx)
{
    if (!ctx) return;
    (void)hipStreamSynchronize(ctx->stream);          // a null handle is the default stream
    if (ctx->engine) train_destroy(ctx->engine);
    if (ctx->avail_pinned) (void)hipHostFree(ctx->avail_pinned);
    for (hipEvent_t ev : ctx->ev_slot) if (ev) (void)hipEventDestroy(ev);
    delete ctx;
}

}  // extern "C"
