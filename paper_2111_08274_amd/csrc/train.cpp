// Host-side schedule of hadfl_local_steps: a fixed launch sequence per sub-step s = 1..E_max, each launch grouped
// over the replicas that still have steps left (a prefix of the replicas ordered by step count, kept in device
// memory).  There is no host loop over replicas and no host read-back inside a cycle.
#include <algorithm>
#include <cstdio>

#include "train.h"
#include "kernels.h"
#include "train_kernels.h"

namespace hadfl {

class TrainEngine {
public:
    hadfl_config cfg;
    NetPlan plan;
    TrainBuffers buf;
    std::vector<int32_t> steps;
    int e_max = 0;
    std::vector<int> n_active;            // n_active[s] = replicas with E_k > s
    // per-tensor activation / gradient offsets (floats) inside one replica's block of `work`
    std::vector<int64_t> act_off, grad_off;
    int64_t rep_block = 0;                // floats of activations + gradients per replica
    std::vector<int64_t> saved_off;       // per layer (BN): offset of saved mean/istd inside the replica block
    int64_t shared_off = 0;               // start of the region shared by all layers (split-K partials, BN partials)
    int64_t shared_floats = 0;
    int64_t bn_off = 0;                   // per-chunk partial sums of the batch-norm reductions (their own region: weight
                                          // gradients may run beside them on the side stream)
    std::vector<int> splits;              // per layer: split-K factor of the weight gradient
    std::vector<int> bn_chunks;           // per layer
    std::vector<char> grad_written;       // scratch for the backward pass
    // ReLU fusion: a ReLU that is the only consumer of a conv / dense / BN / add output is folded into that layer's
    // store (the layer writes the ReLU's output tensor; the ReLU layer itself issues nothing).  Its backward is folded
    // into whoever writes the gradient of that tensor: those kernels zero the gradient where the stored output is not
    // positive, so the tensor's gradient buffer holds the gradient before the ReLU.
    std::vector<int> out_tensor;          // per layer: tensor the layer writes (its own, or the fused ReLU's)
    std::vector<char> skip;               // per layer: fused away
    std::vector<char> fused_relu;         // per layer: applies max(., 0) in its store
    std::vector<char> masked;             // per tensor: gradient writers must apply the (value > 0) mask
    // Pool fusion: a 2x2 max-pool that is the only consumer of a batch-norm layer's (ReLU'd) output is folded into the
    // BN kernels: forward writes the pooled tensor as well, backward forms the full-resolution gradient on the fly from
    // the pooled gradient.  The pool layer itself issues nothing.
    std::vector<int> pool_of;             // per layer: index of the folded pool layer, or -1
    // Statistics fusion (bf16 configuration): a lean convolution whose output feeds a batch norm only leaves the per-channel
    // sums of its output in the BN partial region, and that BN's forward skips its own sums pass.
    std::vector<int> stat_for;            // per layer: the BN layer fed by this convolution's statistics, or -1
    std::vector<int> stat_from;           // per layer (BN): the convolution that supplies them, or -1
    std::vector<int> stat_rows;           // per layer (BN): rows per statistics entry of the latest forward launch
    // The same in the backward pass (bf16 configuration): a lean convolution that is the only consumer of a batch norm's
    // output (after its fused ReLU and folded pool) leaves, from its data-gradient epilogue, the per-channel sums that
    // batch norm's backward pass needs, and the BN skips its own sums pass.
    std::vector<int> bstat_for;           // per layer (conv): the BN layer its data gradient serves, or -1
    std::vector<int> bstat_rows;          // per layer (BN): rows per entry of the latest data-gradient launch (0: none)
    std::vector<int64_t> bstat_rep;       // per layer (BN): floats per replica slot of those entries
    // bf16 configuration: regular convolution layers keep two bf16 weight matrices (forward / data-gradient order)
    std::vector<char> fast;               // per layer: the lean bf16 kernels apply
    std::vector<char> fast32;             // per layer (fp32 configuration): lean fp32 forward / data-gradient kernels apply
    std::vector<int64_t> wf_off, wb_off;  // per layer: offsets (bf16 elements) inside one replica's bf16 weight block
    int64_t wbf_rep = 0;                  // bf16 elements per replica
    int64_t wbf_off = 0;                  // start of the bf16 weight region inside `work` (floats)
    // Option HADFL_OPT_TILE_HINT: 1 makes the lean kernels take their 256 x 256 tiles wherever the layer shape allows,
    // whatever the launch size (lets small problems exercise them); 2 keeps wide-image layers on the general kernels.
    int tile_hint = 0;
    // Weight gradients (and their split-K reduction / fused update) depend only on dY and the stored activations, not on
    // the data-gradient chain, so they run on a second stream beside it; joined before the update kernel.
    // Option HADFL_OPT_SIDE_STREAM = 0 turns this off.
    hipStream_t side = nullptr;
    hipEvent_t ev_fork = nullptr, ev_join = nullptr;
    bool use_side = true;
    // Layers whose weight-gradient kernel applies the update itself (lean kernel, no split): their slices of the
    // parameter rows, ascending; the update kernel runs over the segments in between.
    std::vector<char> fused_update;       // per layer
    std::vector<char> prepped;            // per layer: bf16 copies for the coming sub-step are already written
    std::vector<std::pair<int64_t, int64_t>> update_segments;   // [first, first + count) floats
    // Position tables of the regular convolution layers (see FastConvParams::perm): per layer HW sorted positions
    // followed by HW tap masks, all layers back to back in `tables`; copied to `work` at tab_off by the first run.
    std::vector<int64_t> tab_idx;         // per layer: start inside `tables`, or -1
    std::vector<int32_t> tables;
    int64_t tab_off = 0;                  // start of the table region inside `work` (floats)
    bool tables_uploaded = false;
};

namespace {

int ilog2_exact(int v) { int s = 0; while ((1 << s) < v) ++s; return (1 << s) == v ? s : -1; }

struct Layout {
    std::vector<int64_t> act_off, grad_off, saved_off;
    std::vector<int> splits, bn_chunks;
    int64_t rep_block = 0, shared_floats = 0, bn_floats = 0;
    std::vector<char> fast, fast32;
    std::vector<int64_t> wf_off, wb_off;       // in 2-byte units inside one replica's block of weight copies
    int64_t wbf_rep = 0;
    std::vector<int64_t> tab_idx;
    int64_t tab_ints = 0;
};

bool is_pow2(int v) { return v > 0 && (v & (v - 1)) == 0; }

int64_t up64(int64_t v) { return (v + 63) / 64 * 64; }

// Measured on 32 replicas of the VGG-16 shape: forward and data gradient gain up to 8 x 8 images, the weight gradient up
// to 4 x 4; beyond that the scattered rows of a position-major tile cost more than the skipped taps save.
constexpr int kMaxTablePositions = 64, kMaxTablePositionsWgrad = 16;

Layout make_layout(const hadfl_config& cfg, const NetPlan& plan)
{
    Layout L;
    const int T = (int)plan.tensors.size();
    const int64_t B = cfg.batch;
    L.act_off.assign(T, -1); L.grad_off.assign(T, -1);
    int64_t off = 0;
    for (int t = 1; t < T; ++t) { L.act_off[t] = off; off += up64(B * plan.tensors[t].numel()); }
    for (int t = 1; t < T; ++t) { L.grad_off[t] = off; off += up64(B * plan.tensors[t].numel()); }
    L.saved_off.assign(plan.layers.size(), -1);
    L.splits.assign(plan.layers.size(), 1);
    L.bn_chunks.assign(plan.layers.size(), 1);
    int64_t shared = 0, bn_shared = 0;
    for (size_t i = 0; i < plan.layers.size(); ++i) {
        const Layer& l = plan.layers[i];
        const TensorShape a = plan.tensors[l.in0], r = plan.tensors[l.out];
        if (l.type == HADFL_OP_BN) {
            L.saved_off[i] = off; off += up64(2 * (int64_t)a.c);
            const int64_t rows = B * a.h * a.w;
            int chunks = (int)std::min<int64_t>(128, std::max<int64_t>(1, rows / 128));
            L.bn_chunks[i] = chunks;
            bn_shared = std::max<int64_t>(bn_shared, (int64_t)cfg.n_replicas * chunks * 2 * a.c);
        } else if (l.type == HADFL_OP_CONV || l.type == HADFL_OP_DENSE) {
            // weight gradient: contraction over K = B*Ho*Wo rows; split it until the launch has enough workgroups
            const int64_t K = B * r.h * r.w;
            const int64_t M = (l.type == HADFL_OP_CONV ? (int64_t)l.k * l.k * a.c : a.numel()) + (l.bias ? 1 : 0);
            const int64_t tiles = ((M + 127) / 128) * ((l.cout + 127) / 128);
            int64_t want = (2048 + tiles * cfg.n_replicas - 1) / (tiles * cfg.n_replicas);
            int64_t maxs = std::max<int64_t>(1, K / 128);
            int s = (int)std::max<int64_t>(1, std::min<int64_t>(std::min<int64_t>(want, maxs), 256));
            L.splits[i] = s;
            if (s > 1) shared = std::max<int64_t>(shared, (int64_t)cfg.n_replicas * s * up64(M * l.cout));
        }
    }
    L.rep_block = up64(off);
    L.shared_floats = up64(shared);
    L.fast.assign(plan.layers.size(), 0); L.fast32.assign(plan.layers.size(), 0);
    L.wf_off.assign(plan.layers.size(), -1); L.wb_off.assign(plan.layers.size(), -1);
    if (cfg.bf16) {
        int64_t woff = 0;
        for (size_t i = 0; i < plan.layers.size(); ++i) {
            const Layer& l = plan.layers[i];
            if (l.type != HADFL_OP_CONV || l.in0 == 0) continue;
            const TensorShape a = plan.tensors[l.in0];
            if (l.stride != 1 || 2 * l.pad != l.k - 1 || l.k * l.k > 32) continue;
            if (a.c % 64 != 0 || l.cout % 64 != 0 || !is_pow2(a.h) || !is_pow2(a.w)) continue;
            L.fast[i] = 1;
            L.wf_off[i] = woff; woff += up64(l.w_count);
            L.wb_off[i] = woff; woff += up64(l.w_count);
        }
        L.wbf_rep = woff;
    }
    if (!cfg.bf16) {
        // fp32 configuration: forward and data gradient of the regular layers run in the lean fp32 kernels, which read
        // K-contiguous fp32 copies of the weights (two floats = four 2-byte units per weight and copy pair)
        int64_t woff = 0;
        for (size_t i = 0; i < plan.layers.size(); ++i) {
            const Layer& l = plan.layers[i];
            if (l.type != HADFL_OP_CONV || l.in0 == 0) continue;
            const TensorShape a = plan.tensors[l.in0];
            if (l.stride != 1 || 2 * l.pad != l.k - 1 || l.k * l.k > 32) continue;
            if (a.c % 64 != 0 || l.cout % 64 != 0) continue;      // the data gradient swaps the two channel counts
            L.fast32[i] = 1;
            L.wf_off[i] = woff; woff += up64(2 * l.w_count);
            L.wb_off[i] = woff; woff += up64(2 * l.w_count);
        }
        L.wbf_rep = woff;
    }
    // a lean convolution in front of a batch norm leaves one statistics entry per 128 output rows (at most)
    for (size_t k = 0; k < plan.layers.size(); ++k) {
        const Layer& l = plan.layers[k];
        if (l.type != HADFL_OP_BN || l.in0 < 1 || (!L.fast[l.in0 - 1] && !L.fast32[l.in0 - 1])) continue;
        const TensorShape a = plan.tensors[l.in0];
        bn_shared = std::max<int64_t>(bn_shared, (int64_t)cfg.n_replicas * ((B * a.h * a.w + 127) / 128) * 2 * a.c);
    }
    L.bn_floats = up64(bn_shared);
    // position tables: worth it for small images (many border pixels), and the weight gradient needs slabs of 32
    // contraction indices to hold a single position
    L.tab_idx.assign(plan.layers.size(), -1);
    for (size_t i = 0; i < plan.layers.size(); ++i) {
        if ((!L.fast[i] && !L.fast32[i]) || cfg.batch % 32 != 0) continue;
        const TensorShape a = plan.tensors[plan.layers[i].in0];
        if (a.h * a.w > kMaxTablePositions) continue;
        L.tab_idx[i] = L.tab_ints; L.tab_ints += 2 * (int64_t)a.h * a.w;
    }
    return L;
}

}  // namespace

int64_t train_work_floats(const hadfl_config& cfg, const NetPlan& plan)
{
    if (cfg.net == HADFL_NET_NONE) return 0;
    const Layout L = make_layout(cfg, plan);
    return L.rep_block * cfg.n_replicas + L.shared_floats + L.bn_floats + up64(L.wbf_rep * cfg.n_replicas / 2 + 64) + up64(L.tab_ints);
}

hadfl_status train_create(const hadfl_config& cfg, const NetPlan& plan, const TrainBuffers& buf,
                          const std::vector<int32_t>& steps, const std::vector<int32_t>& order,
                          TrainEngine** out, std::string& err)
{
    (void)order;
    TrainEngine* e = new TrainEngine();
    e->cfg = cfg; e->plan = plan; e->buf = buf; e->steps = steps;
    e->e_max = *std::max_element(steps.begin(), steps.end());
    e->n_active.assign(e->e_max, 0);
    for (int s = 0; s < e->e_max; ++s)
        for (int32_t v : steps) e->n_active[s] += v > s ? 1 : 0;
    const Layout L = make_layout(cfg, plan);
    e->act_off = L.act_off; e->grad_off = L.grad_off; e->saved_off = L.saved_off;
    e->splits = L.splits; e->bn_chunks = L.bn_chunks;
    e->rep_block = L.rep_block;
    e->shared_off = L.rep_block * cfg.n_replicas;
    e->shared_floats = L.shared_floats;
    e->fast = L.fast; e->fast32 = L.fast32; e->wf_off = L.wf_off; e->wb_off = L.wb_off; e->wbf_rep = L.wbf_rep;
    e->bn_off = e->shared_off + L.shared_floats;
    e->wbf_off = e->bn_off + L.bn_floats;
    {
        e->fused_update.assign(plan.layers.size(), 0);
        int64_t pos = 0;
        for (size_t i = 0; i < plan.layers.size(); ++i) {
            const Layer& l = plan.layers[i];
            if (l.type != HADFL_OP_CONV && l.type != HADFL_OP_DENSE) continue;
            // in the weight-gradient epilogue (lean kernels, K not split), or in the split-K reduction of a layer whose
            // fp32 weights nothing reads between its weight gradient and the update: the lean layers' data gradients
            // read the bf16 (fp32 configuration: fp32) copies, a layer on the data set has no data gradient
            const bool in_epilogue = e->fast[i] && e->splits[i] == 1;
            const bool in_reduce = e->splits[i] > 1 && (e->fast[i] || e->fast32[i] || l.in0 == 0);
            if (!in_epilogue && !in_reduce) continue;
            const int64_t cnt = l.w_count + (l.bias ? l.cout : 0);      // bias sits directly behind the weights
            if (l.w_off % 4 != 0 || cnt % 4 != 0 || l.w_off < pos || (l.bias && l.b_off != l.w_off + l.w_count)) continue;
            e->fused_update[i] = 1;
            if (l.w_off > pos) e->update_segments.push_back({pos, l.w_off - pos});
            pos = l.w_off + cnt;
        }
        if (plan.train_end > pos) e->update_segments.push_back({pos, plan.train_end - pos});
    }
    e->tab_off = e->wbf_off + up64(L.wbf_rep * cfg.n_replicas / 2 + 64);
    e->tab_idx = L.tab_idx;
    e->tables.assign((size_t)L.tab_ints, 0);
    for (size_t i = 0; i < plan.layers.size(); ++i) {
        if (L.tab_idx[i] < 0) continue;
        const Layer& l = plan.layers[i];
        const TensorShape a = plan.tensors[l.in0];
        const int hw = a.h * a.w;
        std::vector<uint32_t> mask(hw, 0);
        for (int pos = 0; pos < hw; ++pos)
            for (int t = 0; t < l.k * l.k; ++t) {
                const int yy = pos / a.w + t / l.k - l.pad, xx = pos % a.w + t % l.k - l.pad;
                if (yy >= 0 && yy < a.h && xx >= 0 && xx < a.w) mask[pos] |= 1u << t;
            }
        std::vector<int32_t> perm(hw);
        for (int pos = 0; pos < hw; ++pos) perm[pos] = pos;
        std::stable_sort(perm.begin(), perm.end(), [&](int x, int y) { return mask[x] < mask[y]; });
        for (int ps = 0; ps < hw; ++ps) {
            e->tables[L.tab_idx[i] + ps] = perm[ps];
            e->tables[L.tab_idx[i] + hw + ps] = (int32_t)mask[perm[ps]];
        }
    }
    {
        const int nl = (int)plan.layers.size(), T = (int)plan.tensors.size();
        e->out_tensor.resize(nl); e->skip.assign(nl, 0); e->fused_relu.assign(nl, 0); e->masked.assign(T, 0);
        std::vector<int> consumers(T, 0);
        for (const Layer& l : plan.layers) { consumers[l.in0]++; if (l.type == HADFL_OP_ADD) consumers[l.in1]++; }
        for (int i = 0; i < nl; ++i) e->out_tensor[i] = plan.layers[i].out;
        for (int j = 0; j < nl; ++j) {
            const Layer& r = plan.layers[j];
            if (r.type != HADFL_OP_RELU || r.in0 < 1 || consumers[r.in0] != 1 || r.out == T - 1) continue;
            const int i = r.in0 - 1;                       // layer i writes tensor i + 1
            const int pt = plan.layers[i].type;
            if (pt != HADFL_OP_CONV && pt != HADFL_OP_DENSE && pt != HADFL_OP_BN && pt != HADFL_OP_ADD) continue;
            e->out_tensor[i] = r.out; e->fused_relu[i] = 1; e->skip[j] = 1; e->masked[r.out] = 1;
        }
        e->stat_for.assign(nl, -1); e->stat_from.assign(nl, -1); e->stat_rows.assign(nl, 0);
        for (int k = 0; k < nl; ++k) {
            const Layer& b = plan.layers[k];
            if (b.type != HADFL_OP_BN || b.in0 < 1 || consumers[b.in0] != 1) continue;
            const int i = b.in0 - 1;                        // layer i writes tensor i + 1
            if ((!e->fast[i] && !e->fast32[i]) || plan.layers[i].type != HADFL_OP_CONV || e->out_tensor[i] != b.in0) continue;
            e->stat_for[i] = k; e->stat_from[k] = i;
        }
        e->pool_of.assign(nl, -1);
        const int vec = cfg.bf16 ? 8 : 4;
        for (int j = 0; j < nl; ++j) {
            const Layer& q = plan.layers[j];
            if (q.type != HADFL_OP_MAXPOOL || q.in0 < 1 || consumers[q.in0] != 1) continue;
            int i = -1;                                    // the BN layer that writes the pool's input
            for (int k = 0; k < nl; ++k)
                if (!e->skip[k] && e->out_tensor[k] == q.in0 && plan.layers[k].type == HADFL_OP_BN) i = k;
            if (i < 0) continue;
            const TensorShape t = plan.tensors[q.in0];
            if (t.c % vec != 0 || t.h % 2 != 0 || t.w % 2 != 0) continue;
            e->pool_of[i] = j; e->skip[j] = 1;
        }
        e->bstat_for.assign(nl, -1); e->bstat_rows.assign(nl, 0); e->bstat_rep.assign(nl, 0);
        if (cfg.bf16)
            for (int k = 0; k < nl; ++k) {
                if (plan.layers[k].type != HADFL_OP_BN || e->skip[k]) continue;
                // the tensor the rest of the net sees as this BN's output
                const int t_out = e->pool_of[k] >= 0 ? plan.layers[e->pool_of[k]].out : e->out_tensor[k];
                if (consumers[t_out] != 1) continue;
                for (int j = 0; j < nl; ++j)
                    if (plan.layers[j].type == HADFL_OP_CONV && plan.layers[j].in0 == t_out && e->fast[j]) e->bstat_for[j] = k;
            }
    }
    *out = e;
    return HADFL_OK;
}

void train_set_steps(TrainEngine* e, const std::vector<int32_t>& steps)
{
    e->steps = steps;
    e->e_max = steps.empty() ? 0 : *std::max_element(steps.begin(), steps.end());
    e->n_active.assign(e->e_max, 0);
    for (int s = 0; s < e->e_max; ++s)
        for (int32_t v : steps) e->n_active[s] += v > s ? 1 : 0;
}

void train_set_lr(TrainEngine* e, float lr) { e->cfg.lr = lr; }

void train_set_side_stream(TrainEngine* e, bool on) { e->use_side = on; }
void train_set_tile_hint(TrainEngine* e, int hint) { e->tile_hint = hint; }
bool train_has_momentum(const TrainEngine* e) { return e->buf.mom != nullptr; }

void train_destroy(TrainEngine* e)
{
    if (!e) return;
    if (e->side) { (void)hipStreamSynchronize(e->side); (void)hipStreamDestroy(e->side); }
    if (e->ev_fork) (void)hipEventDestroy(e->ev_fork);
    if (e->ev_join) (void)hipEventDestroy(e->ev_join);
    delete e;
}

namespace {

struct Runner {
    TrainEngine& e;
    hipStream_t s;
    Profiler* prof;
    int na = 0;
    int cur_layer = -1;
    hipError_t rc = hipSuccess;
    const char* failed = nullptr;

    const float* act(int t) const { return t == 0 ? e.buf.x : e.buf.work + e.act_off[t]; }
    float* actw(int t) const { return e.buf.work + e.act_off[t]; }
    float* grad(int t) const { return e.buf.work + e.grad_off[t]; }
    hipStream_t main_stream = nullptr;
    bool forked = false;                  // a flag, not the handle: the caller's stream may be the null stream
    // the launches that follow go to the side stream, ordered after everything enqueued on the main stream so far
    void fork()
    {
        if (!e.use_side || !e.side || rc != hipSuccess) return;
        rc = hipEventRecord(e.ev_fork, s);
        if (rc == hipSuccess) rc = hipStreamWaitEvent(e.side, e.ev_fork, 0);
        if (rc != hipSuccess) { failed = "fork"; return; }
        main_stream = s; s = e.side; forked = true;
    }
    void unfork() { if (forked) { s = main_stream; forked = false; } }
    // the main stream waits for everything enqueued on the side stream
    void join()
    {
        if (!e.use_side || !e.side || rc != hipSuccess) return;
        rc = hipEventRecord(e.ev_join, e.side);
        if (rc == hipSuccess) rc = hipStreamWaitEvent(s, e.ev_join, 0);
        if (rc != hipSuccess) failed = "join";
    }
    float* shared() const { return e.buf.work + e.shared_off; }
    float* bn_shared() const { return e.buf.work + e.bn_off; }
    __bf16* wbf() const { return reinterpret_cast<__bf16*>(e.buf.work + e.wbf_off); }
    const int* perm(size_t i) const { return e.tab_idx[i] < 0 ? nullptr : reinterpret_cast<const int*>(e.buf.work + e.tab_off) + e.tab_idx[i]; }
    const unsigned* posmask(size_t i) const
    {
        const TensorShape a = e.plan.tensors[e.plan.layers[i].in0];
        return e.tab_idx[i] < 0 ? nullptr : reinterpret_cast<const unsigned*>(e.buf.work + e.tab_off) + e.tab_idx[i] + a.h * a.w;
    }

    // K-contiguous copies of layer i's filters for the lean kernels (forward layout and flipped/transposed for the data
    // gradient; bf16, or fp32 in the fp32 configuration), refreshed from the fp32 master for the first n replicas in step
    // order
    void prep_layer(size_t i, int n)
    {
        const int keep_na = na, keep_layer = cur_layer;
        na = n; cur_layer = (int)i;
        const Layer& l = e.plan.layers[i];
        if (e.fast32[i]) {                                   // fp32 configuration: K-contiguous fp32 copies
            WeightPrepF32Params w{};
            w.w = e.buf.replicas + l.w_off; w.w_rep = e.plan.row_stride;
            w.wf = wcopy32(e.wf_off[i]); w.wb = wcopy32(e.wb_off[i]); w.wcopy_rep = e.wbf_rep / 2;
            w.C = e.plan.tensors[l.in0].c; w.N = l.cout; w.taps = l.k * l.k; w.order = e.buf.order;
            run("weight_prep", 0, 12.0 * l.w_count, [&] { return launch_weight_prep_f32(w, na, s); });
        } else {
            WeightPrepParams w{};
            w.w = e.buf.replicas + l.w_off; w.w_rep = e.plan.row_stride;
            w.wf = wbf() + e.wf_off[i]; w.wb = wbf() + e.wb_off[i]; w.wbf_rep = e.wbf_rep;
            w.C = e.plan.tensors[l.in0].c; w.N = l.cout; w.taps = l.k * l.k; w.order = e.buf.order;
            run("weight_prep", 0, 8.0 * l.w_count, [&] { return launch_weight_prep(w, na, s); });
        }
        na = keep_na; cur_layer = keep_layer;
    }
    float* wcopy32(int64_t off) const { return reinterpret_cast<float*>(wbf() + off); }
    void prepare_weights()
    {
        for (size_t i = 0; i < e.plan.layers.size(); ++i) {
            if (!e.fast[i] && !e.fast32[i]) continue;
            if (e.prepped[i]) { e.prepped[i] = 0; continue; }      // written during the previous sub-step's backward pass
            prep_layer(i, na);
        }
    }
    // A layer whose update is fused into its weight-gradient kernel has its final weights of this sub-step as soon as
    // that kernel ends, so the copies for the next sub-step are written right behind it on the same stream, off the
    // forward pass's critical path.  Not before this sub-step's data gradient of the layer has read the old copy:
    // the copy of layer i is therefore issued after the next fork, which follows that data gradient on the main stream.
    int na_next = 0;
    int pending_prep = -1;
    void flush_pending_prep()
    {
        if (pending_prep < 0) return;
        prep_layer((size_t)pending_prep, na_next);
        e.prepped[pending_prep] = 1;
        pending_prep = -1;
    }

    // flops / bytes: algorithmic work of the launch for all active replicas (reported by the profiler)
    template <typename F> void run(const char* name, double flops, double bytes, F&& f)
    {
        if (rc != hipSuccess) return;
        if (prof) {
            if (prof->detail) {
                char tag[64];
                std::snprintf(tag, sizeof(tag), "%s:L%d:n%d", name, cur_layer, na);
                prof->begin(tag, s, flops * na, bytes * na);
            } else {
                prof->begin(name, s, flops * na, bytes * na);
            }
        }
        rc = f();
        if (prof) prof->end(s);
        if (rc != hipSuccess) failed = name;
    }

    hipError_t gemm(const GemmParams& p) const { return e.cfg.bf16 ? launch_gemm_bf16(p, na, s) : launch_gemm(p, na, s); }
    static double gemm_flops(const GemmParams& p) { return 2.0 * p.B * p.Ho * p.Wo * p.R * p.S * (double)p.Cin * p.Cout; }
    // activations are 2 bytes in the bf16 configuration, weights and their gradients 4
    double asz() const { return e.cfg.bf16 ? 0.5 : 1.0; }
    double gemm_bytes(const GemmParams& p) const
    {
        return 4.0 * (asz() * ((double)p.B * p.H * p.W * p.Cin + (double)p.B * p.Ho * p.Wo * p.Cout) + (double)p.R * p.S * p.Cin * p.Cout);
    }

    GemmParams gemm_base(const Layer& l) const
    {
        const TensorShape a = e.plan.tensors[l.in0], r = e.plan.tensors[l.out];
        GemmParams p{};
        p.B = e.cfg.batch;
        if (l.type == HADFL_OP_CONV) {
            p.H = a.h; p.W = a.w; p.Cin = a.c; p.Ho = r.h; p.Wo = r.w; p.Cout = l.cout;
            p.R = p.S = l.k; p.stride = l.stride; p.pad = l.pad;
        } else {
            p.H = p.W = p.Ho = p.Wo = 1; p.Cin = (int)a.numel(); p.Cout = l.cout;
            p.R = p.S = 1; p.stride = 1; p.pad = 0;
        }
        p.splits = 1; p.kchunk = 1 << 30;
        p.hw_shift = ilog2_exact(p.Ho * p.Wo); p.w_shift = ilog2_exact(p.Wo);
        if (p.hw_shift < 0 || p.w_shift < 0) p.hw_shift = p.w_shift = -1;
        p.w = e.buf.replicas + l.w_off; p.w_rep = e.plan.row_stride;
        p.has_bias = l.bias;
        p.order = e.buf.order;
        p.n_samples = e.cfg.n_samples; p.batch = e.cfg.batch; p.sample_sz = e.plan.tensors[0].numel();
        return p;
    }

    void forward_layer(size_t i)
    {
        cur_layer = (int)i;
        if (e.skip[i]) return;
        const Layer& l = e.plan.layers[i];
        const TensorShape a = e.plan.tensors[l.in0], r = e.plan.tensors[l.out];
        const int64_t B = e.cfg.batch;
        const int ot = e.out_tensor[i];
        EwParams q{};
        q.order = e.buf.order; q.B = (int)B; q.H = a.h; q.W = a.w; q.C = a.c; q.bf16 = e.cfg.bf16;
        q.in = act(l.in0); q.in_rep = e.rep_block;
        q.out = actw(ot); q.out_rep = e.rep_block;
        q.relu = e.fused_relu[i];
        q.count = B * r.numel();
        switch (l.type) {
        case HADFL_OP_CONV:
        case HADFL_OP_DENSE: {
            GemmParams p = gemm_base(l);
            p.mode = kFwd;
            p.M = (int)(B * p.Ho * p.Wo); p.N = p.Cout; p.K = p.R * p.S * p.Cin;
            p.a = act(l.in0); p.a_rep = e.rep_block;
            p.cursor = l.in0 == 0 ? e.buf.cursor : nullptr;
            p.a_f32 = l.in0 == 0;
            p.out = actw(ot); p.out_rep = e.rep_block;
            p.relu = e.fused_relu[i];
            {
                FirstConvParams fc;
                if (first_conv(i, fc)) {
                    fc.out = actw(ot); fc.out_rep = e.rep_block; fc.relu = p.relu;
                    run("conv_fwd", gemm_flops(p), gemm_bytes(p), [&] { return launch_conv_first_fwd(fc, na, s); });
                    break;
                }
            }
            if (e.fast[i]) {
                FastConvParams f{};
                f.B = p.B; f.H = p.H; f.W = p.W; f.C = p.Cin; f.N = p.Cout; f.R = p.R; f.S = p.S; f.pad = p.pad;
                f.M = p.M; f.K = p.K;
                f.a = act(l.in0); f.a_rep = e.rep_block;
                f.wmat = wbf() + e.wf_off[i]; f.wmat_rep = e.wbf_rep;
                f.out = actw(ot); f.out_rep = e.rep_block;
                f.bias = l.bias ? e.buf.replicas + l.b_off : nullptr; f.bias_rep = e.plan.row_stride;
                f.relu = p.relu; f.order = e.buf.order; f.tile_hint = e.tile_hint;
                f.perm = perm(i); f.posmask = posmask(i);
                int* srows = nullptr;
                if (e.stat_for[i] >= 0) {
                    f.stat = bn_shared(); f.stat_rep = ((int64_t)p.M + 127) / 128 * 2 * p.Cout;
                    srows = &e.stat_rows[e.stat_for[i]];
                }
                run("conv_fwd", gemm_flops(p), gemm_bytes(p), [&] { return launch_conv_fast(f, 0, na, s, srows); });
                break;
            }
            if (e.fast32[i]) {
                FastConvParams f{};
                f.B = p.B; f.H = p.H; f.W = p.W; f.C = p.Cin; f.N = p.Cout; f.R = p.R; f.S = p.S; f.pad = p.pad;
                f.M = p.M; f.K = p.K;
                f.a = act(l.in0); f.a_rep = e.rep_block;
                f.wmat = reinterpret_cast<const __bf16*>(wcopy32(e.wf_off[i])); f.wmat_rep = e.wbf_rep / 2;
                f.out = actw(ot); f.out_rep = e.rep_block;
                f.bias = l.bias ? e.buf.replicas + l.b_off : nullptr; f.bias_rep = e.plan.row_stride;
                f.relu = p.relu; f.order = e.buf.order; f.tile_hint = e.tile_hint;
                f.perm = perm(i); f.posmask = posmask(i);
                int* srows = nullptr;
                if (e.stat_for[i] >= 0) {
                    f.stat = bn_shared(); f.stat_rep = ((int64_t)p.M + 127) / 128 * 2 * p.Cout;
                    srows = &e.stat_rows[e.stat_for[i]];
                }
                run("conv_fwd", gemm_flops(p), gemm_bytes(p), [&] { return launch_conv_f32_fast(f, 0, na, s, srows); });
                break;
            }
            if (l.type == HADFL_OP_DENSE && l.cout <= 16 && l.in0 != 0 && !p.relu) {
                DenseSmallParams d{};
                d.x = act(l.in0); d.x_rep = e.rep_block; d.w = p.w; d.w_rep = p.w_rep;
                d.out = actw(ot); d.out_rep = e.rep_block;
                d.rows = (int)B; d.K = p.Cin; d.N = l.cout; d.has_bias = l.bias; d.order = e.buf.order; d.bf16 = e.cfg.bf16;
                run("dense_small_fwd", gemm_flops(p), gemm_bytes(p), [&] { return launch_dense_small_fwd(d, na, s); });
                break;
            }
            run(l.type == HADFL_OP_CONV ? "conv_fwd" : "dense_fwd", gemm_flops(p), gemm_bytes(p), [&] { return gemm(p); });
            break; }
        case HADFL_OP_RELU: run("relu_fwd", 0, asz() * (8.0 * q.count), [&] { return launch_relu_fwd(q, na, s); }); break;
        case HADFL_OP_MAXPOOL: run("maxpool_fwd", 0, asz() * (4.0 * (B * a.numel() + q.count)), [&] { return launch_maxpool_fwd(q, na, s); }); break;
        case HADFL_OP_ADD:
            q.in2 = act(l.in1); q.in2_rep = e.rep_block;
            run("add_fwd", 0, asz() * (12.0 * q.count), [&] { return launch_add_fwd(q, na, s); });
            break;
        case HADFL_OP_GAP: run("gap_fwd", 0, asz() * (4.0 * (B * a.numel() + q.count)), [&] { return launch_gap_fwd(q, na, s); }); break;
        case HADFL_OP_BN: {
            BnParams b = bn_params(i);
            b.y = actw(ot); b.relu = e.fused_relu[i];
            if (e.stat_from[i] >= 0 && e.stat_rows[i] > 0) {          // the convolution in front left the sums
                b.stats_done = 1; b.stat_entries = (b.rows + e.stat_rows[i] - 1) / e.stat_rows[i];
                b.partial_rep = ((int64_t)b.rows + 127) / 128 * 2 * b.C;
                const Layer& conv = e.plan.layers[e.stat_from[i]];
                b.stat_shift = conv.bias ? e.buf.replicas + conv.b_off : nullptr; b.stat_shift_rep = e.plan.row_stride;
            }
            if (e.pool_of[i] >= 0) {
                b.pool = 1; b.H = a.h; b.W = a.w;
                b.pool_out = actw(e.plan.layers[e.pool_of[i]].out); b.pool_out_rep = e.rep_block;
            }
            run("bn_fwd", 0, asz() * (8.0 * B * a.numel()), [&] { return launch_bn_fwd(b, na, s); });
            break; }
        }
    }

    // bf16 configuration: the first convolution (data set in) has its own kernels when its footprint fits one MFMA
    bool first_conv(size_t i, FirstConvParams& f) const
    {
        const Layer& l = e.plan.layers[i];
        if (!e.cfg.bf16 || l.type != HADFL_OP_CONV || l.in0 != 0 || l.stride != 1) return false;
        if (l.bias && l.b_off != l.w_off + l.w_count) return false;
        const TensorShape a = e.plan.tensors[0], r = e.plan.tensors[l.out];
        if (r.h != a.h || r.w != a.w) return false;
        f = FirstConvParams{};
        f.x = e.buf.x; f.cursor = e.buf.cursor; f.n_samples = e.cfg.n_samples;
        f.B = e.cfg.batch; f.H = a.h; f.W = a.w; f.C = a.c; f.N = l.cout; f.R = f.S = l.k; f.pad = l.pad;
        f.K = l.k * l.k * a.c; f.M = e.cfg.batch * a.h * a.w;
        f.w = e.buf.replicas + l.w_off; f.w_rep = e.plan.row_stride;
        f.bias = l.bias ? e.buf.replicas + l.b_off : nullptr;
        f.order = e.buf.order;
        return conv_first_supported(f);
    }

    BnParams bn_params(size_t i) const
    {
        const Layer& l = e.plan.layers[i];
        const TensorShape a = e.plan.tensors[l.in0];
        BnParams b{};
        b.x = act(l.in0); b.x_rep = e.rep_block;
        b.y = actw(l.out); b.y_rep = e.rep_block;
        b.params = e.buf.replicas; b.grads = e.buf.grad; b.row_stride = e.plan.row_stride;
        b.w_off = l.w_off; b.stat_off = l.stat_off;
        b.saved = e.buf.work + e.saved_off[i]; b.saved_rep = e.rep_block;
        b.rows = (int)((int64_t)e.cfg.batch * a.h * a.w); b.C = a.c;
        b.chunks = e.bn_chunks[i];
        b.chunk_rows = (b.rows + b.chunks - 1) / b.chunks;
        b.partial = bn_shared(); b.partial_rep = (long long)b.chunks * 2 * a.c;
        b.order = e.buf.order; b.bf16 = e.cfg.bf16;
        return b;
    }

    // d(out) is complete; produce d(in0) (and d(in1)), and the parameter gradients of the layer
    void backward_layer(size_t i)
    {
        cur_layer = (int)i;
        if (e.skip[i]) return;
        const Layer& l = e.plan.layers[i];
        const TensorShape a = e.plan.tensors[l.in0], r = e.plan.tensors[l.out];
        const int64_t B = e.cfg.batch;
        const bool need_din = l.in0 != 0;
        const int acc0 = need_din ? (e.grad_written[l.in0] ? 1 : 0) : 0;
        const int ot = e.out_tensor[i];          // d(loss)/d(this layer's pre-ReLU output) lives in grad(ot)
        const float* mask0 = (need_din && e.masked[l.in0]) ? act(l.in0) : nullptr;
        EwParams q{};
        q.order = e.buf.order; q.B = (int)B; q.H = a.h; q.W = a.w; q.C = a.c; q.bf16 = e.cfg.bf16;
        q.accumulate = acc0;
        q.mask = mask0; q.mask_rep = e.rep_block;
        if (need_din) { q.out = grad(l.in0); q.out_rep = e.rep_block; }
        switch (l.type) {
        case HADFL_OP_CONV:
        case HADFL_OP_DENSE: {
            // weight (and bias) gradient
            GemmParams p = gemm_base(l);
            p.mode = kWgrad;
            p.M = p.R * p.S * p.Cin + (l.bias ? 1 : 0); p.N = p.Cout; p.K = (int)(B * p.Ho * p.Wo);
            p.a = act(l.in0); p.a_rep = e.rep_block;
            p.cursor = l.in0 == 0 ? e.buf.cursor : nullptr;
            p.a_f32 = l.in0 == 0;
            p.dy = grad(ot); p.dy_rep = e.rep_block;
            p.splits = e.splits[i];
            const int64_t mn = (int64_t)p.M * p.N;
            if (p.splits > 1 && e.fast[i]) {
                // The planned split count fills the chip when every replica is active.  A sub-step with fewer active
                // replicas splits K further; the partial-sum buffer (sized for all replicas at the planned count) and
                // K bound how far.  Wide-image layers run the all-taps kernel with one tile per 64 x 64 channel pair.
                const bool wide = ((p.W == 16 || p.W == 32) && p.Cin <= 128 && p.N <= 128) || (p.W == 8 && p.H % 4 == 0);
                const int64_t tiles = wide ? (int64_t)(p.Cin / 64) * (p.N / 64) : ((p.M + 127) / 128) * ((p.N + 127) / 128);
                const int64_t want = (1024 + tiles * na - 1) / (tiles * na);
                const int64_t by_buffer = e.shared_floats / ((int64_t)na * ((mn + 63) / 64 * 64));
                const int64_t by_k = std::max<int64_t>(1, p.K / 512);
                p.splits = (int)std::max<int64_t>(p.splits, std::min<int64_t>(std::min<int64_t>(want, by_buffer), std::min<int64_t>(by_k, 256)));
            }
            if (p.splits > 1) {
                const int unit = e.fast[i] ? 64 : 16;      // slab length of the kernel that will run
                const int slabs = (p.K + unit - 1) / unit;
                p.kchunk = ((slabs + p.splits - 1) / p.splits) * unit;
                p.out_split = (mn + 63) / 64 * 64;
                p.out = shared(); p.out_rep = p.out_split * p.splits;
            } else {
                p.out = e.buf.grad + l.w_off; p.out_rep = e.plan.row_stride;
            }
            fork();
            flush_pending_prep();
            FirstConvParams fc;
            if (first_conv(i, fc)) {
                fc.dy = grad(ot); fc.dy_rep = e.rep_block;
                fc.gout = p.out; fc.gout_rep = p.out_rep; fc.gout_split = p.out_split; fc.splits = p.splits; fc.kchunk = p.kchunk;
                run("conv_wgrad", gemm_flops(p), gemm_bytes(p), [&] { return launch_conv_first_wgrad(fc, na, s); });
            } else
            if (e.fast[i]) {
                FastWgradParams f{};
                f.B = p.B; f.H = p.H; f.W = p.W; f.C = p.Cin; f.N = p.Cout; f.R = p.R; f.S = p.S; f.pad = p.pad;
                f.M = p.M; f.K = p.K; f.kchunk = p.kchunk; f.splits = p.splits; f.w_shift = p.w_shift; f.has_bias = l.bias;
                f.x = act(l.in0); f.x_rep = e.rep_block; f.dy = grad(ot); f.dy_rep = e.rep_block;
                f.out = p.out; f.out_rep = p.out_rep; f.out_split = p.out_split; f.order = e.buf.order;
                if (p.H * p.W <= kMaxTablePositionsWgrad && p.B % 64 == 0) { f.perm = perm(i); f.posmask = posmask(i); }
                f.tile_hint = e.tile_hint;
                if (e.fused_update[i]) {
                    f.sgd_w = e.buf.replicas + l.w_off; f.sgd_buf = e.buf.mom ? e.buf.mom + l.w_off : nullptr;
                    f.lr = e.cfg.lr; f.momentum = e.cfg.momentum;
                }
                run("conv_wgrad", gemm_flops(p), gemm_bytes(p), [&] { return launch_wgrad_fast(f, na, s); });
                if (e.fused_update[i] && na_next > 0) pending_prep = (int)i;
            } else
            {
                run(l.type == HADFL_OP_CONV ? "conv_wgrad" : "dense_wgrad", gemm_flops(p), gemm_bytes(p), [&] { return gemm(p); });
                if (e.fast32[i] && e.fused_update[i] && na_next > 0) pending_prep = (int)i;
            }
            if (p.splits > 1 && e.fused_update[i])
                run("splitk_reduce", 0, 4.0 * mn * (p.splits + 4), [&] {
                    return launch_splitk_reduce_update(shared(), p.out_split, p.splits, e.buf.replicas + l.w_off,
                                                       e.buf.mom ? e.buf.mom + l.w_off : nullptr, e.plan.row_stride, mn, e.cfg.lr,
                                                       e.cfg.momentum, e.buf.order, na, s); });
            else if (p.splits > 1)
                run("splitk_reduce", 0, 4.0 * mn * (p.splits + 1), [&] { return launch_splitk_reduce(shared(), p.out_split, p.splits, e.buf.grad + l.w_off,
                                                                       e.plan.row_stride, mn, e.buf.order, na, s); });
            unfork();
            if (need_din) {
                GemmParams d = gemm_base(l);
                d.mode = kDgrad;
                d.M = (int)(B * d.H * d.W); d.N = d.Cin; d.K = d.R * d.S * d.Cout;
                d.a = grad(ot); d.a_rep = e.rep_block;
                d.out = grad(l.in0); d.out_rep = e.rep_block;
                d.accumulate = acc0;
                d.mask = mask0; d.mask_rep = e.rep_block;
                if (e.fast[i]) {
                    FastConvParams f{};
                    f.B = d.B; f.H = d.H; f.W = d.W; f.C = d.Cout; f.N = d.Cin; f.R = d.R; f.S = d.S; f.pad = d.R - 1 - d.pad;
                    f.M = d.M; f.K = d.K;
                    f.a = grad(ot); f.a_rep = e.rep_block;
                    f.wmat = wbf() + e.wb_off[i]; f.wmat_rep = e.wbf_rep;
                    f.out = grad(l.in0); f.out_rep = e.rep_block;
                    f.mask = mask0; f.mask_rep = e.rep_block; f.accumulate = acc0; f.order = e.buf.order; f.tile_hint = e.tile_hint;
                    f.perm = perm(i); f.posmask = posmask(i);
                    int* brows = nullptr;
                    if (e.bstat_for[i] >= 0 && !acc0) {        // this data gradient is the whole gradient of a BN's output
                        const int k = e.bstat_for[i];
                        f.stat = bn_shared(); f.stat_rep = ((int64_t)d.M + 127) / 128 * 2 * d.N;
                        f.stat_y = act(l.in0); f.stat_y_rep = e.rep_block; f.stat_relu = e.fused_relu[k];
                        e.bstat_rep[k] = f.stat_rep;
                        brows = &e.bstat_rows[k];
                    }
                    run("conv_dgrad", gemm_flops(d), gemm_bytes(d), [&] { return launch_conv_fast(f, 1, na, s, brows); });
                } else if (e.fast32[i]) {
                    FastConvParams f{};
                    f.B = d.B; f.H = d.H; f.W = d.W; f.C = d.Cout; f.N = d.Cin; f.R = d.R; f.S = d.S; f.pad = d.R - 1 - d.pad;
                    f.M = d.M; f.K = d.K;
                    f.a = grad(ot); f.a_rep = e.rep_block;
                    f.wmat = reinterpret_cast<const __bf16*>(wcopy32(e.wb_off[i])); f.wmat_rep = e.wbf_rep / 2;
                    f.out = grad(l.in0); f.out_rep = e.rep_block;
                    f.mask = mask0; f.mask_rep = e.rep_block; f.accumulate = acc0; f.order = e.buf.order; f.tile_hint = e.tile_hint;
                    f.perm = perm(i); f.posmask = posmask(i);
                    run("conv_dgrad", gemm_flops(d), gemm_bytes(d), [&] { return launch_conv_f32_fast(f, 1, na, s); });
                } else
                run(l.type == HADFL_OP_CONV ? "conv_dgrad" : "dense_dgrad", gemm_flops(d), gemm_bytes(d), [&] { return gemm(d); });
            }
            break; }
        case HADFL_OP_RELU:
            q.in = act(l.in0); q.in_rep = e.rep_block; q.in2 = grad(l.out); q.in2_rep = e.rep_block;
            q.count = B * a.numel();
            run("relu_bwd", 0, asz() * (12.0 * q.count), [&] { return launch_relu_bwd(q, na, s); });
            break;
        case HADFL_OP_MAXPOOL:
            q.in = act(l.in0); q.in_rep = e.rep_block; q.in2 = grad(l.out); q.in2_rep = e.rep_block;
            q.count = B * r.numel();
            run("maxpool_bwd", 0, asz() * (4.0 * (2 * B * a.numel() + q.count)), [&] { return launch_maxpool_bwd(q, na, s); });
            break;
        case HADFL_OP_ADD: {
            q.in = grad(ot); q.in_rep = e.rep_block; q.count = B * a.numel();
            run("add_bwd", 0, asz() * (8.0 * q.count), [&] { return launch_pass_grad(q, na, s); });
            EwParams q2 = q;
            if (l.in1 == l.in0) q2.accumulate = 1; else q2.accumulate = e.grad_written[l.in1] ? 1 : 0;
            q2.out = grad(l.in1);
            q2.mask = e.masked[l.in1] ? act(l.in1) : nullptr;
            run("add_bwd", 0, asz() * (8.0 * q.count), [&] { return launch_pass_grad(q2, na, s); });
            e.grad_written[l.in1] = 1;
            break; }
        case HADFL_OP_GAP:
            q.in = grad(l.out); q.in_rep = e.rep_block; q.count = B * a.numel();
            run("gap_bwd", 0, asz() * (4.0 * (q.count + B * a.c)), [&] { return launch_gap_bwd(q, na, s); });
            break;
        case HADFL_OP_BN: {
            BnParams b = bn_params(i);
            b.dy = grad(ot); b.dy_rep = e.rep_block;
            b.y = grad(l.in0); b.y_rep = e.rep_block;
            b.accumulate = acc0;
            b.mask = mask0; b.mask_rep = e.rep_block;
            if (e.pool_of[i] >= 0) {
                b.pool = 1; b.H = a.h; b.W = a.w; b.relu = e.fused_relu[i];
                b.pool_g = grad(e.plan.layers[e.pool_of[i]].out); b.pool_g_rep = e.rep_block;
            }
            if (e.bstat_rows[i] > 0) {                       // the data gradient of the layer above left the sums
                const int64_t rows_out = e.pool_of[i] >= 0 ? b.rows / 4 : b.rows;
                b.bwd_stats_done = 1; b.stat_entries = (int)((rows_out + e.bstat_rows[i] - 1) / e.bstat_rows[i]);
                b.partial_rep = e.bstat_rep[i];
                e.bstat_rows[i] = 0;
            }
            run("bn_bwd", 0, asz() * (12.0 * B * a.numel()), [&] { return launch_bn_bwd(b, na, s); });
            break; }
        }
        if (need_din) e.grad_written[l.in0] = 1;
    }
};

}  // namespace

hadfl_status train_run(TrainEngine* e, hipStream_t s, Profiler* prof, std::string& err)
{
    Runner r{*e, s, (prof && prof->on) ? prof : nullptr};
    const int N = e->cfg.n_replicas;
    r.run("zero_versions", 0, 0, [&] { return launch_fill_u32((uint32_t*)e->buf.versions, 0u, N, s); });
    if (!e->tables_uploaded && !e->tables.empty()) {
        const hipError_t rc = hipMemcpyAsync(e->buf.work + e->tab_off, e->tables.data(), e->tables.size() * sizeof(int32_t), hipMemcpyHostToDevice, s);
        if (rc != hipSuccess) { err = std::string("copy position tables: ") + hipGetErrorString(rc); return HADFL_EDEVICE; }
        e->tables_uploaded = true;
    }
    if (e->use_side && !e->side) {
        if (hipStreamCreateWithFlags(&e->side, hipStreamNonBlocking) != hipSuccess ||
            hipEventCreateWithFlags(&e->ev_fork, hipEventDisableTiming) != hipSuccess ||
            hipEventCreateWithFlags(&e->ev_join, hipEventDisableTiming) != hipSuccess) {
            err = "side stream"; return HADFL_EDEVICE;
        }
    }
    const int T = (int)e->plan.tensors.size();
    e->prepped.assign(e->plan.layers.size(), 0);       // the weights may have changed since the last call (aggregation)
    for (int step = 0; step < e->e_max && r.rc == hipSuccess; ++step) {
        r.na = e->n_active[step];
        r.prepare_weights();
        for (size_t i = 0; i < e->plan.layers.size(); ++i) r.forward_layer(i);
        LossParams lp{};
        lp.logits = r.act(T - 1); lp.logits_rep = e->rep_block;
        lp.dlogits = r.grad(T - 1); lp.dlogits_rep = e->rep_block;
        lp.y = e->buf.y; lp.cursor = e->buf.cursor; lp.n_samples = e->cfg.n_samples; lp.batch = e->cfg.batch;
        lp.n_classes = e->cfg.n_classes; lp.loss = e->buf.loss; lp.order = e->buf.order; lp.bf16 = e->cfg.bf16;
        r.run("softmax_ce", 0, r.asz() * 8.0 * e->cfg.batch * e->cfg.n_classes, [&] { return launch_softmax_ce(lp, r.na, s); });
        e->grad_written.assign(T, 0);
        e->grad_written[T - 1] = 1;
        r.na_next = step + 1 < e->e_max ? e->n_active[step + 1] : 0;
        for (size_t i = e->plan.layers.size(); i-- > 0;) r.backward_layer(i);
        if (r.pending_prep >= 0) { r.fork(); r.flush_pending_prep(); r.unfork(); }
        r.join();
        SgdParams sp{};
        sp.w = e->buf.replicas; sp.g = e->buf.grad; sp.buf = e->buf.mom; sp.row_stride = e->plan.row_stride;
        sp.lr = e->cfg.lr; sp.momentum = e->cfg.momentum;
        sp.cursor = e->buf.cursor; sp.versions = e->buf.versions; sp.order = e->buf.order;
        r.cur_layer = 0;
        // the pieces of the row no weight-gradient kernel has updated already, several per launch; the last launch (there
        // is always one) also advances the replicas' batch cursors and versions
        const size_t nseg = e->update_segments.size();
        for (size_t k0 = 0; k0 < std::max<size_t>(nseg, 1); k0 += kMaxSgdSegments) {
            const size_t k1 = std::min(nseg, k0 + kMaxSgdSegments);
            double floats = 0.0;
            sp.n_seg = (int)(k1 - k0);
            for (size_t k = k0; k < k1; ++k) {
                sp.first[k - k0] = e->update_segments[k].first; sp.count[k - k0] = e->update_segments[k].second;
                floats += (double)e->update_segments[k].second;
            }
            sp.bump = k1 == nseg;
            r.run("sgd", 0, (e->buf.mom ? 20.0 : 12.0) * floats, [&] { return launch_sgd(sp, r.na, s); });
        }
    }
    if (r.rc != hipSuccess) {
        err = std::string("kernel launch failed in ") + (r.failed ? r.failed : "?") + ": " + hipGetErrorString(r.rc);
        return HADFL_EDEVICE;
    }
    return HADFL_OK;
}

}  // namespace hadfl
