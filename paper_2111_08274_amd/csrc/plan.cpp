// Network plans: layer lists of the supported networks, tensor shapes, and the two parameter layouts
// (the dense interface vector documented in hadfl.h and the padded row kept in device memory).
#include "hadfl_internal.h"

namespace hadfl {
namespace {

struct Net {
    std::vector<Layer> L;
    int push(int type, int in0, int in1 = -1, int k = 0, int stride = 0, int pad = 0, int cout = 0, int bias = 0) {
        Layer l;
        l.type = type; l.in0 = in0; l.in1 = in1; l.out = (int)L.size() + 1;
        l.k = k; l.stride = stride; l.pad = pad; l.cout = cout; l.bias = bias;
        L.push_back(l);
        return l.out;
    }
    int conv(int x, int cout, int k, int stride, int pad, bool bias) { return push(HADFL_OP_CONV, x, -1, k, stride, pad, cout, bias); }
    int dense(int x, int cout) { return push(HADFL_OP_DENSE, x, -1, 0, 0, 0, cout, 1); }
    int relu(int x) { return push(HADFL_OP_RELU, x); }
    int pool(int x) { return push(HADFL_OP_MAXPOOL, x); }
    int bn(int x) { return push(HADFL_OP_BN, x); }
    int add(int a, int b) { return push(HADFL_OP_ADD, a, b); }
    int gap(int x) { return push(HADFL_OP_GAP, x); }
};

void net_mlp(Net& n, int n_classes) {
    int h = n.relu(n.dense(0, 128));
    n.dense(h, n_classes);
}

void net_cnn2(Net& n, int n_classes) {
    int t = n.pool(n.relu(n.conv(0, 32, 3, 1, 1, true)));
    t = n.pool(n.relu(n.conv(t, 64, 3, 1, 1, true)));
    n.dense(t, n_classes);
}

// ResNet-18 for 32x32 inputs (He et al. 2016, CIFAR form with the ImageNet widths): 3x3 stem,
// stages of two basic blocks at 64/128/256/512 channels, stride 2 entering stages 2-4 with a
// 1x1 projection shortcut, batch norm after every convolution, average pool, linear classifier.
void net_resnet18(Net& n, int n_classes) {
    int t = n.relu(n.bn(n.conv(0, 64, 3, 1, 1, false)));
    const int widths[4] = {64, 128, 256, 512};
    int cin = 64;
    for (int s = 0; s < 4; ++s)
        for (int b = 0; b < 2; ++b) {
            const int stride = (b == 0 && s > 0) ? 2 : 1;
            const int cout = widths[s];
            int u = n.relu(n.bn(n.conv(t, cout, 3, stride, 1, false)));
            u = n.bn(n.conv(u, cout, 3, 1, 1, false));
            int sc = t;
            if (stride != 1 || cin != cout) sc = n.bn(n.conv(t, cout, 1, stride, 0, false));
            t = n.relu(n.add(u, sc));
            cin = cout;
        }
    n.dense(n.gap(t), n_classes);
}

// VGG-16 (Simonyan & Zisserman 2015, configuration D) with batch norm, for 32x32 inputs.
void net_vgg16(Net& n, int n_classes) {
    const int width[5] = {64, 128, 256, 512, 512}, reps[5] = {2, 2, 3, 3, 3};
    int t = 0;
    for (int g = 0; g < 5; ++g) {
        for (int r = 0; r < reps[g]; ++r) t = n.relu(n.bn(n.conv(t, width[g], 3, 1, 1, true)));
        t = n.pool(t);
    }
    n.dense(t, n_classes);
}

int64_t round_up(int64_t v, int64_t a) { return (v + a - 1) / a * a; }

}  // namespace

hadfl_status build_plan(const hadfl_config& cfg, NetPlan& plan, std::string& err)
{
    plan = NetPlan();
    if (cfg.net == HADFL_NET_NONE) {
        if (cfg.m_none < 1) { err = "m_none must be positive for HADFL_NET_NONE"; return HADFL_EINVAL; }
        plan.m_train = plan.m_total = cfg.m_none;
        plan.train_end = plan.row_stride = round_up(cfg.m_none, kRowAlign);
        plan.segs.push_back({0, 0, cfg.m_none});
        return HADFL_OK;
    }
    Net n;
    const int nc = cfg.n_classes;
    if (nc < 2 && cfg.net != HADFL_NET_CUSTOM) { err = "n_classes must be at least 2"; return HADFL_EINVAL; }
    switch (cfg.net) {
    case HADFL_NET_MLP: net_mlp(n, nc); break;
    case HADFL_NET_CNN2: net_cnn2(n, nc); break;
    case HADFL_NET_RESNET18: net_resnet18(n, nc); break;
    case HADFL_NET_VGG16: net_vgg16(n, nc); break;
    case HADFL_NET_CUSTOM:
        if (!cfg.custom_ops || cfg.n_custom_ops < 1) { err = "custom network without layers"; return HADFL_EINVAL; }
        for (int i = 0; i < cfg.n_custom_ops; ++i) {
            const hadfl_op& o = cfg.custom_ops[i];
            n.push(o.type, o.in0, o.in1, o.k, o.stride, o.pad, o.cout, o.bias ? 1 : 0);
        }
        break;
    default: err = "unknown network"; return HADFL_EINVAL;
    }
    if (cfg.in_dim[0] < 1 || cfg.in_dim[1] < 1 || cfg.in_dim[2] < 1) { err = "in_dim must be positive"; return HADFL_EINVAL; }

    plan.layers = n.L;
    plan.tensors.assign(plan.layers.size() + 1, TensorShape());
    plan.tensors[0].h = cfg.in_dim[0]; plan.tensors[0].w = cfg.in_dim[1]; plan.tensors[0].c = cfg.in_dim[2];
    int64_t if_off = 0, row_off = 0;
    for (size_t i = 0; i < plan.layers.size(); ++i) {
        Layer& l = plan.layers[i];
        if (l.in0 < 0 || l.in0 >= l.out) { err = "layer input must be an earlier tensor"; return HADFL_EINVAL; }
        // tensor 0 is the batch inside the data set, addressed through the replica's batch cursor: only the layers
        // that form GEMM operands from it know how to read it
        if ((l.in0 == 0 && l.type != HADFL_OP_CONV && l.type != HADFL_OP_DENSE) || (l.type == HADFL_OP_ADD && l.in1 == 0)) {
            err = "only a convolution or dense layer may read the input batch"; return HADFL_EUNSUPPORTED;
        }
        const TensorShape a = plan.tensors[l.in0];
        TensorShape r = a;
        switch (l.type) {
        case HADFL_OP_CONV:
            if (l.k < 1 || l.stride < 1 || l.pad < 0 || l.cout < 1) { err = "bad convolution geometry"; return HADFL_EINVAL; }
            r.h = (a.h + 2 * l.pad - l.k) / l.stride + 1;
            r.w = (a.w + 2 * l.pad - l.k) / l.stride + 1;
            r.c = l.cout;
            if (r.h < 1 || r.w < 1) { err = "convolution output is empty"; return HADFL_EINVAL; }
            l.w_count = (int64_t)l.k * l.k * a.c * l.cout;
            break;
        case HADFL_OP_DENSE:
            if (l.cout < 1) { err = "bad dense width"; return HADFL_EINVAL; }
            r.h = r.w = 1; r.c = l.cout;
            l.w_count = a.numel() * l.cout;
            break;
        case HADFL_OP_RELU: break;
        case HADFL_OP_MAXPOOL:
            if (a.h % 2 || a.w % 2) { err = "max-pool needs even height and width"; return HADFL_EINVAL; }
            r.h = a.h / 2; r.w = a.w / 2; break;
        case HADFL_OP_BN: l.w_count = a.c; break;
        case HADFL_OP_ADD: {
            if (l.in1 < 0 || l.in1 >= l.out) { err = "add needs two earlier tensors"; return HADFL_EINVAL; }
            const TensorShape b = plan.tensors[l.in1];
            if (a.h != b.h || a.w != b.w || a.c != b.c) { err = "add operands differ in shape"; return HADFL_EINVAL; }
            break; }
        case HADFL_OP_GAP: r.h = r.w = 1; break;
        default: err = "unknown layer type"; return HADFL_EINVAL;
        }
        plan.tensors[l.out] = r;
        if (l.w_count > 0) {
            const int64_t second = (l.type == HADFL_OP_BN) ? a.c : (l.bias ? l.cout : 0);
            row_off = round_up(row_off, kRowAlign);
            l.w_off = row_off; l.if_w_off = if_off;
            plan.segs.push_back({if_off, row_off, l.w_count + second});   // bias/beta directly follows in both layouts
            if (second) { l.b_off = row_off + l.w_count; l.if_b_off = if_off + l.w_count; }
            row_off += l.w_count + second; if_off += l.w_count + second;
        }
    }
    plan.m_train = if_off;
    plan.train_end = round_up(row_off, kRowAlign);
    row_off = plan.train_end;
    for (Layer& l : plan.layers)
        if (l.type == HADFL_OP_BN) {
            const int c = plan.tensors[l.in0].c;
            l.stat_off = row_off; l.if_stat_off = if_off;
            plan.segs.push_back({if_off, row_off, 2 * (int64_t)c});
            row_off += 2 * (int64_t)c; if_off += 2 * (int64_t)c;
        }
    plan.m_total = if_off;
    plan.row_stride = round_up(row_off, kRowAlign);
    const TensorShape last = plan.tensors.back();
    if (last.h != 1 || last.w != 1 || (cfg.net != HADFL_NET_CUSTOM && last.c != nc) || last.c != cfg.n_classes) {
        err = "network output must be [1][1][n_classes]"; return HADFL_EINVAL;
    }
    return HADFL_OK;
}

}  // namespace hadfl
