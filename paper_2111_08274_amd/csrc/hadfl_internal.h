// Internal declarations shared by the translation units of libhadfl.so (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <string>
#include <vector>

#include "../../include/hadfl.h"

namespace hadfl {

constexpr int kMaxReplicas = 1024;     // selection kernel keeps per-replica state in LDS
constexpr int kRowAlign = 64;          // floats: every layer's slice of a parameter row starts 256-byte aligned

struct TensorShape { int h = 0, w = 0, c = 0; int64_t numel() const { return (int64_t)h * w * c; } };

// One layer of the network plan.  Offsets are in floats inside a (padded) parameter row.
struct Layer {
    int type = 0, in0 = 0, in1 = -1, out = 0;
    int k = 0, stride = 0, pad = 0, cout = 0, bias = 0;
    int64_t w_off = -1;        // weights / gamma (bias or beta follows directly: w_off + w_count)
    int64_t w_count = 0;
    int64_t b_off = -1;
    int64_t stat_off = -1;     // running mean; running variance follows
    // interface (dense) offsets of the same tensors
    int64_t if_w_off = -1, if_b_off = -1, if_stat_off = -1;
};

struct NetPlan {
    std::vector<Layer> layers;
    std::vector<TensorShape> tensors;     // tensors[0] = input sample
    int64_t m_train = 0, m_total = 0;     // interface sizes
    int64_t train_end = 0;                // padded-row extent of the trainable part
    int64_t row_stride = 0;               // padded row length (multiple of kRowAlign)
    // copy segments interface<->row: (if_off, row_off, count)
    struct Seg { int64_t if_off, row_off, count; };
    std::vector<Seg> segs;
};

hadfl_status build_plan(const hadfl_config& cfg, NetPlan& plan, std::string& err);

}  // namespace hadfl
