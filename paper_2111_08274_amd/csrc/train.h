// Local-training engine: the forward / backward / update kernels of hadfl_local_steps and the
// host-side schedule that issues them for all replicas at once.
#pragma once
#include "hadfl_internal.h"

namespace hadfl {

struct Profiler;

struct TrainBuffers {
    float* replicas = nullptr;      // [N][row_stride] parameter rows
    float* mom = nullptr;           // [N][row_stride] momentum buffers (null when momentum == 0)
    float* grad = nullptr;          // [N][row_stride]
    float* work = nullptr;          // activations, activation gradients, split-K partials
    const float* x = nullptr;       // [N][n_samples][H][W][C]
    const int32_t* y = nullptr;     // [N][n_samples]
    int32_t* order = nullptr;       // [N] replica indices sorted by step count, descending
    int32_t* versions = nullptr;    // [N]
    long long* cursor = nullptr;     // [N] steps taken since init
    float* loss = nullptr;          // [N]
};

class TrainEngine;
// Floats of `work` the engine needs for cfg/plan (0 for HADFL_NET_NONE).
int64_t train_work_floats(const hadfl_config& cfg, const NetPlan& plan);
hadfl_status train_create(const hadfl_config& cfg, const NetPlan& plan, const TrainBuffers& buf,
                          const std::vector<int32_t>& steps, const std::vector<int32_t>& order,
                          TrainEngine** out, std::string& err);
// Enqueue every replica's E_k local steps on s.
hadfl_status train_run(TrainEngine* e, hipStream_t s, Profiler* prof, std::string& err);
// New per-replica step counts for the following runs (the caller has already re-sorted and uploaded `order`)
void train_set_steps(TrainEngine* e, const std::vector<int32_t>& steps);
void train_set_lr(TrainEngine* e, float lr);
void train_set_side_stream(TrainEngine* e, bool on);      // weight gradients on the engine's second stream
void train_set_tile_hint(TrainEngine* e, int hint);       // 0 automatic, 1 tall tiles wherever they fit, 2 no wide-image kernels
bool train_has_momentum(const TrainEngine* e);
void train_destroy(TrainEngine* e);

// Event-pair profiler used by hadfl_profile_*.
struct Profiler {
    struct Rec { std::string name; hipEvent_t a, b; double flops, bytes; };
    bool on = false;
    bool detail = false;            // names carry the layer index and the number of active replicas
    std::vector<Rec> recs;
    std::vector<hipEvent_t> pool;
    hipEvent_t get();
    void begin(const char* name, hipStream_t s, double flops = 0.0, double bytes = 0.0);
    void end(hipStream_t s);
    void clear();
    ~Profiler();
};

}  // namespace hadfl
