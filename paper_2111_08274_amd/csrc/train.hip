#include "train.h"
namespace hadfl {
class TrainEngine {};
int64_t train_work_floats(const hadfl_config&, const NetPlan&) { return 0; }
hadfl_status train_create(const hadfl_config&, const NetPlan&, const TrainBuffers&, const std::vector<int32_t>&,
                          const std::vector<int32_t>&, TrainEngine**, std::string& err)
{ err = "training kernels not built"; return HADFL_EUNSUPPORTED; }
hadfl_status train_run(TrainEngine*, hipStream_t, Profiler*, std::string& err) { err = "no engine"; return HADFL_EUNSUPPORTED; }
void train_destroy(TrainEngine*) {}
}
