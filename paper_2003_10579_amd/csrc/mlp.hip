#include "mlp.hpp"

namespace ssgd {
struct MlpState { int unused; };
hipError_t mlp_create(MlpState**, const ssgd_model&, int, int, int, int, double, uint64_t, hipStream_t, std::string* msg) {
    if (msg) *msg = "not built yet";
    return hipErrorNotSupported;
}
hipError_t mlp_run_segment(MlpState*, const Trace&, const WorkerState&, int64_t, int64_t, float*, hipStream_t, double*, int64_t*, std::string* msg) {
    if (msg) *msg = "not built yet";
    return hipErrorNotSupported;
}
float* mlp_params(MlpState*) { return nullptr; }
void mlp_destroy(MlpState*) {}
}  // namespace ssgd
