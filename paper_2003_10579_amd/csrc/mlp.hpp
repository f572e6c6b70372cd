// Two-layer ReLU network (bf16 MFMA contractions, fp32 accumulation): host entry points.
#pragma once
#include <string>

#include "../../include/ssgd.h"
#include "common.hpp"

namespace ssgd {

struct MlpState;

// One state per replica (independent runs that differ in the replica field of their random draws).  The first replica
// (first == nullptr) makes a bf16 copy of the sample matrix as it is at this call; the others read that copy, so the first
// state is destroyed last.
hipError_t mlp_create(MlpState** out, const ssgd_model& model, int P, int m, int variant, int Kcap, double lr,
                      uint64_t seed, int replica, const MlpState* first, hipStream_t stream, std::string* msg);
// Runs updates [v0, v0+n) of all R replicas, whose schedules are already in the trace; agg_out: replica 0's.
// `pieces` (may be null): the schedule of the segment is still being written, piece by piece, on another stream, which
// also copies the trace rows of replica 0 to pinned host memory; piece k (updates [k len, (k + 1) len) of the segment)
// is complete, on the device and in the host copies, once ready[k] has happened.  One replica only.
struct MlpPieces {
    const hipEvent_t* ready;
    int count;
    int64_t len;
    const int32_t* K;      // [n]           host copies, indexed from the segment's first update
    const int32_t* tau;    // [n][Kcap]
    const int32_t* sel;    // [1 + n][Kcap] one row in front: the consume list of update v0 - 1 (unused when v0 = 0)
};
hipError_t mlp_run_segment(MlpState* const* states, int R, const Trace& tr, const WorkerState& ws, int64_t v0, int64_t n,
                           float* agg_out, hipStream_t stream, double* ms_accum, int64_t* launches, std::string* msg,
                           const MlpPieces* pieces = nullptr);
float* mlp_params(MlpState* s);
// Objective over the whole data set at the current parameters, with the trainer's forward pass.
hipError_t mlp_full_loss(MlpState* s, double* out, hipStream_t stream, std::string* msg);
// Its gradient, |w| floats on the host, with the arithmetic of the trainer's gradients.
hipError_t mlp_full_gradient(MlpState* s, float* grad_out_host, hipStream_t stream, std::string* msg);
// Snapshot of everything later updates depend on (host memory; the stream must be idle).
int64_t mlp_state_bytes(MlpState* s);
hipError_t mlp_get_state(MlpState* s, unsigned char* host);
hipError_t mlp_set_state(MlpState* s, const unsigned char* host);
void mlp_destroy(MlpState* s);

}  // namespace ssgd
