// Shared declarations of the library's translation units (host side and kernels).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "rng.hpp"

namespace ssgd {

enum Variant : int32_t { kSync = 0, kBatchSync = 1, kAsync = 2, kBatchAsync = 3 };
enum ModelKind : int32_t { kLsq = 0, kSoftmax = 1, kMlp2 = 2 };

constexpr int kMaxWorkers = 256;   // four workers per lane of one wavefront
constexpr int kClassPad = 16;      // MFMA tile height that holds the class dimension

// Per-update records written by the schedule kernel (one row per update).
struct Trace {
    double* t;        // [R][cap]        clock after the update
    float* loss;      // [R][cap]        mean mini-batch loss of the contributors
    int32_t* K;       // [R][cap]
    int32_t* sel;     // [R][cap][Kcap]  contributing workers in arrival order
    int32_t* tau;     // [R][cap][Kcap]  parameter version each of them read
    int32_t* ord;     // [R][cap][Kcap]  ordinal of the contributed mini-batch
    int64_t cap;
    int32_t Kcap;
};

// Event state of the P workers of every replica, kept across ssgd_run calls.
struct WorkerState {
    double* finish;   // [R][P]  absolute finish time (async)
    int32_t* tau;     // [R][P]  version read
    int32_t* ord;     // [R][P]
    double* clock;    // [R]
    int32_t* curK;    // [R]
    // AdaSync bookkeeping per replica
    double* win_prev; // [R] mean loss of the previous window
    int64_t* win_index;
    double* F0;       // [R] loss of update 0
    int64_t* int_start; // [R] first update of the current interval
    int32_t* crossed; // [R] set by the schedule kernel when the clock crossed an interval boundary
    int64_t* n_done;  // [R] updates scheduled by the last schedule launch
};

struct SchedArgs {
    Trace tr;
    WorkerState ws;
    Dist dist;
    uint64_t seed;
    int32_t P, variant, table_ord;
    int32_t replica0;
    int64_t j0, count;
    double interval_t;   // > 0: stop after the update whose clock crosses a multiple of it
};

void launch_schedule(const SchedArgs& a, int replicas, hipStream_t s);

struct AdaArgs {
    Trace tr;
    WorkerState ws;
    int32_t mode, K0, Kmax, window, P;
    double rel_tol;
    int64_t j_end;     // updates done after this segment
    int32_t window_closed;  // mode 1: the segment ended a window
};
void launch_adasync(const AdaArgs& a, int replicas, hipStream_t s);

// ---- linear models (least squares, softmax regression) ---------------------------------------
struct LinArgs {
    int32_t kind, d, C, m, mp, P, variant;
    const float* X;
    const void* y;
    uint32_t N;
    float lr;
    uint64_t seed;
    int32_t G, S;            // column slices per replica, gradient slots per replica
    int32_t replica0, replicas;
    Trace tr;
    int64_t v0, nsteps;
    float* params;           // [R][nw], standard layout
    float* park;             // [R][G][S][16][threads] parked per-slot gradients (thread-owned layout)
    float* park_small;       // [R][G][S][17]: bias gradient (16) and mean loss (1) of every slot
    float* zpart;            // [R][2][G][maxrows][16] partial logits exchanged inside a cluster
    int32_t maxrows;
    unsigned int* arrive;    // [R][2] arrival counters of the cluster exchange, zero at launch
    int32_t* abort_flag;
    uint32_t spin_limit;
    float* agg_out;          // nullable: averaged gradient of the last update of replica 0
    int32_t* xcc_ids;        // [R][G] XCD each workgroup of a cluster runs on (checked on the device)
    int32_t allow_fast;      // 1: exchange through the shared L2 once a cluster is known to sit on one XCD
    unsigned long long* prof;   // nullable diagnostics: [R][G][8] shader-clock cycles spent per phase
};
int linear_max_resident_groups(int nbw, size_t lds_bytes);
size_t linear_lds_bytes(int nbw, int C, int S);
hipError_t launch_linear(const LinArgs& a, int nbw, hipStream_t s);

}  // namespace ssgd
