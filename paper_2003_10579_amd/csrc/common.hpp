// Shared declarations of the library's translation units (host side and kernels).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <string>

#include "rng.hpp"

namespace ssgd {

enum Variant : int32_t { kSync = 0, kBatchSync = 1, kAsync = 2, kBatchAsync = 3 };
enum ModelKind : int32_t { kLsq = 0, kSoftmax = 1, kMlp2 = 2 };

constexpr int kMaxWorkers = 256;   // four workers per lane of one wavefront
constexpr int kClassPad = 16;      // MFMA tile height that holds the class dimension
constexpr int kArriveStride = 64;  // 32-bit words between the arrival counters of two replicas
constexpr int kArriveFast = 32;

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
    float* park;             // [R][G][S][4][threads][4] parked per-slot gradients: class own_cls + vv, 4 columns of the owner thread
    float* park_small;       // [R][G][S][17]: bias gradient (16) and mean loss (1) of every slot
    float* zpart;            // [R][2][G][maxrows][16] partial logits exchanged inside a cluster
    int32_t maxrows;
    uint32_t* zx;            // [R][3][G][64][16] exchange of the steady-state kernel: every word 0xFFFFFFFF until written
    uint32_t* dx;            // [R][4][64][16] delta on its way from a cluster's helper workgroup to its slices, same convention
    int32_t* fallback;       // [R] set by a cluster that does not sit on one XCD: the replica was left untouched
    unsigned int* arrive;    // [R][kArriveStride] arrival counters of the cluster exchange, zero at launch:
                             // word 0 fenced exchanges, word kArriveFast shared-L2 exchanges (a cache line each)
    int32_t* abort_flag;
    uint32_t spin_limit;
    float* agg_out;          // nullable: averaged gradient of the last update of replica 0
    int32_t* xcc_ids;        // [R][G + 1] XCD each workgroup of a cluster runs on (checked on the device); kernels without a helper use [R][G]
    int32_t allow_fast;      // 1: exchange through the shared L2 once a cluster is known to sit on one XCD
    // Steady-state kernel, full launches only: CUs per XCD and resident workgroups per CU.  When set, the
    // workgroup slots of an XCD are dealt out so that the clusters that share CUs share all of them in pairs
    // (0: clusters take consecutive slots).
    int32_t pair_cus, pair_layers;
    // Steady-state kernel: 1 when the launch has more workgroups than the device has CUs, so that workgroups share
    // CUs.  Polling for the exchange then pauses longer between rounds: the re-reads of a waiting workgroup compete
    // with the memory operations of the one it shares the CU with.
    int32_t shared_cus;
    int32_t prof_wave, prof_a, prof_b;   // diagnostics: wave and the pair of marks of the phase profile
    int32_t debug_flags;                 // test switches set by the host (SSGD_DEBUG_FLAGS): bit 1 makes the odd replicas take the path of a cluster spread over XCDs
    int64_t prof_base;                   // first word of the steady-state kernel's part of prof
    int64_t prof_helper;                 // offset, from prof_base, of the helper workgroups' words (one per replica)
    // Steady-state kernel: 1 for a synchronous variant whose iteration does not fit one 64-row tile.  The rows of the
    // K mini-batches are then taken 64 at a time, each tile through the whole forward / exchange / backward schedule,
    // the gradient summed over the tiles and the update applied after the last one.
    int32_t chunked;
    unsigned long long* prof;   // nullable diagnostics: [R][G][20] cycles per phase (general kernel), then [R][G][2] cycles of the profiled interval (steady-state kernel: compute wave, loader wave)
};
int linear_max_resident_groups(int nbw, size_t lds_bytes);
size_t linear_lds_bytes(int nbw, int C, int S, bool parks);
hipError_t launch_linear(const LinArgs& a, int nbw, hipStream_t s);
// Single-tile steady-state kernel (256 columns per workgroup, same state layout as launch_linear with nbw = 4).
// max_records: the most mini-batches any step of the segment computes.
bool linear_tile_supports(const LinArgs& a, int max_records);
size_t linear_tile_lds_bytes(int C, int S, int Kcap);
int linear_tile_resident_groups(size_t lds_bytes);
hipError_t launch_linear_tile(const LinArgs& a, hipStream_t s);
// Steady-state kernel of K-async with at most 8 workers (linear_defer.hip): one workgroup per CU, the gradients in
// flight in LDS, the gradient contraction of a tile one version behind its forward pass.  Same state layout.
bool linear_defer_supports(const LinArgs& a);
size_t linear_defer_lds_bytes(int C, int S);
int linear_defer_replicas_per_launch(int G, int cus);
hipError_t launch_linear_defer(const LinArgs& a, hipStream_t s);

// Gradient of that objective (full_grad.hip): `scratch` holds full_grad_scratch_floats floats, `out` |w| floats (device).
bool full_grad_supports(int kind, int d, int C);
int64_t full_grad_scratch_floats(int64_t N, int d, int C, int* chunks_out);
hipError_t launch_full_grad(int kind, const float* X, const void* y, int64_t N, int d, int C, const float* w,
                            float* scratch, float* out, int cus, hipStream_t s);
// The static scratch array of full_grad.hip (one copy per GPU, held until the process ends): its size, the per-device
// look-up of its address (call once with the device current), and the address on the current device.
int64_t full_grad_static_scratch_floats();
hipError_t full_grad_static_scratch_prepare();
float* full_grad_static_scratch();
// Objective over the whole data set for one parameter vector of a linear model (full_loss.hip): partial sums of the
// per-sample losses, one fp64 per workgroup.
bool full_loss_supports(int kind, int d, int C);
hipError_t launch_full_loss(int kind, const float* X, const void* y, int64_t N, int d, int C, const float* w, double* partial,
                            int blocks, hipStream_t s);

// Message behind ssgd_last_error(NULL), for the entry points that take no context (api.hip).
void set_global_error(const std::string& msg);

}  // namespace ssgd
