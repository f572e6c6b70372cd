// C ABI of the library (see include/ssgd.h): argument checks, device state, and the
// host loop that alternates schedule segments with gradient/update launches.
#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <string>
#include <vector>

#include "../../include/ssgd.h"
#include "common.hpp"
#include "mlp.hpp"

using namespace ssgd;

namespace {

thread_local std::string g_err;

struct DevBuf {
    void* p = nullptr;
    size_t bytes = 0;
    hipError_t alloc(size_t n) {
        bytes = n;
        return hipMalloc(&p, n ? n : 1);
    }
    void release() { if (p) (void)hipFree(p); p = nullptr; }
    template <class T> T* as() const { return reinterpret_cast<T*>(p); }
};

}  // namespace

struct ssgd_ctx {
    ssgd_model model{};
    int32_t P = 0, K0 = 0, m = 0, mp = 0, variant = 0, R = 0;
    ssgd_adasync ada{};
    Dist dist{};
    DevBuf table;
    double lr = 0;
    uint64_t seed = 0;
    hipStream_t stream = nullptr;
    hipStream_t side = nullptr;     // second stream for the schedule of the network's next piece (default priority)
    int32_t* host_rows = nullptr;   // pinned: copies of replica 0's K, tau and sel rows of the segment being run (network)
    size_t host_rows_words = 0;
    int device = 0;
    int64_t nw = 0;
    int32_t Kcap = 0, S = 0, G = 0, nbw = 0, maxrows = 0, table_ord = 1;
    int tile_resident_groups = 0, defer_per_launch = 0, cu_count = 0;
    LinArgs lin{};
    int64_t j = 0;
    int32_t win_cnt = 0;
    bool broken = false;

    Trace tr{};
    DevBuf tr_t, tr_loss, tr_K, tr_sel, tr_tau, tr_ord;
    WorkerState ws{};
    DevBuf ws_finish, ws_tau, ws_ord, ws_clock, ws_curK, ws_winprev, ws_winidx, ws_F0, ws_intstart, ws_crossed, ws_ndone;
    DevBuf params, park, park_small, zpart, zx, dx, fallback, arrive, abort_flag, xcc_ids, prof;
    int resident_groups = 0;
    size_t lds_bytes = 0;
    std::vector<MlpState*> mlp;      // two-layer network: one state per replica

    double last_ms = 0;
    int64_t last_launches = 0;
    std::string err;
};

namespace {

}  // namespace
namespace ssgd { void set_global_error(const std::string& msg) { g_err = msg; } }
namespace {
ssgd_status fail(ssgd_ctx* c, ssgd_status st, const std::string& msg) {
    if (c) c->err = msg; else g_err = msg;
    return st;
}

#define HIP_OK(c, call)                                                                      \
    do {                                                                                     \
        hipError_t e_ = (call);                                                              \
        if (e_ != hipSuccess)                                                                \
            return fail((c), e_ == hipErrorOutOfMemory ? SSGD_ENOMEM : SSGD_EDEVICE,          \
                        std::string(#call) + ": " + hipGetErrorString(e_));                  \
    } while (0)

__global__ void init_workers_kernel(WorkerState ws, Dist dist, uint64_t seed, int P, int R, int K, int variant,
                                    int table_ord) {
    const int q = blockIdx.x * blockDim.x + threadIdx.x;
    if (q < R) {
        ws.clock[q] = 0.0; ws.curK[q] = K; ws.win_prev[q] = 0.0; ws.win_index[q] = 0; ws.F0[q] = -1.0;
        ws.int_start[q] = 0; ws.crossed[q] = 0; ws.n_done[q] = 0;
    }
    if (q >= R * P) return;
    const int rep = q / P, w = q % P;
    ws.tau[q] = 0; ws.ord[q] = 0;
    // all workers are launched afresh at time 0 (as in the proof of Lemma 4)
    ws.finish[q] = (variant >= kAsync) ? (double)delay(dist, seed, kDelay, 0, rep, P, table_ord, w, 0, 0) : 0.0;
}

__global__ void debug_delay_kernel(Dist dist, const uint32_t* bits, int64_t n, float* out) {
    const int64_t q = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (q < n) out[q] = delay_from_bits(dist, bits[q]);
}

__global__ void debug_batch_kernel(uint64_t seed, uint32_t replica, uint32_t worker, uint32_t ordinal,
                                   uint32_t version, int m, uint32_t N, uint32_t* out) {
    const int s = blockIdx.x * blockDim.x + threadIdx.x;
    if (s < m) out[s] = batch_index(seed, replica, worker, ordinal, version, (uint32_t)s, N);
}

// A plain streaming read: every thread takes 16-byte words a whole grid apart; the words are folded into a value
// that is stored only if it equals a pattern the data will not have, which keeps the loads alive.
typedef uint32_t stream_u32x4 __attribute__((ext_vector_type(4)));
__global__ __launch_bounds__(256) void stream_read_kernel(const stream_u32x4* src, int64_t n16, uint32_t* sink) {
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    stream_u32x4 acc = {0u, 0u, 0u, 0u};
    int64_t q = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    for (; q + 3 * stride < n16; q += 4 * stride) {
        const stream_u32x4 v0 = __builtin_nontemporal_load(src + q), v1 = __builtin_nontemporal_load(src + q + stride);
        const stream_u32x4 v2 = __builtin_nontemporal_load(src + q + 2 * stride), v3 = __builtin_nontemporal_load(src + q + 3 * stride);
        acc ^= v0 ^ v1 ^ v2 ^ v3;
    }
    for (; q < n16; q += stride) acc ^= __builtin_nontemporal_load(src + q);
    if ((acc.x ^ acc.y) == 0x9E3779B9u && (acc.z ^ acc.w) == 0x7F4A7C15u) sink[0] = acc.x;
}

bool dist_ok(const ssgd_delay_dist* d) {
    if (!d) return false;
    switch (d->kind) {
    case SSGD_EXP: return d->rate > 0;
    case SSGD_SHIFTED_EXP: return d->rate > 0 && d->shift >= 0;
    case SSGD_PARETO: return d->alpha > 0 && d->scale > 0;
    case SSGD_TABLE: return d->table != nullptr && d->table_len > 0;
    default: return false;
    }
}

// Host description -> device description; TABLE delays are copied into `table`.
hipError_t make_dist(const ssgd_delay_dist* d, DevBuf* table, Dist* out) {
    out->kind = d->kind;
    out->shift = (float)d->shift; out->rate = (float)d->rate;
    out->alpha = (float)d->alpha; out->scale = (float)d->scale;
    out->table = nullptr; out->table_len = 0;
    if (d->kind == SSGD_TABLE) {
        hipError_t e = table->alloc(sizeof(float) * (size_t)d->table_len);
        if (e != hipSuccess) return e;
        e = hipMemcpy(table->p, d->table, sizeof(float) * (size_t)d->table_len, hipMemcpyHostToDevice);
        if (e != hipSuccess) return e;
        out->table = table->as<float>();
        out->table_len = d->table_len;
    }
    return hipSuccess;
}

ssgd_status grow_trace(ssgd_ctx* c, int64_t need) {
    if (need <= c->tr.cap) return SSGD_OK;
    int64_t cap = std::max<int64_t>(need, std::max<int64_t>(256, 2 * c->tr.cap));
    const int64_t R = c->R, W = c->Kcap, old = c->tr.cap, used = c->j;
    DevBuf nt, nl, nk, ns, na, no;
    // the new arrays are released again if an allocation or a copy fails: the old trace stays in place
    struct Temps { DevBuf* b[6]; bool keep = false; ~Temps() { if (!keep) for (DevBuf* q : b) q->release(); } } temps{{&nt, &nl, &nk, &ns, &na, &no}};
    HIP_OK(c, nt.alloc(sizeof(double) * R * cap));
    HIP_OK(c, nl.alloc(sizeof(float) * R * cap));
    HIP_OK(c, nk.alloc(sizeof(int32_t) * R * cap));
    HIP_OK(c, ns.alloc(sizeof(int32_t) * R * cap * W));
    HIP_OK(c, na.alloc(sizeof(int32_t) * R * cap * W));
    HIP_OK(c, no.alloc(sizeof(int32_t) * R * cap * W));
    if (used > 0) {
        HIP_OK(c, hipStreamSynchronize(c->stream));
        for (int64_t r = 0; r < R; ++r) {
            HIP_OK(c, hipMemcpy(nt.as<double>() + r * cap, c->tr.t + r * old, sizeof(double) * used, hipMemcpyDeviceToDevice));
            HIP_OK(c, hipMemcpy(nl.as<float>() + r * cap, c->tr.loss + r * old, sizeof(float) * used, hipMemcpyDeviceToDevice));
            HIP_OK(c, hipMemcpy(nk.as<int32_t>() + r * cap, c->tr.K + r * old, sizeof(int32_t) * used, hipMemcpyDeviceToDevice));
            HIP_OK(c, hipMemcpy(ns.as<int32_t>() + r * cap * W, c->tr.sel + r * old * W, sizeof(int32_t) * used * W, hipMemcpyDeviceToDevice));
            HIP_OK(c, hipMemcpy(na.as<int32_t>() + r * cap * W, c->tr.tau + r * old * W, sizeof(int32_t) * used * W, hipMemcpyDeviceToDevice));
            HIP_OK(c, hipMemcpy(no.as<int32_t>() + r * cap * W, c->tr.ord + r * old * W, sizeof(int32_t) * used * W, hipMemcpyDeviceToDevice));
        }
    }
    temps.keep = true;
    c->tr_t.release(); c->tr_loss.release(); c->tr_K.release(); c->tr_sel.release(); c->tr_tau.release(); c->tr_ord.release();
    c->tr_t = nt; c->tr_loss = nl; c->tr_K = nk; c->tr_sel = ns; c->tr_tau = na; c->tr_ord = no;
    c->tr.t = nt.as<double>(); c->tr.loss = nl.as<float>(); c->tr.K = nk.as<int32_t>();
    c->tr.sel = ns.as<int32_t>(); c->tr.tau = na.as<int32_t>(); c->tr.ord = no.as<int32_t>();
    c->tr.cap = cap;
    return SSGD_OK;
}

int chunks_for(int n_rec, int mp) {
    if (mp <= 64) { const int rpc = 64 / mp; return (n_rec + rpc - 1) / rpc; }
    return n_rec * ((mp + 63) / 64);
}

// One launch per group of co-resident replicas; `mode` selects the kernel.
enum LinearKernel { kGeneralKernel = 0, kTileKernel = 1, kDeferKernel = 2 };
ssgd_status launch_steps(ssgd_ctx* c, int64_t v0, int64_t n, float* agg_out, int mode,
                         std::vector<std::pair<hipEvent_t, hipEvent_t>>* events) {
    const bool tile = mode != kGeneralKernel;
    // a cluster stays on one XCD (block ids congruent modulo 8), so the resident slots count per XCD
    const int resident = tile ? c->tile_resident_groups : c->resident_groups;
    const int per_launch = mode == kDeferKernel ? c->defer_per_launch : std::max(1, 8 * ((resident / 8) / c->G));
    HIP_OK(c, hipMemsetAsync(c->arrive.p, 0, sizeof(unsigned int) * kArriveStride * c->R, c->stream));
    if (tile) HIP_OK(c, hipMemsetAsync(c->zx.p, 0xFF, sizeof(uint32_t) * 3 * 1024 * (size_t)c->R * c->G, c->stream));
    if (mode == kDeferKernel) {
        HIP_OK(c, hipMemsetAsync(c->dx.p, 0xFF, sizeof(uint32_t) * 4 * 1024 * (size_t)c->R, c->stream));
        HIP_OK(c, hipMemsetAsync(c->fallback.p, 0, sizeof(int32_t) * (size_t)c->R, c->stream));
    }
    if (getenv("SSGD_DEBUG"))
        fprintf(stderr, "ssgd launch: v0=%lld n=%lld tile=%d resident=%d per_launch=%d R=%d\n", (long long)v0, (long long)n,
                (int)tile, resident, per_launch, c->R);
    for (int r0 = 0; r0 < c->R; r0 += per_launch) {
        LinArgs a = c->lin;
        a.replica0 = r0; a.replicas = std::min(per_launch, c->R - r0);
        a.tr = c->tr;
        a.v0 = v0; a.nsteps = n;
        a.agg_out = agg_out;
        a.pair_cus = 0; a.pair_layers = 0;
        a.shared_cus = (a.replicas * c->G > c->cu_count) ? 1 : 0;
        a.prof_wave = 0; a.prof_a = -1; a.prof_b = -1; a.prof_base = (int64_t)c->R * c->G * 20; a.prof_helper = (int64_t)c->R * c->G * 2;
        if (const char* e = getenv("SSGD_PHASE_PROFILE")) (void)sscanf(e, "%d,%d,%d", &a.prof_a, &a.prof_b, &a.prof_wave);
        a.debug_flags = 0;
        if (const char* e = getenv("SSGD_DEBUG_FLAGS")) a.debug_flags = atoi(e);
        if (mode == kTileKernel && a.replicas == per_launch && c->cu_count % 8 == 0 && resident % c->cu_count == 0 && !getenv("SSGD_NO_PAIRING")) {
            a.pair_cus = c->cu_count / 8;
            a.pair_layers = resident / c->cu_count;
            // the dealt-out layout must hold as many clusters per XCD as the consecutive one
            const int nb = a.pair_cus / c->G, Lr = a.pair_cus - nb * c->G;
            if (8 * (nb * a.pair_layers + (Lr * a.pair_layers) / c->G) < a.replicas) { a.pair_cus = 0; a.pair_layers = 0; }
        }
        hipEvent_t e0 = nullptr, e1 = nullptr;
        if (events) {
            HIP_OK(c, hipEventCreate(&e0)); HIP_OK(c, hipEventCreate(&e1));
            HIP_OK(c, hipEventRecord(e0, c->stream));
        }
        HIP_OK(c, mode == kDeferKernel ? launch_linear_defer(a, c->stream)
                                       : (tile ? launch_linear_tile(a, c->stream) : launch_linear(a, c->nbw, c->stream)));
        if (events) { HIP_OK(c, hipEventRecord(e1, c->stream)); events->push_back({e0, e1}); }
    }
    if (mode == kDeferKernel) {
        // A cluster that found itself spread over XCDs has left its replica untouched: those replicas take the same
        // updates through the kernel that can exchange across XCDs.
        std::vector<int32_t> fb((size_t)c->R);
        HIP_OK(c, hipMemcpyAsync(fb.data(), c->fallback.p, sizeof(int32_t) * fb.size(), hipMemcpyDeviceToHost, c->stream));
        HIP_OK(c, hipStreamSynchronize(c->stream));
        bool any = false;
        for (int r = 0; r < c->R; ++r) any = any || fb[r] != 0;
        if (any) {
            HIP_OK(c, hipMemsetAsync(c->arrive.p, 0, sizeof(unsigned int) * kArriveStride * c->R, c->stream));
            HIP_OK(c, hipMemsetAsync(c->zx.p, 0xFF, sizeof(uint32_t) * 3 * 1024 * (size_t)c->R * c->G, c->stream));
            for (int r = 0; r < c->R; ++r) {
                if (!fb[r]) continue;
                LinArgs a = c->lin;
                a.replica0 = r; a.replicas = 1;
                a.tr = c->tr;
                a.v0 = v0; a.nsteps = n;
                a.agg_out = agg_out;
                a.pair_cus = 0; a.pair_layers = 0; a.shared_cus = 0;
                a.prof_wave = 0; a.prof_a = -1; a.prof_b = -1; a.prof_base = (int64_t)c->R * c->G * 20; a.prof_helper = (int64_t)c->R * c->G * 2;
                a.debug_flags = 0;
                if (!linear_tile_supports(a, c->Kcap)) return fail(c, SSGD_EDEVICE, "a cluster was spread over XCDs and no other kernel takes its shape");
                HIP_OK(c, launch_linear_tile(a, c->stream));
            }
        }
    }
    return SSGD_OK;
}

ssgd_status run_segment_linear(ssgd_ctx* c, int64_t v0, int64_t n, float* agg_out,
                               std::vector<std::pair<hipEvent_t, hipEvent_t>>* events) {
    LinArgs& a = c->lin;
    a.kind = c->model.kind; a.d = c->model.d; a.C = (c->model.kind == SSGD_LSQ) ? 1 : c->model.classes;
    a.m = c->m; a.mp = c->mp; a.P = c->P; a.variant = c->variant;
    a.X = c->model.X; a.y = c->model.y; a.N = (uint32_t)c->model.N;
    a.lr = (float)c->lr; a.seed = c->seed;
    a.G = c->G; a.S = c->S;
    a.tr = c->tr;
    a.params = c->params.as<float>(); a.park = c->park.as<float>(); a.park_small = c->park_small.as<float>();
    a.zpart = c->zpart.as<float>(); a.maxrows = c->maxrows;
    a.zx = c->zx.as<uint32_t>();
    a.dx = c->dx.as<uint32_t>();
    a.fallback = c->fallback.as<int32_t>();
    a.arrive = c->arrive.as<unsigned int>();
    a.abort_flag = c->abort_flag.as<int32_t>();
    a.spin_limit = 4000000u;
    if (const char* e = getenv("SSGD_SPIN_LIMIT")) a.spin_limit = (uint32_t)strtoul(e, nullptr, 10);
    a.xcc_ids = c->xcc_ids.as<int32_t>();
    a.allow_fast = 1;
    if (const char* e = getenv("SSGD_EXCHANGE")) a.allow_fast = (strcmp(e, "fenced") == 0) ? 0 : 1;
    a.prof = c->prof.as<unsigned long long>();
    a.agg_out = agg_out;

    // The steady-state kernel runs the steps whose mini-batches fit one tile; step 0 of K-async
    // (all P workers start) and every other shape go through the general kernel.
    bool tile = c->nbw == 4 && c->tile_resident_groups >= c->G;
    bool defer = c->nbw == 4 && c->defer_per_launch >= 1 && c->tile_resident_groups >= c->G;
    if (const char* e = getenv("SSGD_KERNEL")) {          // diagnostics: "general" or "tile" keep the later kernels out
        tile = tile && strcmp(e, "general") != 0;
        defer = defer && strcmp(e, "general") != 0 && strcmp(e, "tile") != 0;
    }
    int64_t head = 0;
    a.v0 = v0;
    a.chunked = 0;
    if (tile || defer) {
        if (c->variant == SSGD_K_ASYNC && v0 == 0) { head = 1; a.v0 = 1; }
        a.chunked = ((c->variant == SSGD_K_SYNC || c->variant == SSGD_K_BATCH_SYNC) && a.mp * c->Kcap > 64) ? 1 : 0;
        tile = tile && linear_tile_supports(a, c->Kcap);
        defer = defer && linear_defer_supports(a);
    }
    if (!tile && !defer && c->variant == SSGD_K_BATCH_ASYNC) return fail(c, SSGD_EINVAL, "K-batch-async: the cluster of this shape does not fit the device");
    if (!tile && !defer) return launch_steps(c, v0, n, agg_out, kGeneralKernel, events);
    if (head > 0) {
        ssgd_status st = launch_steps(c, v0, std::min(head, n), agg_out, kGeneralKernel, events);
        if (st != SSGD_OK) return st;
    }
    if (n > head) return launch_steps(c, v0 + head, n - head, agg_out, defer ? kDeferKernel : kTileKernel, events);
    return SSGD_OK;
}

ssgd_status run_updates(ssgd_ctx* c, int64_t J, float* agg_out) {
    if (c->broken) return fail(c, SSGD_ESTATE, "context is unusable after a device error");
    if (J < 0) return fail(c, SSGD_EINVAL, "J must be >= 0");
    HIP_OK(c, hipSetDevice(c->device));
    std::vector<std::pair<hipEvent_t, hipEvent_t>> events;
    c->last_ms = 0; c->last_launches = 0;
    int64_t remaining = J;
    while (remaining > 0) {
        int64_t seg = remaining;
        if (c->ada.mode == 1) seg = std::min<int64_t>(seg, c->ada.window - c->win_cnt);
        if (c->model.kind == SSGD_MLP2) seg = std::min<int64_t>(seg, 4096);
        ssgd_status st = grow_trace(c, c->j + seg);
        if (st != SSGD_OK) return st;

        SchedArgs sa{};
        sa.tr = c->tr; sa.ws = c->ws; sa.dist = c->dist; sa.seed = c->seed; sa.P = c->P; sa.variant = c->variant;
        sa.table_ord = c->table_ord; sa.replica0 = 0; sa.j0 = c->j; sa.count = seg;
        sa.interval_t = (c->ada.mode >= 2) ? c->ada.interval_t : 0.0;
        // The schedule does not depend on the numerics (K changes only between segments here), so it is written piece by
        // piece on a second stream while the gradient kernels of the piece before run: one wavefront per replica beside
        // kernels that leave it room (the network's updates are separate launches; the steady-state kernel of K-async
        // on the linear models leaves CUs free).  The pieces of the linear models are long: every piece is a launch of
        // its own, which reads the gradients in flight from HBM and writes them back.
        const bool linear_pipe = c->model.kind != SSGD_MLP2 && c->variant == SSGD_K_ASYNC && c->defer_per_launch >= 1 && agg_out == nullptr;
        // (one replica of the network takes the rows of a piece as they come: short pieces, so that the first one of a
        // segment, whose schedule nothing hides, is soon there)
        const int64_t kPiece = c->model.kind == SSGD_MLP2 ? (c->R == 1 ? 16 : 64) : 1024;
        const bool pipelined = (c->model.kind == SSGD_MLP2 || linear_pipe) && c->ada.mode < 2 && seg > kPiece;
        if (pipelined) {
            if (!c->side) HIP_OK(c, hipStreamCreateWithFlags(&c->side, hipStreamNonBlocking));
            hipEvent_t before = nullptr;
            HIP_OK(c, hipEventCreateWithFlags(&before, hipEventDisableTiming));
            hipError_t e = hipEventRecord(before, c->stream);
            if (e == hipSuccess) e = hipStreamWaitEvent(c->side, before, 0);
            std::vector<hipEvent_t> written;
            // One replica of the network: the rows that the host needs of every piece (K, tau, sel of replica 0; one row
            // of sel in front) follow the schedule kernel to pinned memory, and the whole segment is one call below that
            // takes them piece by piece, so that its kernels keep flowing from one piece to the next.
            const bool one_call = c->model.kind == SSGD_MLP2 && c->R == 1;
            const size_t W = (size_t)c->Kcap;
            int32_t *hK = nullptr, *htau = nullptr, *hsel = nullptr;
            if (one_call && e == hipSuccess) {
                const size_t words = (size_t)seg * (1 + 2 * W) + W;
                if (c->host_rows_words < words) {
                    if (c->host_rows) (void)hipHostFree(c->host_rows);
                    c->host_rows = nullptr; c->host_rows_words = 0;
                    e = hipHostMalloc((void**)&c->host_rows, sizeof(int32_t) * words, hipHostMallocDefault);
                    if (e == hipSuccess) c->host_rows_words = words;
                }
                hK = c->host_rows; htau = hK + seg; hsel = htau + (size_t)seg * W;
                if (e == hipSuccess && c->j > 0)
                    e = hipMemcpyAsync(hsel, c->tr.sel + (size_t)(c->j - 1) * W, sizeof(int32_t) * W, hipMemcpyDeviceToHost, c->side);
            }
            for (int64_t off = 0; off < seg && e == hipSuccess; off += kPiece) {
                sa.j0 = c->j + off; sa.count = std::min(kPiece, seg - off);
                launch_schedule(sa, c->R, c->side);
                if (one_call) {
                    const size_t cnt = (size_t)sa.count;
                    e = hipMemcpyAsync(hK + off, c->tr.K + sa.j0, sizeof(int32_t) * cnt, hipMemcpyDeviceToHost, c->side);
                    if (e == hipSuccess) e = hipMemcpyAsync(htau + (size_t)off * W, c->tr.tau + (size_t)sa.j0 * W, sizeof(int32_t) * cnt * W, hipMemcpyDeviceToHost, c->side);
                    if (e == hipSuccess) e = hipMemcpyAsync(hsel + (size_t)(off + 1) * W, c->tr.sel + (size_t)sa.j0 * W, sizeof(int32_t) * cnt * W, hipMemcpyDeviceToHost, c->side);
                    if (e != hipSuccess) break;
                }
                hipEvent_t ev = nullptr;
                e = hipEventCreateWithFlags(&ev, hipEventDisableTiming);
                if (e == hipSuccess) { written.push_back(ev); e = hipEventRecord(ev, c->side); }
            }
            std::string msg;
            size_t k = 0;
            ssgd_status lin_st = SSGD_OK;
            if (one_call && e == hipSuccess) {
                // (the kernels are launched after the host has seen a piece's event: no stream has to wait for it)
                MlpPieces pc{written.data(), (int)written.size(), kPiece, hK, htau, hsel};
                e = mlp_run_segment(c->mlp.data(), c->R, c->tr, c->ws, c->j, seg, agg_out, c->stream, &c->last_ms, &c->last_launches, &msg, &pc);
            }
            for (int64_t off = 0; off < seg && e == hipSuccess && lin_st == SSGD_OK && !one_call; off += kPiece, ++k) {
                e = hipStreamWaitEvent(c->stream, written[k], 0);
                if (e != hipSuccess) break;
                if (c->model.kind == SSGD_MLP2)
                    e = mlp_run_segment(c->mlp.data(), c->R, c->tr, c->ws, c->j + off, std::min(kPiece, seg - off), agg_out, c->stream,
                                        &c->last_ms, &c->last_launches, &msg);
                else
                    lin_st = run_segment_linear(c, c->j + off, std::min(kPiece, seg - off), agg_out, &events);
            }
            if (lin_st != SSGD_OK) {
                (void)hipStreamSynchronize(c->side);
                (void)hipEventDestroy(before);
                for (hipEvent_t ev : written) (void)hipEventDestroy(ev);
                c->broken = true;
                return lin_st;
            }
            if (e != hipSuccess) (void)hipStreamSynchronize(c->side);
            (void)hipEventDestroy(before);
            for (hipEvent_t ev : written) (void)hipEventDestroy(ev);
            if (e != hipSuccess) { c->broken = true; return fail(c, SSGD_EDEVICE, "pipelined segment: " + (msg.empty() ? std::string(hipGetErrorString(e)) : msg)); }
        } else {
            launch_schedule(sa, c->R, c->stream);
            HIP_OK(c, hipGetLastError());
        }
        if (c->ada.mode >= 2) {
            int64_t nd = 0;
            HIP_OK(c, hipMemcpyAsync(&nd, c->ws.n_done, sizeof(nd), hipMemcpyDeviceToHost, c->stream));
            HIP_OK(c, hipStreamSynchronize(c->stream));
            seg = nd;
        }
        if (pipelined) {
            // done above
        } else if (c->model.kind == SSGD_MLP2) {
            std::string msg;
            hipError_t e = mlp_run_segment(c->mlp.data(), c->R, c->tr, c->ws, c->j, seg, agg_out, c->stream, &c->last_ms, &c->last_launches, &msg);
            if (e != hipSuccess) { c->broken = true; return fail(c, SSGD_EDEVICE, "mlp segment: " + msg); }
        } else {
            st = run_segment_linear(c, c->j, seg, agg_out, &events);
            if (st != SSGD_OK) { c->broken = true; return st; }
        }
        c->j += seg;
        remaining -= seg;
        if (c->ada.mode != 0) {
            AdaArgs aa{};
            aa.tr = c->tr; aa.ws = c->ws; aa.mode = c->ada.mode; aa.K0 = c->ada.K0; aa.Kmax = c->ada.Kmax;
            aa.window = c->ada.window; aa.P = c->P; aa.rel_tol = c->ada.rel_tol; aa.j_end = c->j;
            aa.window_closed = 0;
            if (c->ada.mode == 1) {
                c->win_cnt += (int32_t)seg;
                if (c->win_cnt == c->ada.window) { aa.window_closed = 1; c->win_cnt = 0; }
            }
            launch_adasync(aa, c->R, c->stream);
            HIP_OK(c, hipGetLastError());
        }
    }
    HIP_OK(c, hipStreamSynchronize(c->stream));
    for (auto& ev : events) {
        float ms = 0;
        if (hipEventElapsedTime(&ms, ev.first, ev.second) == hipSuccess) { c->last_ms += ms; c->last_launches += 1; }
        (void)hipEventDestroy(ev.first); (void)hipEventDestroy(ev.second);
    }
    int32_t aborted = 0;
    HIP_OK(c, hipMemcpy(&aborted, c->abort_flag.p, sizeof(aborted), hipMemcpyDeviceToHost));
    if (aborted) {
        c->broken = true;
        return fail(c, SSGD_EDEVICE, "cluster exchange timed out: the workgroups of a replica were not co-resident");
    }
    return SSGD_OK;
}

}  // namespace

// the C ABI is all the library exports (everything else is built with hidden visibility)
#pragma GCC visibility push(default)
extern "C" {

ssgd_status ssgd_create(const ssgd_model* model, int32_t P, int32_t K, int32_t m, int32_t variant,
                        const ssgd_delay_dist* dist, double lr, uint64_t seed, int32_t replicas,
                        const ssgd_adasync* adasync, void* hip_stream, ssgd_ctx** out) {
    if (!model || !out) return fail(nullptr, SSGD_EINVAL, "model and out must not be null");
    if (!dist_ok(dist)) return fail(nullptr, SSGD_EINVAL, "invalid delay distribution");
    if (!model->X || !model->y || model->N < 1 || model->N >= (1ll << 32) || model->d < 1)
        return fail(nullptr, SSGD_EINVAL, "invalid data set description");
    if (variant < SSGD_K_SYNC || variant > SSGD_K_BATCH_ASYNC) return fail(nullptr, SSGD_EINVAL, "unknown variant");
    if (P < 1 || P > kMaxWorkers || K < 1 || m < 1 || m > 65535 || replicas < 1 || !(lr >= 0))
        return fail(nullptr, SSGD_EINVAL, "P, K, m, replicas or lr out of range");
    ssgd_adasync ada{};
    ada.mode = 0; ada.K0 = K; ada.Kmax = K; ada.window = 0;
    if (adasync && adasync->mode != 0) {
        ada = *adasync;
        if (ada.mode < 1 || ada.mode > 3 || ada.Kmax < K || ada.K0 < 1) return fail(nullptr, SSGD_EINVAL, "invalid adasync block");
        if (ada.mode == 1 && ada.window < 1) return fail(nullptr, SSGD_EINVAL, "adasync window must be >= 1");
        if (ada.mode >= 2 && (!(ada.interval_t > 0) || replicas != 1)) return fail(nullptr, SSGD_EINVAL, "adasync modes 2, 3 need interval_t > 0 and replicas == 1");
        if (ada.mode == 3 && ada.K0 >= P) return fail(nullptr, SSGD_EINVAL, "adasync mode 3 needs K0 < P");
    }
    const int32_t Kcap = ada.Kmax;
    if ((variant == SSGD_K_SYNC || variant == SSGD_K_ASYNC) && Kcap > P) return fail(nullptr, SSGD_EINVAL, "K must not exceed P");
    if (Kcap > kMaxWorkers) return fail(nullptr, SSGD_EINVAL, "K must not exceed 256");
    if (variant == SSGD_K_BATCH_ASYNC) {
        if (ada.mode >= 2) return fail(nullptr, SSGD_EINVAL, "K-batch-async runs with a fixed K or plateau doubling");
        // the linear models run this variant through the steady-state kernel only
        const int32_t classes = model->kind == SSGD_LSQ ? 1 : model->classes;
        if (model->kind != SSGD_MLP2 && (model->d % 4 != 0 || classes > 15 || Kcap > 64))
            return fail(nullptr, SSGD_EINVAL, "K-batch-async: linear models need d % 4 == 0, at most 15 classes, K <= 64");
    }
    if (model->kind == SSGD_LSQ) {
        if (model->bf16) return fail(nullptr, SSGD_EINVAL, "bf16 is for the MLP only");
    } else if (model->kind == SSGD_SOFTMAX) {
        if (model->classes < 2 || model->classes > kClassPad || model->bf16) return fail(nullptr, SSGD_EINVAL, "softmax needs 2..16 classes, bf16 = 0");
    } else if (model->kind == SSGD_MLP2) {
        // the same limits as mlp_create, so that every invalid shape is refused here, before anything is allocated
        if (model->classes < 2 || model->classes > kClassPad || model->hidden < 128 || model->hidden % 128 || model->d % 128 ||
            !model->bf16 || m > 64 || (replicas > 1 && ada.mode >= 2))
            return fail(nullptr, SSGD_EINVAL, "MLP needs 2..16 classes, hidden % 128 == 0, d % 128 == 0, m <= 64, bf16 = 1; several replicas with a fixed K or plateau doubling only");
    } else {
        return fail(nullptr, SSGD_EINVAL, "unknown model kind");
    }

    ssgd_ctx* c = new (std::nothrow) ssgd_ctx();
    if (!c) return fail(nullptr, SSGD_ENOMEM, "host allocation failed");
    auto bail = [&](ssgd_status st, const std::string& msg) { ssgd_destroy(c); return fail(nullptr, st, msg); };
#define HIP_C(call)                                                                                     \
    do {                                                                                                \
        hipError_t e_ = (call);                                                                         \
        if (e_ != hipSuccess)                                                                           \
            return bail(e_ == hipErrorOutOfMemory ? SSGD_ENOMEM : SSGD_EDEVICE, std::string(#call) + ": " + hipGetErrorString(e_)); \
    } while (0)

    c->model = *model; c->P = P; c->K0 = K; c->m = m; c->mp = (m + 3) / 4 * 4; c->variant = variant; c->R = replicas;
    c->ada = ada; c->lr = lr; c->seed = seed; c->stream = (hipStream_t)hip_stream; c->Kcap = Kcap;
    c->table_ord = (variant == SSGD_K_BATCH_SYNC || variant == SSGD_K_BATCH_ASYNC) ? Kcap + 1 : 1;
    HIP_C(hipGetDevice(&c->device));
    HIP_C(make_dist(dist, &c->table, &c->dist));
    const int64_t R = replicas;
    if (model->kind == SSGD_LSQ) c->nw = model->d;
    else if (model->kind == SSGD_SOFTMAX) c->nw = (int64_t)model->classes * model->d + model->classes;
    else c->nw = (int64_t)model->hidden * model->d + model->hidden + (int64_t)model->classes * model->hidden + model->classes;

    HIP_C(c->ws_finish.alloc(sizeof(double) * R * P)); HIP_C(c->ws_tau.alloc(sizeof(int32_t) * R * P));
    HIP_C(c->ws_ord.alloc(sizeof(int32_t) * R * P)); HIP_C(c->ws_clock.alloc(sizeof(double) * R));
    HIP_C(c->ws_curK.alloc(sizeof(int32_t) * R)); HIP_C(c->ws_winprev.alloc(sizeof(double) * R));
    HIP_C(c->ws_winidx.alloc(sizeof(int64_t) * R)); HIP_C(c->ws_F0.alloc(sizeof(double) * R));
    HIP_C(c->ws_intstart.alloc(sizeof(int64_t) * R)); HIP_C(c->ws_crossed.alloc(sizeof(int32_t) * R));
    HIP_C(c->ws_ndone.alloc(sizeof(int64_t) * R));
    c->ws.finish = c->ws_finish.as<double>(); c->ws.tau = c->ws_tau.as<int32_t>(); c->ws.ord = c->ws_ord.as<int32_t>();
    c->ws.clock = c->ws_clock.as<double>(); c->ws.curK = c->ws_curK.as<int32_t>(); c->ws.win_prev = c->ws_winprev.as<double>();
    c->ws.win_index = c->ws_winidx.as<int64_t>(); c->ws.F0 = c->ws_F0.as<double>(); c->ws.int_start = c->ws_intstart.as<int64_t>();
    c->ws.crossed = c->ws_crossed.as<int32_t>(); c->ws.n_done = c->ws_ndone.as<int64_t>();
    {
        const int n = (int)std::max<int64_t>(R * P, R);
        hipLaunchKernelGGL(init_workers_kernel, dim3((n + 255) / 256), dim3(256), 0, c->stream, c->ws, c->dist, seed, P,
                           (int)R, K, variant, c->table_ord);
        HIP_C(hipGetLastError());
    }
    c->tr.Kcap = Kcap; c->tr.cap = 0;
    HIP_C(c->abort_flag.alloc(sizeof(int32_t)));
    HIP_C(hipMemsetAsync(c->abort_flag.p, 0, sizeof(int32_t), c->stream));

    if (model->kind == SSGD_MLP2) {
        std::string msg;
        for (int r = 0; r < replicas; ++r) {
            MlpState* ms = nullptr;
            hipError_t e = mlp_create(&ms, *model, P, m, variant, Kcap, lr, seed, r, c->mlp.empty() ? nullptr : c->mlp[0], c->stream, &msg);
            if (e != hipSuccess)
                return bail(e == hipErrorOutOfMemory ? SSGD_ENOMEM : (e == hipErrorInvalidValue ? SSGD_EINVAL : SSGD_EDEVICE), "mlp_create: " + msg);
            c->mlp.push_back(ms);
        }
    } else {
        const int d = model->d;
        c->nbw = d <= 64 ? 1 : (d <= 128 ? 2 : 4);
        if (const char* e = getenv("SSGD_NBW")) { const int v = atoi(e); if (v == 1 || v == 2 || v == 4) c->nbw = v; }
        if (variant == SSGD_K_BATCH_ASYNC) c->nbw = 4;   // only the steady-state kernel runs this variant: one wide slice for small d
        const int SL = 64 * c->nbw;
        c->G = (d + SL - 1) / SL;
        const bool async = variant == SSGD_K_ASYNC || variant == SSGD_K_BATCH_ASYNC;   // gradients are parked per worker
        c->S = async ? P : Kcap;
        const int C = model->kind == SSGD_LSQ ? 1 : model->classes;
        c->maxrows = 64 * chunks_for(async ? std::max(P, Kcap) : Kcap, c->mp);
        c->lds_bytes = linear_lds_bytes(c->nbw, C, c->S, async);
        if (variant == SSGD_K_BATCH_ASYNC) {
            // the general kernel is never used for this variant; what has to fit is the steady-state kernel's LDS
            if (linear_tile_lds_bytes(C, c->S, Kcap) > 160 * 1024) return bail(SSGD_EINVAL, "too many gradient slots for the LDS of one workgroup");
            c->lds_bytes = std::min<size_t>(c->lds_bytes, 160 * 1024);
        }
        if (c->lds_bytes > 160 * 1024) return bail(SSGD_EINVAL, "too many gradient slots for the LDS of one workgroup");
        c->resident_groups = linear_max_resident_groups(c->nbw, c->lds_bytes);
        if (c->resident_groups < c->G) return bail(SSGD_EINVAL, "d is too large for a co-resident cluster of workgroups");
        { hipDeviceProp_t prop; HIP_C(hipGetDeviceProperties(&prop, c->device)); c->cu_count = prop.multiProcessorCount; }
        if (c->nbw == 4 && C <= 15 && linear_tile_lds_bytes(C, c->S, Kcap) <= 160 * 1024)
            c->tile_resident_groups = linear_tile_resident_groups(linear_tile_lds_bytes(C, c->S, Kcap));
        if (c->nbw == 4 && C <= 15 && variant == SSGD_K_ASYNC && c->S <= 8 && linear_defer_lds_bytes(C, c->S) <= 160 * 1024)
            c->defer_per_launch = linear_defer_replicas_per_launch(c->G, c->cu_count);
        HIP_C(c->params.alloc(sizeof(float) * R * c->nw));
        HIP_C(hipMemsetAsync(c->params.p, 0, sizeof(float) * R * c->nw, c->stream));
        const size_t park_n = (size_t)R * c->G * c->S * 16 * SL;
        HIP_C(c->park.alloc(sizeof(float) * park_n));
        HIP_C(hipMemsetAsync(c->park.p, 0, sizeof(float) * park_n, c->stream));
        HIP_C(c->park_small.alloc(sizeof(float) * R * c->G * c->S * 17));
        HIP_C(hipMemsetAsync(c->park_small.p, 0, sizeof(float) * R * c->G * c->S * 17, c->stream));
        HIP_C(c->zpart.alloc(sizeof(float) * R * 2 * c->G * c->maxrows * 16));
        HIP_C(c->zx.alloc(sizeof(uint32_t) * 3 * 1024 * (size_t)R * c->G));
        HIP_C(c->dx.alloc(sizeof(uint32_t) * 4 * 1024 * (size_t)R));
        HIP_C(c->fallback.alloc(sizeof(int32_t) * (size_t)R));
        HIP_C(c->xcc_ids.alloc(sizeof(int32_t) * R * (c->G + 1)));
        HIP_C(hipMemsetAsync(c->xcc_ids.p, 0xFF, sizeof(int32_t) * R * (c->G + 1), c->stream));
        if (getenv("SSGD_PHASE_PROFILE")) {
            HIP_C(c->prof.alloc(sizeof(unsigned long long) * (R * c->G * 22 + R)));
            HIP_C(hipMemsetAsync(c->prof.p, 0, sizeof(unsigned long long) * (R * c->G * 22 + R), c->stream));
        }
        HIP_C(c->arrive.alloc(sizeof(unsigned int) * kArriveStride * R));
        HIP_C(hipMemsetAsync(c->arrive.p, 0, sizeof(unsigned int) * kArriveStride * R, c->stream));
        // set-up for ssgd_full_gradient_static: this device's address of the library's static scratch array
        HIP_C(full_grad_static_scratch_prepare());
    }
    HIP_C(hipStreamSynchronize(c->stream));
#undef HIP_C
    *out = c;
    return SSGD_OK;
}

ssgd_status ssgd_run(ssgd_ctx* ctx, int64_t J) {
    if (!ctx) return fail(nullptr, SSGD_EINVAL, "null context");
    return run_updates(ctx, J, nullptr);
}

ssgd_status ssgd_reserve_trace(ssgd_ctx* ctx, int64_t updates) {
    if (!ctx) return fail(nullptr, SSGD_EINVAL, "null context");
    if (updates < 0) return fail(ctx, SSGD_EINVAL, "updates must be >= 0");
    HIP_OK(ctx, hipSetDevice(ctx->device));
    return grow_trace(ctx, ctx->j + updates);
}

ssgd_status ssgd_step(ssgd_ctx* ctx, float* agg_grad_out) {
    if (!ctx) return fail(nullptr, SSGD_EINVAL, "null context");
    return run_updates(ctx, 1, agg_grad_out);
}

int64_t ssgd_param_count(const ssgd_ctx* ctx) { return ctx ? ctx->nw : -1; }
int64_t ssgd_updates_done(const ssgd_ctx* ctx) { return ctx ? ctx->j : -1; }
int32_t ssgd_trace_width(const ssgd_ctx* ctx) { return ctx ? ctx->Kcap : -1; }

int32_t ssgd_current_K(const ssgd_ctx* ctx, int32_t replica) {
    if (!ctx || replica < 0 || replica >= ctx->R) return -1;
    int32_t K = -1;
    if (hipSetDevice(ctx->device) != hipSuccess) return -1;
    if (hipMemcpy(&K, ctx->ws.curK + replica, sizeof(K), hipMemcpyDeviceToHost) != hipSuccess) return -1;
    return K;
}

ssgd_status ssgd_get_trace(ssgd_ctx* c, int32_t replica, int64_t from, int64_t n, double* t, float* loss,
                           int32_t* K, int32_t* sel, int32_t* staleness, int32_t* ordinal) {
    if (!c) return fail(nullptr, SSGD_EINVAL, "null context");
    if (replica < 0 || replica >= c->R || from < 0 || n < 0 || from + n > c->j) return fail(c, SSGD_EINVAL, "trace range out of bounds");
    if (n == 0) return SSGD_OK;
    HIP_OK(c, hipSetDevice(c->device));
    HIP_OK(c, hipStreamSynchronize(c->stream));
    const int64_t cap = c->tr.cap, W = c->Kcap, base = (int64_t)replica * cap + from;
    if (t) HIP_OK(c, hipMemcpy(t, c->tr.t + base, sizeof(double) * n, hipMemcpyDeviceToHost));
    if (loss) HIP_OK(c, hipMemcpy(loss, c->tr.loss + base, sizeof(float) * n, hipMemcpyDeviceToHost));
    if (K) HIP_OK(c, hipMemcpy(K, c->tr.K + base, sizeof(int32_t) * n, hipMemcpyDeviceToHost));
    if (sel) HIP_OK(c, hipMemcpy(sel, c->tr.sel + base * W, sizeof(int32_t) * n * W, hipMemcpyDeviceToHost));
    if (ordinal) HIP_OK(c, hipMemcpy(ordinal, c->tr.ord + base * W, sizeof(int32_t) * n * W, hipMemcpyDeviceToHost));
    if (staleness) {
        HIP_OK(c, hipMemcpy(staleness, c->tr.tau + base * W, sizeof(int32_t) * n * W, hipMemcpyDeviceToHost));
        for (int64_t q = 0; q < n; ++q)
            for (int64_t l = 0; l < W; ++l) {
                int32_t& v = staleness[q * W + l];
                if (v >= 0) v = (int32_t)(from + q) - v;   // j - tau
            }
    }
    return SSGD_OK;
}

ssgd_status ssgd_get_params(ssgd_ctx* c, int32_t replica, float* w_out) {
    if (!c || !w_out) return fail(c, SSGD_EINVAL, "null argument");
    if (replica < 0 || replica >= c->R) return fail(c, SSGD_EINVAL, "replica out of range");
    HIP_OK(c, hipSetDevice(c->device));
    HIP_OK(c, hipStreamSynchronize(c->stream));
    const float* src = c->model.kind == SSGD_MLP2 ? mlp_params(c->mlp[(size_t)replica]) : c->params.as<float>() + (int64_t)replica * c->nw;
    HIP_OK(c, hipMemcpy(w_out, src, sizeof(float) * c->nw, hipMemcpyDeviceToHost));
    return SSGD_OK;
}

ssgd_status ssgd_set_params(ssgd_ctx* c, int32_t replica, const float* w_in) {
    if (!c || !w_in) return fail(c, SSGD_EINVAL, "null argument");
    if (replica < 0 || replica >= c->R) return fail(c, SSGD_EINVAL, "replica out of range");
    HIP_OK(c, hipSetDevice(c->device));
    HIP_OK(c, hipStreamSynchronize(c->stream));
    float* dst = c->model.kind == SSGD_MLP2 ? mlp_params(c->mlp[(size_t)replica]) : c->params.as<float>() + (int64_t)replica * c->nw;
    HIP_OK(c, hipMemcpy(dst, w_in, sizeof(float) * c->nw, hipMemcpyHostToDevice));
    return SSGD_OK;
}

ssgd_status ssgd_force_K(ssgd_ctx* c, int32_t K) {
    if (!c) return fail(nullptr, SSGD_EINVAL, "null context");
    if (K < 1 || K > c->Kcap) return fail(c, SSGD_EINVAL, "K out of range");
    HIP_OK(c, hipSetDevice(c->device));
    HIP_OK(c, hipStreamSynchronize(c->stream));
    std::vector<int32_t> ks(c->R, K);
    HIP_OK(c, hipMemcpy(c->ws.curK, ks.data(), sizeof(int32_t) * c->R, hipMemcpyHostToDevice));
    return SSGD_OK;
}

ssgd_status ssgd_full_loss(ssgd_ctx* c, int32_t replica, double* loss_out) {
    if (!c || !loss_out) return fail(c, SSGD_EINVAL, "null argument");
    if (replica < 0 || replica >= c->R) return fail(c, SSGD_EINVAL, "replica out of range");
    if (c->broken) return fail(c, SSGD_ESTATE, "context is unusable after a device error");
    const int C = c->model.kind == SSGD_LSQ ? 1 : c->model.classes;
    if (c->model.kind == SSGD_MLP2) {
        HIP_OK(c, hipSetDevice(c->device));
        std::string msg;
        HIP_OK(c, hipStreamSynchronize(c->stream));
        hipError_t em = mlp_full_loss(c->mlp[(size_t)replica], loss_out, c->stream, &msg);
        if (em == hipErrorOutOfMemory) return fail(c, SSGD_ENOMEM, "full objective: " + msg);
        if (em != hipSuccess) return fail(c, SSGD_EDEVICE, "full objective: " + msg);
        return SSGD_OK;
    }
    if (!full_loss_supports(c->model.kind, c->model.d, C))
        return fail(c, SSGD_EINVAL, "the full objective of the linear models needs d % 4 == 0");
    HIP_OK(c, hipSetDevice(c->device));
    const int blocks = std::max(1, c->cu_count);
    DevBuf partial;
    HIP_OK(c, partial.alloc(sizeof(double) * blocks));
    hipError_t e = launch_full_loss(c->model.kind, c->model.X, c->model.y, c->model.N, c->model.d, C,
                                    c->params.as<float>() + (int64_t)replica * c->nw, partial.as<double>(), blocks, c->stream);
    std::vector<double> h(blocks);
    if (e == hipSuccess) e = hipMemcpyAsync(h.data(), partial.p, sizeof(double) * blocks, hipMemcpyDeviceToHost, c->stream);
    if (e == hipSuccess) e = hipStreamSynchronize(c->stream);
    partial.release();
    if (e != hipSuccess) return fail(c, SSGD_EDEVICE, std::string("full objective: ") + hipGetErrorString(e));
    double s = 0.0;
    for (double v : h) s += v;
    *loss_out = s / (double)c->model.N;
    return SSGD_OK;
}

ssgd_status ssgd_full_gradient(ssgd_ctx* c, int32_t replica, float* grad_out) {
    if (!c || !grad_out) return fail(c, SSGD_EINVAL, "null argument");
    if (replica < 0 || replica >= c->R) return fail(c, SSGD_EINVAL, "replica out of range");
    if (c->broken) return fail(c, SSGD_ESTATE, "context is unusable after a device error");
    const int C = c->model.kind == SSGD_LSQ ? 1 : c->model.classes;
    if (c->model.kind == SSGD_MLP2) {
        HIP_OK(c, hipSetDevice(c->device));
        HIP_OK(c, hipStreamSynchronize(c->stream));
        std::string msg;
        hipError_t em = mlp_full_gradient(c->mlp[(size_t)replica], grad_out, c->stream, &msg);
        if (em == hipErrorOutOfMemory) return fail(c, SSGD_ENOMEM, "full gradient: " + msg);
        if (em != hipSuccess) return fail(c, SSGD_EDEVICE, "full gradient: " + msg);
        return SSGD_OK;
    }
    if (!full_grad_supports(c->model.kind, c->model.d, C))
        return fail(c, SSGD_EINVAL, "the full gradient of the linear models needs d % 4 == 0");
    HIP_OK(c, hipSetDevice(c->device));
    DevBuf scratch, out;
    hipError_t e = scratch.alloc(sizeof(float) * (size_t)full_grad_scratch_floats(c->model.N, c->model.d, C, nullptr));
    if (e == hipSuccess) e = out.alloc(sizeof(float) * (size_t)c->nw);
    if (e != hipSuccess) { scratch.release(); out.release(); return fail(c, SSGD_ENOMEM, "full gradient: device allocation failed"); }
    e = launch_full_grad(c->model.kind, c->model.X, c->model.y, c->model.N, c->model.d, C,
                         c->params.as<float>() + (int64_t)replica * c->nw, scratch.as<float>(), out.as<float>(), c->cu_count, c->stream);
    if (e == hipSuccess) e = hipMemcpyAsync(grad_out, out.p, sizeof(float) * (size_t)c->nw, hipMemcpyDeviceToHost, c->stream);
    if (e == hipSuccess) e = hipStreamSynchronize(c->stream);
    scratch.release(); out.release();
    if (e != hipSuccess) return fail(c, SSGD_EDEVICE, std::string("full gradient: ") + hipGetErrorString(e));
    return SSGD_OK;
}

ssgd_status ssgd_full_gradient_static(ssgd_ctx* c, int32_t replica, float* grad_out_device) {
    if (!c || !grad_out_device) return fail(c, SSGD_EINVAL, "null argument");
    if (replica < 0 || replica >= c->R) return fail(c, SSGD_EINVAL, "replica out of range");
    if (c->broken) return fail(c, SSGD_ESTATE, "context is unusable after a device error");
    const int C = c->model.kind == SSGD_LSQ ? 1 : c->model.classes;
    if (c->model.kind == SSGD_MLP2 || !full_grad_supports(c->model.kind, c->model.d, C))
        return fail(c, SSGD_EINVAL, "the full gradient is built for the linear models with d % 4 == 0");
    const int64_t need = full_grad_scratch_floats(c->model.N, c->model.d, C, nullptr);
    if (need > full_grad_static_scratch_floats())
        return fail(c, SSGD_EINVAL, "the data set needs " + std::to_string(need) + " floats of scratch memory, the static array holds " +
                                        std::to_string(full_grad_static_scratch_floats()) + " (16 N + min(64, ceil(N / 256)) classes (d + 1))");
    HIP_OK(c, hipSetDevice(c->device));
    float* work = full_grad_static_scratch();
    if (!work) return fail(c, SSGD_ESTATE, "the static scratch array was not set up on this device");
    // every word of the scratch memory that the kernels read has been written by this call before (the per-sample
    // deltas of rows 0 .. N-1, the partial sums of all chunks, classes and columns), so nothing has to be cleared
    HIP_OK(c, launch_full_grad(c->model.kind, c->model.X, c->model.y, c->model.N, c->model.d, C,
                               c->params.as<float>() + (int64_t)replica * c->nw, work, grad_out_device, c->cu_count, c->stream));
    return SSGD_OK;
}

ssgd_status ssgd_get_workers(ssgd_ctx* c, int32_t replica, int32_t* tau, int32_t* ord, double* finish) {
    if (!c) return fail(nullptr, SSGD_EINVAL, "null context");
    if (replica < 0 || replica >= c->R) return fail(c, SSGD_EINVAL, "replica out of range");
    if (c->variant != SSGD_K_ASYNC && c->variant != SSGD_K_BATCH_ASYNC)
        return fail(c, SSGD_EINVAL, "the synchronous variants keep no mini-batch in flight between updates");
    HIP_OK(c, hipSetDevice(c->device));
    HIP_OK(c, hipStreamSynchronize(c->stream));
    const size_t off = (size_t)replica * c->P;
    if (tau) HIP_OK(c, hipMemcpy(tau, c->ws.tau + off, sizeof(int32_t) * c->P, hipMemcpyDeviceToHost));
    if (ord) HIP_OK(c, hipMemcpy(ord, c->ws.ord + off, sizeof(int32_t) * c->P, hipMemcpyDeviceToHost));
    if (finish) HIP_OK(c, hipMemcpy(finish, c->ws.finish + off, sizeof(double) * c->P, hipMemcpyDeviceToHost));
    return SSGD_OK;
}

extern "C++" {
namespace {

// Snapshot layout: header, then the trace of the updates done (replica by replica), then every device buffer that
// later updates depend on, each as raw bytes in the order of state_buffers().
struct StateHeader {
    char magic[8];
    int64_t total_bytes;
    int32_t kind, d, classes, hidden, P, m, variant, R, Kcap, S, G, ada_mode;
    int64_t N, nw, j, mlp_bytes;
    uint64_t seed;
    int32_t win_cnt, reserved;
};

std::vector<DevBuf*> state_buffers(ssgd_ctx* c) {
    std::vector<DevBuf*> b = {&c->ws_finish, &c->ws_tau, &c->ws_ord, &c->ws_clock, &c->ws_curK, &c->ws_winprev, &c->ws_winidx,
                              &c->ws_F0, &c->ws_intstart, &c->ws_crossed, &c->ws_ndone};
    if (c->model.kind != SSGD_MLP2) { b.push_back(&c->params); b.push_back(&c->park); b.push_back(&c->park_small); }
    return b;
}

int64_t trace_bytes(const ssgd_ctx* c, int64_t j) {
    return (int64_t)c->R * j * (int64_t)(sizeof(double) + sizeof(float) + sizeof(int32_t) + 3 * sizeof(int32_t) * c->Kcap);
}

StateHeader make_header(ssgd_ctx* c) {
    StateHeader h{};
    memcpy(h.magic, "SSGDST01", 8);
    h.kind = c->model.kind; h.d = c->model.d; h.classes = c->model.classes; h.hidden = c->model.hidden;
    h.P = c->P; h.m = c->m; h.variant = c->variant; h.R = c->R; h.Kcap = c->Kcap; h.S = c->S; h.G = c->G;
    h.ada_mode = c->ada.mode; h.N = c->model.N; h.nw = c->nw; h.j = c->j; h.seed = c->seed; h.win_cnt = c->win_cnt;
    h.mlp_bytes = 0;
    for (MlpState* ms : c->mlp) h.mlp_bytes += mlp_state_bytes(ms);
    int64_t n = (int64_t)sizeof(StateHeader) + trace_bytes(c, c->j) + h.mlp_bytes;
    for (DevBuf* b : state_buffers(c)) n += (int64_t)b->bytes;
    h.total_bytes = n;
    return h;
}

}  // namespace
}  // extern "C++"

ssgd_status ssgd_state_bytes(ssgd_ctx* c, int64_t* bytes) {
    if (!c || !bytes) return fail(c, SSGD_EINVAL, "null argument");
    *bytes = make_header(c).total_bytes;
    return SSGD_OK;
}

ssgd_status ssgd_get_state(ssgd_ctx* c, void* host_buf, int64_t bytes) {
    if (!c || !host_buf) return fail(c, SSGD_EINVAL, "null argument");
    if (c->broken) return fail(c, SSGD_ESTATE, "context is unusable after a device error");
    const StateHeader h = make_header(c);
    if (bytes < h.total_bytes) return fail(c, SSGD_EINVAL, "buffer smaller than ssgd_state_bytes");
    HIP_OK(c, hipSetDevice(c->device));
    HIP_OK(c, hipStreamSynchronize(c->stream));
    unsigned char* out = static_cast<unsigned char*>(host_buf);
    memcpy(out, &h, sizeof(h));
    size_t off = sizeof(h);
    const int64_t j = c->j, W = c->Kcap, cap = c->tr.cap;
    for (int64_t r = 0; r < c->R && j > 0; ++r) {
        HIP_OK(c, hipMemcpy(out + off, c->tr.t + r * cap, sizeof(double) * j, hipMemcpyDeviceToHost)); off += sizeof(double) * j;
        HIP_OK(c, hipMemcpy(out + off, c->tr.loss + r * cap, sizeof(float) * j, hipMemcpyDeviceToHost)); off += sizeof(float) * j;
        HIP_OK(c, hipMemcpy(out + off, c->tr.K + r * cap, sizeof(int32_t) * j, hipMemcpyDeviceToHost)); off += sizeof(int32_t) * j;
        HIP_OK(c, hipMemcpy(out + off, c->tr.sel + r * cap * W, sizeof(int32_t) * j * W, hipMemcpyDeviceToHost)); off += sizeof(int32_t) * j * W;
        HIP_OK(c, hipMemcpy(out + off, c->tr.tau + r * cap * W, sizeof(int32_t) * j * W, hipMemcpyDeviceToHost)); off += sizeof(int32_t) * j * W;
        HIP_OK(c, hipMemcpy(out + off, c->tr.ord + r * cap * W, sizeof(int32_t) * j * W, hipMemcpyDeviceToHost)); off += sizeof(int32_t) * j * W;
    }
    for (DevBuf* b : state_buffers(c)) {
        HIP_OK(c, hipMemcpy(out + off, b->p, b->bytes, hipMemcpyDeviceToHost));
        off += b->bytes;
    }
    for (MlpState* ms : c->mlp) {
        HIP_OK(c, mlp_get_state(ms, out + off));
        off += (size_t)mlp_state_bytes(ms);
    }
    return SSGD_OK;
}

ssgd_status ssgd_set_state(ssgd_ctx* c, const void* host_buf, int64_t bytes) {
    if (!c || !host_buf) return fail(c, SSGD_EINVAL, "null argument");
    if (c->broken) return fail(c, SSGD_ESTATE, "context is unusable after a device error");
    if (bytes < (int64_t)sizeof(StateHeader)) return fail(c, SSGD_EINVAL, "not a state snapshot");
    StateHeader h;
    memcpy(&h, host_buf, sizeof(h));
    if (memcmp(h.magic, "SSGDST01", 8) != 0) return fail(c, SSGD_EINVAL, "not a state snapshot");
    // the snapshot must come from a context of the same configuration
    StateHeader mine = make_header(c);
    if (h.kind != mine.kind || h.d != mine.d || h.classes != mine.classes || h.hidden != mine.hidden || h.P != mine.P ||
        h.m != mine.m || h.variant != mine.variant || h.R != mine.R || h.Kcap != mine.Kcap || h.S != mine.S || h.G != mine.G ||
        h.ada_mode != mine.ada_mode || h.N != mine.N || h.nw != mine.nw || h.seed != mine.seed || h.mlp_bytes != mine.mlp_bytes)
        return fail(c, SSGD_EINVAL, "the snapshot was taken from a context of another configuration");
    // Everything the header claims is checked against this context before the context is touched: the number of
    // updates must be one whose trace fits the buffer handed in, and the total must be what this configuration
    // writes for that many updates.
    const int64_t per_update = trace_bytes(c, 1);
    int64_t fixed = (int64_t)sizeof(StateHeader) + h.mlp_bytes;
    for (DevBuf* b : state_buffers(c)) fixed += (int64_t)b->bytes;
    if (h.j < 0 || h.total_bytes > bytes || h.total_bytes < fixed || (h.total_bytes - fixed) / per_update < h.j ||
        fixed + trace_bytes(c, h.j) != h.total_bytes)
        return fail(c, SSGD_EINVAL, "truncated or malformed state snapshot");
    HIP_OK(c, hipSetDevice(c->device));
    HIP_OK(c, hipStreamSynchronize(c->stream));
    // room for the snapshot's trace; the updates done so far stay valid until the copies below begin
    ssgd_status st = grow_trace(c, std::max(h.j, c->j));
    if (st != SSGD_OK) return st;
    // from here on a failed copy leaves a mixture of two runs behind: the context is marked unusable
    struct Guard { ssgd_ctx* c; bool ok = false; ~Guard() { if (!ok) c->broken = true; } } guard{c};
    const unsigned char* in = static_cast<const unsigned char*>(host_buf);
    size_t off = sizeof(h);
    const int64_t j = h.j, W = c->Kcap, cap = c->tr.cap;
    for (int64_t r = 0; r < c->R && j > 0; ++r) {
        HIP_OK(c, hipMemcpy(c->tr.t + r * cap, in + off, sizeof(double) * j, hipMemcpyHostToDevice)); off += sizeof(double) * j;
        HIP_OK(c, hipMemcpy(c->tr.loss + r * cap, in + off, sizeof(float) * j, hipMemcpyHostToDevice)); off += sizeof(float) * j;
        HIP_OK(c, hipMemcpy(c->tr.K + r * cap, in + off, sizeof(int32_t) * j, hipMemcpyHostToDevice)); off += sizeof(int32_t) * j;
        HIP_OK(c, hipMemcpy(c->tr.sel + r * cap * W, in + off, sizeof(int32_t) * j * W, hipMemcpyHostToDevice)); off += sizeof(int32_t) * j * W;
        HIP_OK(c, hipMemcpy(c->tr.tau + r * cap * W, in + off, sizeof(int32_t) * j * W, hipMemcpyHostToDevice)); off += sizeof(int32_t) * j * W;
        HIP_OK(c, hipMemcpy(c->tr.ord + r * cap * W, in + off, sizeof(int32_t) * j * W, hipMemcpyHostToDevice)); off += sizeof(int32_t) * j * W;
    }
    for (DevBuf* b : state_buffers(c)) {
        HIP_OK(c, hipMemcpy(b->p, in + off, b->bytes, hipMemcpyHostToDevice));
        off += b->bytes;
    }
    for (MlpState* ms : c->mlp) {
        HIP_OK(c, mlp_set_state(ms, in + off));
        off += (size_t)mlp_state_bytes(ms);
    }
    c->j = h.j;
    c->win_cnt = h.win_cnt;
    guard.ok = true;
    return SSGD_OK;
}

ssgd_status ssgd_debug_delays(const ssgd_delay_dist* dist, const uint32_t* bits, int64_t n, float* out) {
    if (!dist_ok(dist) || dist->kind == SSGD_TABLE || !bits || !out || n < 0) return fail(nullptr, SSGD_EINVAL, "invalid argument");
    if (n == 0) return SSGD_OK;
    DevBuf b, o, tbl;
    Dist dd;
    ssgd_ctx* c = nullptr;
    HIP_OK(c, make_dist(dist, &tbl, &dd));
    HIP_OK(c, b.alloc(sizeof(uint32_t) * n));
    HIP_OK(c, o.alloc(sizeof(float) * n));
    HIP_OK(c, hipMemcpy(b.p, bits, sizeof(uint32_t) * n, hipMemcpyHostToDevice));
    hipLaunchKernelGGL(debug_delay_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, nullptr, dd, b.as<uint32_t>(), n, o.as<float>());
    HIP_OK(c, hipGetLastError());
    HIP_OK(c, hipMemcpy(out, o.p, sizeof(float) * n, hipMemcpyDeviceToHost));
    b.release(); o.release(); tbl.release();
    return SSGD_OK;
}

ssgd_status ssgd_debug_batch(uint64_t seed, uint32_t replica, uint32_t worker, uint32_t ordinal, uint32_t version,
                             int32_t m, int64_t N, uint32_t* out) {
    if (!out || m < 1 || N < 1 || N >= (1ll << 32)) return fail(nullptr, SSGD_EINVAL, "invalid argument");
    DevBuf o;
    ssgd_ctx* c = nullptr;
    HIP_OK(c, o.alloc(sizeof(uint32_t) * m));
    hipLaunchKernelGGL(debug_batch_kernel, dim3((m + 255) / 256), dim3(256), 0, nullptr, seed, replica, worker, ordinal, version, m, (uint32_t)N, o.as<uint32_t>());
    HIP_OK(c, hipGetLastError());
    HIP_OK(c, hipMemcpy(out, o.p, sizeof(uint32_t) * m, hipMemcpyDeviceToHost));
    o.release();
    return SSGD_OK;
}

ssgd_status ssgd_stream_read_rate(const void* data, int64_t bytes, int32_t passes, void* hip_stream, double* bytes_per_s) {
    if (!data || !bytes_per_s || bytes < 16 || passes < 1 || ((uintptr_t)data & 15u) != 0)
        return fail(nullptr, SSGD_EINVAL, "stream read: a 16-byte aligned device buffer of at least 16 bytes and passes >= 1");
    ssgd_ctx* c = nullptr;
    hipStream_t stream = (hipStream_t)hip_stream;
    int dev = 0, cus = 0;
    HIP_OK(c, hipGetDevice(&dev));
    HIP_OK(c, hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev));
    DevBuf sink;
    HIP_OK(c, sink.alloc(sizeof(uint32_t)));
    hipEvent_t e0 = nullptr, e1 = nullptr;
    hipError_t e = hipEventCreate(&e0);
    if (e == hipSuccess) e = hipEventCreate(&e1);
    const int64_t n16 = bytes / 16;
    const int blocks = std::max(1, cus) * 8;
    if (e == hipSuccess) {
        hipLaunchKernelGGL(stream_read_kernel, dim3(blocks), dim3(256), 0, stream, (const stream_u32x4*)data, n16, sink.as<uint32_t>());   // warm-up
        e = hipEventRecord(e0, stream);
    }
    for (int p = 0; p < passes && e == hipSuccess; ++p)
        hipLaunchKernelGGL(stream_read_kernel, dim3(blocks), dim3(256), 0, stream, (const stream_u32x4*)data, n16, sink.as<uint32_t>());
    if (e == hipSuccess) e = hipEventRecord(e1, stream);
    if (e == hipSuccess) e = hipEventSynchronize(e1);
    float ms = 0.0f;
    if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
    if (e == hipSuccess) e = hipGetLastError();
    if (e0) (void)hipEventDestroy(e0);
    if (e1) (void)hipEventDestroy(e1);
    sink.release();
    if (e != hipSuccess) return fail(nullptr, SSGD_EDEVICE, std::string("stream read: ") + hipGetErrorString(e));
    *bytes_per_s = (double)(n16 * 16) * passes / ((double)ms * 1e-3);
    return SSGD_OK;
}

const char* ssgd_last_error(const ssgd_ctx* ctx) { return ctx ? ctx->err.c_str() : g_err.c_str(); }

ssgd_status ssgd_last_kernel_ms(const ssgd_ctx* ctx, double* avg_ms, int64_t* launches) {
    if (!ctx) return SSGD_EINVAL;
    if (avg_ms) *avg_ms = ctx->last_launches ? ctx->last_ms / (double)ctx->last_launches : 0.0;
    if (launches) *launches = ctx->last_launches;
    return SSGD_OK;
}

void ssgd_destroy(ssgd_ctx* c) {
    if (!c) return;
    (void)hipSetDevice(c->device);
    (void)hipStreamSynchronize(c->stream);
    if (c->prof.p) {
        // diagnostics requested through SSGD_PHASE_PROFILE=a,b[,wave]: mean cycles per update between mark a and the
        // next mark b of one wave per workgroup (marks below 16: compute waves, from 16: loader waves)
        std::vector<unsigned long long> h((size_t)c->R * c->G * 2 + (size_t)c->R);
        if (hipMemcpy(h.data(), c->prof.as<unsigned long long>() + (size_t)c->R * c->G * 20, h.size() * sizeof(unsigned long long), hipMemcpyDeviceToHost) == hipSuccess && c->j > 0) {
            double tot[2] = {0, 0}, helper = 0;
            const size_t nslice = (size_t)c->R * c->G * 2;
            for (size_t q = 0; q < nslice; ++q) tot[q % 2] += (double)h[q];
            for (size_t q = nslice; q < h.size(); ++q) helper += (double)h[q];
            // marks from 32 on belong to the helper workgroups (one per replica) of the kernel that has them
            const double per = helper > 0 ? helper / ((double)c->R * (double)c->j) : (tot[0] + tot[1]) / ((double)c->R * c->G * (double)c->j);
            fprintf(stderr, "ssgd phase profile %s: %.0f cycles per update and workgroup\n", getenv("SSGD_PHASE_PROFILE"), per);
        }
    }
    if (c->xcc_ids.p && getenv("SSGD_DEBUG")) {
        // placement of the last launch: XCD, shader engine and CU of every workgroup of the first clusters
        std::vector<int32_t> h((size_t)c->R * c->G);
        if (hipMemcpy(h.data(), c->xcc_ids.p, h.size() * sizeof(int32_t), hipMemcpyDeviceToHost) == hipSuccess)
            for (int r = 0; r < c->R; ++r) {
                fprintf(stderr, "ssgd placement replica %d:", r);
                for (int g = 0; g < c->G; ++g) {
                    const int v = h[(size_t)r * c->G + g], hw = v >> 8;
                    fprintf(stderr, " x%d.se%d.cu%d", v & 0xFF, (hw >> 13) & 7, (hw >> 8) & 15);
                }
                fprintf(stderr, "\n");
            }
    }
    for (size_t r = c->mlp.size(); r-- > 0;) mlp_destroy(c->mlp[r]);   // the first one owns what the others share
    if (c->side) (void)hipStreamDestroy(c->side);
    if (c->host_rows) (void)hipHostFree(c->host_rows);
    DevBuf* bufs[] = {&c->table, &c->tr_t, &c->tr_loss, &c->tr_K, &c->tr_sel, &c->tr_tau, &c->tr_ord, &c->ws_finish,
                      &c->ws_tau, &c->ws_ord, &c->ws_clock, &c->ws_curK, &c->ws_winprev, &c->ws_winidx, &c->ws_F0,
                      &c->ws_intstart, &c->ws_crossed, &c->ws_ndone, &c->params, &c->park, &c->park_small, &c->zpart, &c->zx, &c->dx, &c->fallback,
                      &c->arrive, &c->abort_flag, &c->xcc_ids, &c->prof};
    for (DevBuf* b : bufs) b->release();
    delete c;
}

}  // extern "C"
#pragma GCC visibility pop
