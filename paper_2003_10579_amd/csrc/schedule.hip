// Event process of the parameter server (Sec. 2.2) on the device: random delays
// (Sec. 3.1), K-of-P selection of the earliest finishers, staleness bookkeeping.
//
// One wavefront simulates one replica; each lane owns up to four of the P <= 256
// workers.  The delays do not depend on the data, so a whole segment of updates is
// scheduled before any gradient is taken; the gradient kernels then read the trace.
#include "common.hpp"

namespace ssgd {
namespace {

constexpr int NQ = kMaxWorkers / 64;

struct Best { double key; int32_t id; };

__device__ __forceinline__ bool before(double ka, int32_t ia, double kb, int32_t ib) {
    return ka < kb || (ka == kb && ia < ib);   // ties go to the lower worker id
}

// Smallest (key, id) over the wavefront, known to every lane afterwards.
__device__ __forceinline__ Best wave_min(Best b) {
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const double ok = __shfl_xor(b.key, off, 64);
        const int32_t oi = __shfl_xor(b.id, off, 64);
        if (before(ok, oi, b.key, b.id)) { b.key = ok; b.id = oi; }
    }
    return b;
}

__device__ __forceinline__ Best local_min(const double (&key)[NQ], uint32_t skip, int lane, int P) {
    Best b{__longlong_as_double(0x7FF0000000000000LL), 0x7FFFFFFF};
#pragma unroll
    for (int q = 0; q < NQ; ++q) {
        const int w = lane + 64 * q;
        if (w < P && !((skip >> q) & 1u) && before(key[q], w, b.key, b.id)) { b.key = key[q]; b.id = w; }
    }
    return b;
}

__global__ __launch_bounds__(64) void schedule_kernel(SchedArgs a) {
    const int lane = threadIdx.x;
    const int rep = a.replica0 + blockIdx.x;
    const int P = a.P, Kcap = a.tr.Kcap;
    const int64_t cap = a.tr.cap;
    double* tr_t = a.tr.t + (int64_t)rep * cap;
    int32_t* tr_K = a.tr.K + (int64_t)rep * cap;
    int32_t* tr_sel = a.tr.sel + (int64_t)rep * cap * Kcap;
    int32_t* tr_tau = a.tr.tau + (int64_t)rep * cap * Kcap;
    int32_t* tr_ord = a.tr.ord + (int64_t)rep * cap * Kcap;

    const int K = a.ws.curK[rep];
    double clock = a.ws.clock[rep];
    double key[NQ];
    int32_t tau[NQ], ord[NQ];
#pragma unroll
    for (int q = 0; q < NQ; ++q) {
        const int w = lane + 64 * q;
        key[q] = 0.0; tau[q] = 0; ord[q] = 0;
        if (w < P && a.variant >= kAsync) {
            key[q] = a.ws.finish[(int64_t)rep * P + w];
            tau[q] = a.ws.tau[(int64_t)rep * P + w];
            ord[q] = a.ws.ord[(int64_t)rep * P + w];
        }
    }

    int64_t done = 0;
    int crossed = 0;
    for (; done < a.count; ++done) {
        const int64_t j = a.j0 + done;
        const uint32_t ver = (uint32_t)j;
        for (int l = lane; l < Kcap; l += 64) {
            tr_sel[j * Kcap + l] = -1; tr_tau[j * Kcap + l] = -1; tr_ord[j * Kcap + l] = -1;
        }
        double t_new = clock;
        if (a.variant == kSync || a.variant == kBatchSync) {
            // every worker starts a fresh mini-batch at t_j with w_j
#pragma unroll
            for (int q = 0; q < NQ; ++q) {
                const int w = lane + 64 * q;
                ord[q] = 0;
                if (w < P) key[q] = (double)delay(a.dist, a.seed, kDelay, 0, rep, P, a.table_ord, w, 0, ver);
            }
            uint32_t taken = 0;
            double last = 0.0;
            for (int l = 0; l < K; ++l) {
                const Best b = wave_min(local_min(key, taken, lane, P));
                last = b.key;
                if ((b.id & 63) == lane) {
                    const int q = b.id >> 6;
#pragma unroll
                    for (int qq = 0; qq < NQ; ++qq) {
                        if (qq != q) continue;
                        tr_sel[j * Kcap + l] = b.id; tr_tau[j * Kcap + l] = (int32_t)j; tr_ord[j * Kcap + l] = ord[qq];
                        if (a.variant == kSync) {
                            taken |= 1u << qq;
                        } else {
                            // K-batch-sync: the worker starts its next mini-batch at the same w_j
                            ord[qq] += 1;
                            if (l + 1 < K)
                                key[qq] = key[qq] + (double)delay(a.dist, a.seed, kDelay, 0, rep, P, a.table_ord,
                                                                  b.id, ord[qq], ver);
                        }
                    }
                }
            }
            t_new = clock + last;
        } else {
            // K-async: the K earliest finishers contribute; only they restart, at t_{j+1}
            uint32_t taken = 0;
            for (int l = 0; l < K; ++l) {
                const Best b = wave_min(local_min(key, taken, lane, P));
                t_new = b.key;
                if ((b.id & 63) == lane) {
                    const int q = b.id >> 6;
#pragma unroll
                    for (int qq = 0; qq < NQ; ++qq) {
                        if (qq != q) continue;
                        tr_sel[j * Kcap + l] = b.id; tr_tau[j * Kcap + l] = tau[qq]; tr_ord[j * Kcap + l] = 0;
                        taken |= 1u << qq;
                    }
                }
            }
#pragma unroll
            for (int q = 0; q < NQ; ++q) {
                if (!((taken >> q) & 1u)) continue;
                const int w = lane + 64 * q;
                tau[q] = (int32_t)(j + 1);
                key[q] = t_new + (double)delay(a.dist, a.seed, kDelay, 0, rep, P, a.table_ord, w, 0, ver + 1u);
            }
        }
        if (lane == 0) { tr_t[j] = t_new; tr_K[j] = K; }
        const double t_prev = clock;
        clock = t_new;
        if (a.interval_t > 0.0 && floor(t_new / a.interval_t) > floor(t_prev / a.interval_t)) {
            crossed = 1; ++done; break;
        }
    }

#pragma unroll
    for (int q = 0; q < NQ; ++q) {
        const int w = lane + 64 * q;
        if (w < P && a.variant >= kAsync) {
            a.ws.finish[(int64_t)rep * P + w] = key[q];
            a.ws.tau[(int64_t)rep * P + w] = tau[q];
            a.ws.ord[(int64_t)rep * P + w] = ord[q];
        }
    }
    if (lane == 0) { a.ws.clock[rep] = clock; a.ws.n_done[rep] = done; a.ws.crossed[rep] = crossed; }
}

// AdaSync controller (Sec. 6): one thread per replica, run after the gradient kernels of a segment.
__global__ void adasync_kernel(AdaArgs a, int replicas) {
    const int rep = blockIdx.x * blockDim.x + threadIdx.x;
    if (rep >= replicas) return;
    const float* loss = a.tr.loss + (int64_t)rep * a.tr.cap;
    int K = a.ws.curK[rep];
    if (a.j_end >= 1 && a.ws.F0[rep] < 0.0) a.ws.F0[rep] = (double)loss[0];
    if (a.mode == 1) {
        if (!a.window_closed) return;
        double s = 0.0;
        for (int64_t j = a.j_end - a.window; j < a.j_end; ++j) s += (double)loss[j];
        const double mean = s / (double)a.window;
        if (a.ws.win_index[rep] >= 1 && mean > (1.0 - a.rel_tol) * a.ws.win_prev[rep]) {
            K = 2 * K; if (K > a.Kmax) K = a.Kmax;
        }
        a.ws.win_prev[rep] = mean;
        a.ws.win_index[rep] += 1;
    } else {
        if (!a.ws.crossed[rep]) return;
        double s = 0.0;
        const int64_t j0 = a.ws.int_start[rep];
        for (int64_t j = j0; j < a.j_end; ++j) s += (double)loss[j];
        const double Fstart = s / (double)(a.j_end - j0);
        a.ws.int_start[rep] = a.j_end;
        if (K < a.Kmax && Fstart > 0.0) {
            const double ratio = a.ws.F0[rep] / Fstart;
            double Knew;
            if (a.mode == 2) {
                Knew = (double)a.K0 * sqrt(ratio);                       // Algorithm 1
            } else {
                const double q = (double)a.K0 * a.K0 / (double)(a.P - a.K0) * ratio;   // App. D, K-sync
                Knew = 0.5 * (-q + sqrt(q * q + 4.0 * q * (double)a.P));
            }
            int Ki = (int)floor(Knew + 0.5);
            if (Ki < K) Ki = K;
            if (Ki > a.Kmax) Ki = a.Kmax;
            K = Ki;
        }
    }
    a.ws.curK[rep] = K;
}

}  // namespace

void launch_schedule(const SchedArgs& a, int replicas, hipStream_t s) {
    hipLaunchKernelGGL(schedule_kernel, dim3(replicas), dim3(64), 0, s, a);
}

void launch_adasync(const AdaArgs& a, int replicas, hipStream_t s) {
    hipLaunchKernelGGL(adasync_kernel, dim3((replicas + 63) / 64), dim3(64), 0, s, a, replicas);
}

}  // namespace ssgd
