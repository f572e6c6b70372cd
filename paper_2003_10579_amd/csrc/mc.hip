// Monte-Carlo estimate of the runtime per iteration T (Sec. 2.3; Lemma 1: K-sync
// T = X_{K:P}; Lemma 2: K-batch-sync; Lemma 3: K-async; the simulation of Fig. 6).
//
// One wavefront owns a trial: it draws the P fresh delays, sorts them once (all the
// order statistics X_{1:P}..X_{P:P} at one stroke, bitonic network over lanes x
// registers), and then runs, for every K, the variant's event process for chain_len
// updates.  The K-async process only depends on the multiset of finish times, so
// the state is a sorted array: T = key[K-1] - t, the first K keys are replaced by
// t_new + fresh delays, and the array is sorted again.
#include <algorithm>
#include <string>
#include <vector>

#include "../../include/ssgd.h"
#include "common.hpp"

namespace ssgd {
namespace {

struct McArgs {
    Dist dist;
    uint64_t seed;
    int32_t variant, P, Kmin, Kmax, chain_len;
    int32_t nslices;     // block b takes the values K = Kmin + b % nslices, + nslices, ...: small accumulators, many waves per CU
    int64_t trial0, trials;
    double* partial;     // [blocks][nK*chain_len][2]
    double* per_trial;   // nullable
};

__device__ __forceinline__ double inf64() { return __longlong_as_double(0x7FF0000000000000LL); }

// Ascending bitonic sort of 64*NQ keys; position p = q*64 + lane.
template <int NQ, typename T>
__device__ __forceinline__ void sort_keys(T (&key)[NQ], int lane) {
    constexpr int N = 64 * NQ;
#pragma unroll
    for (int k = 2; k <= N; k <<= 1) {
#pragma unroll
        for (int j = k >> 1; j > 0; j >>= 1) {
            if (j < 64) {
#pragma unroll
                for (int q = 0; q < NQ; ++q) {
                    const int p = q * 64 + lane;
                    const T other = __shfl_xor(key[q], j, 64);
                    const bool up = (p & k) == 0, lower = (p & j) == 0;
                    key[q] = (up == lower) ? fmin(key[q], other) : fmax(key[q], other);
                }
            } else {
                const int dq = j >> 6;
#pragma unroll
                for (int q = 0; q < NQ; ++q) {
                    if ((q & dq) == 0) {
                        const int p = q * 64 + lane;
                        const bool up = (p & k) == 0;
                        const T a = key[q], b = key[q | dq];
                        key[q] = up ? fmin(a, b) : fmax(a, b);
                        key[q | dq] = up ? fmax(a, b) : fmin(a, b);
                    }
                }
            }
        }
    }
}

// Positions [0, B) sorted in descending order, B a power of two below the array size: the network of sort_keys
// turned round, the other positions untouched.
template <int NQ, int B>
__device__ __forceinline__ void sort_prefix_descending(double (&key)[NQ], int lane) {
#pragma unroll
    for (int k = 2; k <= B; k <<= 1) {
#pragma unroll
        for (int j = k >> 1; j > 0; j >>= 1) {
            if (j < 64) {
#pragma unroll
                for (int q = 0; q < NQ; ++q) {
                    if (q * 64 >= B) continue;
                    const int p = q * 64 + lane;
                    const double other = __shfl_xor(key[q], j, 64);
                    const bool down = (p & k) == 0, lower = (p & j) == 0;
                    const double v = (down == lower) ? fmax(key[q], other) : fmin(key[q], other);
                    key[q] = (p < B) ? v : key[q];
                }
            } else {
                const int dq = j >> 6;
#pragma unroll
                for (int q = 0; q < NQ; ++q) {
                    if ((q & dq) == 0 && (q | dq) < NQ && (q | dq) * 64 < B) {
                        const int p = q * 64 + lane;
                        const bool down = (p & k) == 0;
                        const double a = key[q], b = key[q | dq];
                        key[q] = down ? fmax(a, b) : fmin(a, b);
                        key[q | dq] = down ? fmin(a, b) : fmax(a, b);
                    }
                }
            }
        }
    }
}

// The array was ascending and its first K keys have been replaced (K wave-uniform): sorted again.  The first B
// positions, B the power of two that covers K, are sorted in descending order; together with the untouched
// ascending rest that is a bitonic sequence, which one merge pass sorts.
template <int NQ>
__device__ __forceinline__ void resort_prefix(double (&key)[NQ], int lane, int K) {
    constexpr int N = 64 * NQ;
    if (2 * K > N) { sort_keys<NQ, double>(key, lane); return; }
    if (K > 64) { if constexpr (NQ > 2) sort_prefix_descending<NQ, 128>(key, lane); }
    else if (K > 32) sort_prefix_descending<NQ, 64>(key, lane);
    else if (K > 16) sort_prefix_descending<NQ, 32>(key, lane);
    else if (K > 8) sort_prefix_descending<NQ, 16>(key, lane);
    else if (K > 4) sort_prefix_descending<NQ, 8>(key, lane);
    else if (K > 2) sort_prefix_descending<NQ, 4>(key, lane);
    else if (K > 1) sort_prefix_descending<NQ, 2>(key, lane);
#pragma unroll
    for (int j = N >> 1; j > 0; j >>= 1) {
        if (j < 64) {
#pragma unroll
            for (int q = 0; q < NQ; ++q) {
                const double other = __shfl_xor(key[q], j, 64);
                key[q] = ((lane & j) == 0) ? fmin(key[q], other) : fmax(key[q], other);
            }
        } else {
            const int dq = j >> 6;
#pragma unroll
            for (int q = 0; q < NQ; ++q) {
                if ((q & dq) == 0) {
                    const double a = key[q], b = key[q | dq];
                    key[q] = fmin(a, b);
                    key[q | dq] = fmax(a, b);
                }
            }
        }
    }
}

// key at position pos (wave-uniform pos), known to every lane
template <int NQ>
__device__ __forceinline__ double key_at(const double (&key)[NQ], int pos) {
    double v = 0.0;
#pragma unroll
    for (int q = 0; q < NQ; ++q)
        if ((pos >> 6) == q) v = __shfl(key[q], pos & 63, 64);
    return v;
}

struct Best { double key; int32_t id; };
template <int NQ>
__device__ __forceinline__ Best wave_argmin(const double (&key)[NQ], int lane) {
    Best b{inf64(), 0x7FFFFFFF};
#pragma unroll
    for (int q = 0; q < NQ; ++q) {
        const int w = q * 64 + lane;
        if (key[q] < b.key || (key[q] == b.key && w < b.id)) { b.key = key[q]; b.id = w; }
    }
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const double ok = __shfl_xor(b.key, off, 64);
        const int32_t oi = __shfl_xor(b.id, off, 64);
        if (ok < b.key || (ok == b.key && oi < b.id)) { b.key = ok; b.id = oi; }
    }
    return b;
}

template <int NQ>
__global__ __launch_bounds__(64) void mc_kernel(McArgs a) {
    extern __shared__ double acc[];   // [values of K of this block][chain_len][2]
    const int lane = threadIdx.x;
    const int P = a.P, L = a.chain_len, nK = a.Kmax - a.Kmin + 1;
    const int slice = blockIdx.x % a.nslices, group = blockIdx.x / a.nslices, groups = gridDim.x / a.nslices;
    const int cells = ((nK - slice + a.nslices - 1) / a.nslices) * L;
    const int cells_max = ((nK + a.nslices - 1) / a.nslices) * L;
    for (int c = lane; c < 2 * cells; c += 64) acc[c] = 0.0;
    __syncthreads();

    for (int64_t q0 = group; q0 < a.trials; q0 += groups) {
        const uint32_t trial = (uint32_t)(a.trial0 + q0);
        // fresh launch: P delays, shared by every K
        double base[NQ];
#pragma unroll
        for (int q = 0; q < NQ; ++q) {
            const int w = q * 64 + lane;
            base[q] = (w < P) ? (double)delay(a.dist, a.seed, kMonteCarlo, 0, trial, P, 1, w, 0, 0) : inf64();
        }
        if (a.variant == kBatchAsync) {
            // No worker ever waits, whatever K is: the pushes of all workers merged in time order are one sequence
            // shared by every K, and update l happens at push l K (the superposition of renewal processes behind
            // Lemma 5).  The sequence goes to LDS; worker w's n-th delay is keyed by (worker w, version n).
            double* push = acc + 2 * cells_max;
            const int npush = L * a.Kmax;
            double key[NQ];
            uint32_t started[NQ];
#pragma unroll
            for (int q = 0; q < NQ; ++q) { key[q] = base[q]; started[q] = 0; }
            if (lane == 0) push[0] = 0.0;
            for (int n = 1; n <= npush; ++n) {
                const Best b = wave_argmin<NQ>(key, lane);
                if (lane == 0) push[n] = b.key;
                if ((b.id & 63) == lane) {
#pragma unroll
                    for (int q = 0; q < NQ; ++q)
                        if ((b.id >> 6) == q) {
                            started[q] += 1;
                            key[q] = key[q] + (double)delay(a.dist, a.seed, kMonteCarlo, 0, trial, P, 1, b.id, 0, started[q]);
                        }
                }
            }
            __syncthreads();
            for (int c = lane; c < cells; c += 64) {       // one lane per (K, update) cell of this block
                const int kk = c / L, l = c - kk * L;
                const int K = a.Kmin + slice + kk * a.nslices;
                const double T = push[(l + 1) * K] - push[l * K];
                acc[2 * c] += T;
                acc[2 * c + 1] += T * T;
                if (a.per_trial) a.per_trial[(q0 * nK + (K - a.Kmin)) * L + l] = T;
            }
            __syncthreads();
            continue;
        }
        // the fresh draws are fp32 values: sorted as such (half the register traffic of the network), then widened
        double sorted0[NQ];
        {
            float fresh[NQ];
#pragma unroll
            for (int q = 0; q < NQ; ++q) fresh[q] = (float)base[q];
            sort_keys<NQ, float>(fresh, lane);
#pragma unroll
            for (int q = 0; q < NQ; ++q) sorted0[q] = (double)fresh[q];
        }

        for (int K = a.Kmin + slice; K <= a.Kmax; K += a.nslices) {
            double key[NQ];
            double t = 0.0;
#pragma unroll
            for (int q = 0; q < NQ; ++q) key[q] = (a.variant == kBatchSync) ? base[q] : sorted0[q];
            for (int l = 0; l < L; ++l) {
                double t_new;
                if (a.variant == kAsync) {
                    t_new = key_at<NQ>(key, K - 1);
                    // the a-th earliest finisher restarts at t_new with the a-th fresh delay
#pragma unroll
                    for (int q = 0; q < NQ; ++q) {
                        if (q * 64 >= K) continue;        // wave-uniform: no key of this register restarts
                        const int p = q * 64 + lane;
                        if (p < K) key[q] = t_new + (double)delay(a.dist, a.seed, kMonteCarlo, (uint32_t)K, trial, P, 1, p, 0, l + 1);
                    }
                    if (l + 1 < L) resort_prefix<NQ>(key, lane, K);
                } else {
                    if (l > 0) {
#pragma unroll
                        for (int q = 0; q < NQ; ++q) {
                            const int w = q * 64 + lane;
                            key[q] = (w < P) ? (double)delay(a.dist, a.seed, kMonteCarlo, (uint32_t)K, trial, P, 1, w, 0, l) : inf64();
                        }
                        if (a.variant == kSync) sort_keys<NQ, double>(key, lane);
                    }
                    if (a.variant == kSync) {
                        t_new = t + key_at<NQ>(key, K - 1);
                    } else {
                        double last = 0.0;
                        for (int pop = 0; pop < K; ++pop) {
                            const Best b = wave_argmin<NQ>(key, lane);
                            last = b.key;
                            if (pop + 1 < K && (b.id & 63) == lane) {
                                const double x = (double)delay(a.dist, a.seed, kMonteCarlo, (uint32_t)K, trial, P, 1, pop, 1, l);
#pragma unroll
                                for (int q = 0; q < NQ; ++q)
                                    if ((b.id >> 6) == q) key[q] = key[q] + x;
                            }
                        }
                        t_new = t + last;
                    }
                }
                const double T = t_new - t;
                t = t_new;
                const int cell = ((K - a.Kmin) / a.nslices) * L + l;
                if (lane == 0) {
                    acc[2 * cell] += T;
                    acc[2 * cell + 1] += T * T;
                    if (a.per_trial) a.per_trial[(q0 * nK + (K - a.Kmin)) * L + l] = T;
                }
            }
        }
    }
    __syncthreads();
    for (int c = lane; c < 2 * cells; c += 64) a.partial[(int64_t)blockIdx.x * 2 * cells_max + c] = acc[c];
}

}  // namespace
}  // namespace ssgd

using namespace ssgd;

namespace {
void mc_fail(const std::string& m) { set_global_error(m); }
}  // namespace

extern "C" __attribute__((visibility("default"))) ssgd_status ssgd_runtime_mc(int32_t variant, int32_t P, int32_t Kmin, int32_t Kmax,
                                       const ssgd_delay_dist* dist, int64_t trial0, int64_t trials,
                                       int32_t chain_len, uint64_t seed, void* hip_stream, double* mean,
                                       double* var, double* sum, double* sumsq, double* per_trial) {
    if (!dist || dist->kind == SSGD_TABLE || dist->kind < 0 || dist->kind > SSGD_PARETO) { mc_fail("invalid distribution"); return SSGD_EINVAL; }
    if ((dist->kind != SSGD_PARETO && !(dist->rate > 0)) || (dist->kind == SSGD_PARETO && (!(dist->alpha > 0) || !(dist->scale > 0)))) { mc_fail("invalid distribution parameters"); return SSGD_EINVAL; }
    if (variant < SSGD_K_SYNC || variant > SSGD_K_BATCH_ASYNC) { mc_fail("unknown variant"); return SSGD_EINVAL; }
    if (P < 1 || P > kMaxWorkers || Kmin < 1 || Kmax < Kmin || chain_len < 1 || trials < 1 || trial0 < 0 || trial0 + trials > (1ll << 32)) { mc_fail("P, K range, chain_len or trials out of range"); return SSGD_EINVAL; }
    if (variant != SSGD_K_BATCH_SYNC && variant != SSGD_K_BATCH_ASYNC && Kmax > P) { mc_fail("K must not exceed P"); return SSGD_EINVAL; }
    if (Kmax > 65535) { mc_fail("K too large"); return SSGD_EINVAL; }
    const int nK = Kmax - Kmin + 1;
    const int64_t cells = (int64_t)nK * chain_len;
    // accumulators of at most 5 KB per wavefront, so that 32 of them fit a CU
    int nslices = 1;
    while (nslices < nK && (int64_t)((nK + nslices - 1) / nslices) * chain_len * 16 > 5120) ++nslices;
    const int64_t cells_max = (int64_t)((nK + nslices - 1) / nslices) * chain_len;
    size_t lds = sizeof(double) * 2 * cells_max;
    if (variant == SSGD_K_BATCH_ASYNC) lds += sizeof(double) * ((size_t)chain_len * Kmax + 1);   // the push sequence of a trial
    if (lds > 64 * 1024) { mc_fail("chain_len (K-batch-async: chain_len * Kmax) too large for one launch"); return SSGD_EINVAL; }
    if (per_trial && trials * cells > (1ll << 27)) { mc_fail("per_trial output limited to 2^27 values"); return SSGD_EINVAL; }
    hipStream_t st = (hipStream_t)hip_stream;
    McArgs a{};
    a.dist.kind = dist->kind; a.dist.shift = (float)dist->shift; a.dist.rate = (float)dist->rate;
    a.dist.alpha = (float)dist->alpha; a.dist.scale = (float)dist->scale; a.dist.table = nullptr; a.dist.table_len = 0;
    a.seed = seed; a.variant = variant; a.P = P; a.Kmin = Kmin; a.Kmax = Kmax; a.chain_len = chain_len;
    a.trial0 = trial0; a.trials = trials; a.nslices = nslices;
    int dev = 0; hipDeviceProp_t prop;
    if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess) { mc_fail("no device"); return SSGD_EDEVICE; }
    const int64_t groups = std::max<int64_t>(1, std::min<int64_t>(trials, (int64_t)prop.multiProcessorCount * 32 / nslices));
    const int64_t blocks = groups * nslices;
    void *d_partial = nullptr, *d_pt = nullptr;
    ssgd_status rc = SSGD_OK;
    std::vector<double> host((size_t)(blocks * 2 * cells_max));
    do {
        if (hipMalloc(&d_partial, sizeof(double) * blocks * 2 * cells_max) != hipSuccess) { mc_fail("hipMalloc"); rc = SSGD_ENOMEM; break; }
        if (per_trial && hipMalloc(&d_pt, sizeof(double) * trials * cells) != hipSuccess) { mc_fail("hipMalloc"); rc = SSGD_ENOMEM; break; }
        a.partial = (double*)d_partial; a.per_trial = (double*)d_pt;
        const int nq = (P + 63) / 64;
        if (nq == 1) hipLaunchKernelGGL(mc_kernel<1>, dim3((unsigned)blocks), dim3(64), lds, st, a);
        else if (nq == 2) hipLaunchKernelGGL(mc_kernel<2>, dim3((unsigned)blocks), dim3(64), lds, st, a);
        else hipLaunchKernelGGL(mc_kernel<4>, dim3((unsigned)blocks), dim3(64), lds, st, a);
        hipError_t e = hipGetLastError();
        if (e == hipSuccess) e = hipStreamSynchronize(st);
        if (e == hipSuccess) e = hipMemcpy(host.data(), d_partial, sizeof(double) * host.size(), hipMemcpyDeviceToHost);
        if (e == hipSuccess && per_trial) e = hipMemcpy(per_trial, d_pt, sizeof(double) * trials * cells, hipMemcpyDeviceToHost);
        if (e != hipSuccess) { mc_fail(std::string("mc kernel: ") + hipGetErrorString(e)); rc = SSGD_EDEVICE; break; }
        for (int64_t c = 0; c < cells; ++c) {
            // cell (K, update) lives in the blocks of slice (K - Kmin) % nslices, at its place among their values of K
            const int64_t kk = c / chain_len, l = c % chain_len;
            const int64_t local = (kk / nslices) * chain_len + l;
            double s = 0.0, s2 = 0.0;
            for (int64_t b = kk % nslices; b < blocks; b += nslices) { s += host[(b * cells_max + local) * 2]; s2 += host[(b * cells_max + local) * 2 + 1]; }
            if (sum) sum[c] = s;
            if (sumsq) sumsq[c] = s2;
            if (mean) mean[c] = s / (double)trials;
            if (var) var[c] = trials > 1 ? (s2 - s * s / (double)trials) / (double)(trials - 1) : 0.0;
        }
    } while (0);
    if (d_partial) (void)hipFree(d_partial);
    if (d_pt) (void)hipFree(d_pt);
    return rc;
}
