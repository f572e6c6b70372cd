// Event process of the parameter server (Sec. 2.2) on the device: random delays
// (Sec. 3.1), K-of-P selection of the earliest finishers, staleness bookkeeping.
//
// One wavefront simulates one replica; each lane owns up to four of the P <= 256
// workers.  The delays do not depend on the data, so a whole segment of updates is
// scheduled before any gradient is taken; the gradient kernels then read the trace.
#include "common.hpp"

namespace ssgd {
namespace {


struct Best { double key; int32_t id; };

__device__ __forceinline__ bool before(double ka, int32_t ia, double kb, int32_t ib) {
    return ka < kb || (ka == kb && ia < ib);   // ties go to the lower worker id
}

// Smallest (key, id) over the first `width` lanes (a power of two covering every worker), known to every
// lane afterwards.  The butterfly carries the key only; the owner is found with a ballot, and the rare
// tie between lanes goes to the lowest worker id.
template <int CTRL>
__device__ __forceinline__ double dpp_fetch(double k) {
    const long long b = __double_as_longlong(k);
    const int lo = __builtin_amdgcn_update_dpp(0, (int)(uint32_t)b, CTRL, 0xF, 0xF, false);
    const int hi = __builtin_amdgcn_update_dpp(0, (int)(uint32_t)((unsigned long long)b >> 32), CTRL, 0xF, 0xF, false);
    return __longlong_as_double((long long)(((unsigned long long)(uint32_t)hi << 32) | (uint32_t)lo));
}

__device__ __forceinline__ Best wave_min(Best b, int width) {
    double k = b.key;
    // inside a row of 16 lanes the exchange is a data-parallel-primitive move (no LDS round trip):
    // lane ^ 1, lane ^ 2, then the mirrored lane of the other half of 8, then of 16
    if (width > 1) { const double o = dpp_fetch<0xB1>(k); k = o < k ? o : k; }     // quad_perm [1,0,3,2]
    if (width > 2) { const double o = dpp_fetch<0x4E>(k); k = o < k ? o : k; }     // quad_perm [2,3,0,1]
    if (width > 4) { const double o = dpp_fetch<0x141>(k); k = o < k ? o : k; }    // row_half_mirror
    if (width > 8) { const double o = dpp_fetch<0x140>(k); k = o < k ? o : k; }    // row_mirror
    for (int off = 16; off < width; off <<= 1) {
        const double ok = __shfl_xor(k, off, 64);
        k = ok < k ? ok : k;
    }
    const long long kb = __double_as_longlong(k);
    const uint32_t lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)kb);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)((unsigned long long)kb >> 32));
    const double kmin = __longlong_as_double((long long)(((unsigned long long)hi << 32) | lo));
    unsigned long long mask = __ballot(b.key == kmin && b.id != 0x7FFFFFFF);
    int best = 0x7FFFFFFF;
    while (mask) {
        const int l = __builtin_ctzll(mask);
        mask &= mask - 1;
        const int id = __builtin_amdgcn_readlane(b.id, l);
        best = id < best ? id : best;
    }
    return Best{kmin, best};
}

template <int NQ>
__device__ __forceinline__ Best local_min(const double (&key)[NQ], uint32_t skip, int lane, int P) {
    Best b{__longlong_as_double(0x7FF0000000000000LL), 0x7FFFFFFF};
#pragma unroll
    for (int q = 0; q < NQ; ++q) {
        const int w = lane + 64 * q;
        if (w < P && !((skip >> q) & 1u) && before(key[q], w, b.key, b.id)) { b.key = key[q]; b.id = w; }
    }
    return b;
}

// NQ: workers per lane (1 while P <= 64).  TABLE: delays come from a table in memory; kept out of the common
// instantiation, whose loop then holds no load and never waits for its own trace stores.
template <int NQ, bool TABLE>
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

    auto draw_delay = [&](uint32_t worker, uint32_t ordinal, uint32_t version) -> float {
        if constexpr (TABLE) return delay(a.dist, a.seed, kDelay, 0, rep, P, a.table_ord, worker, ordinal, version);
        else return delay_from_bits(a.dist, draw(a.seed, kDelay, 0, rep, worker, ordinal, version).x);
    };
    int width = 1;
    while (width < P && width < 64) width <<= 1;
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
    if (NQ == 1 && !TABLE && a.variant == kAsync && P <= 16 && !(a.interval_t > 0.0)) {
        // K-async with few workers, in a loop of its own: every lane ranks its worker's finish time against all
        // P of them, which gives the K earliest in consume-list order at once.  The delay a worker would draw if
        // it restarted now depends on (worker, version) only: the 64 lanes draw it for 64 / width versions in one go.
        const int wmask = width - 1, per = 64 / width;
        const int me = lane & wmask;
        float ahead = 0.0f;
        int64_t ahead_base = a.j0 + 1 - per;         // refilled before the first use
        double mine = key[0];
        int32_t mytau = tau[0];
        for (; done < a.count; ++done) {
            const int64_t j = a.j0 + done;
            const int slot = (int)(j + 1 - ahead_base);
            if (slot >= per) {
                ahead_base = j + 1;
                ahead = 0.0f;
                if (me < P) ahead = draw_delay((uint32_t)me, 0, (uint32_t)(ahead_base + lane / width));
            }
            const float restart = __shfl(ahead, me + width * (slot >= per ? 0 : slot), 64);
            const long long bits = __double_as_longlong(mine);
            int rank = 0;
            for (int w = 0; w < P; ++w) {
                const uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)bits, w);
                const uint32_t hi = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)((unsigned long long)bits >> 32), w);
                const double other = __longlong_as_double((long long)(((unsigned long long)hi << 32) | lo));
                rank += before(other, w, mine, lane) ? 1 : 0;
            }
            const int last = __builtin_ctzll(__ballot(lane < P && rank == K - 1));
            const uint32_t tlo = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)bits, last);
            const uint32_t thi = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)((unsigned long long)bits >> 32), last);
            const double t_new = __longlong_as_double((long long)(((unsigned long long)thi << 32) | tlo));
            if (lane < P && rank < K) {
                tr_sel[j * Kcap + rank] = lane; tr_tau[j * Kcap + rank] = mytau; tr_ord[j * Kcap + rank] = 0;
                mytau = (int32_t)(j + 1);
                mine = t_new + (double)restart;
            }
            for (int l = K + lane; l < Kcap; l += 64) {
                tr_sel[j * Kcap + l] = -1; tr_tau[j * Kcap + l] = -1; tr_ord[j * Kcap + l] = -1;
            }
            if (lane == 0) { tr_t[j] = t_new; tr_K[j] = K; }
            clock = t_new;
        }
        key[0] = mine; tau[0] = mytau;
    }
    if (!TABLE && a.variant == kAsync && K >= 8 && 18 * K >= P * NQ && (NQ > 1 || P > 16) && !(a.interval_t > 0.0)) {
        // K-async with many contributors per update: K rounds of a wave-wide argmin (0.4 us each) cost more than
        // ranking every worker's finish time against all P of them (one pass over the workers, whatever K is: 22 us
        // at P = 256), which also gives the K earliest in consume-list order.
        for (; done < a.count; ++done) {
            const int64_t j = a.j0 + done;
            double nd[NQ];
            int rank[NQ];
#pragma unroll
            for (int q = 0; q < NQ; ++q) {
                const int w = lane + 64 * q;
                nd[q] = (w < P) ? (double)draw_delay(w, 0, (uint32_t)j + 1u) : 0.0;
                rank[q] = 0;
            }
#pragma unroll
            for (int qo = 0; qo < NQ; ++qo) {
                const long long bits = __double_as_longlong(key[qo]);
                const int lim = min(64, P - 64 * qo);                  // workers held in register qo
                for (int l = 0; l < lim; ++l) {
                    const uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)bits, l);
                    const uint32_t hi = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)((unsigned long long)bits >> 32), l);
                    const double other = __longlong_as_double((long long)(((unsigned long long)hi << 32) | lo));
                    const int wo = l + 64 * qo;
#pragma unroll
                    for (int q = 0; q < NQ; ++q) rank[q] += before(other, wo, key[q], lane + 64 * q) ? 1 : 0;
                }
            }
            // the K-th earliest finish time is the time of the update
            double t_new = 0.0;
#pragma unroll
            for (int q = 0; q < NQ; ++q) {
                const unsigned long long m = __ballot(lane + 64 * q < P && rank[q] == K - 1);
                if (m != 0ull) {
                    const int l = __builtin_ctzll(m);
                    const long long bits = __double_as_longlong(key[q]);
                    const uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)bits, l);
                    const uint32_t hi = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)((unsigned long long)bits >> 32), l);
                    t_new = __longlong_as_double((long long)(((unsigned long long)hi << 32) | lo));
                }
            }
#pragma unroll
            for (int q = 0; q < NQ; ++q) {
                const int w = lane + 64 * q;
                if (w < P && rank[q] < K) {
                    tr_sel[j * Kcap + rank[q]] = w; tr_tau[j * Kcap + rank[q]] = tau[q]; tr_ord[j * Kcap + rank[q]] = 0;
                    tau[q] = (int32_t)(j + 1);
                    key[q] = t_new + nd[q];
                }
            }
            for (int l = K + lane; l < Kcap; l += 64) {
                tr_sel[j * Kcap + l] = -1; tr_tau[j * Kcap + l] = -1; tr_ord[j * Kcap + l] = -1;
            }
            if (lane == 0) { tr_t[j] = t_new; tr_K[j] = K; }
            clock = t_new;
        }
    }
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
                if (w < P) key[q] = (double)draw_delay(w, 0, ver);
            }
            uint32_t taken = 0;
            double last = 0.0;
            for (int l = 0; l < K; ++l) {
                const Best b = wave_min(local_min(key, taken, lane, P), width);
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
                                key[qq] = key[qq] + (double)draw_delay(b.id, ord[qq], ver);
                        }
                    }
                }
            }
            t_new = clock + last;
        } else if (a.variant == kBatchAsync) {
            // K-batch-async: the K earliest mini-batches contribute, whoever computed them.  A worker that pushes
            // one of the first K-1 re-reads the parameters (still w_j) and starts its next mini-batch at once; the
            // K-th push triggers update j, and that worker reads w_{j+1}.
            for (int l = 0; l < K; ++l) {
                const Best b = wave_min(local_min(key, 0u, lane, P), width);
                t_new = b.key;
                if ((b.id & 63) == lane) {
                    const int q = b.id >> 6;
#pragma unroll
                    for (int qq = 0; qq < NQ; ++qq) {
                        if (qq != q) continue;
                        tr_sel[j * Kcap + l] = b.id; tr_tau[j * Kcap + l] = tau[qq]; tr_ord[j * Kcap + l] = ord[qq];
                        if (l + 1 < K) {
                            if (tau[qq] == (int32_t)j) ord[qq] += 1; else { tau[qq] = (int32_t)j; ord[qq] = 0; }
                            key[qq] = key[qq] + (double)draw_delay(b.id, ord[qq], ver);
                        } else {
                            tau[qq] = (int32_t)(j + 1); ord[qq] = 0;
                            key[qq] = t_new + (double)draw_delay(b.id, 0, ver + 1u);
                        }
                    }
                }
            }
        } else {
            // K-async: the K earliest finishers contribute; only they restart, at t_{j+1}.  The delay a
            // worker would draw if it restarted now depends on (worker, version) only, so every lane
            // draws it up front, off the selection's dependency chain.
            double nd[NQ];
#pragma unroll
            for (int q = 0; q < NQ; ++q) {
                const int w = lane + 64 * q;
                nd[q] = 0.0;
                if (w < P) nd[q] = (double)draw_delay(w, 0, ver + 1u);
            }
            uint32_t taken = 0;
            for (int l = 0; l < K; ++l) {
                const Best b = wave_min(local_min(key, taken, lane, P), width);
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
                tau[q] = (int32_t)(j + 1);
                key[q] = t_new + nd[q];
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
    const bool table = a.dist.kind == 3;
    if (a.P <= 64) {
        if (table) hipLaunchKernelGGL((schedule_kernel<1, true>), dim3(replicas), dim3(64), 0, s, a);
        else hipLaunchKernelGGL((schedule_kernel<1, false>), dim3(replicas), dim3(64), 0, s, a);
    } else {
        if (table) hipLaunchKernelGGL((schedule_kernel<kMaxWorkers / 64, true>), dim3(replicas), dim3(64), 0, s, a);
        else hipLaunchKernelGGL((schedule_kernel<kMaxWorkers / 64, false>), dim3(replicas), dim3(64), 0, s, a);
    }
}

void launch_adasync(const AdaArgs& a, int replicas, hipStream_t s) {
    hipLaunchKernelGGL(adasync_kernel, dim3((replicas + 63) / 64), dim3(64), 0, s, a, replicas);
}

}  // namespace ssgd
