// Mini-batch gradients of the linear models at possibly stale parameters, the
// K-gradient aggregate and the parameter-server update (Sec. 2.2, Eq. (2), Eq. (3)).
//
// One persistent launch runs a whole segment of updates.  Each replica is a
// "cluster" of G workgroups; workgroup s owns the column slice [s*SL, (s+1)*SL) of
// the sample matrix, of the weights and of every parked gradient, so the update
// and the staleness bookkeeping never leave the workgroup.  Per step v:
//   1. compute list of v (the mini-batches that start at parameter version v): the
//      rows are in LDS; partial logits X_slice W_slice^T on the fp32 MFMA units;
//   2. one exchange of partial logits inside the cluster (arrival counter in HBM);
//   3. residual / softmax, then the gradient slice delta^T X_slice (MFMA) from the same
//      LDS tile; a gradient that update v consumes is added to the aggregate in
//      registers, any other is parked per slot (a K-async worker keeps it until it is selected);
//   4. update v: w -= (lr/K) sum over the consume list of update v.
// The schedule (who starts, who is consumed, K) was written by the schedule kernel and
// does not depend on the numerics, so the rows of step v+1 are gathered from HBM while
// step v computes.  Waves are specialised for that: the vector-memory counter of a wave
// retires in order, so a wave that had the long HBM gather in flight would stall on it
// at the first cache-resident load it needs.  Compute waves never touch the sample
// matrix; loader waves hold the next tile in registers and only join the barriers.
#include "common.hpp"

namespace ssgd {
namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int ROWS = 64;   // rows of one LDS tile
constexpr int ZB = 6;      // partial-logit blocks fetched per batch of the exchange

struct ChunkMap {
    int n_chunks, rpc, spr;
};

__device__ __forceinline__ ChunkMap chunk_map(int n_rec, int mp) {
    ChunkMap c;
    if (mp <= ROWS) { c.rpc = ROWS / mp; c.spr = 1; c.n_chunks = (n_rec + c.rpc - 1) / c.rpc; }
    else { c.rpc = 1; c.spr = (mp + ROWS - 1) / ROWS; c.n_chunks = n_rec * c.spr; }
    return c;
}

// Exchange buffer accesses.  Fenced mode: plain accesses ordered by agent-scope
// release/acquire fences.  Fast mode: every access is an agent-scope relaxed atomic (served by
// the L2 that all workgroups of a cluster share, never by a CU's L1), ordered by the completion
// of the stores before the arrival counter is raised.
__device__ __forceinline__ void exch_store(float* p, f32x4 v, bool fast) {
    if (fast) {
#pragma unroll
        for (int e = 0; e < 4; ++e) __hip_atomic_store(p + e, v[e], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    } else {
        *reinterpret_cast<f32x4*>(p) = v;
    }
}

__device__ __forceinline__ f32x4 exch_load(const float* p, bool fast) {
    if (fast) {
        f32x4 v;
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] = __hip_atomic_load(p + e, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        return v;
    }
    return *reinterpret_cast<const f32x4*>(p);
}

constexpr int loader_waves(int nbw) { return nbw; }

template <int NBW>
__global__ __launch_bounds__(64 * (NBW + loader_waves(NBW)), 4) void linear_cluster_kernel(LinArgs a) {
    constexpr int SL = 64 * NBW;            // columns per workgroup
    constexpr int NTC = 64 * NBW;           // compute threads (waves 0 .. NBW-1)
    constexpr int LW = loader_waves(NBW);   // loader waves
    constexpr int NTL = 64 * LW;
    constexpr int CPR = SL / 4;             // float4 chunks per tile row
    constexpr int RB = 4 / NBW;             // 16-row blocks per compute wave in the forward pass
    constexpr int LLOADS = ROWS * CPR / NTL;   // float4 loads per loader thread per tile

    // cluster id / slice id from the block id: consecutive block ids go to different XCDs, so
    // all slices of one cluster take block ids that are congruent modulo 8 and share one L2.
    const int xcd = blockIdx.x & 7, slot_in_xcd = blockIdx.x >> 3;
    const int cluster = (slot_in_xcd / a.G) * 8 + xcd;
    const int slice = slot_in_xcd % a.G;
    if (cluster >= a.replicas) return;
    const int rep = a.replica0 + cluster;

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const bool loader = tid >= NTC;
    const int lt = tid - NTC;               // loader thread index
    const int d = a.d, C = a.C, m = a.m, mp = a.mp, P = a.P, S = a.S, G = a.G;
    const int Kcap = a.tr.Kcap;
    const int64_t cap = a.tr.cap;
    const int64_t nw = (a.kind == kLsq) ? d : (int64_t)C * d + C;
    const int col0 = slice * SL;
    const bool async = a.variant == kAsync;

    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    float* tile = reinterpret_cast<float*>(smem);            // [64][SL], 16-byte chunks xor-swizzled by row
    float* wlds = tile + ROWS * SL;                          // [C][SL], same swizzle: the weights live here
    float* zbuf = wlds + C * SL;                             // [64][16] logits, then delta
    uint32_t* rowid = reinterpret_cast<uint32_t*>(zbuf + ROWS * 16);   // [64]
    float* ylab = reinterpret_cast<float*>(rowid + ROWS);    // [64] label (int bits) or target
    float* lossrow = ylab + ROWS;                            // [64]
    float* bias = lossrow + ROWS;                            // [16]
    float* small = bias + 16;                                // [S][17] bias gradient + loss per slot
    int* stop = reinterpret_cast<int*>(small + S * 17);      // [4]: stop flag, exchange mode, same-XCD flag
    unsigned char* fresh = reinterpret_cast<unsigned char*>(stop + 4);   // [S] slot is consumed by this update

    const int32_t* tr_K = a.tr.K + (int64_t)rep * cap;
    const int32_t* tr_sel = a.tr.sel + (int64_t)rep * cap * Kcap;
    const int32_t* tr_tau = a.tr.tau + (int64_t)rep * cap * Kcap;
    const int32_t* tr_ord = a.tr.ord + (int64_t)rep * cap * Kcap;
    float* tr_loss = a.tr.loss + (int64_t)rep * cap;
    float* params = a.params + (int64_t)rep * nw;
    float* park = a.park + ((int64_t)rep * G + slice) * S * 16 * NTC;
    float* small_g = a.park_small + ((int64_t)rep * G + slice) * S * 17;
    float* zpart = a.zpart + (int64_t)rep * 2 * G * a.maxrows * 16;
    unsigned long long* arrive = a.arrive + rep;
    int32_t* xcc_ids = a.xcc_ids + (int64_t)rep * G;
    const float inv_m = 1.0f / (float)m;
    const bool vec_ok = (d % 4) == 0;
    const int nquad = (C + 3) / 4;       // 4-class groups that carry data

    // Workgroup barrier.  Loader waves must not wait for their gathers here, so they only make
    // their LDS writes visible; compute waves use the full barrier (their global stores complete).
    auto wg_barrier = [&]() {
        if (loader) {
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
            __builtin_amdgcn_s_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
        } else {
            __syncthreads();
        }
    };

    // ---- compute threads: share of the parameters: class 4*(lane/16)+v, columns own_col..own_col+3
    const int own_ch = 16 * wave + (lane & 15);
    const int own_col = col0 + 4 * own_ch;
    const int own_cls = 4 * (lane >> 4);
    if (!loader) {
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int cls = own_cls + v;
            if (cls < C) {
                f32x4 val;
#pragma unroll
                for (int c = 0; c < 4; ++c) val[c] = (own_col + c < d) ? params[(int64_t)cls * d + own_col + c] : 0.0f;
                *reinterpret_cast<f32x4*>(wlds + cls * SL + ((own_ch ^ (cls & 15)) << 2)) = val;
            }
        }
        if (tid < 16) bias[tid] = (a.kind == kSoftmax && tid < C) ? params[(int64_t)C * d + tid] : 0.0f;
        for (int q = tid; q < S * 17; q += NTC) small[q] = small_g[q];
        if (tid == 0) {
            stop[0] = __hip_atomic_load(a.abort_flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            stop[1] = 0;   // exchange mode: fenced until the cluster is known to share an XCD
            stop[2] = 0;
            // XCC_ID hardware register: the XCD this workgroup runs on
            const int my_xcc = (int)(__builtin_amdgcn_s_getreg((3 << 11) | 20) & 0xF);
            __hip_atomic_store(xcc_ids + slice, my_xcc, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
    wg_barrier();
    if (stop[0] != 0) return;

    // record r of the compute list of version ver -> (worker, ordinal)
    auto rec_worker = [&](int64_t ver, int r) -> int {
        if (async) return (ver == 0) ? r : tr_sel[(ver - 1) * Kcap + r];
        return tr_sel[ver * Kcap + r];
    };
    auto rec_ord = [&](int64_t ver, int r) -> int { return async ? 0 : tr_ord[ver * Kcap + r]; };

    // The two roles run separate loops (so that the registers that hold the next tile are not
    // live in the compute code) and meet at the same sequence of workgroup barriers:
    //   per step:  single-tile step: T | S X | (Z D) | U          T tile in LDS, S exchange stores done,
    //              multi-tile step:  (T F)* | S X | (T Z D R)* | U   X exchange complete, Z logits in LDS,
    //   D delta in LDS, R tile may be rewritten, F forward done, U update done; one more after the loop.
    if (loader) {
        // =============================== loader waves ===============================
        auto lbar = [&]() {
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
            __builtin_amdgcn_s_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
        };
        f32x4 pref[LLOADS];      // the tile gathered ahead
        uint32_t row_id = 0xFFFFFFFFu;   // sample id / label of tile row `lane`
        float row_lab = 0.0f;
        bool have_pref = false;

        // Loader wave lw issues, per instruction i, one 16-byte load per lane that covers RPI whole tile
        // rows: rows (lw + LW*i)*RPI + j, j < RPI, lane -> (j = lane / CPR, chunk = lane % CPR).  The row's
        // sample id comes from lane `row` of this wave through readlane, so the row base stays scalar.
        constexpr int RPI = 64 / CPR;
        const int lw = __builtin_amdgcn_readfirstlane(lt >> 6);
        const int sub = lane / CPR, lch = lane % CPR;
        const int lcol = col0 + 4 * lch;

        auto fetch = [&](int64_t ver, int nrec_v, const ChunkMap& cmv, int chunk) {
            int r, s;
            bool ok;
            if (mp <= ROWS) { r = chunk * cmv.rpc + lane / mp; s = lane % mp; ok = lane < cmv.rpc * mp && r < nrec_v && s < m; }
            else { r = chunk / cmv.spr; s = ROWS * (chunk % cmv.spr) + lane; ok = s < m; }
            row_id = 0xFFFFFFFFu;
            row_lab = 0.0f;
            if (ok) {
                row_id = batch_index(a.seed, (uint32_t)rep, (uint32_t)rec_worker(ver, r), (uint32_t)rec_ord(ver, r),
                                     (uint32_t)ver, (uint32_t)s, a.N);
                row_lab = (a.kind == kLsq) ? reinterpret_cast<const float*>(a.y)[row_id]
                                           : __int_as_float(reinterpret_cast<const int32_t*>(a.y)[row_id]);
            }
#pragma unroll
            for (int i = 0; i < LLOADS; ++i) {
                const int row0 = (lw + LW * i) * RPI;
                uint32_t id = (uint32_t)__builtin_amdgcn_readlane((int)row_id, row0);
#pragma unroll
                for (int j = 1; j < RPI; ++j) {
                    const uint32_t idj = (uint32_t)__builtin_amdgcn_readlane((int)row_id, row0 + j);
                    if (sub == j) id = idj;
                }
                f32x4 val = {0.0f, 0.0f, 0.0f, 0.0f};
                if (id != 0xFFFFFFFFu) {
                    const float* src = a.X + (int64_t)id * d + lcol;
                    if (vec_ok) {
                        if (lcol + 3 < d) val = *reinterpret_cast<const f32x4*>(src);
                    } else {
                        if (lcol + 0 < d) val.x = src[0];
                        if (lcol + 1 < d) val.y = src[1];
                        if (lcol + 2 < d) val.z = src[2];
                        if (lcol + 3 < d) val.w = src[3];
                    }
                }
                pref[i] = val;
            }
        };
        auto publish = [&]() {
#pragma unroll
            for (int i = 0; i < LLOADS; ++i) {
                const int row = (lw + LW * i) * RPI + sub;
                *reinterpret_cast<f32x4*>(tile + row * SL + ((lch ^ (row & 15)) << 2)) = pref[i];
            }
            if (lt < ROWS) { rowid[lt] = row_id; ylab[lt] = row_lab; }
        };

        for (int64_t step = 0; step < a.nsteps; ++step) {
            const int64_t v = a.v0 + step;
            const int Kv = tr_K[v];
            const int n_rec = async ? ((v == 0) ? P : tr_K[v - 1]) : Kv;
            const ChunkMap cm = chunk_map(n_rec, mp);
            const bool single = cm.n_chunks == 1;
            if (single) {
                if (!have_pref) fetch(v, n_rec, cm, 0);
                publish();
                lbar();                                     // T
                // the rows of step v+1 are gathered now and stay in registers until step v is done
                have_pref = false;
                if (step + 1 < a.nsteps) {
                    const int nrec_n = async ? Kv : tr_K[v + 1];
                    const ChunkMap cmn = chunk_map(nrec_n, mp);
                    if (cmn.n_chunks == 1) { fetch(v + 1, nrec_n, cmn, 0); have_pref = true; }
                }
            } else {
                have_pref = false;
                for (int chunk = 0; chunk < cm.n_chunks; ++chunk) {
                    fetch(v, n_rec, cm, chunk);
                    publish();
                    lbar();                                 // T
                    lbar();                                 // F
                }
            }
            lbar();                                         // S
            lbar();                                         // X
            if (stop[0] != 0) return;
            for (int chunk = 0; chunk < cm.n_chunks; ++chunk) {
                if (!single) { fetch(v, n_rec, cm, chunk); publish(); lbar(); }   // T
                lbar();                                     // Z
                lbar();                                     // D
                if (!single) lbar();                        // R
            }
            lbar();                                         // U
        }
        lbar();
        return;
    }

    // ================================= compute waves =================================
    unsigned long long ph[8] = {0, 0, 0, 0, 0, 0, 0, 0}, tprev = 0;
    const bool profiling = a.prof != nullptr && tid == 0;
    auto mark = [&](int phase) {
        if (profiling) { const unsigned long long now = clock64(); ph[phase] += now - tprev; tprev = now; }
    };

    for (int64_t step = 0; step < a.nsteps; ++step) {
        const int64_t v = a.v0 + step;
        if (profiling) tprev = clock64();
        const bool fast = stop[1] != 0;
        const int par = (int)((a.arrive_base + (unsigned long long)step) & 1ull);
        float* zp_mine = zpart + ((int64_t)par * G + slice) * a.maxrows * 16;
        const float* zp_all = zpart + (int64_t)par * G * a.maxrows * 16;

        // ---- lists of step v
        const int Kv = tr_K[v];
        const int n_rec = async ? ((v == 0) ? P : tr_K[v - 1]) : Kv;
        const ChunkMap cm = chunk_map(n_rec, mp);
        const bool single = cm.n_chunks == 1;

        auto forward = [&](int chunk) {
            // partial logits of the tile: D[class][row] += W[class][k] * X[row][k] over this slice
#pragma unroll
            for (int b = 0; b < RB; ++b) {
                const int rb = wave * RB + b;
                const int row = 16 * rb + (lane & 15);
                f32x4 acc0 = {0.f, 0.f, 0.f, 0.f}, acc1 = {0.f, 0.f, 0.f, 0.f};
                const int cls = lane & 15;
#pragma unroll 4
                for (int s = 0; s < SL / 16; ++s) {
                    const int ch = 4 * s + (lane >> 4);
                    f32x4 wv = {0.f, 0.f, 0.f, 0.f};
                    if (cls < C) wv = *reinterpret_cast<const f32x4*>(wlds + cls * SL + ((ch ^ cls) << 2));
                    const f32x4 xv = *reinterpret_cast<const f32x4*>(tile + row * SL + ((ch ^ (row & 15)) << 2));
                    acc0 = __builtin_amdgcn_mfma_f32_16x16x4f32(wv.x, xv.x, acc0, 0, 0, 0);
                    acc1 = __builtin_amdgcn_mfma_f32_16x16x4f32(wv.y, xv.y, acc1, 0, 0, 0);
                    acc0 = __builtin_amdgcn_mfma_f32_16x16x4f32(wv.z, xv.z, acc0, 0, 0, 0);
                    acc1 = __builtin_amdgcn_mfma_f32_16x16x4f32(wv.w, xv.w, acc1, 0, 0, 0);
                }
                const f32x4 out = acc0 + acc1;   // lane: classes 4*(lane/16)+0..3 of row `row`
                if ((lane >> 4) < nquad)
                    exch_store(zp_mine + ((int64_t)chunk * ROWS + row) * 16 + 4 * (lane >> 4), out, fast);
            }
        };

        // ---- phase 1: partial logits of every chunk
        if (single) {
            __syncthreads();                                // T: tile, row ids and labels of step v are in LDS
            forward(0);
        } else {
            for (int chunk = 0; chunk < cm.n_chunks; ++chunk) {
                __syncthreads();                            // T
                forward(chunk);
                __syncthreads();                            // F
            }
        }
        mark(0);

        float gsum[16];
        float bsum = 0.0f;
#pragma unroll
        for (int e = 0; e < 16; ++e) gsum[e] = 0.0f;

        // which slots does update v take from this very step (tau == v)?
        for (int s = tid; s < S; s += NTC) {
            unsigned char f = 0;
            if (!async) f = s < Kv;
            else
                for (int l = 0; l < Kv; ++l)
                    if (tr_sel[v * Kcap + l] == s && tr_tau[v * Kcap + l] == (int32_t)v) f = 1;
            fresh[s] = f;
        }

        // ---- phase 2: exchange inside the cluster
        __syncthreads();                                    // S: every thread's exchange stores have completed
        if (G > 1 && tid == 0) {
            if (fast) __hip_atomic_fetch_add(arrive, 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            else __hip_atomic_fetch_add(arrive, 1ull, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
        }
        mark(1);
        // while the exchange is in flight: the part of update v that earlier steps parked
        for (int l = 0; l < Kv; ++l) {
            if (tr_tau[v * Kcap + l] == (int32_t)v) continue;
            const int slot = async ? tr_sel[v * Kcap + l] : l;
            const float* pk = park + (int64_t)slot * 16 * NTC + tid;
#pragma unroll
            for (int vv = 0; vv < 4; ++vv)
#pragma unroll
                for (int c = 0; c < 4; ++c)
                    if (own_cls + vv < C) gsum[vv * 4 + c] += pk[(vv * 4 + c) * NTC];
            if (tid < 17) bsum += small[slot * 17 + tid];
        }
        mark(2);
        if (G > 1 && tid == 0) {
            const unsigned long long target = (a.arrive_base + (unsigned long long)step + 1ull) * (unsigned long long)G;
            uint32_t spins = 0;
            for (;;) {
                const unsigned long long got = fast ? __hip_atomic_load(arrive, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)
                                                    : __hip_atomic_load(arrive, __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_AGENT);
                if (got >= target) break;
                __builtin_amdgcn_s_sleep(1);
                if (++spins > a.spin_limit ||
                    __hip_atomic_load(a.abort_flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0) {
                    __hip_atomic_store(a.abort_flag, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    stop[0] = 1;
                    break;
                }
            }
            if (!fast && a.allow_fast && stop[0] == 0) {
                // first exchange of the launch: do all slices of this cluster share an XCD (one L2)?
                int same = 1;
                const int mine = __hip_atomic_load(xcc_ids + slice, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                for (int g = 0; g < G; ++g)
                    if (__hip_atomic_load(xcc_ids + g, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != mine) same = 0;
                stop[2] = same;
            }
        }
        __syncthreads();                                    // X
        if (G > 1 && !fast) __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
        if (stop[0] != 0) return;   // uniform: every thread reads the same LDS word
        mark(3);

        // ---- phase 3: residual / softmax and the gradient slices
        for (int chunk = 0; chunk < cm.n_chunks; ++chunk) {
            if (!single) __syncthreads();                   // T
            // full logits of the 64 rows: sum of the G partials in slice order
            for (int q = tid; q < ROWS * 4; q += NTC) {
                f32x4 z = {0.f, 0.f, 0.f, 0.f};
                if ((q & 3) < nquad) {
                    const float* src = zp_all + (int64_t)chunk * ROWS * 16 + 4 * q;
                    for (int g0 = 0; g0 < G; g0 += ZB) {
                        f32x4 part[ZB];
#pragma unroll
                        for (int i = 0; i < ZB; ++i)
                            if (g0 + i < G) part[i] = exch_load(src + (int64_t)(g0 + i) * a.maxrows * 16, fast);
#pragma unroll
                        for (int i = 0; i < ZB; ++i)
                            if (g0 + i < G) z += part[i];
                    }
                }
                *reinterpret_cast<f32x4*>(zbuf + 4 * q) = z;
            }
            __syncthreads();                                // Z
            if (tid < ROWS) {
                float* z = zbuf + tid * 16;
                float dl[16];
                float loss = 0.0f;
                const bool ok = rowid[tid] != 0xFFFFFFFFu;
                if (a.kind == kLsq) {
                    const float r = z[0] - ylab[tid];
                    dl[0] = ok ? r * inv_m : 0.0f;
                    loss = ok ? 0.5f * r * r : 0.0f;
#pragma unroll
                    for (int c = 1; c < 16; ++c) dl[c] = 0.0f;
                } else {
                    const int lab = __float_as_int(ylab[tid]);
                    float zmax = -3.0e38f;
#pragma unroll
                    for (int c = 0; c < 16; ++c) {
                        dl[c] = z[c] + bias[c];
                        if (c < C) zmax = fmaxf(zmax, dl[c]);
                    }
                    float den = 0.0f;
#pragma unroll
                    for (int c = 0; c < 16; ++c) {
                        const float e = (c < C) ? expf(dl[c] - zmax) : 0.0f;
                        den += e;
                        if (c == lab) loss = -(dl[c] - zmax);
                        dl[c] = e;
                    }
                    loss = ok ? loss + logf(den) : 0.0f;
                    const float inv = 1.0f / den;
#pragma unroll
                    for (int c = 0; c < 16; ++c) {
                        const float p = dl[c] * inv - ((c == lab) ? 1.0f : 0.0f);
                        dl[c] = (ok && c < C) ? p * inv_m : 0.0f;
                    }
                }
#pragma unroll
                for (int c = 0; c < 16; ++c) z[c] = dl[c];
                lossrow[tid] = loss * inv_m;
            }
            __syncthreads();                                // D

            // per record of this chunk: bias gradient, loss, and the gradient slice
            const int nseg = (mp <= ROWS) ? cm.rpc : 1;
            for (int sg = 0; sg < nseg; ++sg) {
                int r, row_lo, row_hi;
                bool first;
                if (mp <= ROWS) { r = chunk * cm.rpc + sg; row_lo = sg * mp; row_hi = row_lo + mp; first = true; }
                else {
                    r = chunk / cm.spr;
                    const int sub = chunk % cm.spr;
                    row_lo = 0; row_hi = min(ROWS, mp - ROWS * sub); first = (sub == 0);
                }
                if (r >= n_rec) break;
                const int slot = async ? rec_worker(v, r) : r;
                const bool is_fresh = fresh[slot] != 0;
                if (tid < 17) {
                    float sacc = 0.0f;
                    if (tid < 16) { for (int row = row_lo; row < row_hi; ++row) sacc += zbuf[row * 16 + tid]; }
                    else { for (int row = row_lo; row < row_hi; ++row) sacc += lossrow[row]; }
                    if (is_fresh) bsum += sacc;
                    else small[slot * 17 + tid] = first ? sacc : small[slot * 17 + tid] + sacc;
                }
                f32x4 acc[4];
#pragma unroll
                for (int c = 0; c < 4; ++c) acc[c] = f32x4{0.f, 0.f, 0.f, 0.f};
                for (int ks = row_lo / 4; ks < row_hi / 4; ++ks) {
                    const int row = 4 * ks + (lane >> 4);
                    const float dv = zbuf[row * 16 + (lane & 15)];
                    const f32x4 xv = *reinterpret_cast<const f32x4*>(tile + row * SL + ((own_ch ^ (row & 15)) << 2));
                    acc[0] = __builtin_amdgcn_mfma_f32_16x16x4f32(dv, xv.x, acc[0], 0, 0, 0);
                    acc[1] = __builtin_amdgcn_mfma_f32_16x16x4f32(dv, xv.y, acc[1], 0, 0, 0);
                    acc[2] = __builtin_amdgcn_mfma_f32_16x16x4f32(dv, xv.z, acc[2], 0, 0, 0);
                    acc[3] = __builtin_amdgcn_mfma_f32_16x16x4f32(dv, xv.w, acc[3], 0, 0, 0);
                }
                if (is_fresh) {
#pragma unroll
                    for (int vv = 0; vv < 4; ++vv)
#pragma unroll
                        for (int c = 0; c < 4; ++c) gsum[vv * 4 + c] += acc[c][vv];
                } else {
                    float* pk = park + (int64_t)slot * 16 * NTC + tid;
#pragma unroll
                    for (int vv = 0; vv < 4; ++vv)
#pragma unroll
                        for (int c = 0; c < 4; ++c) {
                            if (own_cls + vv < C) {
                                float g = acc[c][vv];
                                if (!first) g += pk[(vv * 4 + c) * NTC];
                                pk[(vv * 4 + c) * NTC] = g;
                            }
                        }
                }
            }
            if (!single) __syncthreads();                   // R: the tile is rewritten by the next chunk
        }
        mark(4);

        // ---- phase 4: update v (each compute thread owns its weights; nobody reads them before the barrier)
        {
            const float scale = (float)((double)a.lr / (double)Kv);
#pragma unroll
            for (int vv = 0; vv < 4; ++vv) {
                const int cls = own_cls + vv;
                if (cls < C) {
                    f32x4* wp = reinterpret_cast<f32x4*>(wlds + cls * SL + ((own_ch ^ (cls & 15)) << 2));
                    f32x4 w = *wp;
#pragma unroll
                    for (int c = 0; c < 4; ++c) w[c] -= scale * gsum[vv * 4 + c];
                    *wp = w;
                }
            }
            if (tid == 16 && slice == 0) tr_loss[v] = bsum / (float)Kv;
            if (a.agg_out != nullptr && rep == 0) {
                const float invK = 1.0f / (float)Kv;
#pragma unroll
                for (int vv = 0; vv < 4; ++vv)
#pragma unroll
                    for (int c = 0; c < 4; ++c) {
                        const int cls = own_cls + vv, col = own_col + c;
                        if (cls < C && col < d) a.agg_out[(int64_t)cls * d + col] = gsum[vv * 4 + c] * invK;
                    }
                if (a.kind == kSoftmax && slice == 0 && tid < C) a.agg_out[(int64_t)C * d + tid] = bsum * invK;
            }
            if (tid == 0 && stop[2] != 0) stop[1] = 1;   // later exchanges of this launch use the shared L2
            __syncthreads();                                // U: the row threads of phase 3 have read the bias
            if (a.kind == kSoftmax && tid < C) bias[tid] -= scale * bsum;
        }
        mark(5);
    }
    if (profiling)
        for (int q = 0; q < 8; ++q) a.prof[((int64_t)rep * G + slice) * 8 + q] += ph[q];
    __syncthreads();

    // ---- leave the state in HBM for the next launch
#pragma unroll
    for (int vv = 0; vv < 4; ++vv) {
        const int cls = own_cls + vv;
        if (cls < C) {
            const f32x4 w = *reinterpret_cast<const f32x4*>(wlds + cls * SL + ((own_ch ^ (cls & 15)) << 2));
#pragma unroll
            for (int c = 0; c < 4; ++c)
                if (own_col + c < d) params[(int64_t)cls * d + own_col + c] = w[c];
        }
    }
    if (a.kind == kSoftmax && slice == 0 && tid < C) params[(int64_t)C * d + tid] = bias[tid];
    for (int q = tid; q < S * 17; q += NTC) small_g[q] = small[q];
}

template <int NBW>
hipError_t launch_t(const LinArgs& a, hipStream_t s) {
    const size_t lds = linear_lds_bytes(NBW, a.C, a.S);
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(linear_cluster_kernel<NBW>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    const int groups = (a.replicas + 7) / 8;
    hipLaunchKernelGGL(linear_cluster_kernel<NBW>, dim3(groups * 8 * a.G), dim3(64 * (NBW + loader_waves(NBW))), lds, s, a);
    return hipGetLastError();
}

template <int NBW>
int resident_t(size_t lds_bytes) {
    int per_cu = 0;
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(linear_cluster_kernel<NBW>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes) != hipSuccess) return 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, linear_cluster_kernel<NBW>, 64 * (NBW + loader_waves(NBW)),
                                                     lds_bytes) != hipSuccess) return 0;
    return per_cu;
}

}  // namespace

size_t linear_lds_bytes(int nbw, int C, int S) {
    const size_t SL = 64 * (size_t)nbw;
    const size_t words = ROWS * SL + (size_t)C * SL + ROWS * 16 + 3 * ROWS + 16 + (size_t)S * 17 + 4;
    return sizeof(float) * words + (((size_t)S + 15) / 16) * 16;
}

int linear_max_resident_groups(int nbw, size_t lds_bytes) {
    int dev = 0;
    hipDeviceProp_t prop;
    if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess) return 0;
    const int per_cu = nbw == 1 ? resident_t<1>(lds_bytes) : (nbw == 2 ? resident_t<2>(lds_bytes) : resident_t<4>(lds_bytes));
    return per_cu * prop.multiProcessorCount;
}

hipError_t launch_linear(const LinArgs& a, int nbw, hipStream_t s) {
    if (nbw == 1) return launch_t<1>(a, s);
    if (nbw == 2) return launch_t<2>(a, s);
    return launch_t<4>(a, s);
}

}  // namespace ssgd
