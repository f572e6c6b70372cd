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
// does not depend on the numerics, so everything about step v+1 that comes from HBM (its
// rows, labels and lists) is fetched while step v computes.  Waves are specialised for
// that: the vector-memory counter of a wave retires in order, so a wave that had the long
// HBM gather in flight would stall on it at the first cache-resident load it needs.
// Compute waves never touch the sample matrix or the schedule; loader waves hold the next
// tile in registers, publish it to LDS when the tile is free, and only join the barriers.
#include "common.hpp"

namespace ssgd {
namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr int ROWS = 64;   // rows of one LDS tile
constexpr int ZB = 12;     // partial-logit blocks fetched per batch of the exchange
constexpr int KC = 32;     // list entries per step that the loader waves publish in LDS
// cache policy of the exchange loads: agent-coherent (sc1), i.e. never served by a CU's L1
constexpr int kCoherentLoad = 16;

struct ChunkMap {
    int n_chunks, rpc, spr;
};

__device__ __forceinline__ ChunkMap chunk_map(int n_rec, int mp) {
    ChunkMap c;
    if (mp <= ROWS) { c.rpc = ROWS / mp; c.spr = 1; c.n_chunks = (n_rec + c.rpc - 1) / c.rpc; }
    else { c.rpc = 1; c.spr = (mp + ROWS - 1) / ROWS; c.n_chunks = n_rec * c.spr; }
    return c;
}

__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* p, uint32_t bytes) {
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p), 0, (int)bytes, 0x00020000);
}

// NBW: 64-column blocks per workgroup; VEC: d is a multiple of 4, rows can be read 16 bytes at a time;
// BIG: the lists of a step may be longer than the KC entries the loader waves publish in LDS, so the
// compute waves read them from HBM (kept out of the common instantiation: a possible global load
// in the middle of a phase makes the compiler wait for every outstanding store there).
template <int NBW, bool VEC, bool BIG, bool PROF>
__global__ __launch_bounds__(128 * NBW, 4) void linear_cluster_kernel(LinArgs a) {
    constexpr int SL = 64 * NBW;            // columns per workgroup
    constexpr int NTC = 64 * NBW;           // compute threads (waves 0 .. NBW-1)
    constexpr int LW = NBW;                 // loader waves (waves NBW .. 2 NBW-1)
    constexpr int NTL = 64 * LW;
    constexpr int CPR = SL / 4;             // float4 chunks per tile row
    constexpr int RB = 4 / NBW;             // 16-row blocks per compute wave in the forward pass
    constexpr int LLOADS = ROWS * CPR / NTL;   // float4 loads per loader thread per tile (= 16)
    constexpr int RPI = 64 / CPR;           // whole tile rows covered by one wave-wide load instruction

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
    const int Ssm = async ? S : 0;                           // the synchronous variants never park a gradient
    float* small = bias + 16;                                // [Ssm][17] bias gradient + loss per parked slot
    int* stop = reinterpret_cast<int*>(small + Ssm * 17);      // [4]: stop flag, exchange mode, same-XCD flag
    int* sched = stop + 4;                                   // [4 + 3 KC] lists of the step, from the loader
    int* s_sel = sched + 4;                                  // [KC] consume list of update v: slot
    int* s_tau = s_sel + KC;                                 // [KC]                          version read
    int* s_slot = s_tau + KC;                                // [KC] compute list of v: slot of record r
    unsigned char* fresh = reinterpret_cast<unsigned char*>(s_slot + KC);   // [S] slot computed and consumed in v

    const int32_t* tr_K = a.tr.K + (int64_t)rep * cap;
    const int32_t* tr_sel = a.tr.sel + (int64_t)rep * cap * Kcap;
    const int32_t* tr_tau = a.tr.tau + (int64_t)rep * cap * Kcap;
    const int32_t* tr_ord = a.tr.ord + (int64_t)rep * cap * Kcap;
    float* tr_loss = a.tr.loss + (int64_t)rep * cap;
    float* params = a.params + (int64_t)rep * nw;
    float* park = a.park + ((int64_t)rep * G + slice) * S * 16 * NTC;
    float* small_g = a.park_small + ((int64_t)rep * G + slice) * S * 17;
    float* zpart = a.zpart + (int64_t)rep * 2 * G * a.maxrows * 16;
    unsigned int* arrive = a.arrive + kArriveStride * rep;   // fenced exchanges; word kArriveFast: shared-L2 exchanges
    int32_t* xcc_ids = a.xcc_ids + (int64_t)rep * G;
    const float inv_m = 1.0f / (float)m;
    const int nquad = (C + 3) / 4;       // 4-class groups that carry data

    // record r of the compute list of version ver -> (worker, ordinal)
    auto rec_worker = [&](int64_t ver, int r) -> int {
        if (async) return (ver == 0) ? r : tr_sel[(ver - 1) * Kcap + r];
        return tr_sel[ver * Kcap + r];
    };
    auto rec_ord = [&](int64_t ver, int r) -> int { return async ? 0 : tr_ord[ver * Kcap + r]; };

    // The two roles run separate loops (so that the registers that hold the next tile are not
    // live in the compute code) and meet at the same sequence of workgroup barriers:
    //   one at the start; per step (T F)* | S X | (T' Z D R)* | U with T' and R only in multi-tile
    //   steps and (T F)* = T alone in a single-tile step; one more after the loop.
    //   T tile in LDS, F forward done, S exchange stores done, X exchange complete, Z logits in
    //   LDS, D delta in LDS, R tile may be rewritten, U update done.
    if (loader) {
        // =============================== loader waves ===============================
        // They never wait for their gathers at a barrier: only their LDS writes are made visible.
        auto lbar = [&]() {
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
            __builtin_amdgcn_s_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
        };
        lbar();
        if (stop[0] != 0) return;

        f32x4 pref[LLOADS];              // the tile gathered ahead
        uint32_t row_id = 0xFFFFFFFFu;   // sample id / label of tile row `lane`
        float row_lab = 0.0f;
        // lists of the step the tile belongs to (lane l: entry l; wave-uniform: n_K, n_rec)
        int n_K = 0, n_nrec = 0, n_sel = 0, n_tau = 0, n_slot = 0;
        uint32_t n_fresh = 0;            // bit q: slot lane + 64 q
        // When every list fits the lanes of a wave, the lists are fetched two steps ahead with plain
        // vector loads (lane l: entry l) and everything else is derived from them with lane shuffles,
        // so that no step of the loader waits for a dependent chain of loads.
        const bool lanes_ok = Kcap <= 64;
        int q_sel = -1, q_tau = -1, q_ord = 0;   // raw lists of version q_ver, loads possibly still in flight
        int64_t q_ver = -1;
        int cur_sel = -1;                        // raw consume list of the step whose tile is held

        // Loader wave lw issues, per instruction i, one 16-byte load per lane that covers RPI whole tile
        // rows: rows (lw + LW*i)*RPI + j, j < RPI, lane -> (j = lane / CPR, chunk = lane % CPR).  The row's
        // sample id comes from lane `row` of this wave through readlane, so the row base stays scalar.
        const int lw = __builtin_amdgcn_readfirstlane(lt >> 6);
        const int sub = lane / CPR, lch = lane % CPR;
        const int lcol = col0 + 4 * lch;

        auto fetch_lists = [&](int64_t ver) {
            n_K = tr_K[ver];
            n_nrec = async ? ((ver == 0) ? P : tr_K[ver - 1]) : n_K;
            n_sel = 0; n_tau = -1; n_slot = 0; n_fresh = 0;
            if (lane < n_K && lane < KC) {
                n_tau = tr_tau[ver * Kcap + lane];
                n_sel = async ? tr_sel[ver * Kcap + lane] : lane;
            }
            if (lane < n_nrec && lane < KC) n_slot = async ? rec_worker(ver, lane) : lane;
            for (int q = 0; q * 64 < S; ++q) {
                const int s = lane + 64 * q;
                bool f = false;
                if (s < S) {
                    if (!async) f = s < n_K;
                    else
                        for (int l = 0; l < n_K; ++l)
                            if (tr_sel[ver * Kcap + l] == s && tr_tau[ver * Kcap + l] == (int32_t)ver) f = true;
                }
                if (f) n_fresh |= 1u << q;
            }
        };

        auto gather_rows = [&]() {
#pragma unroll
            for (int i = 0; i < LLOADS; ++i) {
                const int row0 = (lw + LW * i) * RPI;
                f32x4 val = {0.0f, 0.0f, 0.0f, 0.0f};
                // the sample matrix streams through the L2 once: non-temporal loads, so that the parked
                // gradients and the exchange buffers stay resident
                if constexpr (VEC && RPI == 1) {
                    // one row per instruction: scalar row base (buffer descriptor), one constant lane offset;
                    // lanes past the end of the row read zeros (out-of-range buffer access)
                    const uint32_t id = (uint32_t)__builtin_amdgcn_readlane((int)row_id, row0);
                    if (id != 0xFFFFFFFFu) {
                        const __amdgpu_buffer_rsrc_t xr = make_rsrc(a.X + (int64_t)id * d, (uint32_t)d * 4u);
                        val = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(xr, lcol * 4, 0, 2));
                    }
                } else {
                    uint32_t id = (uint32_t)__builtin_amdgcn_readlane((int)row_id, row0);
#pragma unroll
                    for (int j = 1; j < RPI; ++j) {
                        const uint32_t idj = (uint32_t)__builtin_amdgcn_readlane((int)row_id, row0 + j);
                        if (sub == j) id = idj;
                    }
                    if (id != 0xFFFFFFFFu) {
                        const float* src = a.X + (int64_t)id * d + lcol;
                        if constexpr (VEC) {
                            if (lcol + 3 < d) val = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(src));
                        } else {
                            if (lcol + 0 < d) val.x = __builtin_nontemporal_load(src + 0);
                            if (lcol + 1 < d) val.y = __builtin_nontemporal_load(src + 1);
                            if (lcol + 2 < d) val.z = __builtin_nontemporal_load(src + 2);
                            if (lcol + 3 < d) val.w = __builtin_nontemporal_load(src + 3);
                        }
                    }
                }
                pref[i] = val;
            }
        };
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
            gather_rows();
        };
        const bool lprof = PROF && lt == 0;
        unsigned long long lph[8] = {0, 0, 0, 0, 0, 0, 0, 0}, lprev = 0;
        auto lmark = [&](int q) {
            if constexpr (PROF) { if (lprof) { const unsigned long long now = clock64(); lph[q] += now - lprev; lprev = now; } }
        };
        auto issue_lists = [&](int64_t ver) {
            q_sel = -1; q_tau = -1; q_ord = 0;
            if (lane < Kcap) {
                q_sel = tr_sel[ver * Kcap + lane];
                q_tau = tr_tau[ver * Kcap + lane];
                if (!async) q_ord = tr_ord[ver * Kcap + lane];
            }
            q_ver = ver;
        };
        // Everything of version ver >= 1 from the lane-resident lists; false if that step needs several tiles.
        auto prefetch_fast = [&](int64_t ver, int Kprev, bool lists_of_next) -> bool {
            if (lprof) lprev = clock64();
            if (q_ver != ver) issue_lists(ver);
            const int l_sel = q_sel, l_tau = q_tau, l_ord = q_ord;
            const int K = __popcll(__ballot(l_sel >= 0));
            lmark(0);
            const int nrec = async ? Kprev : K;
            const ChunkMap cmn = chunk_map(nrec, mp);
            if (cmn.n_chunks != 1) return false;
            n_K = K; n_nrec = nrec;
            n_tau = (lane < K) ? l_tau : -1;
            n_sel = (lane < K) ? (async ? l_sel : lane) : 0;
            n_slot = (lane < nrec) ? (async ? cur_sel : lane) : 0;
            n_fresh = 0;
            for (int q = 0; q * 64 < S; ++q) {
                const int s = lane + 64 * q;
                bool f = false;
                if (!async) f = s < K;
                else
                    for (int l = 0; l < K; ++l)
                        if (__builtin_amdgcn_readlane(l_sel, l) == s && __builtin_amdgcn_readlane(l_tau, l) == (int32_t)ver) f = true;
                if (f && s < S) n_fresh |= 1u << q;
            }
            lmark(1);
            const int r = lane / mp, sidx = lane % mp;
            const bool ok = lane < cmn.rpc * mp && r < nrec && sidx < m;
            const int worker = __shfl(async ? cur_sel : l_sel, r, 64);
            const int ordinal = async ? 0 : __shfl(l_ord, r, 64);
            row_id = 0xFFFFFFFFu;
            row_lab = 0.0f;
            if (ok) {
                row_id = batch_index(a.seed, (uint32_t)rep, (uint32_t)worker, (uint32_t)ordinal, (uint32_t)ver,
                                     (uint32_t)sidx, a.N);
                row_lab = (a.kind == kLsq) ? reinterpret_cast<const float*>(a.y)[row_id]
                                           : __int_as_float(reinterpret_cast<const int32_t*>(a.y)[row_id]);
            }
            cur_sel = l_sel;
            // Everything derived from the lists is final before any gather is issued: the gathers are the
            // youngest vector-memory operations of this wave until the tile is published, and the counter
            // retires in order, so a load consumed after them would wait for all of them.
            asm volatile("" : "+v"(n_sel), "+v"(n_tau), "+v"(n_slot), "+v"(n_fresh), "+v"(cur_sel), "+v"(row_id) : : "memory");
            lmark(2);
            if (lists_of_next) issue_lists(ver + 1);
            __builtin_amdgcn_sched_barrier(0);
            lmark(3);
            gather_rows();
            lmark(4);
            return true;
        };
        auto publish = [&](bool with_lists) {
#pragma unroll
            for (int i = 0; i < LLOADS; ++i) {
                const int row = (lw + LW * i) * RPI + sub;
                *reinterpret_cast<f32x4*>(tile + row * SL + ((lch ^ (row & 15)) << 2)) = pref[i];
            }
            if (lt < ROWS) {
                rowid[lt] = row_id; ylab[lt] = row_lab;
                if (with_lists) {
                    if (lt == 0) { sched[0] = n_K; sched[1] = n_nrec; }
                    if (lt < KC) { s_sel[lt] = n_sel; s_tau[lt] = n_tau; s_slot[lt] = n_slot; }
                    for (int q = 0; q * 64 < S; ++q)
                        if (lt + 64 * q < S) fresh[lt + 64 * q] = (unsigned char)((n_fresh >> q) & 1u);
                }
            }
        };

        unsigned long long lq0 = 0, lq1 = 0;
        int64_t step = 0;
        while (step < a.nsteps) {
            int64_t v = a.v0 + step;
            // ---- steady state: consecutive single-tile steps whose lists fit the lanes
            bool fast_ok = false;
            if (lanes_ok && (!async || v >= 1)) {
                cur_sel = -1;
                if (async && lane < Kcap) cur_sel = tr_sel[(v - 1) * Kcap + lane];
                const int Kprev = __popcll(__ballot(cur_sel >= 0));
                fast_ok = prefetch_fast(v, Kprev, step + 1 < a.nsteps);
            }
            if (fast_ok) {
                for (;;) {
                    const unsigned long long lt0 = lprof ? clock64() : 0;
                    const int Kv = n_K;
                    publish(true);
                    if (lprof) lq1 += clock64() - lt0;
                    lbar();                                 // T
                    const unsigned long long lt1 = lprof ? clock64() : 0;
                    bool more = false;
                    if (step + 1 < a.nsteps) {
                        // everything of step v+1 is fetched now and stays in registers until step v is done
                        more = prefetch_fast(v + 1, Kv, step + 2 < a.nsteps);
                    }
                    if (lprof) lq0 += clock64() - lt1;
                    lbar();                                 // S
                    lbar();                                 // X
                    if (stop[0] != 0) return;
                    lbar();                                 // Z
                    lbar();                                 // D
                    lbar();                                 // U
                    ++step; ++v;
                    if (!more) break;
                }
                continue;
            }
            // ---- any other step: fetched when it is needed
            fetch_lists(v);
            const int n_rec = n_nrec;
            const ChunkMap cm = chunk_map(n_rec, mp);
            const bool single = cm.n_chunks == 1;
            fetch(v, n_rec, cm, 0);
            publish(true);
            lbar();                                         // T (chunk 0)
            if (!single) {
                lbar();                                     // F (chunk 0)
                for (int chunk = 1; chunk < cm.n_chunks; ++chunk) {
                    fetch(v, n_rec, cm, chunk);
                    publish(false);
                    lbar();                                 // T
                    lbar();                                 // F
                }
            }
            lbar();                                         // S
            lbar();                                         // X
            if (stop[0] != 0) return;
            for (int chunk = 0; chunk < cm.n_chunks; ++chunk) {
                if (!single) { fetch(v, n_rec, cm, chunk); publish(false); lbar(); }   // T'
                lbar();                                     // Z
                lbar();                                     // D
                if (!single) lbar();                        // R
            }
            lbar();                                         // U
            ++step;
        }
        if (lprof) {
            for (int q = 0; q < 8; ++q) a.prof[((int64_t)rep * G + slice) * 20 + 12 + q] += lph[q];
            a.prof[((int64_t)rep * G + slice) * 20 + 6] += lq0;   // loader: work between T and S
            a.prof[((int64_t)rep * G + slice) * 20 + 7] += lq1;   // loader: step start to tile published
        }
        lbar();
        return;
    }

    // ================================= compute waves =================================
    // share of the parameters: class 4*(lane/16)+v, columns own_col..own_col+3
    const int own_ch = 16 * wave + (lane & 15);
    const int own_col = col0 + 4 * own_ch;
    const int own_cls = 4 * (lane >> 4);
    const bool bias_owner = wave == 0 && (lane & 15) == 0;   // classes own_cls .. own_cls+3 of the bias
    const bool loss_owner = tid == ((C < 16) ? 48 : 0);      // the thread that receives the loss sums
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
    for (int q = tid; q < Ssm * 17; q += NTC) small[q] = small_g[q];
    if (tid == 0) {
        stop[0] = __hip_atomic_load(a.abort_flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        stop[1] = 0;   // exchange mode: fenced until the cluster is known to share an XCD
        stop[2] = 0;
        // XCC_ID hardware register: the XCD this workgroup runs on
        const int my_xcc = (int)(__builtin_amdgcn_s_getreg((3 << 11) | 20) & 0xF);
        __hip_atomic_store(xcc_ids + slice, my_xcc, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    __syncthreads();
    if (stop[0] != 0) return;

    // Barrier that orders LDS only.  The full __syncthreads also waits for every outstanding global
    // store of the wave (parked gradients, trace), which no barrier but S needs.
    auto cbar = [&]() {
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
        __builtin_amdgcn_s_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
    };

    // Exchange through the L2 that the cluster shares ("fast"): buffer accesses whose loads are
    // marked workgroup-coherent, so they are served by the L2 and never by this CU's L1; stores
    // write through to the L2; the arrival counter is an L2 atomic.  Otherwise ("fenced"):
    // plain accesses ordered by agent-scope release / acquire.
    const __amdgpu_buffer_rsrc_t zrsrc = make_rsrc(zpart, (uint32_t)(2u * G * a.maxrows * 16u * sizeof(float)));
    const __amdgpu_buffer_rsrc_t crsrc = make_rsrc(arrive, kArriveStride * 4u);
    // parked gradients of this workgroup: plane e of slot s at byte ((s*16 + e)*NTC + tid)*4.  Lanes whose
    // classes do not exist use an offset past the end: such loads return zero and such stores are dropped.
    const __amdgpu_buffer_rsrc_t prsrc = make_rsrc(park, (uint32_t)S * 16u * NTC * 4u);
    int pk_off[4];
#pragma unroll
    for (int vv = 0; vv < 4; ++vv) pk_off[vv] = (own_cls + vv < C) ? (vv * NTC + tid) * 16 : (int)0x80000000;
    uint32_t n_fenced = 0, n_fast = 0;       // exchanges of each kind so far in this launch

    unsigned long long ph[12] = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0}, tprev = 0;
    const bool profiling = PROF && tid == 0;
    auto mark = [&](int phase) {
        if constexpr (PROF) { if (profiling) { const unsigned long long now = clock64(); ph[phase] += now - tprev; tprev = now; } }
    };

    for (int64_t step = 0; step < a.nsteps; ++step) {
        const int64_t v = a.v0 + step;
        if (profiling) tprev = clock64();
        const bool fast = stop[1] != 0;
        const int par = (int)(step & 1);
        const int zoff_mine = (par * G + slice) * a.maxrows * 16;   // in floats, inside this replica's buffer
        const int zoff_all = par * G * a.maxrows * 16;

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
                if ((lane >> 4) < nquad) {
                    const int off = zoff_mine + (chunk * ROWS + row) * 16 + 4 * (lane >> 4);
                    if (fast) __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, out), zrsrc, off * 4, 0, 0);
                    else *reinterpret_cast<f32x4*>(zpart + off) = out;
                }
            }
        };

        // ---- phase 1: partial logits of every chunk
        cbar();                                             // T: tile, row ids, labels and lists of step v are in LDS
        const int Kv = sched[0], n_rec = sched[1];
        constexpr bool direct = BIG;
        const ChunkMap cm = chunk_map(n_rec, mp);
        const bool single = cm.n_chunks == 1;
        auto cons_slot = [&](int l) -> int {
            if constexpr (direct) return async ? tr_sel[v * Kcap + l] : l; else return s_sel[l];
        };
        auto cons_tau = [&](int l) -> int {
            if constexpr (direct) return tr_tau[v * Kcap + l]; else return s_tau[l];
        };
        auto rec_slot = [&](int r) -> int {
            if constexpr (direct) return async ? rec_worker(v, r) : r; else return s_slot[r];
        };
        forward(0);
        if (!single) {
            cbar();                                         // F
            for (int chunk = 1; chunk < cm.n_chunks; ++chunk) {
                cbar();                                     // T
                forward(chunk);
                cbar();                                     // F
            }
        }
        mark(0);

        float gsum[16];          // this thread's part of sum_l g_l
        float bg[4] = {0.f, 0.f, 0.f, 0.f};   // bias owners: sum_l of the bias gradient, classes own_cls..+3
        float lsum = 0.0f;       // loss owner: sum_l of the mini-batch losses
#pragma unroll
        for (int e = 0; e < 16; ++e) gsum[e] = 0.0f;

        // ---- phase 2: exchange inside the cluster
        __syncthreads();                                    // S: every thread's exchange stores have completed
        if (G > 1 && tid == 0) {
            if (fast) (void)__builtin_amdgcn_raw_ptr_buffer_atomic_add_i32(1, crsrc, kArriveFast * 4, 0, 0);
            else __hip_atomic_fetch_add(arrive, 1u, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
        }
        mark(1);
        // while the exchange is in flight: the part of update v that earlier steps parked
        for (int l = 0; l < Kv; ++l) {
            if (cons_tau(l) == (int32_t)v) continue;
            const int slot = cons_slot(l);
            // all 16 planes are loaded without a branch (planes of unused classes hold zeros), so that the
            // loads are issued back to back instead of one predicated block and one wait per element
            const int soff = __builtin_amdgcn_readfirstlane(slot) * 16 * NTC * 4;
            f32x4 pv[4];
#pragma unroll
            for (int vv = 0; vv < 4; ++vv)
                pv[vv] = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(prsrc, pk_off[vv], soff, 0));
#pragma unroll
            for (int e = 0; e < 16; ++e) gsum[e] += pv[e >> 2][e & 3];
            if (bias_owner) {
#pragma unroll
                for (int vv = 0; vv < 4; ++vv) bg[vv] += small[slot * 17 + own_cls + vv];
                if (loss_owner) lsum += small[slot * 17 + 16];
            }
        }
        mark(2);
        if (G > 1 && tid == 0) {
            const uint32_t target = (fast ? n_fast + 1u : n_fenced + 1u) * (uint32_t)G;
            uint32_t spins = 0;
            for (;;) {
                const uint32_t got = fast ? __builtin_amdgcn_raw_buffer_load_b32(crsrc, kArriveFast * 4, 0, kCoherentLoad)
                                          : __hip_atomic_load(arrive, __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_AGENT);
                asm volatile("" ::: "memory");   // the load is repeated every turn
                if ((int32_t)(got - target) >= 0) break;
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
        if (fast) ++n_fast; else ++n_fenced;
        cbar();                                             // X
        if (G > 1 && !fast) __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
        if (stop[0] != 0) return;   // uniform: every thread reads the same LDS word
        mark(3);

        // ---- phase 3: residual / softmax and the gradient slices
        for (int chunk = 0; chunk < cm.n_chunks; ++chunk) {
            if (!single) cbar();                            // T'
            // full logits of the 64 rows: sum of the G partials in slice order
            for (int q = tid; q < ROWS * 4; q += NTC) {
                f32x4 z = {0.f, 0.f, 0.f, 0.f};
                if ((q & 3) < nquad) {
                    const int off = zoff_all + chunk * ROWS * 16 + 4 * q;
                    for (int g0 = 0; g0 < G; g0 += ZB) {
                        // straight-line batch: slices past the end re-read the last one and are not added
                        f32x4 part[ZB];
                        if (fast) {
#pragma unroll
                            for (int i = 0; i < ZB; ++i) {
                                const int o = off + min(g0 + i, G - 1) * a.maxrows * 16;
                                part[i] = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(zrsrc, o * 4, 0, kCoherentLoad));
                            }
                        } else {
#pragma unroll
                            for (int i = 0; i < ZB; ++i) {
                                const int o = off + min(g0 + i, G - 1) * a.maxrows * 16;
                                part[i] = *reinterpret_cast<const f32x4*>(zpart + o);
                            }
                        }
#pragma unroll
                        for (int i = 0; i < ZB; ++i) {
                            const float keep = (g0 + i < G) ? 1.0f : 0.0f;
                            z += part[i] * keep;
                        }
                    }
                }
                *reinterpret_cast<f32x4*>(zbuf + 4 * q) = z;
            }
            cbar();                                         // Z
            mark(8);
            // residual / softmax: four threads per row, each with four classes
            for (int t = tid; t < ROWS * 4; t += NTC) {
                const int row = t >> 2, qd = t & 3;
                f32x4 zz = *reinterpret_cast<const f32x4*>(zbuf + row * 16 + 4 * qd);
                const bool ok = rowid[row] != 0xFFFFFFFFu;
                f32x4 dl = {0.f, 0.f, 0.f, 0.f};
                float loss = 0.0f;
                if (a.kind == kLsq) {
                    const float r = zbuf[row * 16] - ylab[row];   // every thread of the row reads it before any writes
                    if (ok) loss = 0.5f * r * r;
                    if (qd == 0 && ok) dl.x = r * inv_m;
                } else {
                    const int lab = __float_as_int(ylab[row]);
                    float zmax = -3.0e38f;
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        zz[e] += bias[4 * qd + e];
                        if (4 * qd + e < C) zmax = fmaxf(zmax, zz[e]);
                    }
                    zmax = fmaxf(zmax, __shfl_xor(zmax, 1, 64));
                    zmax = fmaxf(zmax, __shfl_xor(zmax, 2, 64));
                    float den = 0.0f, lt_ = 0.0f;
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const float ex = (4 * qd + e < C) ? expf(zz[e] - zmax) : 0.0f;
                        den += ex;
                        if (4 * qd + e == lab) lt_ = -(zz[e] - zmax);
                        dl[e] = ex;
                    }
                    den += __shfl_xor(den, 1, 64);
                    den += __shfl_xor(den, 2, 64);
                    lt_ += __shfl_xor(lt_, 1, 64);
                    lt_ += __shfl_xor(lt_, 2, 64);
                    loss = ok ? lt_ + logf(den) : 0.0f;
                    const float inv = 1.0f / den;
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const float pr = dl[e] * inv - ((4 * qd + e == lab) ? 1.0f : 0.0f);
                        dl[e] = (ok && 4 * qd + e < C) ? pr * inv_m : 0.0f;
                    }
                }
                // with fewer than 16 classes the unused class 15 carries the row loss, so that one
                // contraction with a column of ones yields the bias gradient and the loss sum
                if (C < 16 && qd == 3) dl.w = loss * inv_m;
                *reinterpret_cast<f32x4*>(zbuf + row * 16 + 4 * qd) = dl;
                if (qd == 0) lossrow[row] = loss * inv_m;
            }
            cbar();                                         // D
            mark(9);

            // per record of this chunk: the gradient slice delta^T X; wave 0 also contracts delta and
            // the row losses with a column of ones, which gives the bias gradient and the loss sum
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
                const int slot = rec_slot(r);
                const bool is_fresh = fresh[slot] != 0;
                f32x4 acc[4], accb = {0.f, 0.f, 0.f, 0.f}, accl = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int c = 0; c < 4; ++c) acc[c] = f32x4{0.f, 0.f, 0.f, 0.f};
                auto contract = [&](float dv, const f32x4& xv, int row) {
                    acc[0] = __builtin_amdgcn_mfma_f32_16x16x4f32(dv, xv.x, acc[0], 0, 0, 0);
                    acc[1] = __builtin_amdgcn_mfma_f32_16x16x4f32(dv, xv.y, acc[1], 0, 0, 0);
                    acc[2] = __builtin_amdgcn_mfma_f32_16x16x4f32(dv, xv.z, acc[2], 0, 0, 0);
                    acc[3] = __builtin_amdgcn_mfma_f32_16x16x4f32(dv, xv.w, acc[3], 0, 0, 0);
                    if (wave == 0) {
                        accb = __builtin_amdgcn_mfma_f32_16x16x4f32(dv, 1.0f, accb, 0, 0, 0);
                        if (C == 16) {
                            const float lv = ((lane & 15) == 0) ? lossrow[row] : 0.0f;
                            accl = __builtin_amdgcn_mfma_f32_16x16x4f32(lv, 1.0f, accl, 0, 0, 0);
                        }
                    }
                };
                int ks = row_lo / 4;
                const int ks_end = row_hi / 4;
                for (; ks + 4 <= ks_end; ks += 4) {     // operands of four steps are read before their MFMAs
                    float dv[4];
                    f32x4 xv[4];
#pragma unroll
                    for (int u = 0; u < 4; ++u) {
                        const int row = 4 * (ks + u) + (lane >> 4);
                        dv[u] = zbuf[row * 16 + (lane & 15)];
                        xv[u] = *reinterpret_cast<const f32x4*>(tile + row * SL + ((own_ch ^ (row & 15)) << 2));
                    }
#pragma unroll
                    for (int u = 0; u < 4; ++u) contract(dv[u], xv[u], 4 * (ks + u) + (lane >> 4));
                }
                for (; ks < ks_end; ++ks) {
                    const int row = 4 * ks + (lane >> 4);
                    const float dv = zbuf[row * 16 + (lane & 15)];
                    const f32x4 xv = *reinterpret_cast<const f32x4*>(tile + row * SL + ((own_ch ^ (row & 15)) << 2));
                    contract(dv, xv, row);
                }
                const float lval = (C < 16) ? accb[3] : accl[0];   // loss sum of the record, in the loss owner
                mark(4);
                if (is_fresh) {
#pragma unroll
                    for (int vv = 0; vv < 4; ++vv)
#pragma unroll
                        for (int c = 0; c < 4; ++c) gsum[vv * 4 + c] += acc[c][vv];
                    if (bias_owner) {
#pragma unroll
                        for (int vv = 0; vv < 4; ++vv) bg[vv] += accb[vv];
                        if (loss_owner) lsum += lval;
                    }
                } else {
                    const int soff = __builtin_amdgcn_readfirstlane(slot) * 16 * NTC * 4;
                    f32x4 old[4];
                    if (!first) {
#pragma unroll
                        for (int vv = 0; vv < 4; ++vv)
                            old[vv] = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(prsrc, pk_off[vv], soff, 0));
                    }
#pragma unroll
                    for (int vv = 0; vv < 4; ++vv) {
                        f32x4 g = {acc[0][vv], acc[1][vv], acc[2][vv], acc[3][vv]};
                        if (!first) g += old[vv];
                        // the slot offset goes into the vector offset: a 16-byte buffer store whose scalar offset is a
                        // register has lost data here when the next instruction rewrote its source registers
                        __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, g), prsrc, pk_off[vv] + soff, 0, 0);
                    }
                    if (bias_owner) {
#pragma unroll
                        for (int vv = 0; vv < 4; ++vv) {
                            float* sp = small + slot * 17 + own_cls + vv;
                            *sp = first ? accb[vv] : *sp + accb[vv];
                        }
                        if (loss_owner) {
                            float* sp = small + slot * 17 + 16;
                            *sp = first ? lval : *sp + lval;
                        }
                    }
                }
                mark(11);
            }
            if (!single) cbar();                            // R: the tile is rewritten by the next chunk
        }
        mark(10);

        // ---- phase 4: update v (each compute thread owns its weights; nobody reads them before the barrier)
        {
            const float scale = a.lr / (float)Kv;
            const float invK = 1.0f / (float)Kv;
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
            if (loss_owner && slice == 0) tr_loss[v] = lsum * invK;
            if (a.agg_out != nullptr && rep == 0) {
#pragma unroll
                for (int vv = 0; vv < 4; ++vv)
#pragma unroll
                    for (int c = 0; c < 4; ++c) {
                        const int cls = own_cls + vv, col = own_col + c;
                        if (cls < C && col < d) a.agg_out[(int64_t)cls * d + col] = gsum[vv * 4 + c] * invK;
                    }
                if (a.kind == kSoftmax && slice == 0 && bias_owner) {
#pragma unroll
                    for (int vv = 0; vv < 4; ++vv)
                        if (own_cls + vv < C) a.agg_out[(int64_t)C * d + own_cls + vv] = bg[vv] * invK;
                }
            }
            if (tid == 0 && stop[2] != 0) stop[1] = 1;   // later exchanges of this launch use the shared L2
            cbar();                                         // U: the row threads of phase 3 have read the bias
            if (a.kind == kSoftmax && bias_owner) {
#pragma unroll
                for (int vv = 0; vv < 4; ++vv)
                    if (own_cls + vv < C) bias[own_cls + vv] -= scale * bg[vv];
            }
        }
        mark(5);
    }
    if (profiling)
        for (int q = 0; q < 12; ++q)
            if (q < 6 || q > 7) a.prof[((int64_t)rep * G + slice) * 20 + q] += ph[q];
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
    for (int q = tid; q < Ssm * 17; q += NTC) small_g[q] = small[q];
}

template <int NBW, bool VEC, bool BIG, bool PROF>
hipError_t launch_p(const LinArgs& a, hipStream_t s) {
    const size_t lds = linear_lds_bytes(NBW, a.C, a.S, a.variant == kAsync);
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(linear_cluster_kernel<NBW, VEC, BIG, PROF>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    const int groups = (a.replicas + 7) / 8;
    hipLaunchKernelGGL((linear_cluster_kernel<NBW, VEC, BIG, PROF>), dim3(groups * 8 * a.G), dim3(128 * NBW), lds, s, a);
    return hipGetLastError();
}

template <int NBW, bool VEC, bool BIG>
hipError_t launch_t(const LinArgs& a, hipStream_t s) {
    // the instrumented build exists for the common instantiation only
    if constexpr (VEC && !BIG) { if (a.prof != nullptr) return launch_p<NBW, VEC, BIG, true>(a, s); }
    return launch_p<NBW, VEC, BIG, false>(a, s);
}

template <int NBW, bool VEC, bool BIG>
int resident_one(size_t lds_bytes) {
    int per_cu = 0;
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(linear_cluster_kernel<NBW, VEC, BIG, false>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes) != hipSuccess) return 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, linear_cluster_kernel<NBW, VEC, BIG, false>, 128 * NBW, lds_bytes) != hipSuccess) return 0;
    return per_cu;
}

template <int NBW>
int resident_t(size_t lds_bytes) {
    const int r[4] = {resident_one<NBW, true, false>(lds_bytes), resident_one<NBW, true, true>(lds_bytes),
                      resident_one<NBW, false, false>(lds_bytes), resident_one<NBW, false, true>(lds_bytes)};
    int m = r[0];
    for (int q = 1; q < 4; ++q) m = r[q] < m ? r[q] : m;
    return m;
}

template <int NBW>
hipError_t launch_n(const LinArgs& a, hipStream_t s) {
    const bool vec = (a.d % 4) == 0;
    const bool big = a.tr.Kcap > KC || a.P > KC;
    if (vec) return big ? launch_t<NBW, true, true>(a, s) : launch_t<NBW, true, false>(a, s);
    return big ? launch_t<NBW, false, true>(a, s) : launch_t<NBW, false, false>(a, s);
}

}  // namespace

size_t linear_lds_bytes(int nbw, int C, int S, bool parks) {
    const size_t SL = 64 * (size_t)nbw;
    const size_t words = ROWS * SL + (size_t)C * SL + ROWS * 16 + 3 * ROWS + 16 + (parks ? (size_t)S * 17 : 0) + 4 + 4 + 3 * KC;
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
    if (nbw == 1) return launch_n<1>(a, s);
    if (nbw == 2) return launch_n<2>(a, s);
    return launch_n<4>(a, s);
}

}  // namespace ssgd
