// Steady-state kernel of the linear models (Sec. 2.2, Eq. (2), Eq. (3)) for the common shape:
// every step's mini-batches fit one 64-row tile (records * padded m <= 64), at most 15 classes,
// rows readable 16 bytes at a time.  Same cluster decomposition, state layout and arithmetic as
// the general kernel (linear.hip), which runs every other shape and may be mixed with this one
// launch by launch; what differs is the schedule inside a step:
//
//   TU  tile, lists and the updated weights are in LDS          (workgroup barrier)
//       partial logits on the fp32 MFMA units, stored to the cluster's exchange buffer;
//       each wave waits for its own stores and adds 1 to the arrival counter;
//       while the other slices arrive: the parked (stale) part of update v is summed;
//       each wave polls the counter, then sums the G partials of its 16 rows and goes
//       straight on to residual / softmax in registers
//   D   delta in LDS                                            (workgroup barrier)
//       gradient slices delta^T X per record; added to the aggregate or parked
//   B   the tile has been read                                   (workgroup barrier)
//       compute waves: w -= (lr/K) * aggregate;  loader waves: next tile -> LDS
//
// Four compute waves, four loader waves.  A wave's vector-memory counter retires in order,
// so the long HBM gathers live in waves of their own: the loader waves fetch everything of
// step v+1 (lists, sample ids, labels, rows) while step v computes, hold the rows in
// registers, and copy them to LDS between B and TU.
#include "common.hpp"

namespace ssgd {
namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr int ROWS = 64;        // rows of the LDS tile
constexpr int SL = 256;         // columns per workgroup
constexpr int NTC = 256;        // compute threads
constexpr int LW = 4;           // loader waves
constexpr int LLOADS = 16;      // 16-byte loads per loader lane per tile
constexpr int KC = 32;          // list entries per step
constexpr int kAgentLoad = 16;  // cache policy: served by the L2, never by a CU's L1
constexpr int kStream = 2;      // cache policy: non-temporal
constexpr uint32_t kNoRow = 0xFFFFFFFFu;
constexpr int kOutOfRange = (int)0x80000000;   // buffer offset past any buffer: loads give 0, stores are dropped

__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* p, uint32_t bytes) {
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p), 0, (int)bytes, 0x00020000);
}

struct Lds {
    float* tile;      // [64][SL]  16-byte chunk c of row r at chunk position c ^ (r & 15)
    float* wlds;      // [C][SL]   same swizzle, keyed by the class
    float* zbuf;      // [64][16]  delta
    uint32_t* rowid;  // [64]
    float* ylab;      // [64]
    float* bias;      // [16]
    float* small;     // [S][17]   bias gradient and mean loss of every parked slot
    int* ctl;         // [8]: 0 stop, 1 exchange through the shared L2, 2 cluster shares an XCD, 3 K, 4 records
    int* s_sel;       // [KC] consume list of update v: slot
    int* s_tau;       // [KC]                          version read
    int* s_slot;      // [KC] compute list of v: slot of record r
    int* s_fresh;     // [KC]                    record r is consumed by update v itself
};

__device__ __forceinline__ Lds carve(unsigned char* smem, int C, int S) {
    Lds l;
    l.tile = reinterpret_cast<float*>(smem);
    l.wlds = l.tile + ROWS * SL;
    l.zbuf = l.wlds + C * SL;
    l.rowid = reinterpret_cast<uint32_t*>(l.zbuf + ROWS * 16);
    l.ylab = reinterpret_cast<float*>(l.rowid + ROWS);
    l.bias = l.ylab + ROWS;
    l.small = l.bias + 16;
    l.ctl = reinterpret_cast<int*>(l.small + S * 17);
    l.s_sel = l.ctl + 8;
    l.s_tau = l.s_sel + KC;
    l.s_slot = l.s_tau + KC;
    l.s_fresh = l.s_slot + KC;
    return l;
}

__device__ __forceinline__ void lds_barrier() {
    // orders LDS traffic only: outstanding global loads and stores stay in flight
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

template <int KIND, bool PROF>
__global__ __launch_bounds__(512, 4) void linear_tile_kernel(LinArgs a) {
    // consecutive block ids go to different XCDs: all slices of one cluster take block ids that
    // are congruent modulo 8 and share one L2
    const int xcd = blockIdx.x & 7, slot_in_xcd = blockIdx.x >> 3;
    const int cluster = (slot_in_xcd / a.G) * 8 + xcd;
    const int slice = slot_in_xcd % a.G;
    if (cluster >= a.replicas) return;
    const int rep = a.replica0 + cluster;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int d = a.d, C = a.C, m = a.m, mp = a.mp, S = a.S, G = a.G;
    const int Kcap = a.tr.Kcap;
    const int64_t cap = a.tr.cap;
    const int col0 = slice * SL;
    const bool async = a.variant == kAsync;

    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    const Lds L = carve(smem, C, S);

    if (wave >= 4) {
        // =============================== loader waves ===============================
        const int lw = wave - 4;
        const int32_t* tr_sel = a.tr.sel + (int64_t)rep * cap * Kcap;
        const int32_t* tr_tau = a.tr.tau + (int64_t)rep * cap * Kcap;
        const int32_t* tr_ord = a.tr.ord + (int64_t)rep * cap * Kcap;
        const __amdgpu_buffer_rsrc_t xrsrc = make_rsrc(a.X, (uint32_t)((uint64_t)a.N * d * 4u));
        const uint32_t row_bytes = (uint32_t)d * 4u;

        // tile row `lane` is sample s_of of record r_of
        const int r_of = lane / mp, s_of = lane % mp;
        const bool samp_ok = s_of < m;
        // Row lw + 4 i of the tile is fetched by instruction i of this wave, one 16-byte chunk per lane.
        // The swizzle is applied on the global side: lane l fetches chunk l ^ key and writes position l.
        int goff[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int key = (lw + 4 * q) & 15;
            const int col = col0 + 4 * (lane ^ key);
            goff[q] = (col < d) ? col * 4 : kOutOfRange;    // past the end of the row: zeros
        }
        float* const my_tile = L.tile + lw * SL + lane * 4;

        f32x4 pref[LLOADS];
        uint32_t row_id = kNoRow;
        float row_lab = 0.0f;
        int n_K = 0, n_nrec = 0, n_sel = 0, n_tau = -1, n_slot = 0, n_fresh = 0;
        int q_sel = -1, q_tau = -1, q_ord = 0;   // lane l: entry l of the consume list of a later version, in flight
        int cur_sel = -1;                        // consume list of the version before the one being prepared

        unsigned long long lph[4] = {0, 0, 0, 0}, lprev = 0;
        const bool lprof = PROF && tid == NTC;
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
        };
        // Everything of version `ver` from the lists in q_*; leaves the gathers in flight.
        auto prepare = [&](int64_t ver, bool more) {
            const int l_sel = q_sel, l_tau = q_tau, l_ord = q_ord;
            const int K = __popcll(__ballot(l_sel >= 0));
            const int nrec = async ? __popcll(__ballot(cur_sel >= 0)) : K;
            const int rec_worker = async ? cur_sel : l_sel;      // lane r: worker of record r
            const int rec_slot = async ? cur_sel : lane;
            int fr = (!async && lane < K) ? 1 : 0;
            if (async)
                for (int l = 0; l < K; ++l)
                    if (__builtin_amdgcn_readlane(l_tau, l) == (int32_t)ver && __builtin_amdgcn_readlane(l_sel, l) == rec_slot) fr = 1;
            n_K = K; n_nrec = nrec;
            n_tau = (lane < K) ? l_tau : -1;
            n_sel = (lane < K) ? (async ? l_sel : lane) : 0;
            n_slot = (lane < nrec) ? rec_slot : 0;
            n_fresh = (lane < nrec) ? fr : 0;
            const int worker = __shfl(rec_worker, r_of, 64);
            const int ordinal = async ? 0 : __shfl(l_ord, r_of, 64);
            row_id = kNoRow;
            row_lab = 0.0f;
            if (samp_ok && r_of < nrec) {
                row_id = batch_index(a.seed, (uint32_t)rep, (uint32_t)worker, (uint32_t)ordinal, (uint32_t)ver,
                                     (uint32_t)s_of, a.N);
                row_lab = (KIND == kLsq) ? reinterpret_cast<const float*>(a.y)[row_id]
                                         : __int_as_float(reinterpret_cast<const int32_t*>(a.y)[row_id]);
            }
            cur_sel = l_sel;
            // The lists are consumed before the gathers are issued: the gathers are the youngest
            // vector-memory operations of this wave until the tile is published.
            asm volatile("" : "+v"(n_sel), "+v"(n_tau), "+v"(n_slot), "+v"(n_fresh), "+v"(cur_sel), "+v"(row_id) : : "memory");
            if (more) issue_lists(ver + 1);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int i = 0; i < LLOADS; ++i) {
                // rows without a sample read row 0; their delta is zero
                uint32_t id = (uint32_t)__builtin_amdgcn_readlane((int)row_id, lw + 4 * i);
                id = (id == kNoRow) ? 0u : id;
                pref[i] = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(xrsrc, goff[i & 3], (int)(id * row_bytes), kStream));
            }
        };
        auto publish = [&]() {
#pragma unroll
            for (int i = 0; i < LLOADS; ++i) *reinterpret_cast<f32x4*>(my_tile + 4 * i * SL) = pref[i];
            if (lw == 0) {
                L.rowid[lane] = row_id; L.ylab[lane] = row_lab;
                if (lane == 0) { L.ctl[3] = n_K; L.ctl[4] = n_nrec; }
                if (lane < KC) { L.s_sel[lane] = n_sel; L.s_tau[lane] = n_tau; L.s_slot[lane] = n_slot; L.s_fresh[lane] = n_fresh; }
            }
        };

        lds_barrier();                               // the compute waves have set up the control words
        if (L.ctl[0] != 0) return;
        if (async && lane < Kcap) cur_sel = tr_sel[(a.v0 - 1) * Kcap + lane];   // v0 >= 1 for K-async
        issue_lists(a.v0);
        prepare(a.v0, a.nsteps > 1);
        for (int64_t step = 0; step < a.nsteps; ++step) {
            if constexpr (PROF) { if (lprof) lprev = clock64(); }
            publish();
            lmark(0);
            lds_barrier();                           // TU
            if (step + 1 < a.nsteps) prepare(a.v0 + step + 1, step + 2 < a.nsteps);
            lmark(1);
            lds_barrier();                           // D
            if (L.ctl[0] != 0) return;
            lmark(2);
            lds_barrier();                           // B
            lmark(3);
        }
        if constexpr (PROF) {
            if (lprof)
                for (int q = 0; q < 4; ++q) a.prof[((int64_t)rep * G + slice) * 20 + 12 + q] += lph[q];
        }
        return;
    }

    // ================================= compute waves =================================
    const int64_t nw = (KIND == kLsq) ? d : (int64_t)C * d + C;
    float* params = a.params + (int64_t)rep * nw;
    float* park = a.park + ((int64_t)rep * G + slice) * S * 16 * NTC;
    float* small_g = a.park_small + ((int64_t)rep * G + slice) * S * 17;
    float* zpart = a.zpart + (int64_t)rep * 2 * G * a.maxrows * 16;
    unsigned int* arrive = a.arrive + 2 * rep;     // [0] fenced exchanges, [1] shared-L2 exchanges of this launch
    const float inv_m = 1.0f / (float)m;
    const int nquad = (C + 3) / 4;

    // share of the parameters: classes own_cls .. own_cls+3, columns own_col .. own_col+3
    const int own_ch = 16 * wave + (lane & 15);
    const int own_col = col0 + 4 * own_ch;
    const int own_cls = 4 * (lane >> 4);
    const bool bias_owner = wave == 0 && (lane & 15) == 0;
    const bool loss_owner = tid == 48;             // class 15 of the delta tile carries the row losses
#pragma unroll
    for (int v = 0; v < 4; ++v) {
        const int cls = own_cls + v;
        if (cls < C) {
            f32x4 val;
#pragma unroll
            for (int c = 0; c < 4; ++c) val[c] = (own_col + c < d) ? params[(int64_t)cls * d + own_col + c] : 0.0f;
            *reinterpret_cast<f32x4*>(L.wlds + cls * SL + ((own_ch ^ cls) << 2)) = val;
        }
    }
    if (tid < 16) L.bias[tid] = (KIND == kSoftmax && tid < C) ? params[(int64_t)C * d + tid] : 0.0f;
    for (int q = tid; q < S * 17; q += NTC) L.small[q] = small_g[q];
    if (tid == 0) {
        L.ctl[0] = __hip_atomic_load(a.abort_flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        L.ctl[1] = 0;   // fenced until the cluster is known to share an XCD
        L.ctl[2] = 0;
        const int my_xcc = (int)(__builtin_amdgcn_s_getreg((3 << 11) | 20) & 0xF);   // XCC_ID
        __hip_atomic_store(a.xcc_ids + (int64_t)rep * G + slice, my_xcc, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    __syncthreads();
    if (L.ctl[0] != 0) return;

    const __amdgpu_buffer_rsrc_t zrsrc = make_rsrc(zpart, (uint32_t)(2u * G * a.maxrows * 16u * sizeof(float)));
    const __amdgpu_buffer_rsrc_t crsrc = make_rsrc(arrive, 8u);
    // parked gradients of this workgroup: plane e = 4 vv + c of slot s at float (s*16 + e)*NTC + tid
    const __amdgpu_buffer_rsrc_t prsrc = make_rsrc(park, (uint32_t)S * 16u * NTC * 4u);
    int pk_off[4];
#pragma unroll
    for (int vv = 0; vv < 4; ++vv) pk_off[vv] = (own_cls + vv < C) ? (vv * 4 * NTC + tid) * 4 : kOutOfRange;
    // forward: rows 16 wave .. 16 wave + 15; row / class index of this lane in the MFMA operands
    const int f_row = 16 * wave + (lane & 15);
    const int f_cls = lane & 15;
    const float* const f_x = L.tile + f_row * SL;
    const float* const f_w = L.wlds + f_cls * SL;
    // exchange: this lane's 16 bytes (4 classes of one row) inside one slice's block
    const int z_store = (f_row * 16 + 4 * (lane >> 4)) * 4;
    const int z_store_off = ((lane >> 4) < nquad) ? z_store : kOutOfRange;
    const int z_row = tid >> 2, z_qd = tid & 3;             // row / class quad of the softmax phase
    const int z_load_off = (z_qd < nquad) ? (z_row * 16 + 4 * z_qd) * 4 : kOutOfRange;
    const int slice_bytes = a.maxrows * 16 * 4;

    uint32_t n_fenced = 0, n_fast = 0;       // exchanges of each kind so far in this launch
    unsigned long long ph[8] = {0, 0, 0, 0, 0, 0, 0, 0}, tprev = 0;
    const bool profiling = PROF && tid == 0;
    auto mark = [&](int phase) {
        if constexpr (PROF) { if (profiling) { const unsigned long long now = clock64(); ph[phase] += now - tprev; tprev = now; } }
    };

    for (int64_t step = 0; step < a.nsteps; ++step) {
        const int64_t v = a.v0 + step;
        if constexpr (PROF) { if (profiling) tprev = clock64(); }
        lds_barrier();                                      // TU
        mark(0);
        const bool fast = L.ctl[1] != 0;
        const int Kv = __builtin_amdgcn_readfirstlane(L.ctl[3]);
        const int n_rec = __builtin_amdgcn_readfirstlane(L.ctl[4]);
        const int par = (int)(step & 1);

        // ---- partial logits of rows 16 wave ..: D[class][row] += W[class][k] X[row][k] over this slice
        {
            f32x4 acc0 = {0.f, 0.f, 0.f, 0.f}, acc1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll 4
            for (int s = 0; s < SL / 16; ++s) {
                const int ch = 4 * s + (lane >> 4);
                f32x4 wv = {0.f, 0.f, 0.f, 0.f};
                if (f_cls < C) wv = *reinterpret_cast<const f32x4*>(f_w + ((ch ^ f_cls) << 2));
                const f32x4 xv = *reinterpret_cast<const f32x4*>(f_x + ((ch ^ (f_row & 15)) << 2));
                acc0 = __builtin_amdgcn_mfma_f32_16x16x4f32(wv.x, xv.x, acc0, 0, 0, 0);
                acc1 = __builtin_amdgcn_mfma_f32_16x16x4f32(wv.y, xv.y, acc1, 0, 0, 0);
                acc0 = __builtin_amdgcn_mfma_f32_16x16x4f32(wv.z, xv.z, acc0, 0, 0, 0);
                acc1 = __builtin_amdgcn_mfma_f32_16x16x4f32(wv.w, xv.w, acc1, 0, 0, 0);
            }
            const f32x4 out = acc0 + acc1;   // classes 4*(lane/16)+0..3 of row f_row
            __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, out), zrsrc, z_store_off,
                                                   (par * G + slice) * slice_bytes, 0);
        }
        // ---- arrival: this wave's stores are in the L2 (shared-L2 mode) or released to the device
        if (fast) {
            __builtin_amdgcn_s_waitcnt(0x0F70);              // vmcnt(0): the stores have been acknowledged
            if (lane == 0) (void)__builtin_amdgcn_raw_ptr_buffer_atomic_add_i32(1, crsrc, 4, 0, 0);
        } else {
            if (lane == 0) __hip_atomic_fetch_add(arrive, 1u, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
        }
        mark(1);

        // ---- while the other slices arrive: the part of update v that earlier steps parked
        float gsum[16];
        float bg[4] = {0.f, 0.f, 0.f, 0.f};
        float lsum = 0.0f;
#pragma unroll
        for (int e = 0; e < 16; ++e) gsum[e] = 0.0f;
        for (int l = 0; l < Kv; ++l) {
            if (L.s_tau[l] == (int32_t)v) continue;
            const int slot = __builtin_amdgcn_readfirstlane(L.s_sel[l]);
            const int soff = slot * 16 * NTC * 4;
            float pv[16];
#pragma unroll
            for (int e = 0; e < 16; ++e)
                pv[e] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(prsrc, pk_off[e >> 2], soff + (e & 3) * NTC * 4, 0));
#pragma unroll
            for (int e = 0; e < 16; ++e) gsum[e] += pv[e];
            if (bias_owner) {
#pragma unroll
                for (int vv = 0; vv < 4; ++vv) bg[vv] += L.small[slot * 17 + own_cls + vv];
                if (loss_owner) lsum += L.small[slot * 17 + 16];
            }
        }
        mark(2);

        // ---- every wave polls the counter itself: all 4 G waves of the cluster have arrived
        {
            const uint32_t target = (fast ? n_fast + 1u : n_fenced + 1u) * (uint32_t)(4 * G);
            uint32_t spins = 0;
            for (;;) {
                uint32_t got = fast ? __builtin_amdgcn_raw_buffer_load_b32(crsrc, 4, 0, kAgentLoad)
                                    : __hip_atomic_load(arrive, __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_AGENT);
                asm volatile("" ::: "memory");   // the load is repeated every turn
                got = (uint32_t)__builtin_amdgcn_readfirstlane((int)got);
                if ((int32_t)(got - target) >= 0) break;
                __builtin_amdgcn_s_sleep(1);
                ++spins;
                if (spins > a.spin_limit ||
                    ((spins & 63u) == 0 && __hip_atomic_load(a.abort_flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0)) {
                    if (lane == 0) {
                        __hip_atomic_store(a.abort_flag, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                        L.ctl[0] = 1;
                    }
                    break;
                }
            }
            if (!fast && a.allow_fast && tid == 0) {
                // first exchange of the launch: do all slices of this cluster share an XCD (one L2)?
                const int32_t* ids = a.xcc_ids + (int64_t)rep * G;
                int same = 1;
                const int mine = __hip_atomic_load(ids + slice, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                for (int g = 0; g < G; ++g)
                    if (__hip_atomic_load(ids + g, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != mine) same = 0;
                L.ctl[2] = same;
            }
            if (fast) ++n_fast; else ++n_fenced;
        }
        mark(3);

        // ---- full logits of row z_row (sum of the G partials in slice order), then residual / softmax
        {
            f32x4 zz = {0.f, 0.f, 0.f, 0.f};
            const int zbase = par * G * slice_bytes;
            for (int g0 = 0; g0 < G; g0 += 12) {
                // straight-line batch: slices past the end re-read the last one and are not added
                f32x4 part[12];
#pragma unroll
                for (int i = 0; i < 12; ++i)
                    part[i] = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(
                        zrsrc, z_load_off, zbase + min(g0 + i, G - 1) * slice_bytes, kAgentLoad));
#pragma unroll
                for (int i = 0; i < 12; ++i) {
                    const float keep = (g0 + i < G) ? 1.0f : 0.0f;
                    zz += part[i] * keep;
                }
            }
            mark(4);
            const bool ok = L.rowid[z_row] != kNoRow;
            f32x4 dl = {0.f, 0.f, 0.f, 0.f};
            float loss = 0.0f;
            if constexpr (KIND == kLsq) {
                const float z0 = __shfl(zz.x, lane & ~3, 64);
                const float r = z0 - L.ylab[z_row];
                if (ok) loss = 0.5f * r * r;
                if (z_qd == 0 && ok) dl.x = r * inv_m;
            } else {
                const int lab = __float_as_int(L.ylab[z_row]);
                float zmax = -3.0e38f;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    zz[e] += L.bias[4 * z_qd + e];
                    if (4 * z_qd + e < C) zmax = fmaxf(zmax, zz[e]);
                }
                zmax = fmaxf(zmax, __shfl_xor(zmax, 1, 64));
                zmax = fmaxf(zmax, __shfl_xor(zmax, 2, 64));
                float den = 0.0f, lt_ = 0.0f;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const float ex = (4 * z_qd + e < C) ? expf(zz[e] - zmax) : 0.0f;
                    den += ex;
                    if (4 * z_qd + e == lab) lt_ = -(zz[e] - zmax);
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
                    const float pr = dl[e] * inv - ((4 * z_qd + e == lab) ? 1.0f : 0.0f);
                    dl[e] = (ok && 4 * z_qd + e < C) ? pr * inv_m : 0.0f;
                }
            }
            // the unused class 15 carries the row loss, so that one contraction with a column of ones
            // yields the bias gradient and the loss sum
            if (z_qd == 3) dl.w = loss * inv_m;
            *reinterpret_cast<f32x4*>(L.zbuf + z_row * 16 + 4 * z_qd) = dl;
        }
        lds_barrier();                                      // D
        if (L.ctl[0] != 0) return;   // uniform: every thread reads the same LDS word
        mark(5);

        // ---- per record: the gradient slice delta^T X; wave 0 also contracts delta with a column of
        //      ones, which gives the bias gradient and (class 15) the loss sum
        for (int r = 0; r < n_rec; ++r) {
            const int slot = __builtin_amdgcn_readfirstlane(L.s_slot[r]);
            const bool is_fresh = __builtin_amdgcn_readfirstlane(L.s_fresh[r]) != 0;
            f32x4 acc[4], accb = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int c = 0; c < 4; ++c) acc[c] = f32x4{0.f, 0.f, 0.f, 0.f};
            auto contract = [&](float dv, const f32x4& xv) {
                acc[0] = __builtin_amdgcn_mfma_f32_16x16x4f32(dv, xv.x, acc[0], 0, 0, 0);
                acc[1] = __builtin_amdgcn_mfma_f32_16x16x4f32(dv, xv.y, acc[1], 0, 0, 0);
                acc[2] = __builtin_amdgcn_mfma_f32_16x16x4f32(dv, xv.z, acc[2], 0, 0, 0);
                acc[3] = __builtin_amdgcn_mfma_f32_16x16x4f32(dv, xv.w, acc[3], 0, 0, 0);
                if (wave == 0) accb = __builtin_amdgcn_mfma_f32_16x16x4f32(dv, 1.0f, accb, 0, 0, 0);
            };
            int ks = r * mp / 4;
            const int ks_end = ks + mp / 4;
            for (; ks + 4 <= ks_end; ks += 4) {     // operands of four steps are read before their MFMAs
                float dv[4];
                f32x4 xv[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int row = 4 * (ks + u) + (lane >> 4);
                    dv[u] = L.zbuf[row * 16 + (lane & 15)];
                    xv[u] = *reinterpret_cast<const f32x4*>(L.tile + row * SL + ((own_ch ^ (row & 15)) << 2));
                }
#pragma unroll
                for (int u = 0; u < 4; ++u) contract(dv[u], xv[u]);
            }
            for (; ks < ks_end; ++ks) {
                const int row = 4 * ks + (lane >> 4);
                const float dv = L.zbuf[row * 16 + (lane & 15)];
                const f32x4 xv = *reinterpret_cast<const f32x4*>(L.tile + row * SL + ((own_ch ^ (row & 15)) << 2));
                contract(dv, xv);
            }
            if (is_fresh) {
#pragma unroll
                for (int vv = 0; vv < 4; ++vv)
#pragma unroll
                    for (int c = 0; c < 4; ++c) gsum[vv * 4 + c] += acc[c][vv];
                if (bias_owner) {
#pragma unroll
                    for (int vv = 0; vv < 4; ++vv) bg[vv] += accb[vv];
                    if (loss_owner) lsum += accb[3];
                }
            } else {
                const int soff = slot * 16 * NTC * 4;
#pragma unroll
                for (int vv = 0; vv < 4; ++vv)
#pragma unroll
                    for (int c = 0; c < 4; ++c)
                        __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(uint32_t, acc[c][vv]), prsrc, pk_off[vv],
                                                              soff + c * NTC * 4, 0);
                if (bias_owner) {
#pragma unroll
                    for (int vv = 0; vv < 4; ++vv) L.small[slot * 17 + own_cls + vv] = accb[vv];
                    if (loss_owner) L.small[slot * 17 + 16] = accb[3];
                }
            }
        }
        mark(6);
        lds_barrier();                                      // B: the loader waves may rewrite the tile and the lists
        // ---- update v: each compute thread owns its weights; nobody reads them before TU
        {
            const float scale = a.lr / (float)Kv;
            const float invK = 1.0f / (float)Kv;
#pragma unroll
            for (int vv = 0; vv < 4; ++vv) {
                const int cls = own_cls + vv;
                if (cls < C) {
                    f32x4* wp = reinterpret_cast<f32x4*>(L.wlds + cls * SL + ((own_ch ^ cls) << 2));
                    f32x4 w = *wp;
#pragma unroll
                    for (int c = 0; c < 4; ++c) w[c] -= scale * gsum[vv * 4 + c];
                    *wp = w;
                }
            }
            if (loss_owner && slice == 0) a.tr.loss[(int64_t)rep * cap + v] = lsum * invK;
            if (KIND == kSoftmax && bias_owner) {
#pragma unroll
                for (int vv = 0; vv < 4; ++vv)
                    if (own_cls + vv < C) L.bias[own_cls + vv] -= scale * bg[vv];
            }
            if (tid == 0 && L.ctl[2] != 0) L.ctl[1] = 1;   // later exchanges of this launch use the shared L2
        }
        mark(7);
    }
    if constexpr (PROF) {
        if (profiling)
            for (int q = 0; q < 8; ++q) a.prof[((int64_t)rep * G + slice) * 20 + q] += ph[q];
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();   // compute waves only would do, but every wave of the workgroup counts
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");

    // ---- leave the state in HBM for the next launch
#pragma unroll
    for (int vv = 0; vv < 4; ++vv) {
        const int cls = own_cls + vv;
        if (cls < C) {
            const f32x4 w = *reinterpret_cast<const f32x4*>(L.wlds + cls * SL + ((own_ch ^ cls) << 2));
#pragma unroll
            for (int c = 0; c < 4; ++c)
                if (own_col + c < d) params[(int64_t)cls * d + own_col + c] = w[c];
        }
    }
    if (KIND == kSoftmax && slice == 0 && tid < C) params[(int64_t)C * d + tid] = L.bias[tid];
    for (int q = tid; q < S * 17; q += NTC) small_g[q] = L.small[q];
}

template <int KIND, bool PROF>
hipError_t launch_k(const LinArgs& a, size_t lds, hipStream_t s) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(linear_tile_kernel<KIND, PROF>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    const int groups = (a.replicas + 7) / 8;
    hipLaunchKernelGGL((linear_tile_kernel<KIND, PROF>), dim3(groups * 8 * a.G), dim3(512), lds, s, a);
    return hipGetLastError();
}

}  // namespace

size_t linear_tile_lds_bytes(int C, int S) {
    const size_t words = (size_t)ROWS * SL + (size_t)C * SL + ROWS * 16 + 2 * ROWS + 16 + (size_t)S * 17 + 8 + 4 * KC;
    return sizeof(float) * words;
}

bool linear_tile_supports(const LinArgs& a, int max_records) {
    if (a.C > 15 || (a.d % 4) != 0 || a.tr.Kcap > KC || max_records > KC) return false;
    if (a.mp * max_records > ROWS) return false;
    if ((uint64_t)a.N * (uint64_t)a.d * 4u >= (1ull << 32)) return false;   // one buffer descriptor spans the sample matrix
    if (a.agg_out != nullptr) return false;
    if (a.variant == kAsync && a.v0 < 1) return false;    // step 0 of K-async starts all P workers
    if (a.variant == kBatchAsync) return false;
    return linear_tile_lds_bytes(a.C, a.S) <= 160 * 1024;
}

int linear_tile_resident_groups(size_t lds_bytes) {
    int dev = 0, per_cu = 0;
    hipDeviceProp_t prop;
    if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess) return 0;
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(linear_tile_kernel<kSoftmax, false>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes) != hipSuccess) return 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, linear_tile_kernel<kSoftmax, false>, 512, lds_bytes) != hipSuccess) return 0;
    return per_cu * prop.multiProcessorCount;
}

hipError_t launch_linear_tile(const LinArgs& a, hipStream_t s) {
    const size_t lds = linear_tile_lds_bytes(a.C, a.S);
    const bool prof = a.prof != nullptr;
    if (a.kind == kLsq) return prof ? launch_k<kLsq, true>(a, lds, s) : launch_k<kLsq, false>(a, lds, s);
    return prof ? launch_k<kSoftmax, true>(a, lds, s) : launch_k<kSoftmax, false>(a, lds, s);
}

}  // namespace ssgd
