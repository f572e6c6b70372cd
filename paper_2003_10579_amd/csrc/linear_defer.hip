// Steady-state kernel of K-async SGD on the linear models (Sec. 2.2, Eq. (3)) for the shapes of the headline
// configuration: at most 8 workers, mini-batches padded to a multiple of 16 rows, every version's mini-batches in one
// 64-row tile.  Same state in HBM between launches and the same arithmetic as linear_tile.hip; what differs is who does
// what, when, and where the gradients in flight live.
//
// A replica is a cluster of G + 1 workgroups on one XCD (they meet in its L2):
//
//   * G slice workgroups, one per CU, each owning 256 columns of the parameters.  A slice workgroup never waits
//     for a trip through the L2 in the common case.  Per version v it runs, on the fp32 MFMA units, the partial
//     logits of tile v (which need w_v) and the gradient contraction delta^T X of tile v-1, whose delta has come
//     back in the meantime.  A gradient g(w_v, xi) is needed by the update that consumes it, and the schedule
//     (which does not depend on the numerics, Sec. 3.1) says which one that is: unless it is update v itself, the
//     contraction may run one version late.  The rows it needs are copied from the LDS tile into registers (in
//     the layout of the MFMA operand) while the tile is there, so the tile is free for the next version as soon as
//     the forward pass has read it.  The gradients of the mini-batches in flight (one slot per worker; Eq. (3)
//     uses each at the update that its worker's push belongs to) stay in LDS for the whole launch: read from HBM
//     when the launch starts, written back when it ends, never in between.
//   * One helper workgroup on a CU of its own, whose memory pipeline carries no row gathers (a load that queues
//     behind 64 KB of gathers waits for them).  It polls the partial logits of the G slices, adds them in slice
//     order, takes residual / softmax and stores delta (64 x 16 words) for the slices to fetch; it owns the bias,
//     the bias gradients in flight and the loss record.
//
// Slice workgroup, version v (four compute waves, four loader waves, no workgroup barrier between them: LDS counters):
//   compute: wait for w_v (all four waves have applied update v-1) and for tile v;
//            partial logits of tile v -> exchange buffer; along the way the rows of tile v -> registers in the layout
//            of the gradient contraction, and delta_{v-1} is asked for; the tile in LDS is let go;
//            gradient contraction of tile v-1 from registers -> LDS slot of each mini-batch's worker;
//            sum of the slots that update v consumes; if update v consumes a mini-batch of version v itself, wait for
//            delta_v and contract tile v now; w_{v+1} = w_v - (lr/K) sum
//   loaders: wait until tile v-1 has been let go; tile v from registers -> LDS; sample ids and gathers of tile v+2
//            into the registers that tile v left (two sets take turns)
#include <algorithm>
#include <type_traits>

#include "common.hpp"

namespace ssgd {
namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4v __attribute__((ext_vector_type(4)));

constexpr int ROWS = 64;        // rows of the LDS tile
constexpr int SL = 256;         // columns per slice workgroup
constexpr int NTC = 256;        // compute threads
constexpr int LLOADS = 16;      // 16-byte loads per loader lane per tile
constexpr int SMAX = 8;         // gradient slots (workers) and list entries per step
constexpr int kAgentLoad = 16;  // cache policy: served by the L2, never by a CU's L1
constexpr int kStream = 2;      // cache policy: non-temporal
constexpr uint32_t kNoRow = 0xFFFFFFFFu;
constexpr uint32_t kSentinel = 0xFFFFFFFFu;    // an exchange word that has not been written yet
constexpr int kOutOfRange = (int)0x80000000;   // buffer offset past any buffer: loads give 0, stores are dropped

__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* p, uint32_t bytes) {
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p), 0, (int)bytes, 0x00020000);
}

__device__ __forceinline__ float quad_xor1(float x) {
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0xB1, 0xF, 0xF, false));   // quad_perm [1,0,3,2]
}
__device__ __forceinline__ float quad_xor2(float x) {
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0x4E, 0xF, 0xF, false));   // quad_perm [2,3,0,1]
}
__device__ __forceinline__ float quad_lane0(float x) {
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0x00, 0xF, 0xF, false));   // quad_perm [0,0,0,0]
}

// a wave gives up its wait: the launch is aborted (every workgroup of every cluster sees the flag in its own waits)
__device__ __forceinline__ bool give_up(const LinArgs& a, uint32_t spins) {
    return spins > a.spin_limit ||
           ((spins & 63u) == 0 && __hip_atomic_load(a.abort_flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0);
}

// What one version's tile consists of, derived from the trace rows (lane l holds entry l of a list): the
// mini-batches that start at w_ver are those of the workers that update ver - 1 consumed; update ver consumes K
// gradients, parked ones (version read < ver) and, possibly, some of the mini-batches of this very tile.
struct TileMeta {
    int K = 0, nrec = 0, nstale = 0, fresh = 0;
    int stale = 0, stale_pos = SMAX;   // lane l < K: slot of entry l and, if it is parked, its place in the compact list
    int rec_word = 0;                  // lane r < nrec: slot of record r; bit 16: consumed by update ver itself
    int worker = -1;                   // lane r: worker of record r
};
struct ListReader {
    const int32_t* tr_sel;
    const int32_t* tr_tau;
    int Kcap, lane;
    int q_sel = -1, q_tau = -1;        // entry `lane` of the consume list of a later version, in flight
    int cur_sel = -1;                  // consume list of the version before the one being prepared
    __device__ __forceinline__ void issue(int64_t ver) {
        q_sel = -1; q_tau = -1;
        if (lane < Kcap) {
            q_sel = tr_sel[ver * Kcap + lane];
            q_tau = tr_tau[ver * Kcap + lane];
        }
    }
    __device__ __forceinline__ void start(int64_t v0) {      // v0 >= 1
        if (lane < Kcap) cur_sel = tr_sel[(v0 - 1) * Kcap + lane];
        issue(v0);
    }
    __device__ __forceinline__ void take(TileMeta& t, int64_t ver, bool more) {
        const int l_sel = q_sel, l_tau = q_tau;
        const int K = __popcll(__ballot(l_sel >= 0));
        const int nrec = __popcll(__ballot(cur_sel >= 0));
        const int rec_slot = cur_sel;
        int fr = 0;
        for (int l = 0; l < K; ++l)
            if (__builtin_amdgcn_readlane(l_tau, l) == (int32_t)ver && __builtin_amdgcn_readlane(l_sel, l) == rec_slot) fr = 1;
        t.K = K;
        const bool is_stale = lane < K && l_tau != (int32_t)ver;
        const unsigned long long smask = __ballot(is_stale);
        t.nstale = __popcll(smask);
        t.stale = l_sel;
        t.stale_pos = is_stale ? __popcll(smask & ((1ull << lane) - 1ull)) : SMAX;
        t.nrec = nrec;
        t.rec_word = (lane < nrec) ? (rec_slot | (fr << 16)) : 0;
        t.fresh = (__ballot(lane < nrec && fr != 0) != 0ull) ? 1 : 0;
        t.worker = cur_sel;
        cur_sel = l_sel;
        asm volatile("" : "+v"(t.stale), "+v"(t.stale_pos), "+v"(t.rec_word), "+v"(t.worker), "+v"(cur_sel) : : "memory");
        if (more) issue(ver + 1);
    }
};

// Spins until the LDS counter has reached `target`; false if the launch was given up meanwhile.
__device__ __forceinline__ bool wait_count(const LinArgs& a, int* ctl, int which, int target) {
    uint32_t spins = 0;
    while (__builtin_amdgcn_readfirstlane(__hip_atomic_load(ctl + which, __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_WORKGROUP)) < target) {
        __builtin_amdgcn_s_sleep(1);
        ++spins;
        if ((spins & 255u) == 0) {
            if (__builtin_amdgcn_readfirstlane(__hip_atomic_load(ctl, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP)) != 0) return false;
            if ((spins >> 8) > a.spin_limit || __hip_atomic_load(a.abort_flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0) {
                if ((threadIdx.x & 63) == 0) {
                    __hip_atomic_store(a.abort_flag, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    __hip_atomic_store(ctl, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
                }
                return false;
            }
        }
    }
    return true;
}
__device__ __forceinline__ void bump(int* ctl, int which) {
    if ((threadIdx.x & 63) == 0) __hip_atomic_fetch_add(ctl + which, 1, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_WORKGROUP);
}

// ============================================================================================================
// Helper workgroup: four softmax waves (thread -> row tid / 4 of the tile, classes 4 (tid % 4) .. + 3) and one
// clerk wave.  The softmax waves do nothing but what the slices wait for: poll the partial logits, add them, take
// residual / softmax with the bias and the labels that the clerk has put into LDS, store delta, and leave the column
// sums of delta (bias gradient, loss) in LDS for the clerk.  The clerk wave (lane -> row of the tile for the labels,
// lane -> class for the sums) reads the schedule, draws the sample ids and fetches the labels of the next version,
// keeps the bias and the bias gradients in flight, and writes the loss record.  They meet through two LDS counters:
//   sums   += 1 by every softmax wave once its column sums of version s are in LDS    (complete at 4 (s + 1))
//   meta    = s + 1 by the clerk once bias and labels of version s are in LDS
// LDS: colsum[2][4][16], biasbuf[2][16], labbuf[2][64], small[S][17], counters.
// ============================================================================================================
template <int KIND, bool PROF>
__device__ __forceinline__ void helper_role(const LinArgs& a, int rep, unsigned char* smem) {
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int d = a.d, C = a.C, m = a.m, mp = a.mp, S = a.S, G = a.G;
    const int64_t cap = a.tr.cap;
    float* colsum = reinterpret_cast<float*>(smem);          // [2][4][16], per step parity
    float* biasbuf = colsum + 128;                           // [2][16]
    uint32_t* labbuf = reinterpret_cast<uint32_t*>(biasbuf + 32);   // [2][64] label (or target) bits; kNoRow: no sample in this row
    int* cnt = reinterpret_cast<int*>(labbuf + 128);         // [4]: 0 stop, 1 sums, 2 meta
    float* small = reinterpret_cast<float*>(cnt + 4);        // [S][17]
    constexpr int kSums = 1, kMeta = 2;
    const int64_t nw = (KIND == kLsq) ? d : (int64_t)C * d + C;
    float* params = a.params + (int64_t)rep * nw;
    float* small_g = a.park_small + (int64_t)rep * G * S * 17;      // slice 0's copy is read; every slice's is written back
    for (int q = tid; q < S * 17; q += 5 * 64) small[q] = small_g[q];
    if (tid < 4) cnt[tid] = 0;
    __syncthreads();

    uint32_t h_acc = 0, h_t0 = 0;            // diagnostics: cycles between two marks (numbered from 32) of one wave
    auto hmark = [&](int q) {
        if constexpr (PROF) {
            if (wave == a.prof_wave) {
                if (32 + q == a.prof_a) h_t0 = (uint32_t)clock64();
                if (32 + q == a.prof_b) h_acc += (uint32_t)clock64() - h_t0;
            }
        }
    };
    auto hprof_out = [&]() {
        if constexpr (PROF) {
            if (wave == a.prof_wave && lane == 0) a.prof[(int64_t)a.prof_base + (int64_t)a.prof_helper + rep] += h_acc;
        }
    };

    if (wave == 4) {
        // ===================================== clerk =====================================
        ListReader lists{a.tr.sel + (int64_t)rep * cap * a.tr.Kcap, a.tr.tau + (int64_t)rep * cap * a.tr.Kcap, a.tr.Kcap, lane};
        TileMeta cur, nxt;
        const int rec_of = lane / mp, smp_of = lane % mp;          // tile row `lane` is sample smp_of of record rec_of
        // label (or target) bits of tile row `lane` of version `ver`; leaves the load in flight
        auto row_label = [&](const TileMeta& t, int64_t ver) -> uint32_t {
            const int worker = __shfl(t.worker, min(rec_of, 63), 64);
            if (!(smp_of < m && rec_of < t.nrec)) return kNoRow;
            const uint32_t row_id = batch_index(a.seed, (uint32_t)rep, (uint32_t)worker, 0u, (uint32_t)ver, (uint32_t)smp_of, a.N);
            return reinterpret_cast<const uint32_t*>(a.y)[row_id];
        };
        float bias_c = (KIND == kSoftmax && lane < C) ? params[(int64_t)C * d + lane] : 0.0f;     // lane c: bias of class c
        lists.start(a.v0);
        lists.take(cur, a.v0, a.nsteps > 1);
        labbuf[lane] = row_label(cur, a.v0);
        if (lane < 16) biasbuf[lane] = bias_c;
        if (lane == 0) __hip_atomic_store(cnt + kMeta, 1, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_WORKGROUP);
        const int gpr = mp >> 4;                       // groups of 16 rows per mini-batch
        for (int64_t step = 0; step < a.nsteps; ++step) {
            const int64_t v = a.v0 + step;
            const int par = (int)(step & 1);
            hmark(0);
            // the next version's lists and labels: asked for before the wait, stored after it
            uint32_t lab_nxt = kNoRow;
            if (step + 1 < a.nsteps) {
                lists.take(nxt, v + 1, step + 2 < a.nsteps);
                lab_nxt = row_label(nxt, v + 1);
            }
            hmark(1);
            if (!wait_count(a, cnt, kSums, (int)(4 * (step + 1)))) return;      // the column sums of version v are complete
            hmark(2);
            // Bias gradient (classes 0..C-1) and mean loss (class 15) of every mini-batch of the tile: summed over the
            // consume list of update v like the weight gradients, or parked in the worker's slot.  Lane c takes class c.
            {
                const int c = lane & 15;
                const int sidx = (c == 15) ? 16 : c;          // the slot record keeps the loss in word 16
                float tot = 0.0f;
                for (int i = 0; i < cur.nstale; ++i) {
                    // entry i of the compact list of parked gradients: the lane whose stale_pos is i holds its slot
                    const unsigned long long who = __ballot(cur.stale_pos == i);
                    const int slot = __builtin_amdgcn_readlane(cur.stale, (int)__builtin_ctzll(who | (1ull << 63)));
                    tot += small[slot * 17 + sidx];
                }
                for (int r = 0; r < cur.nrec; ++r) {
                    float prt = 0.0f;
                    for (int g = 0; g < gpr; ++g) prt += colsum[par * 64 + (r * gpr + g) * 16 + c];
                    const int word = __builtin_amdgcn_readlane(cur.rec_word, r);
                    if ((word >> 16) != 0) tot += prt;
                    else if (lane < 16) small[(word & 0xFFFF) * 17 + sidx] = prt;
                }
                const float invK = 1.0f / (float)cur.K;
                if (KIND == kSoftmax && lane < C) bias_c -= (a.lr * invK) * tot;
                if (lane == 15) a.tr.loss[(int64_t)rep * cap + v] = tot * invK;
                // the averaged gradient of replica 0, when the caller asked for it: bias part
                if (KIND == kSoftmax && a.agg_out != nullptr && rep == 0 && lane < C) a.agg_out[(int64_t)C * d + lane] = tot * invK;
            }
            hmark(3);
            if (step + 1 < a.nsteps) {
                // (the softmax waves are done with the buffers of version v - 1, which version v + 1 takes over: they
                // read them before they left their column sums of version v - 1, let alone v)
                labbuf[(1 - par) * 64 + lane] = lab_nxt;
                if (lane < 16) biasbuf[(1 - par) * 16 + lane] = bias_c;
                if (lane == 0) __hip_atomic_store(cnt + kMeta, (int)(step + 2), __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_WORKGROUP);
            }
            cur = nxt;
            hmark(4);
        }
        hprof_out();
        // ---- leave the state in HBM for the next launch (every slice's copy of the bias gradients in flight)
        if (KIND == kSoftmax && lane < C) params[(int64_t)C * d + lane] = bias_c;
        for (int g = 0; g < G; ++g)
            for (int q = lane; q < S * 17; q += 64) small_g[(int64_t)g * S * 17 + q] = small[q];
        return;
    }

    // ===================================== softmax waves =====================================
    const int nquad = (C + 3) / 4;
    const int z_row = tid >> 2, z_qd = tid & 3;
    const int z_load_off = (z_qd < nquad) ? (z_row * 16 + 4 * z_qd) * 4 : kOutOfRange;
    // delta goes out as [row % 4][class][row / 4]: the slices read it as the first operand of their MFMAs, where a lane
    // takes one class of rows 4 kk + lane / 16 for all sixteen kk
    const int dT_off = (((z_row & 3) * 16 + 4 * z_qd) * 16 + (z_row >> 2)) * 4;      // class 4 z_qd; + 64 bytes per class
    const float inv_m = 1.0f / (float)m;
    const __amdgpu_buffer_rsrc_t ersrc = make_rsrc(a.zx + (int64_t)rep * 3 * G * 1024, (uint32_t)(3u * G * 4096u));
    const __amdgpu_buffer_rsrc_t drsrc = make_rsrc(a.dx + (int64_t)rep * 4 * 1024, 4u * 4096u);

    // The partial logits of this thread's row from the slices of one batch (up to 12), 16 bytes each.
    u32x4v part[12];
    auto ask = [&](int buf, int g0) {
        const int xbase = buf * G * 4096;
#pragma unroll
        for (int i = 0; i < 12; ++i)
            part[i] = __builtin_amdgcn_raw_buffer_load_b128(ersrc, z_load_off, xbase + min(g0 + i, G - 1) * 4096, kAgentLoad);
    };
    ask(0, 0);
    for (int64_t step = 0; step < a.nsteps; ++step) {
        const int buf = (int)(step % 3);
        const int par = (int)(step & 1);
        hmark(0);
        // ---- full logits of row z_row: the partial logits of the G slices, polled until none of the words is the
        //      sentinel, added in slice order
        f32x4 zz = {0.f, 0.f, 0.f, 0.f};
        {
            uint32_t spins = 0;
            for (int g0 = 0; g0 < G; g0 += 12) {
                if (g0 > 0) ask(buf, g0);
                for (;;) {
                    asm volatile("" ::: "memory");   // the loads are repeated every round
                    uint32_t top = 0u;
#pragma unroll
                    for (int i = 0; i < 12; ++i) top = max(max(top, max(part[i].x, part[i].y)), max(part[i].z, part[i].w));
                    if (__ballot(top == kSentinel) == 0ull) break;
                    ++spins;
                    if (give_up(a, spins)) {
                        if (lane == 0) {
                            __hip_atomic_store(a.abort_flag, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                            __hip_atomic_store(cnt, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
                        }
                        return;
                    }
                    ask(buf, g0);
                }
#pragma unroll
                for (int i = 0; i < 12; ++i)
                    if (g0 + i < G) zz += __builtin_bit_cast(f32x4, part[i]);
            }
        }
        // everything this wave has stored so far (the re-arming stores of the version before among it) is in the L2;
        // those stores are a whole version old, so this costs nothing
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        hmark(1);
        // ---- The delta buffer of two versions on is re-armed.  It holds the delta of two versions ago; every slice
        //      has stored its partial logits of this version, which it does after it has taken the delta of the
        //      version before into registers, so that buffer is read no more.  No wait is needed here: this wave's
        //      next data store to these words is two versions away, and before the slices look at them they have seen
        //      the delta of the next version, which goes out after a wait for this wave's loads that covers the
        //      stores issued now (loads and stores share the wave's counter).
        {
            uint32_t sv = kSentinel;
            asm volatile("" : "+v"(sv));
#pragma unroll
            for (int e = 0; e < 4; ++e) __builtin_amdgcn_raw_buffer_store_b32(sv, drsrc, dT_off + 64 * e, (int)((step + 2) % 4) * 4096, 0);
        }
        // ---- bias and labels of this version (the clerk has had a whole version's time for them)
        if (!wait_count(a, cnt, kMeta, (int)(step + 1))) return;
        const uint32_t lab_bits = labbuf[par * 64 + z_row];
        const f32x4 b4 = *reinterpret_cast<const f32x4*>(biasbuf + par * 16 + 4 * z_qd);
        const bool ok = lab_bits != kNoRow;
        // ---- residual / softmax.  The slices wait for delta: it is stored as soon as it is known, the row loss (which
        //      needs a logarithm) follows.
        f32x4 dl = {0.f, 0.f, 0.f, 0.f};
        float loss = 0.0f;
        float s_den = 1.0f, s_lt = 0.0f;
        if constexpr (KIND == kLsq) {
            const float z0 = quad_lane0(zz.x);
            const float r = z0 - __uint_as_float(lab_bits);
            if (ok) loss = 0.5f * r * r;
            if (z_qd == 0 && ok) dl.x = r * inv_m;
        } else {
            const int lab = (int)lab_bits;
            float zmax = -3.0e38f;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                zz[e] += b4[e];
                if (4 * z_qd + e < C) zmax = fmaxf(zmax, zz[e]);
            }
            zmax = fmaxf(zmax, quad_xor1(zmax));
            zmax = fmaxf(zmax, quad_xor2(zmax));
            float den = 0.0f, lt_ = 0.0f;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float ex = (4 * z_qd + e < C) ? expf(zz[e] - zmax) : 0.0f;
                den += ex;
                if (4 * z_qd + e == lab) lt_ = -(zz[e] - zmax);
                dl[e] = ex;
            }
            den += quad_xor1(den);
            den += quad_xor2(den);
            const float inv = 1.0f / den;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float pr = dl[e] * inv - ((4 * z_qd + e == lab) ? 1.0f : 0.0f);
                dl[e] = (ok && 4 * z_qd + e < C) ? pr * inv_m : 0.0f;
            }
            s_den = den; s_lt = lt_;
        }
        // ---- delta goes out.  (Class 15 of a row, which does not exist, will carry the row loss in this workgroup's
        //      column sums; the slices get a zero there.)
        {
            u32x4v ob = __builtin_bit_cast(u32x4v, dl);
#pragma unroll
            for (int c = 0; c < 4; ++c) ob[c] = (ob[c] == kSentinel) ? 0x7FC00000u : ob[c];   // a NaN that is not the sentinel
#pragma unroll
            for (int e = 0; e < 4; ++e) __builtin_amdgcn_raw_buffer_store_b32(ob[e], drsrc, dT_off + 64 * e, (int)(step % 4) * 4096, 0);
        }
        hmark(2);
        {
            // this thread's words of the partial logits are re-armed for the exchange three versions on (a slice writes
            // them again only after it has seen the delta of the next version, which goes out after a wait that covers
            // these stores)
            uint32_t sv = kSentinel;
            asm volatile("" : "+v"(sv));
            const u32x4v arm = {sv, sv, sv, sv};
            for (int g = 0; g < G; ++g) __builtin_amdgcn_raw_buffer_store_b128(arm, ersrc, z_load_off, (buf * G + g) * 4096, 0);
            // and the first look at the next version's partial logits is asked for
            if (step + 1 < a.nsteps) ask((int)((step + 1) % 3), 0);
        }
        // ---- row loss and column sums for the clerk
        if constexpr (KIND == kSoftmax) {
            float lt_ = s_lt;
            lt_ += quad_xor1(lt_);
            lt_ += quad_xor2(lt_);
            loss = ok ? lt_ + logf(s_den) : 0.0f;
        }
        // the unused class 15 carries the row loss: the column sums of delta then hold the bias gradient and the loss
        if (z_qd == 3) dl.w = loss * inv_m;
        {
            // over this wave's 16 rows (one group of 16 rows never straddles two mini-batches)
            f32x4 cs = dl;
#pragma unroll
            for (int o = 4; o < 64; o <<= 1) {
#pragma unroll
                for (int e = 0; e < 4; ++e) cs[e] += __shfl_xor(cs[e], o, 64);
            }
            if (lane < 4) *reinterpret_cast<f32x4*>(colsum + par * 64 + wave * 16 + 4 * lane) = cs;
        }
        bump(cnt, kSums);
        hmark(3);
    }
    hprof_out();
}

// ============================================================================================================
// Slice workgroup.  After the set-up its eight waves never meet at a workgroup barrier: the loader waves stall
// wherever the memory system makes them wait with their gathers, and nothing the compute waves do may depend on
// that beyond the tile itself.  Three counters in LDS carry the hand-over instead (a wave's LDS operations are
// performed in the order it issued them, so a counter that a wave bumps after its writes, or after its reads,
// says that they are done):
//   ready  += 1 by every loader wave once its rows of tile s are in LDS            (tile s complete at 4 (s + 1))
//   taken  += 1 by every compute wave once it has read tile s for the last time    (tile s free at 4 (s + 1))
//   stepped += 1 by every compute wave once its share of w_{s+1} is in LDS         (w_{s+1} complete at 4 (s + 1))
// ============================================================================================================
struct Lds {
    float* tile;      // [64][SL]   16-byte chunk c of row r at chunk position c ^ (r & 15)
    float* wlds;      // [C][SL]    same swizzle, keyed by the class
    float* park;      // [S][C][SL] gradient of the mini-batch in flight of every worker, plain layout
    int* ctl;         // [4]: 0 stop, 1 ready, 2 taken, 3 stepped
    int* stp;         // [2][4] per step parity: K, records, parked gradients that the update consumes, 1 if it consumes a record of its own version
    int* s_stale;     // [2][8] slots of those parked gradients, in the order of the consume list
    int* s_rec;       // [2][8] slot of record r; bit 16: consumed by the update of its own version
};

__device__ __forceinline__ Lds carve(unsigned char* smem, int C, int S) {
    Lds l;
    l.tile = reinterpret_cast<float*>(smem);
    l.wlds = l.tile + ROWS * SL;
    l.park = l.wlds + C * SL;
    l.ctl = reinterpret_cast<int*>(l.park + S * C * SL);
    l.stp = l.ctl + 4;
    l.s_stale = l.stp + 8;
    l.s_rec = l.s_stale + 2 * SMAX;
    return l;
}

template <int KIND, bool PROF, int MPK>
__device__ __forceinline__ void slice_role(const LinArgs& a, int rep, int slice, unsigned char* smem) {
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int d = a.d, C = a.C, m = a.m, S = a.S, G = a.G;
    const int mp = MPK > 0 ? MPK : a.mp;      // rows per mini-batch in the tile: known when the kernel is compiled, as a rule
    const int Kcap = a.tr.Kcap;
    const int64_t cap = a.tr.cap;
    const int col0 = slice * SL;
    const Lds L = carve(smem, C, S);
    constexpr int kReady = 1, kTaken = 2, kStepped = 3;

    if (wave >= 4) {
        // =============================== loader waves ===============================
        const int lw = wave - 4;
        const __amdgpu_buffer_rsrc_t xrsrc = make_rsrc(a.X, (uint32_t)((uint64_t)a.N * d * 4u));
        const uint32_t row_bytes = (uint32_t)d * 4u;
        // tile row `lane` is sample s_of of record r_of
        const int r_of = lane / mp, s_of = lane % mp;
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

        // Two sets of prefetch registers and tile descriptions, used in turn: tile s sits in set s & 1 until the compute
        // waves have let go of tile s - 1; as soon as it is in LDS, the gathers of tile s + 2 are issued into its set.
        f32x4 pref[2][LLOADS];
        TileMeta meta[2];
        ListReader lists{a.tr.sel + (int64_t)rep * cap * Kcap, a.tr.tau + (int64_t)rep * cap * Kcap, Kcap, lane};

        uint32_t lp_acc = 0, lp_t0 = 0;  // diagnostics: cycles between two marks, summed in scalar registers
        const bool lprof = PROF && lw == a.prof_wave;
        auto lmark = [&](int q) {
            if constexpr (PROF) {
                if (lprof) {
                    if (16 + q == a.prof_a) lp_t0 = (uint32_t)clock64();
                    if (16 + q == a.prof_b) lp_acc += (uint32_t)clock64() - lp_t0;
                }
            }
        };
        // Sample ids of the tile of version `ver`; leaves the gathers in flight.
        auto make_tile = [&](const TileMeta& t, f32x4 (&pf)[LLOADS], int64_t ver) {
            const int worker = __shfl(t.worker, min(r_of, 63), 64);
            uint32_t row_id = kNoRow;
            if (s_of < m && r_of < t.nrec)
                row_id = batch_index(a.seed, (uint32_t)rep, (uint32_t)worker, 0u, (uint32_t)ver, (uint32_t)s_of, a.N);
            asm volatile("" : "+v"(row_id) : : "memory");
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int i = 0; i < LLOADS; ++i) {
                // rows without a sample read row 0; their delta is zero
                uint32_t id = (uint32_t)__builtin_amdgcn_readlane((int)row_id, lw + 4 * i);
                id = (id == kNoRow) ? 0u : id;
                pf[i] = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(xrsrc, goff[i & 3], (int)(id * row_bytes), kStream));
            }
        };
        auto publish = [&](const TileMeta& t, const f32x4 (&pf)[LLOADS], int par) {
#pragma unroll
            for (int i = 0; i < LLOADS; ++i) *reinterpret_cast<f32x4*>(my_tile + 4 * i * SL) = pf[i];
            if (lw == 0) {
                if (lane == 0) {
                    L.stp[par * 4 + 0] = t.K; L.stp[par * 4 + 1] = t.nrec; L.stp[par * 4 + 2] = t.nstale; L.stp[par * 4 + 3] = t.fresh;
                }
                if (t.stale_pos < SMAX) L.s_stale[par * SMAX + t.stale_pos] = t.stale;
                if (lane < SMAX) L.s_rec[par * SMAX + lane] = t.rec_word;
            }
        };

        __syncthreads();                             // the compute waves have set up the control words and the slots
        if (L.ctl[0] != 0) return;
        lists.start(a.v0);
        lists.take(meta[0], a.v0, a.nsteps > 1);
        make_tile(meta[0], pref[0], a.v0);
        if (a.nsteps > 1) {
            lists.take(meta[1], a.v0 + 1, a.nsteps > 2);
            make_tile(meta[1], pref[1], a.v0 + 1);
        }
        // One tile with compile-time register set Q = step & 1.
        auto one_step = [&](auto qc, int64_t step) {
            constexpr int Q = decltype(qc)::value;
            lmark(0);
            if (!wait_count(a, L.ctl, kTaken, (int)(4 * step))) return false;      // tile step - 1 has been read
            lmark(1);
            publish(meta[Q], pref[Q], Q);
            bump(L.ctl, kReady);
            lmark(2);
            if (step + 2 < a.nsteps) {
                lists.take(meta[Q], a.v0 + step + 2, step + 3 < a.nsteps);
                make_tile(meta[Q], pref[Q], a.v0 + step + 2);
            }
            lmark(3);
            return true;
        };
        for (int64_t step = 0; step < a.nsteps; step += 2) {
            if (!one_step(std::integral_constant<int, 0>{}, step)) return;
            if (step + 1 < a.nsteps && !one_step(std::integral_constant<int, 1>{}, step + 1)) return;
        }
        if constexpr (PROF) {
            if (lprof && lane == 0) a.prof[(int64_t)a.prof_base + ((int64_t)rep * G + slice) * 2 + 1] += lp_acc;
        }
        return;
    }

    // ================================= compute waves =================================
    const int64_t nw = (KIND == kLsq) ? d : (int64_t)C * d + C;
    float* params = a.params + (int64_t)rep * nw;
    float* park_g = a.park + ((int64_t)rep * G + slice) * S * 16 * NTC;
    const int nquad = (C + 3) / 4;

    // share of the parameters: classes own_cls .. own_cls+3, columns own_col .. own_col+3
    const int own_ch = 16 * wave + (lane & 15);
    const int own_col = col0 + 4 * own_ch;
    const int own_cls = 4 * (lane >> 4);
    // Lanes of classes that do not exist (the class dimension is padded to 16 for the MFMA units) own nothing.  Their
    // LDS reads go to the last class that exists, so that no read needs a branch; what they compute is never stored.
    int slot_row[4];         // float offset of (class own_cls + vv, chunk own_ch) inside a slot of L.park, clamped
    int w_off[4];            // float offset of the same element in L.wlds (swizzled), clamped
#pragma unroll
    for (int vv = 0; vv < 4; ++vv) {
        const int cls = min(own_cls + vv, C - 1);
        slot_row[vv] = cls * SL + 4 * own_ch;
        w_off[vv] = cls * SL + ((own_ch ^ cls) << 2);
    }
    f32x4 w_own[4];
#pragma unroll
    for (int v = 0; v < 4; ++v) {
        const int cls = own_cls + v;
        w_own[v] = f32x4{0.f, 0.f, 0.f, 0.f};
        if (cls < C) {
#pragma unroll
            for (int c = 0; c < 4; ++c) w_own[v][c] = (own_col + c < d) ? params[(int64_t)cls * d + own_col + c] : 0.0f;
            *reinterpret_cast<f32x4*>(L.wlds + w_off[v]) = w_own[v];
        }
    }
    // the gradients in flight: HBM layout 16 bytes at ((slot * 4 + vv) * NTC + tid) * 16 -> this thread's words of the slot
    for (int s = 0; s < S; ++s) {
#pragma unroll
        for (int vv = 0; vv < 4; ++vv) {
            const int cls = own_cls + vv;
            if (cls < C)
                *reinterpret_cast<f32x4*>(L.park + ((s * C + cls) * SL + 4 * own_ch)) =
                    *reinterpret_cast<const f32x4*>(park_g + ((int64_t)(s * 4 + vv) * NTC + tid) * 4);
        }
    }
    if (tid == 0) {
        L.ctl[0] = __hip_atomic_load(a.abort_flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        L.ctl[1] = 0; L.ctl[2] = 0; L.ctl[3] = 0;
    }
    __syncthreads();
    if (L.ctl[0] != 0) return;

    // exchange: three buffers of G x 64 x 16 words (partial logits, written here) and three of 64 x 16 words (delta,
    // written by the helper; four of those), used in turn; a word is the sentinel until it has been written
    const __amdgpu_buffer_rsrc_t ersrc = make_rsrc(a.zx + (int64_t)rep * 3 * G * 1024, (uint32_t)(3u * G * 4096u));
    const __amdgpu_buffer_rsrc_t drsrc = make_rsrc(a.dx + (int64_t)rep * 4 * 1024, 4u * 4096u);
    // forward: rows 16 wave .. 16 wave + 15; row / class index of this lane in the MFMA operands
    const int f_row = 16 * wave + (lane & 15);
    const int f_key = min(lane & 15, C - 1);     // lanes of classes that do not exist read the last class
    const float* f_xa[4];
    const float* f_wa[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int kx = f_row & 15;
        f_xa[j] = L.tile + f_row * SL + ((4 * (j ^ (kx >> 2)) + ((lane >> 4) ^ (kx & 3))) << 2);
        f_wa[j] = L.wlds + f_key * SL + ((4 * (j ^ (f_key >> 2)) + ((lane >> 4) ^ (f_key & 3))) << 2);
    }
    const int z_store = (f_row * 16 + 4 * (lane >> 4)) * 4;
    const int z_store_off = ((lane >> 4) < nquad) ? z_store : kOutOfRange;
    const int b_lo = lane >> 4, b_cls = lane & 15;
    // The rows of the tile as the second operand of the gradient contraction: k-step kk covers rows 4 kk .. 4 kk + 3,
    // this lane takes row 4 kk + lane / 16, chunk own_ch.  The swizzle key of that row is 4 (kk % 4) + lane / 16: four
    // base addresses, the rest is a constant offset of 16 rows per (kk / 4).
    const float* r_xa[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) r_xa[u] = L.tile + (4 * u + b_lo) * SL + ((own_ch ^ (4 * u + b_lo)) << 2);
    // delta as the first operand: the helper stores it as [row % 4][class][row / 4], so that this lane's sixteen values
    // (row 4 kk + lane / 16, class lane % 16, kk = 0 .. 15) are 64 consecutive bytes
    const int d_off = (b_lo * 16 + b_cls) * 64;

    uint32_t p_acc = 0, p_t0 = 0;            // diagnostics, as in the loader waves
    const bool profiling = PROF && wave == a.prof_wave;
    auto mark = [&](int phase) {
        if constexpr (PROF) {
            if (profiling) {
                if (phase == a.prof_a) p_t0 = (uint32_t)clock64();
                if (phase == a.prof_b) p_acc += (uint32_t)clock64() - p_t0;
            }
        }
    };

    f32x4 xb[2][16];         // set s & 1: rows 4 kk + lane / 16 of tile s, chunk own_ch
    float gsum[16];          // this thread's part of sum_l g_l of the update in progress: gsum[4 vv + c]
    u32x4v da[4];            // delta of the tile whose gradient contraction comes next
    bool pend = false;       // the tile before this one still waits for its gradient contraction
    int pend_words = 0, pend_nrec = 0, pend_buf = 0;    // lane r < 8: slot word of its record r; delta buffer of that tile

    auto ask_delta = [&](int buf) {
#pragma unroll
        for (int q = 0; q < 4; ++q) da[q] = __builtin_amdgcn_raw_buffer_load_b128(drsrc, d_off + 16 * q, buf * 4096, kAgentLoad);
    };
    // all 16 words of every lane have been written by the helper?  Otherwise they are asked for again.
    auto await_delta = [&](int buf) -> bool {
        uint32_t spins = 0;
        for (;;) {
            asm volatile("" ::: "memory");
            uint32_t top = 0u;
#pragma unroll
            for (int q = 0; q < 4; ++q) top = max(max(top, max(da[q].x, da[q].y)), max(da[q].z, da[q].w));
            if (__ballot(top == kSentinel) == 0ull) return true;
            ++spins;
            if (give_up(a, spins) || __builtin_amdgcn_readfirstlane(__hip_atomic_load(L.ctl, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP)) != 0) {
                if (lane == 0) {
                    __hip_atomic_store(a.abort_flag, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    __hip_atomic_store(L.ctl, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
                }
                return false;
            }
            __builtin_amdgcn_s_sleep(1);
            ask_delta(buf);
        }
    };
    // Gradient contraction of a tile's rows (in registers) with the delta in da, mini-batch by mini-batch (mp rows
    // each, a multiple of 16).  A mini-batch that the update in progress consumes itself (`now`, bit 16 of its word) is
    // added to gsum; every other one goes to the LDS slot of its worker.
    auto backward = [&](const f32x4 (&xr)[16], int words, int n_rec, bool now) {
        const int rows_used = n_rec * mp;
        f32x4 acc[4];
#pragma unroll
        for (int g = 0; g < 4; ++g) {                 // groups of 16 rows
            const bool first = (16 * g) % mp == 0, last = (16 * (g + 1)) % mp == 0;     // of their mini-batch
            if (16 * g < rows_used) {
                if (first) {
#pragma unroll
                    for (int c = 0; c < 4; ++c) acc[c] = f32x4{0.f, 0.f, 0.f, 0.f};
                }
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int kk = 4 * g + u;
                    const float dk = __uint_as_float(da[g][u]);
#pragma unroll
                    for (int c = 0; c < 4; ++c) acc[c] = __builtin_amdgcn_mfma_f32_16x16x4f32(dk, xr[kk][c], acc[c], 0, 0, 0);
                }
                if (last) {
                    const int r = (16 * (g + 1)) / mp - 1;
                    const int word = __builtin_amdgcn_readlane(words, r);
                    if (now && (word >> 16) != 0) {
#pragma unroll
                        for (int vv = 0; vv < 4; ++vv)
#pragma unroll
                            for (int c = 0; c < 4; ++c) gsum[vv * 4 + c] += acc[c][vv];
                    } else {
                        float* slot = L.park + (word & 0xFFFF) * C * SL;
#pragma unroll
                        for (int vv = 0; vv < 4; ++vv)
                            if (own_cls + vv < C) *reinterpret_cast<f32x4*>(slot + slot_row[vv]) = f32x4{acc[0][vv], acc[1][vv], acc[2][vv], acc[3][vv]};
                    }
                }
            }
        }
    };

    // One version with compile-time register set Q = step & 1.
    auto one_step = [&](auto qc, int64_t step) -> bool {
        constexpr int Q = decltype(qc)::value;
        mark(9);
        if (!wait_count(a, L.ctl, kStepped, (int)(4 * step))) return false;          // w_v is complete
        if (!wait_count(a, L.ctl, kReady, (int)(4 * (step + 1)))) return false;      // tile v is complete
        mark(0);
        const int buf = (int)(step % 3), dbuf = (int)(step % 4);
        const int4 stp4 = *reinterpret_cast<const int4*>(L.stp + Q * 4);
        const int Kv = __builtin_amdgcn_readfirstlane(stp4.x);
        const int n_rec = __builtin_amdgcn_readfirstlane(stp4.y);
        const int n_stale = __builtin_amdgcn_readfirstlane(stp4.z);
        const bool fresh = __builtin_amdgcn_readfirstlane(stp4.w) != 0;
        const int st_lane = L.s_stale[Q * SMAX + (lane & (SMAX - 1))];
        const int rec_lane = L.s_rec[Q * SMAX + (lane & (SMAX - 1))];

        // ---- partial logits of rows 16 wave ..: D[class][row] += W[class][k] X[row][k] over this slice, the operands
        //      read from LDS two rounds ahead of their MFMAs; along the way, one k-step per round, the tile's rows in
        //      the layout of the gradient contraction -> registers
        f32x4 out;
        {
            f32x4 acc0 = {0.f, 0.f, 0.f, 0.f}, acc1 = {0.f, 0.f, 0.f, 0.f};
            auto w_at = [&](int s) { return *reinterpret_cast<const f32x4*>(f_wa[s & 3] + (s >> 2) * 64); };
            auto x_at = [&](int s) { return *reinterpret_cast<const f32x4*>(f_xa[s & 3] + (s >> 2) * 64); };
            f32x4 w0 = w_at(0), x0 = x_at(0), w1 = w_at(1), x1 = x_at(1);
#pragma unroll
            for (int s = 0; s < SL / 16; ++s) {
                f32x4 w2 = w1, x2 = x1;
                if (s + 2 < SL / 16) { w2 = w_at(s + 2); x2 = x_at(s + 2); }
                xb[Q][s] = *reinterpret_cast<const f32x4*>(r_xa[s & 3] + (s >> 2) * 16 * SL);
                // half-way through: the delta of the tile before, which the helper has stored by now as a rule
                if (s == SL / 32 && pend) ask_delta(pend_buf);
                __builtin_amdgcn_sched_barrier(0);   // keep the reads ahead of the MFMAs
                acc0 = __builtin_amdgcn_mfma_f32_16x16x4f32(w0.x, x0.x, acc0, 0, 0, 0);
                acc1 = __builtin_amdgcn_mfma_f32_16x16x4f32(w0.y, x0.y, acc1, 0, 0, 0);
                acc0 = __builtin_amdgcn_mfma_f32_16x16x4f32(w0.z, x0.z, acc0, 0, 0, 0);
                acc1 = __builtin_amdgcn_mfma_f32_16x16x4f32(w0.w, x0.w, acc1, 0, 0, 0);
                w0 = w1; x0 = x1; w1 = w2; x1 = x2;
            }
            out = acc0 + acc1;   // classes 4*(lane/16)+0..3 of row f_row
        }
        bump(L.ctl, kTaken);                                 // this wave is done with the tile in LDS
        mark(1);
        // The delta of the tile before is awaited before the partial logits are stored: a wave's stores and loads share
        // one counter, and a wait for these loads with a store in flight would wait for the store's trip to the L2 too.
        if (pend && !await_delta(pend_buf)) return false;
        mark(2);
        {
            u32x4v ob = __builtin_bit_cast(u32x4v, out);
#pragma unroll
            for (int c = 0; c < 4; ++c) ob[c] = (ob[c] == kSentinel) ? 0x7FC00000u : ob[c];   // a NaN that is not the sentinel
            // (16-byte buffer stores carry their whole offset in the vector register)
            __builtin_amdgcn_raw_buffer_store_b128(ob, ersrc, z_store_off + (buf * G + slice) * 4096, 0, 0);
        }

        mark(10);
        // ---- the gradient contraction of the tile before
        if (pend) backward(xb[1 - Q], pend_words, pend_nrec, false);
        pend = false;
        mark(3);

        // ---- the parked part of update v, in the order of the consume list (two slots are read at a time)
        {
            // (entries past the end of the list hold whatever an earlier step left: clamped, read, and not used)
            auto slot_at = [&](int i) { return L.park + min(max(__builtin_amdgcn_readlane(st_lane, i), 0), S - 1) * C * SL; };
            const float* s0 = slot_at(0);
            const float* s1 = slot_at(n_stale > 1 ? 1 : 0);
            f32x4 pa[4];
#pragma unroll
            for (int vv = 0; vv < 4; ++vv) pa[vv] = *reinterpret_cast<const f32x4*>(s0 + slot_row[vv]);
#pragma unroll
            for (int vv = 0; vv < 4; ++vv) {
                const f32x4 pb = *reinterpret_cast<const f32x4*>(s1 + slot_row[vv]);
#pragma unroll
                for (int c = 0; c < 4; ++c) gsum[vv * 4 + c] = (n_stale > 0 ? pa[vv][c] : 0.0f) + (n_stale > 1 ? pb[c] : 0.0f);
            }
            mark(11);
            for (int i = 2; i < n_stale; ++i) {
                const float* sl = slot_at(i);
#pragma unroll
                for (int vv = 0; vv < 4; ++vv) {
                    const f32x4 pv = *reinterpret_cast<const f32x4*>(sl + slot_row[vv]);
#pragma unroll
                    for (int c = 0; c < 4; ++c) gsum[vv * 4 + c] += pv[c];
                }
            }
        }
        mark(4);
        if (fresh) {
            // update v consumes a mini-batch that started at w_v: its gradient cannot wait
            mark(12);
            ask_delta(dbuf);
            if (!await_delta(dbuf)) return false;
            mark(13);
            backward(xb[Q], rec_lane, n_rec, true);
        } else {
            pend = true;
            pend_words = rec_lane;
            pend_nrec = n_rec;
            pend_buf = dbuf;
        }
        mark(5);
        // ---- update v: each compute thread owns its weights and keeps them in registers; the forward passes read the LDS copy
        {
            const float scale = a.lr / (float)Kv;
            const int ocl = own_cls;
#pragma unroll
            for (int vv = 0; vv < 4; ++vv) {
#pragma unroll
                for (int c = 0; c < 4; ++c) w_own[vv][c] -= scale * gsum[vv * 4 + c];
                if (ocl + vv < C) *reinterpret_cast<f32x4*>(L.wlds + w_off[vv]) = w_own[vv];
            }
            bump(L.ctl, kStepped);
            if (a.agg_out != nullptr && rep == 0) {
                // the averaged gradient of replica 0, when the caller asked for it
                const float invK = 1.0f / (float)Kv;
                int ocol = own_col;
                asm volatile("" : "+v"(ocol));
#pragma unroll
                for (int vv = 0; vv < 4; ++vv) {
                    const int cls = ocl + vv;
                    if (cls < C)
#pragma unroll
                        for (int c = 0; c < 4; ++c)
                            if (ocol + c < d) a.agg_out[(int64_t)cls * d + ocol + c] = gsum[vv * 4 + c] * invK;
                }
            }
        }
        mark(6);
        return true;
    };
    for (int64_t step = 0; step < a.nsteps; step += 2) {
        if (!one_step(std::integral_constant<int, 0>{}, step)) return;
        if (step + 1 < a.nsteps && !one_step(std::integral_constant<int, 1>{}, step + 1)) return;
    }
    // the last tile's gradients go to their slots like all the others
    if (pend) {
        ask_delta(pend_buf);
        if (!await_delta(pend_buf)) return;
        if ((a.nsteps & 1) != 0) backward(xb[0], pend_words, pend_nrec, false);
        else backward(xb[1], pend_words, pend_nrec, false);
    }
    if constexpr (PROF) {
        if (profiling && lane == 0) a.prof[(int64_t)a.prof_base + ((int64_t)rep * G + slice) * 2] += p_acc;
    }

    // ---- leave the state in HBM for the next launch: every thread its own words of the weights and of the slots
#pragma unroll
    for (int vv = 0; vv < 4; ++vv) {
        const int cls = own_cls + vv;
        if (cls < C) {
#pragma unroll
            for (int c = 0; c < 4; ++c)
                if (own_col + c < d) params[(int64_t)cls * d + own_col + c] = w_own[vv][c];
        }
    }
    for (int s = 0; s < S; ++s) {
#pragma unroll
        for (int vv = 0; vv < 4; ++vv) {
            const int cls = own_cls + vv;
            if (cls < C)
                *reinterpret_cast<f32x4*>(park_g + ((int64_t)(s * 4 + vv) * NTC + tid) * 4) =
                    *reinterpret_cast<const f32x4*>(L.park + ((s * C + cls) * SL + 4 * own_ch));
        }
    }
}

template <int KIND, bool PROF, int MPK>
__global__ __launch_bounds__(512, 2) void linear_defer_kernel(LinArgs a) {
    // consecutive block ids go to different XCDs: all workgroups of one cluster take block ids that are congruent
    // modulo 8 and share one L2
    const int xcd = blockIdx.x & 7, slot_in_xcd = blockIdx.x >> 3;
    const int pos = slot_in_xcd / (a.G + 1), role = slot_in_xcd % (a.G + 1);
    const int cluster = pos * 8 + xcd;
    if (cluster >= a.replicas) return;
    const int rep = a.replica0 + cluster;
    const bool helper = role == a.G;
    if (helper && threadIdx.x >= 5 * 64) return;   // the helper has five waves

    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    __shared__ int same_xcd;

    // ---- Before anything is changed: the G + 1 workgroups of the cluster meet (an arrival counter in the L2, released
    //      and acquired at device scope) and compare the XCDs they run on.  The exchange below relies on one shared L2;
    //      a cluster that is spread over XCDs leaves everything as it is and tells the host, which runs the replica
    //      through the kernel that can exchange across XCDs.
    if (threadIdx.x == 0) {
        int32_t* ids = a.xcc_ids + (int64_t)rep * (a.G + 1);
        unsigned int* arrive = a.arrive + kArriveStride * rep;
        const int my_xcc = (int)(__builtin_amdgcn_s_getreg((3 << 11) | 20) & 0xF);
        const int hw_id = (int)__builtin_amdgcn_s_getreg((15 << 11) | 4);
        __hip_atomic_store(ids + role, my_xcc | (hw_id << 8), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __hip_atomic_fetch_add(arrive, 1u, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
        uint32_t spins = 0;
        int ok = 1;
        while (__hip_atomic_load(arrive, __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_AGENT) < (unsigned)(a.G + 1)) {
            __builtin_amdgcn_s_sleep(8);
            if (give_up(a, ++spins)) {
                __hip_atomic_store(a.abort_flag, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                ok = -1;
                break;
            }
        }
        if (ok > 0) {
            for (int g = 0; g <= a.G; ++g)
                if ((__hip_atomic_load(ids + g, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) & 0xFF) != my_xcc) ok = 0;
            if ((a.debug_flags & 2) != 0 && (rep & 1) != 0) ok = 0;      // test switch of the host: odd replicas take the path of a spread cluster
        }
        same_xcd = ok;
    }
    __syncthreads();
    if (same_xcd <= 0) {
        if (same_xcd == 0 && helper && threadIdx.x == 0) a.fallback[rep] = 1;
        return;
    }

    if (helper) helper_role<KIND, PROF>(a, rep, smem);
    else slice_role<KIND, PROF, MPK>(a, rep, role, smem);
}

template <int KIND, bool PROF, int MPK>
hipError_t launch_m(const LinArgs& a, size_t lds, hipStream_t s) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(linear_defer_kernel<KIND, PROF, MPK>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    const int groups = (a.replicas + 7) / 8;
    hipLaunchKernelGGL((linear_defer_kernel<KIND, PROF, MPK>), dim3(groups * 8 * (a.G + 1)), dim3(512), lds, s, a);
    return hipGetLastError();
}

// the padded mini-batch size is a compile-time constant for 16, 32 and 64 rows (48 runs through the general code)
template <int KIND, bool PROF>
hipError_t launch_d(const LinArgs& a, size_t lds, hipStream_t s) {
    switch (a.mp) {
    case 16: return launch_m<KIND, PROF, 16>(a, lds, s);
    case 32: return launch_m<KIND, PROF, 32>(a, lds, s);
    case 64: return launch_m<KIND, PROF, 64>(a, lds, s);
    default: return launch_m<KIND, PROF, 0>(a, lds, s);
    }
}

}  // namespace

size_t linear_defer_lds_bytes(int C, int S) {
    const size_t slice_words = (size_t)ROWS * SL + (size_t)C * SL + (size_t)S * C * SL + 4 + 8 + 4 * SMAX;
    const size_t helper_words = 128 + 32 + 128 + 4 + (size_t)S * 17;
    return sizeof(float) * std::max(slice_words, helper_words);
}

bool linear_defer_supports(const LinArgs& a) {
    if (a.variant != kAsync || a.v0 < 1 || a.chunked || !a.allow_fast) return false;     // step 0 of K-async starts all P workers
    if (a.C > 15 || (a.d % 4) != 0 || (a.mp % 16) != 0 || a.mp > ROWS) return false;
    if (a.S > SMAX || a.P > SMAX || a.tr.Kcap > SMAX || a.tr.Kcap * a.mp > ROWS) return false;
    if ((uint64_t)a.N * (uint64_t)a.d * 4u >= (1ull << 32)) return false;   // one buffer descriptor spans the sample matrix
    return linear_defer_lds_bytes(a.C, a.S) <= 160 * 1024;
}

// Replicas per launch: every slice workgroup takes a CU of its own (its LDS leaves no room for a second workgroup), the
// helpers go to CUs that the slices leave free; the clusters of a launch are dealt out over the 8 XCDs.
int linear_defer_replicas_per_launch(int G, int cus) {
    const int per_xcd = cus / 8;
    int clusters = per_xcd / G;
    while (clusters > 0 && clusters * (G + 1) > per_xcd) --clusters;   // a helper asks for the same LDS: a CU of its own
    return 8 * clusters;
}

hipError_t launch_linear_defer(const LinArgs& a, hipStream_t s) {
    const size_t lds = linear_defer_lds_bytes(a.C, a.S);
    const bool prof = a.prof != nullptr;
    if (a.kind == kLsq) return prof ? launch_d<kLsq, true>(a, lds, s) : launch_d<kLsq, false>(a, lds, s);
    return prof ? launch_d<kSoftmax, true>(a, lds, s) : launch_d<kSoftmax, false>(a, lds, s);
}

}  // namespace ssgd
