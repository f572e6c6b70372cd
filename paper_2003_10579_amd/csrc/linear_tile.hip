// Steady-state kernel of the linear models (Sec. 2.2, Eq. (2), Eq. (3)) for the common shapes:
// at most 15 classes, rows readable 16 bytes at a time, and either every step's mini-batches
// fit one 64-row tile (records * padded m <= 64) or the variant is synchronous, in which case
// the rows of an iteration's K mini-batches are taken 64 at a time: every tile goes through the
// schedule below, the gradient is summed over the tiles and the update follows the last one.
// Same cluster decomposition, state layout and arithmetic as the general kernel (linear.hip),
// which runs every other shape and may be mixed with this one launch by launch; what differs
// is the schedule inside a step:
//
//   TU  tile, lists and the updated weights are in LDS          (workgroup barrier)
//       partial logits on the fp32 MFMA units, stored to the cluster's exchange buffer;
//       the parked (stale) part of update v is fetched while the stores travel;
//       each wave polls the partial logits of its 16 rows from all G slices (a word is a
//       sentinel until it has been written), sums them in slice order and goes straight on
//       to residual / softmax in registers; the buffer of the exchange before is re-armed.
//       A cluster that does not sit on one XCD (no shared L2) exchanges through released
//       stores and an arrival counter instead, as does the first exchange of every launch.
//   D   delta in LDS                                            (workgroup barrier)
//       gradient slices delta^T X per record; added to the aggregate or parked;
//       a loader wave sums delta's columns: bias gradient, loss, bias step
//   B   the tile has been read                                   (workgroup barrier)
//       compute waves: w -= (lr/K) * aggregate (after the last tile of the update);
//       loader waves: next tile -> LDS
//
// Four compute waves, four loader waves.  A wave's vector-memory counter retires in order,
// so the long HBM gathers live in waves of their own: the loader waves fetch everything of
// the next tile (lists, sample ids, labels, rows) while the current one is computed, hold the
// rows in registers, and copy them to LDS between B and TU.
#include "common.hpp"

namespace ssgd {
namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr int ROWS = 64;        // rows of the LDS tile
constexpr int SL = 256;         // columns per workgroup
constexpr int NTC = 256;        // compute threads
constexpr int LLOADS = 16;      // 16-byte loads per loader lane per tile
constexpr int KC = 64;          // list entries per step (one lane of a wave each)
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
    int* ctl;         // [8]: 0 stop, 1 exchange through the shared L2, 2 cluster shares an XCD, 3 exchanges seen by wave 0,
                      //      4 K, 5 records, 6 parked gradients that update v consumes
    int* s_stale;     // [KC] slots of those parked gradients, in the order of the consume list
    int* s_rec;       // [KC] compute list of v: slot of record r; bit 16: consumed by update v itself
};

// (kc: places of the two lists, 32 or 64: the second workgroup of a CU fits only while the lists are short)
__device__ __forceinline__ Lds carve(unsigned char* smem, int C, int S, int kc) {
    Lds l;
    l.tile = reinterpret_cast<float*>(smem);
    l.wlds = l.tile + ROWS * SL;
    l.zbuf = l.wlds + C * SL;
    l.rowid = reinterpret_cast<uint32_t*>(l.zbuf + ROWS * 16);
    l.ylab = reinterpret_cast<float*>(l.rowid + ROWS);
    l.bias = l.ylab + ROWS;
    l.ctl = reinterpret_cast<int*>(l.bias + 16);      // 16-byte aligned: words 4..7 are read as one vector
    l.s_stale = l.ctl + 8;
    l.s_rec = l.s_stale + kc;
    l.small = reinterpret_cast<float*>(l.s_rec + kc);
    return l;
}

// value of lane ^ 1 / lane ^ 2 inside a quad: a data-parallel-primitive move, no LDS round trip
__device__ __forceinline__ float quad_xor1(float x) {
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0xB1, 0xF, 0xF, false));   // quad_perm [1,0,3,2]
}
__device__ __forceinline__ float quad_xor2(float x) {
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0x4E, 0xF, 0xF, false));   // quad_perm [2,3,0,1]
}
__device__ __forceinline__ float quad_lane0(float x) {
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0x00, 0xF, 0xF, false));   // quad_perm [0,0,0,0]
}

__device__ __forceinline__ void lds_barrier() {
    // orders LDS traffic only: outstanding global loads and stores stay in flight
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

template <int KIND, bool PROF, bool WHOLE, bool CHUNKED, bool BATCH>
__global__ __launch_bounds__(512, 4) void linear_tile_kernel(LinArgs a) {
    // consecutive block ids go to different XCDs: all slices of one cluster take block ids that
    // are congruent modulo 8 and share one L2
    const int xcd = blockIdx.x & 7, slot_in_xcd = blockIdx.x >> 3;
    int pos = slot_in_xcd / a.G, slice = slot_in_xcd % a.G;
    if (a.pair_cus > 0) {
        // The dispatcher hands the first pair_cus slots of an XCD to distinct CUs and the next pair_cus slots
        // to the same CUs again.  A cluster takes G CUs of one such layer, so the clusters on those G CUs
        // share them with each other only and run in alternation; the CUs left over hold one more cluster.
        const int L = a.pair_cus, layers = a.pair_layers;
        const int layer = slot_in_xcd / L, cu = slot_in_xcd % L;
        const int nb = L / a.G, Lr = L - nb * a.G;
        if (cu < nb * a.G) { pos = (cu / a.G) * layers + layer; slice = cu % a.G; }
        else { const int rem = (cu - nb * a.G) + layer * Lr; pos = nb * layers + rem / a.G; slice = rem % a.G; }
    }
    const int cluster = pos * 8 + xcd;
    if (cluster >= a.replicas) return;
    const int rep = a.replica0 + cluster;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int d = a.d, C = a.C, m = a.m, mp = a.mp, S = a.S, G = a.G;
    const int Kcap = a.tr.Kcap;
    const int64_t cap = a.tr.cap;
    const int col0 = slice * SL;
    const bool async = a.variant == kAsync;
    // A tile holds whole records of mp rows; when an iteration spans several tiles, a tile is one block of 64 rows
    // of the iteration's mini-batches, all of them part of the update.
    // (read from the arguments where it is possible at all: as a compile-time constant it led the compiler to keep
    // two tiles of gathered rows alive and spill them)
    const bool chunked = CHUNKED && a.chunked != 0;
    // K-batch-async with mini-batches of more than 64 rows: a tile is one block of 64 rows of one record; the record's
    // gradient is summed over its tiles in the slot of its worker
    const int spr = (BATCH && mp > ROWS) ? (mp + ROWS - 1) / ROWS : 1;      // tiles per record
    const int mpt = (chunked || spr > 1) ? ROWS : mp;

    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    const int kc = Kcap > 32 ? KC : 32;      // places of the lists in LDS
    const Lds L = carve(smem, C, S, kc);

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
        int n_K = 0, n_nrec = 0, n_nstale = 0, n_stale = 0, n_stale_pos = KC, n_rec_word = 0;
        int q_sel = -1, q_tau = -1, q_ord = 0;   // lane l: entry l of the consume list of a later version, in flight
        int cur_sel = -1;                        // consume list of the version before the one being prepared

        // diagnostics: cycles between passing mark prof_a and the next passing of mark prof_b, summed in scalar registers
        uint32_t lp_acc = 0, lp_t0 = 0;
        const bool lprof = PROF && lw == a.prof_wave;
        auto lmark = [&](int q) {
            if constexpr (PROF) {
                if (lprof) {
                    if (16 + q == a.prof_a) lp_t0 = (uint32_t)clock64();
                    if (16 + q == a.prof_b) lp_acc += (uint32_t)clock64() - lp_t0;
                }
            }
        };

        auto issue_lists = [&](int64_t ver) {
            q_sel = -1; q_tau = -1; q_ord = 0;
            if (lane < Kcap) {
                q_sel = tr_sel[ver * Kcap + lane];
                q_tau = tr_tau[ver * Kcap + lane];
                if (!async) q_ord = tr_ord[ver * Kcap + lane];
            }
        };
        // The lists of version `ver` (in flight in q_*) become the description of its tiles.
        int h_worker = -1, h_ord = 0, h_nrec = 0, h_tiles = 1;
        // K-batch-async: the records of a version are described piecewise (version 0 has P + K - 1 of them):
        // the first `h_first` start a worker's mini-batch 0 (version 0: worker = record index; later: the worker whose
        // push triggered the update before), record h_first + j is the restart after push j of this update (lane j)
        int h_first = 0, h_trig = 0, h_trig_fresh = 0, h_nstale = 0;
        int h_rw = 0, h_ro = 0, h_rf = 0;        // lane j: worker, ordinal, consumed-by-this-update flag of restart j
        int h_csel = -1, h_ctau = -1, h_cord = 0;   // lane l: entry l of the consume list of the version
        const int rpt = spr > 1 ? 1 : ROWS / mp; // K-batch-async: whole records per tile (or one block of a record)
        auto take_lists = [&](int64_t ver, bool more) {
            const int l_sel = q_sel, l_tau = q_tau, l_ord = q_ord;
            const int K = __popcll(__ballot(l_sel >= 0));
            int nrec = async ? __popcll(__ballot(cur_sel >= 0)) : K;
            int rec_slot = async ? cur_sel : lane;
            int rec_ord = async ? 0 : l_ord;
            int fr = (!async && lane < K) ? 1 : 0;
            if (async)
                for (int l = 0; l < K; ++l)
                    if (__builtin_amdgcn_readlane(l_tau, l) == (int32_t)ver && __builtin_amdgcn_readlane(l_sel, l) == rec_slot) fr = 1;
            if constexpr (BATCH) {
                // Mini-batches that start at version ver: at ver = 0 every worker's first one, later the one of the
                // worker whose push triggered update ver - 1; then, for each of the first K - 1 pushes of update ver,
                // the next mini-batch of the pushing worker (ordinal: how many it has started at this version).
                const int Kprev = __popcll(__ballot(cur_sel >= 0));
                h_first = (ver == 0) ? a.P : 1;
                nrec = h_first + K - 1;
                h_trig = (ver == 0) ? 0 : __builtin_amdgcn_readlane(cur_sel, max(Kprev - 1, 0));
                h_rw = l_sel;
                h_ro = (l_tau == (int32_t)ver) ? l_ord + 1 : 0;
                h_rf = 0;          // is restart `lane` consumed by update ver itself?  and the trigger's mini-batch?
                h_trig_fresh = 0;
                for (int q = 0; q < K; ++q) {
                    const int cs = __builtin_amdgcn_readlane(l_sel, q), ct = __builtin_amdgcn_readlane(l_tau, q),
                              co = __builtin_amdgcn_readlane(l_ord, q);
                    if (ct == (int32_t)ver && cs == h_rw && co == h_ro) h_rf = 1;
                    if (ct == (int32_t)ver && cs == h_trig && co == 0) h_trig_fresh = 1;
                }
                h_csel = l_sel; h_ctau = l_tau; h_cord = l_ord;
            }
            n_K = K;
            // parked gradients that update ver consumes: entries whose version is older, compacted
            const bool is_stale = lane < K && l_tau != (int32_t)ver;
            const unsigned long long smask = __ballot(is_stale);
            n_nstale = __popcll(smask);
            n_stale = (async || BATCH) ? l_sel : lane;
            n_stale_pos = is_stale ? __popcll(smask & ((1ull << lane) - 1ull)) : KC;
            if (chunked) {
                // every tile is one record of 64 rows that update ver consumes itself
                n_nrec = 1;
                n_rec_word = (lane == 0) ? (1 << 16) : 0;
            } else {
                n_nrec = nrec;
                n_rec_word = (lane < nrec) ? (rec_slot | (fr << 16)) : 0;      // K-batch-async: set per tile below
            }
            h_worker = async ? cur_sel : l_sel;      // lane r: worker of record r (not K-batch-async)
            h_ord = rec_ord;
            h_nrec = nrec;
            h_tiles = chunked ? max(1, (nrec * mp + ROWS - 1) / ROWS) : 1;
            if constexpr (BATCH) {
                h_nstale = n_nstale;
                h_tiles = spr > 1 ? max(1, nrec * spr) : max(1, (nrec + rpt - 1) / rpt);
            }
            cur_sel = l_sel;
            asm volatile("" : "+v"(n_stale), "+v"(n_stale_pos), "+v"(n_rec_word), "+v"(cur_sel), "+v"(h_worker), "+v"(h_ord) : : "memory");
            if constexpr (BATCH) asm volatile("" : "+v"(h_rw), "+v"(h_ro), "+v"(h_rf), "+v"(h_csel), "+v"(h_ctau), "+v"(h_cord) : : "memory");
            if (more) issue_lists(ver + 1);
        };
        // Tile `t` of version `ver`: sample ids and labels; leaves the gathers in flight.
        auto make_tile = [&](int64_t ver, int t) {
            int rec = r_of, smp = s_of;
            if (chunked) { const int q = t * ROWS + lane; rec = q / mp; smp = q - rec * mp; }
            int worker, ordinal;
            if constexpr (BATCH) {
                // records t * rpt .. of the version; the parked part of the update comes with the first tile
                const int tr0 = spr > 1 ? t / spr : t * rpt;       // first record of the tile
                const int blk = spr > 1 ? t % spr : 0;             // which block of 64 rows of its record
                rec = (r_of < rpt) ? tr0 + r_of : 0x7FFFFFF;
                if (spr > 1) { rec = tr0; smp = ROWS * blk + lane; }
                n_nrec = spr > 1 ? 1 : min(rpt, h_nrec - t * rpt);
                n_nstale = (t == 0) ? h_nstale : 0;
                // worker, ordinal and consumed-by-this-update flag of record q
                auto describe = [&](int q, int& w, int& o, int& f) {
                    const int j = min(max(q - h_first, 0), 63);
                    const int rw = __shfl(h_rw, j, 64), ro = __shfl(h_ro, j, 64), rf = __shfl(h_rf, j, 64);
                    if (q >= h_first) { w = rw; o = ro; f = rf; }
                    else if (ver != 0) { w = h_trig; o = 0; f = h_trig_fresh; }
                    else { w = q; o = 0; f = -1; }          // version 0: looked up below
                };
                int fr;
                describe(rec, worker, ordinal, fr);
                int qw, qo, qf;
                describe(tr0 + lane, qw, qo, qf);
                if (ver == 0) {
                    // every worker's first mini-batch: consumed by update 0 if the list holds (worker, version 0, ordinal 0)
                    const int Kv = n_K;
                    int hit = 0;
                    for (int e = 0; e < Kv; ++e)
                        if (__builtin_amdgcn_readlane(h_csel, e) == qw && __builtin_amdgcn_readlane(h_ctau, e) == 0 &&
                            __builtin_amdgcn_readlane(h_cord, e) == 0) hit = 1;
                    if (qf < 0) qf = hit;
                }
                // bit 16: consumed by the update of its own version; bit 17: the record goes on in the next tile; bit 18: it
                // began in an earlier tile
                n_rec_word = (lane < n_nrec) ? (qw | (qf << 16) | ((blk + 1 < spr ? 1 : 0) << 17) | ((blk > 0 ? 1 : 0) << 18)) : 0;
            } else {
                worker = __shfl(h_worker, min(rec, 63), 64);
                ordinal = __shfl(h_ord, min(rec, 63), 64);
            }
            row_id = kNoRow;
            row_lab = 0.0f;
            if (smp < m && rec < h_nrec) {
                row_id = batch_index(a.seed, (uint32_t)rep, (uint32_t)worker, (uint32_t)ordinal, (uint32_t)ver,
                                     (uint32_t)smp, a.N);
                row_lab = (KIND == kLsq) ? reinterpret_cast<const float*>(a.y)[row_id]
                                         : __int_as_float(reinterpret_cast<const int32_t*>(a.y)[row_id]);
            }
            // The lists are consumed before the gathers are issued: the gathers are the youngest
            // vector-memory operations of this wave until the tile is published.
            asm volatile("" : "+v"(row_id) : : "memory");
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int i = 0; i < LLOADS; ++i) {
                // rows without a sample read row 0; their delta is zero
                uint32_t id = (uint32_t)__builtin_amdgcn_readlane((int)row_id, lw + 4 * i);
                id = (id == kNoRow) ? 0u : id;
                pref[i] = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(xrsrc, goff[i & 3], (int)(id * row_bytes), kStream));
            }
        };
        // flags: bit 0 last tile of its update, bit 1 first tile of its update
        auto publish = [&](int flags) {
#pragma unroll
            for (int i = 0; i < LLOADS; ++i) *reinterpret_cast<f32x4*>(my_tile + 4 * i * SL) = pref[i];
            if (lw == 0) {
                L.rowid[lane] = row_id; L.ylab[lane] = row_lab;
                if (lane == 0) { L.ctl[4] = n_K; L.ctl[5] = n_nrec; L.ctl[6] = n_nstale; L.ctl[7] = flags; }
                if (n_stale_pos < kc) L.s_stale[n_stale_pos] = n_stale;
                if (lane < kc) L.s_rec[lane] = n_rec_word;
            }
        };

        // Loader wave 0, between D and B: the column sums of the delta tile per record, i.e. the bias
        // gradient (classes 0..C-1) and the mean mini-batch loss (class 15), summed over the consume
        // list of update v like the weight gradients; then the bias step and the loss record.
        float run_tot = 0.0f;      // sums of the earlier tiles of the same update
        auto bias_and_loss = [&](int64_t v, int flags) {
            const int Kv = __builtin_amdgcn_readfirstlane(L.ctl[4]);
            const int n_rec = __builtin_amdgcn_readfirstlane(L.ctl[5]);
            const int n_st = __builtin_amdgcn_readfirstlane(L.ctl[6]);
            // lane = class + 16 * (record within a batch of four records)
            const int c = lane & 15, grp = lane >> 4;
            const int sidx = (c == 15) ? 16 : c;          // the slot record keeps the loss in word 16
            float tot = 0.0f;
            for (int i = 0; i < n_st; ++i) {
                const float was = L.small[__builtin_amdgcn_readfirstlane(L.s_stale[i]) * 17 + sidx];
                if (grp == 0) tot += was;
            }
            for (int r0 = 0; r0 < n_rec; r0 += 4) {
                const int r = r0 + grp;
                const bool have = r < n_rec;
                const float* zp = L.zbuf + (have ? r : 0) * mpt * 16 + c;
                float p0 = 0.0f, p1 = 0.0f;
                int i0 = 0;
                for (; i0 + 16 <= mpt; i0 += 16) {     // sixteen rows in flight
                    float t[16];
#pragma unroll
                    for (int i = 0; i < 16; ++i) t[i] = zp[(i0 + i) * 16];
#pragma unroll
                    for (int i = 0; i < 16; i += 2) { p0 += t[i]; p1 += t[i + 1]; }
                }
                for (; i0 < mpt; i0 += 4) {
                    float t[4];
#pragma unroll
                    for (int i = 0; i < 4; ++i) t[i] = zp[(i0 + i) * 16];
                    p0 += t[0] + t[2];
                    p1 += t[1] + t[3];
                }
                const float part = p0 + p1;
                const int word = have ? L.s_rec[r] : 0;
                if (have) {
                    if (((word >> 16) & 1) != 0) tot += part;
                    else if (((word >> 18) & 1) != 0) L.small[(word & 0xFFFF) * 17 + sidx] += part;    // a later block of its record
                    else L.small[(word & 0xFFFF) * 17 + sidx] = part;
                }
            }
            tot += __shfl_xor(tot, 16, 64);
            tot += __shfl_xor(tot, 32, 64);
            if ((flags & 2) == 0) tot += run_tot;
            run_tot = tot;
            if ((flags & 1) != 0) {
                if (KIND == kSoftmax && lane < C) L.bias[lane] -= (a.lr / (float)Kv) * tot;
                if (lane == 15 && slice == 0) a.tr.loss[(int64_t)rep * cap + v] = tot * (1.0f / (float)Kv);
                // the averaged gradient of replica 0, when the caller asked for it: bias part
                if (KIND == kSoftmax && a.agg_out != nullptr && rep == 0 && slice == 0 && lane < C)
                    a.agg_out[(int64_t)C * d + lane] = tot * (1.0f / (float)Kv);
            }
        };

        lds_barrier();                               // the compute waves have set up the control words
        if (L.ctl[0] != 0) return;
        if ((async || (BATCH && a.v0 >= 1)) && lane < Kcap) cur_sel = tr_sel[(a.v0 - 1) * Kcap + lane];   // v0 >= 1 for K-async
        issue_lists(a.v0);
        take_lists(a.v0, a.nsteps > 1);
        make_tile(a.v0, 0);
        for (int64_t step = 0; step < a.nsteps; ++step) {
            const int tiles = h_tiles;               // of update a.v0 + step
            for (int t = 0; t < tiles; ++t) {
                lmark(4);
                const int flags = (t + 1 == tiles ? 1 : 0) | (t == 0 ? 2 : 0);
                publish(flags);
                lmark(0);
                lds_barrier();                       // TU
                if (t + 1 < tiles) {
                    make_tile(a.v0 + step, t + 1);
                } else if (step + 1 < a.nsteps) {
                    take_lists(a.v0 + step + 1, step + 2 < a.nsteps);
                    make_tile(a.v0 + step + 1, 0);
                }
                lmark(1);
                lds_barrier();                       // D
                if (L.ctl[0] != 0) return;
                if (lw == 0) bias_and_loss(a.v0 + step, flags);
                lmark(2);
                lds_barrier();                       // B
                lmark(3);
            }
        }
        if constexpr (PROF) {
            if (lprof && lane == 0) a.prof[(int64_t)a.prof_base + ((int64_t)rep * G + slice) * 2 + 1] += lp_acc;
        }
        lds_barrier();                               // the compute waves' last LDS writes
        return;
    }

    // ================================= compute waves =================================
    const int64_t nw = (KIND == kLsq) ? d : (int64_t)C * d + C;
    float* params = a.params + (int64_t)rep * nw;
    float* park = a.park + ((int64_t)rep * G + slice) * S * 16 * NTC;
    float* small_g = a.park_small + ((int64_t)rep * G + slice) * S * 17;
    float* zpart = a.zpart + (int64_t)rep * 2 * G * a.maxrows * 16;
    unsigned int* arrive = a.arrive + kArriveStride * rep;   // fenced exchanges; word kArriveFast: shared-L2 exchanges
    const float inv_m = 1.0f / (float)m;
    const int nquad = (C + 3) / 4;

    // share of the parameters: classes own_cls .. own_cls+3, columns own_col .. own_col+3
    const int own_ch = 16 * wave + (lane & 15);
    const int own_col = col0 + 4 * own_ch;
    const int own_cls = 4 * (lane >> 4);
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
        L.ctl[3] = 0;
        // XCC_ID in the low byte (what the same-XCD check compares); HW_ID (CU, shader engine) above it, for diagnostics
        const int my_xcc = (int)(__builtin_amdgcn_s_getreg((3 << 11) | 20) & 0xF);
        const int hw_id = (int)__builtin_amdgcn_s_getreg((15 << 11) | 4);
        __hip_atomic_store(a.xcc_ids + (int64_t)rep * G + slice, my_xcc | (hw_id << 8), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    __syncthreads();
    if (L.ctl[0] != 0) return;

    const __amdgpu_buffer_rsrc_t zrsrc = make_rsrc(zpart, (uint32_t)(2u * G * a.maxrows * 16u * sizeof(float)));
    // shared-L2 exchange: three buffers of G x 64 x 16 words used in turn; a word is the sentinel until written
    const __amdgpu_buffer_rsrc_t ersrc = make_rsrc(a.zx + (int64_t)rep * 3 * G * 1024, (uint32_t)(3u * G * 4096u));
    constexpr uint32_t kSentinel = 0xFFFFFFFFu;
    // parked gradients of this workgroup: class own_cls + vv of slot s, 4 columns: 16 bytes at ((s*4 + vv)*NTC + tid)*16
    const __amdgpu_buffer_rsrc_t prsrc = make_rsrc(park, (uint32_t)S * 16u * NTC * 4u);
    int pk_off[4];
#pragma unroll
    for (int vv = 0; vv < 4; ++vv) pk_off[vv] = (own_cls + vv < C) ? (vv * NTC + tid) * 16 : kOutOfRange;
    // forward: rows 16 wave .. 16 wave + 15; row / class index of this lane in the MFMA operands
    const int f_row = 16 * wave + (lane & 15);
    // lanes of classes that do not exist read the last class: their logits are never used
    const int f_key = min(lane & 15, C - 1);
    // k-block s covers 16-byte chunks 4 s + lane/16 of the row; with the swizzle key split as
    // key = 4 k2 + k0 its position is 16 (s / 4) + 4 ((s % 4) ^ k2) + ((lane / 16) ^ k0): four base
    // addresses per operand, the rest is a constant offset
    const float* f_xa[4];
    const float* f_wa[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int kx = f_row & 15;
        f_xa[j] = L.tile + f_row * SL + ((4 * (j ^ (kx >> 2)) + ((lane >> 4) ^ (kx & 3))) << 2);
        f_wa[j] = L.wlds + f_key * SL + ((4 * (j ^ (f_key >> 2)) + ((lane >> 4) ^ (f_key & 3))) << 2);
    }
    // exchange: this lane's 16 bytes (4 classes of one row) inside one slice's block
    const int z_store = (f_row * 16 + 4 * (lane >> 4)) * 4;
    const int z_store_off = ((lane >> 4) < nquad) ? z_store : kOutOfRange;
    const int z_row = tid >> 2, z_qd = tid & 3;             // row / class quad of the softmax phase
    const int z_load_off = (z_qd < nquad) ? (z_row * 16 + 4 * z_qd) * 4 : kOutOfRange;
    const int slice_bytes = a.maxrows * 16 * 4;

    uint32_t n_fenced = 0, n_fast = 0;       // exchanges of each kind so far in this launch
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

    float gsum[16];          // this thread's part of sum_l g_l of the update in progress: gsum[4 vv + c]
    for (int64_t step = 0; step < a.nsteps; ++step) {
      for (bool last_tile = false; !last_tile;) {           // the tiles of update a.v0 + step
        mark(14);
        lds_barrier();                                      // TU
        mark(0);
        const bool fast = L.ctl[1] != 0;
        const int4 ctl4 = *reinterpret_cast<const int4*>(L.ctl + 4);
        const int2 st01 = *reinterpret_cast<const int2*>(L.s_stale);
        const int2 rec01 = *reinterpret_cast<const int2*>(L.s_rec);     // records 0 and 1, read ahead of their use
        const int Kv = __builtin_amdgcn_readfirstlane(ctl4.x);
        const int n_rec = __builtin_amdgcn_readfirstlane(ctl4.y);
        const int n_stale = __builtin_amdgcn_readfirstlane(ctl4.z);
        const int tile_flags = __builtin_amdgcn_readfirstlane(ctl4.w);
        last_tile = (tile_flags & 1) != 0;
        const int par = (int)(step & 1);
        // An opaque zero: addresses built from it are recomputed every step instead of being kept in
        // registers across the whole loop (they would be spilled to scratch memory).
        int opq = 0;
        asm volatile("" : "+s"(opq));

        // ---- partial logits of rows 16 wave ..: D[class][row] += W[class][k] X[row][k] over this slice;
        //      the operands of the next k-block are read from LDS before the MFMAs of this one are issued
        {
            f32x4 acc0 = {0.f, 0.f, 0.f, 0.f}, acc1 = {0.f, 0.f, 0.f, 0.f};
            f32x4 wv = *reinterpret_cast<const f32x4*>(f_wa[0]);
            f32x4 xv = *reinterpret_cast<const f32x4*>(f_xa[0]);
#pragma unroll
            for (int s = 0; s < SL / 16; ++s) {
                f32x4 wn = wv, xn = xv;
                if (s + 1 < SL / 16) {
                    wn = *reinterpret_cast<const f32x4*>(f_wa[(s + 1) & 3] + ((s + 1) >> 2) * 64);
                    xn = *reinterpret_cast<const f32x4*>(f_xa[(s + 1) & 3] + ((s + 1) >> 2) * 64);
                }
                __builtin_amdgcn_sched_barrier(0);   // keep the reads ahead of the MFMAs
                acc0 = __builtin_amdgcn_mfma_f32_16x16x4f32(wv.x, xv.x, acc0, 0, 0, 0);
                acc1 = __builtin_amdgcn_mfma_f32_16x16x4f32(wv.y, xv.y, acc1, 0, 0, 0);
                acc0 = __builtin_amdgcn_mfma_f32_16x16x4f32(wv.z, xv.z, acc0, 0, 0, 0);
                acc1 = __builtin_amdgcn_mfma_f32_16x16x4f32(wv.w, xv.w, acc1, 0, 0, 0);
                wv = wn; xv = xn;
            }
            const f32x4 out = acc0 + acc1;   // classes 4*(lane/16)+0..3 of row f_row
            mark(8);
            // 16-byte buffer stores carry their whole offset in the vector register: with the scalar offset in a
            // register, such a store has lost data here when the next instruction rewrote its source registers
            if (fast) {
                // the re-arming stores of the last exchange are in the L2 before this exchange's data can be seen
                asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
                u32x4 ob = __builtin_bit_cast(u32x4, out);
#pragma unroll
                for (int c = 0; c < 4; ++c) ob[c] = (ob[c] == kSentinel) ? 0x7FC00000u : ob[c];   // a NaN that is not the sentinel
                __builtin_amdgcn_raw_buffer_store_b128(ob, ersrc, z_store_off + (int)((n_fast % 3u) * G + slice) * 4096, 0, 0);
            } else {
                __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, out), zrsrc,
                                                       z_store_off + (par * G + slice) * slice_bytes, 0, 0);
            }
        }
        // ---- the part of update v that earlier steps parked: the first two such gradients are fetched
        //      while the exchange stores are on their way
        auto park_load = [&](int slot, f32x4 (&pv)[4]) {
            // classes that do not exist are out of range and read as zero
            const int soff = __builtin_amdgcn_readfirstlane(slot) * 16 * NTC * 4;
#pragma unroll
            for (int vv = 0; vv < 4; ++vv)
                pv[vv] = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(prsrc, pk_off[vv], soff, 0));
        };
        f32x4 pva[4], pvb[4];
#pragma unroll
        for (int vv = 0; vv < 4; ++vv) { pva[vv] = f32x4{0.f, 0.f, 0.f, 0.f}; pvb[vv] = f32x4{0.f, 0.f, 0.f, 0.f}; }
        if (n_stale > 0) park_load(st01.x, pva);
        if (n_stale > 1) park_load(st01.y, pvb);
        mark(9);
        // ---- arrival: this wave's stores are in the L2 (shared-L2 mode) or released to the device
        // ---- arrival.  Shared-L2 mode needs none: the readers poll the data words themselves.  Otherwise the
        //      wave's stores are released to the device and counted.
        if (!fast && lane == 0) __hip_atomic_fetch_add(arrive, 1u, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
        mark(1);

        if ((tile_flags & 2) != 0) {
#pragma unroll
            for (int e = 0; e < 16; ++e) gsum[e] = pva[e >> 2][e & 3] + pvb[e >> 2][e & 3];
        }
        for (int i = 2; i < n_stale; ++i) {     // further parked gradients (K > 2)
            park_load(L.s_stale[i], pva);
#pragma unroll
            for (int e = 0; e < 16; ++e) gsum[e] += pva[e >> 2][e & 3];
        }
        mark(2);

        // ---- wave 0 polls the counter in the L2 (all 4 G compute waves of the cluster have arrived) and
        //      relays the result through an LDS word, which the other waves poll
        if (!fast) {
            const uint32_t target = (n_fenced + 1u) * (uint32_t)(4 * G);
            const int want = (int)(n_fenced + 1u);
            if (wave == 0) {
                uint32_t spins = 0;
                for (;;) {
                    uint32_t got = __hip_atomic_load(arrive, __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_AGENT);
                    asm volatile("" ::: "memory");   // the load is repeated every turn
                    got = (uint32_t)__builtin_amdgcn_readfirstlane((int)got);
                    if ((int32_t)(got - target) >= 0) break;
                    __builtin_amdgcn_s_sleep(8);
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
                if (lane == 0) __hip_atomic_store(&L.ctl[3], want, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
            } else {
                while (__builtin_amdgcn_readfirstlane(__hip_atomic_load(&L.ctl[3], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP)) < want)
                    __builtin_amdgcn_s_sleep(1);
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
            }
            if (a.allow_fast && tid == 0) {
                // first exchange of the launch: do all slices of this cluster share an XCD (one L2)?
                const int32_t* ids = a.xcc_ids + (int64_t)rep * G;
                int same = 1;
                const int mine = __hip_atomic_load(ids + slice, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) & 0xFF;
                for (int g = 0; g < G; ++g)
                    if ((__hip_atomic_load(ids + g, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) & 0xFF) != mine) same = 0;
                L.ctl[2] = same;
            }
            ++n_fenced;
        }
        mark(3);

        // ---- full logits of row z_row (sum of the G partials in slice order), then residual / softmax
        {
            f32x4 zz = {0.f, 0.f, 0.f, 0.f};
            if (fast) {
                // Poll the partial logits themselves: a batch of slices has arrived for this wave when none of
                // the words its lanes need is the sentinel, i.e. when the largest word read is not all ones.
                // A round re-reads the whole batch; the slices are added in order once it is complete.
                const int xbase = (int)((n_fast % 3u) * G) * 4096;
                uint32_t spins = 0;
                for (int g0 = 0; g0 < G; g0 += 12) {
                    u32x4 part[12];
                    for (;;) {
#pragma unroll
                        for (int i = 0; i < 12; ++i)
                            part[i] = __builtin_amdgcn_raw_buffer_load_b128(ersrc, z_load_off, xbase + min(g0 + i, G - 1) * 4096, kAgentLoad);
                        asm volatile("" ::: "memory");   // the loads are repeated every round
                        uint32_t top = 0u;
#pragma unroll
                        for (int i = 0; i < 12; ++i) top = max(max(top, max(part[i].x, part[i].y)), max(part[i].z, part[i].w));
                        if (__ballot(top == kSentinel) == 0ull) break;
                        // with another workgroup on this CU, re-reading at once would slow its memory operations
                        if (a.shared_cus) __builtin_amdgcn_s_sleep(32); else __builtin_amdgcn_s_sleep(2);
                        ++spins;
                        if (spins > a.spin_limit ||
                            ((spins & 63u) == 0 && __hip_atomic_load(a.abort_flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0)) {
                            if (lane == 0) {
                                __hip_atomic_store(a.abort_flag, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                                L.ctl[0] = 1;
                            }
                            break;         // give up: the launch is aborted at the next barrier
                        }
                    }
                    if (g0 + 12 <= G) {
#pragma unroll
                        for (int i = 0; i < 12; ++i) zz += __builtin_bit_cast(f32x4, part[i]);
                    } else {
                        // the last, partial batch re-read its final slice in the unused places
#pragma unroll
                        for (int i = 0; i < 12; ++i)
                            if (g0 + i < G) zz += __builtin_bit_cast(f32x4, part[i]);
                    }
                }
                // Every slice of this exchange has been written, so every workgroup has finished reading the one
                // before it: this wave's rows of that buffer are re-armed for their next use.
                uint32_t sv = kSentinel;
                asm volatile("" : "+v"(sv));      // built here, not kept in registers across the loop
                const u32x4 arm = {sv, sv, sv, sv};
                __builtin_amdgcn_raw_buffer_store_b128(arm, ersrc, z_store_off + (int)(((n_fast + 2u) % 3u) * G + slice) * 4096, 0, 0);
                ++n_fast;
            } else {
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
            }
            mark(4);
            const bool ok = L.rowid[z_row] != kNoRow;
            f32x4 dl = {0.f, 0.f, 0.f, 0.f};
            float loss = 0.0f;
            if constexpr (KIND == kLsq) {
                const float z0 = quad_lane0(zz.x);
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
                lt_ += quad_xor1(lt_);
                lt_ += quad_xor2(lt_);
                loss = ok ? lt_ + logf(den) : 0.0f;
                const float inv = 1.0f / den;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const float pr = dl[e] * inv - ((4 * z_qd + e == lab) ? 1.0f : 0.0f);
                    dl[e] = (ok && 4 * z_qd + e < C) ? pr * inv_m : 0.0f;
                }
            }
            // the unused class 15 carries the row loss: the column sums of the delta tile (taken by a
            // loader wave) then hold the bias gradient and the loss sum
            if (z_qd == 3) dl.w = loss * inv_m;
            *reinterpret_cast<f32x4*>(L.zbuf + z_row * 16 + 4 * z_qd) = dl;
        }
        mark(13);
        lds_barrier();                                      // D
        if (L.ctl[0] != 0) return;   // uniform: every thread reads the same LDS word
        mark(5);

        // ---- per record: the gradient slice delta^T X, in groups of four k-steps (16 rows); the operands
        //      of the next group are read from LDS before the MFMAs of this one are issued
        {
            const int kpr = mpt >> 2;              // k-steps per record
            const int ngrp = (kpr + 3) >> 2;       // groups per record
            const int b_lo = lane >> 4, b_cls = lane & 15;
            auto load_group = [&](int r, int g, float (&dv)[4], f32x4 (&xv)[4]) {
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int k = 4 * g + u;
                    const int row = r * mpt + 4 * min(k, kpr - 1) + b_lo;
                    dv[u] = L.zbuf[row * 16 + b_cls];   // k-steps past the record are masked when they are used
                    xv[u] = *reinterpret_cast<const f32x4*>(L.tile + row * SL + ((own_ch ^ (row & 15)) << 2));
                }
            };
            f32x4 acc[4];
#pragma unroll
            for (int c = 0; c < 4; ++c) acc[c] = f32x4{0.f, 0.f, 0.f, 0.f};
            auto contract = [&](int g, const float (&dv)[4], const f32x4 (&xv)[4]) {
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const float da = (4 * g + u < kpr) ? dv[u] : 0.0f;   // k-steps past the record contribute nothing
                    acc[0] = __builtin_amdgcn_mfma_f32_16x16x4f32(da, xv[u].x, acc[0], 0, 0, 0);
                    acc[1] = __builtin_amdgcn_mfma_f32_16x16x4f32(da, xv[u].y, acc[1], 0, 0, 0);
                    acc[2] = __builtin_amdgcn_mfma_f32_16x16x4f32(da, xv[u].z, acc[2], 0, 0, 0);
                    acc[3] = __builtin_amdgcn_mfma_f32_16x16x4f32(da, xv[u].w, acc[3], 0, 0, 0);
                }
            };
            // record r is complete: add it to the aggregate of update v, or park it in its slot
            auto finish = [&](int r) {
                if constexpr (PROF) { asm volatile("" : "+v"(acc[0]), "+v"(acc[1]), "+v"(acc[2]), "+v"(acc[3])); mark(11); }
                const int word = __builtin_amdgcn_readfirstlane(r == 0 ? rec01.x : (r == 1 ? rec01.y : L.s_rec[r]));
                bool to_sum = ((word >> 16) & 1) != 0;
                if constexpr (BATCH) {
                    // A record of several tiles is summed in its worker's slot (free by now: what it held was consumed
                    // by an earlier update or with the first tile of this one): later blocks add what is there, and
                    // only the last one goes to the aggregate if the update consumes the record itself.
                    if (((word >> 18) & 1) != 0) {
                        const int soff = (word & 0xFFFF) * 16 * NTC * 4;
#pragma unroll
                        for (int vv = 0; vv < 4; ++vv) {
                            const f32x4 pv = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(prsrc, pk_off[vv], soff, 0));
#pragma unroll
                            for (int c = 0; c < 4; ++c) acc[c][vv] += pv[c];
                        }
                    }
                    if (((word >> 17) & 1) != 0) to_sum = false;
                }
                if (to_sum) {
#pragma unroll
                    for (int vv = 0; vv < 4; ++vv)
#pragma unroll
                        for (int c = 0; c < 4; ++c) gsum[vv * 4 + c] += acc[c][vv];
                } else {
                    const int soff = (word & 0xFFFF) * 16 * NTC * 4;
#pragma unroll
                    for (int vv = 0; vv < 4; ++vv) {
                        const f32x4 gv = {acc[0][vv], acc[1][vv], acc[2][vv], acc[3][vv]};
                        __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, gv), prsrc, pk_off[vv] + soff, 0, 0);
                    }
                }
#pragma unroll
                for (int c = 0; c < 4; ++c) acc[c] = f32x4{0.f, 0.f, 0.f, 0.f};
                mark(12);
            };
            if constexpr (WHOLE) {
                // Whole groups of 16 rows only, at most four of them: the tile and delta addresses are four base
                // addresses (one per k-step of a group, carrying the swizzle key of its rows) plus constants, and
                // two register sets take turns, one being read from LDS while the MFMAs of the other are issued.
                int olo = b_lo, och = own_ch, ocl = b_cls;
                asm volatile("" : "+v"(olo), "+v"(och), "+v"(ocl));   // rebuilt every step, not kept across the loop
                const float* bx[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) bx[u] = L.tile + (4 * u + olo) * SL + ((och ^ (4 * u + olo)) << 2);
                const float* bz = L.zbuf + olo * 16 + ocl;
                // half-group h: k-steps 2 h and 2 h + 1, i.e. rows 8 h .. 8 h + 7
                auto fetch = [&](int h, float (&dv)[2], f32x4 (&xv)[2]) {
#pragma unroll
                    for (int u = 0; u < 2; ++u) {
                        dv[u] = bz[(8 * h + 4 * u) * 16];
                        xv[u] = *reinterpret_cast<const f32x4*>(bx[2 * (h & 1) + u] + 16 * (h >> 1) * SL);
                    }
                };
                auto mac = [&](bool first, const float (&dv)[2], const f32x4 (&xv)[2]) {
#pragma unroll
                    for (int u = 0; u < 2; ++u) {
#pragma unroll
                        for (int c = 0; c < 4; ++c) {
                            const f32x4 init = (first && u == 0) ? f32x4{0.f, 0.f, 0.f, 0.f} : acc[c];
                            acc[c] = __builtin_amdgcn_mfma_f32_16x16x4f32(dv[u], xv[u][c], init, 0, 0, 0);
                        }
                    }
                };
                auto done = [&](int r) {
                    if constexpr (PROF) { asm volatile("" : "+v"(acc[0]), "+v"(acc[1]), "+v"(acc[2]), "+v"(acc[3])); mark(11); }
                    const int word = __builtin_amdgcn_readfirstlane(r == 0 ? rec01.x : rec01.y);
                    if (((word >> 16) & 1) != 0) {
#pragma unroll
                        for (int vv = 0; vv < 4; ++vv)
#pragma unroll
                            for (int c = 0; c < 4; ++c) gsum[vv * 4 + c] += acc[c][vv];
                    } else {
                        const int soff = (word & 0xFFFF) * 16 * NTC * 4;
#pragma unroll
                        for (int vv = 0; vv < 4; ++vv) {
                            const f32x4 gv = {acc[0][vv], acc[1][vv], acc[2][vv], acc[3][vv]};
                            __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, gv), prsrc, pk_off[vv] + soff, 0, 0);
                        }
                    }
                    mark(12);
                };
                float da[2], db[2];
                f32x4 xa[2], xb[2];
                const int H = n_rec * (mpt >> 3);         // half-groups in the tile: 0, 4 or 8
                if (H > 0) {
                    fetch(0, da, xa);
                    fetch(1, db, xb);
                    __builtin_amdgcn_sched_barrier(0);
                    mac(true, da, xa);
                    fetch(2, da, xa);
                    __builtin_amdgcn_sched_barrier(0);
                    mac(false, db, xb);
                    fetch(3, db, xb);
                    __builtin_amdgcn_sched_barrier(0);
                    mac(false, da, xa);
                    if (H > 4) fetch(4, da, xa);
                    __builtin_amdgcn_sched_barrier(0);
                    mac(false, db, xb);
                    if (H > 4) {
                        const bool two = mpt == 32;         // the second record starts with half-group 4
                        if (two) done(0);
                        fetch(5, db, xb);
                        __builtin_amdgcn_sched_barrier(0);
                        if (two) mac(true, da, xa); else mac(false, da, xa);
                        fetch(6, da, xa);
                        __builtin_amdgcn_sched_barrier(0);
                        mac(false, db, xb);
                        fetch(7, db, xb);
                        __builtin_amdgcn_sched_barrier(0);
                        mac(false, da, xa);
                        __builtin_amdgcn_sched_barrier(0);
                        mac(false, db, xb);
                        done(two ? 1 : 0);
                    } else {
                        done(0);
                    }
                }
            } else {
                // the operands of the next group are read into a second register set before the MFMAs of this one
                float dv[4];
                f32x4 xv[4];
                int r = opq, g = 0;
                if (n_rec > 0) load_group(r, 0, dv, xv);
                while (r < n_rec) {
                    int rn = r, gn = g + 1;
                    if (gn == ngrp) { gn = 0; rn = r + 1; }
                    float dn[4];
                    f32x4 xn[4];
    #pragma unroll
                    for (int u = 0; u < 4; ++u) { dn[u] = dv[u]; xn[u] = xv[u]; }
                    if (rn < n_rec) load_group(rn, gn, dn, xn);
                    __builtin_amdgcn_sched_barrier(0);   // keep the reads ahead of the MFMAs
                    contract(g, dv, xv);
                    if (rn != r) finish(r);
    #pragma unroll
                    for (int u = 0; u < 4; ++u) { dv[u] = dn[u]; xv[u] = xn[u]; }
                    r = rn; g = gn;
                }
            }
        }
        mark(6);
        lds_barrier();                                      // B: the loader waves may rewrite the tile and the lists
        // ---- update v: each compute thread owns its weights; nobody reads them before TU
        if (last_tile) {
            const float scale = a.lr / (float)Kv;
            int och = own_ch, ocl = own_cls;
            asm volatile("" : "+v"(och), "+v"(ocl));   // the four addresses below are rebuilt here, not kept across the loop
#pragma unroll
            for (int vv = 0; vv < 4; ++vv) {
                const int cls = ocl + vv;
                if (cls < C) {
                    f32x4* wp = reinterpret_cast<f32x4*>(L.wlds + cls * SL + ((och ^ cls) << 2));
                    f32x4 w = *wp;
#pragma unroll
                    for (int c = 0; c < 4; ++c) w[c] -= scale * gsum[vv * 4 + c];
                    *wp = w;
                }
            }
            if (a.agg_out != nullptr && rep == 0) {
                // the averaged gradient of replica 0, when the caller asked for it
                const float invK = 1.0f / (float)Kv;
#pragma unroll
                for (int vv = 0; vv < 4; ++vv) {
                    const int cls = own_cls + vv;
                    if (cls < C)
#pragma unroll
                        for (int c = 0; c < 4; ++c)
                            if (own_col + c < d) a.agg_out[(int64_t)cls * d + own_col + c] = gsum[vv * 4 + c] * invK;
                }
            }
        }
        if (tid == 0 && L.ctl[2] != 0) L.ctl[1] = 1;   // later exchanges of this launch use the shared L2
        mark(7);
      }
    }
    if constexpr (PROF) {
        if (profiling && lane == 0) a.prof[(int64_t)a.prof_base + ((int64_t)rep * G + slice) * 2] += p_acc;
    }
    lds_barrier();

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

template <int KIND, bool PROF, bool WHOLE, bool CHUNKED, bool BATCH>
hipError_t launch_w(const LinArgs& a, size_t lds, hipStream_t s) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(linear_tile_kernel<KIND, PROF, WHOLE, CHUNKED, BATCH>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    const int groups = (a.replicas + 7) / 8;
    const int blocks = a.pair_cus > 0 ? 8 * a.pair_cus * a.pair_layers : groups * 8 * a.G;
    hipLaunchKernelGGL((linear_tile_kernel<KIND, PROF, WHOLE, CHUNKED, BATCH>), dim3(blocks), dim3(512), lds, s, a);
    return hipGetLastError();
}

// WHOLE: every record is a whole number of 32-row blocks, so the gradient contraction is fully unrolled;
// CHUNKED: an iteration spans several tiles; BATCH: K-batch-async record lists
template <int KIND, bool PROF>
hipError_t launch_k(const LinArgs& a, size_t lds, hipStream_t s) {
    if (a.chunked) return launch_w<KIND, PROF, true, true, false>(a, lds, s);      // tiles of one 64-row record
    const bool whole = a.mp == 32 || a.mp == 64;
    if (a.variant == kBatchAsync)        // (no phase profile for this variant)
        return whole ? launch_w<KIND, false, true, false, true>(a, lds, s) : launch_w<KIND, false, false, false, true>(a, lds, s);
    return whole ? launch_w<KIND, PROF, true, false, false>(a, lds, s) : launch_w<KIND, PROF, false, false, false>(a, lds, s);
}

}  // namespace

size_t linear_tile_lds_bytes(int C, int S, int Kcap) {
    const size_t words = (size_t)ROWS * SL + (size_t)C * SL + ROWS * 16 + 2 * ROWS + 16 + 8 + 2 * (Kcap > 32 ? 64 : 32) + (size_t)S * 17;
    return sizeof(float) * words;
}

bool linear_tile_supports(const LinArgs& a, int max_records) {
    if (a.C > 15 || (a.d % 4) != 0 || a.tr.Kcap > KC || max_records > KC) return false;
    if (a.mp * max_records > ROWS && !a.chunked && a.variant != kBatchAsync) return false;
    if (a.chunked && a.variant == kAsync) return false;
    if ((uint64_t)a.N * (uint64_t)a.d * 4u >= (1ull << 32)) return false;   // one buffer descriptor spans the sample matrix
    if (a.variant == kBatchAsync) {
        // whole records per tile, or tiles of one record; the consume list and the restarts of an update sit in one lane each
        return linear_tile_lds_bytes(a.C, a.S, a.tr.Kcap) <= 160 * 1024;
    }
    if (a.variant == kAsync && a.v0 < 1) return false;    // step 0 of K-async starts all P workers
    return linear_tile_lds_bytes(a.C, a.S, a.tr.Kcap) <= 160 * 1024;
}

int linear_tile_resident_groups(size_t lds_bytes) {
    int dev = 0, per_cu = 0;
    hipDeviceProp_t prop;
    if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess) return 0;
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(linear_tile_kernel<kSoftmax, false, false, false, false>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes) != hipSuccess) return 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, linear_tile_kernel<kSoftmax, false, false, false, false>, 512, lds_bytes) != hipSuccess) return 0;
    return per_cu * prop.multiProcessorCount;
}

hipError_t launch_linear_tile(const LinArgs& a, hipStream_t s) {
    const size_t lds = linear_tile_lds_bytes(a.C, a.S, a.tr.Kcap);
    const bool prof = a.prof != nullptr;
    if (a.kind == kLsq) return prof ? launch_k<kLsq, true>(a, lds, s) : launch_k<kLsq, false>(a, lds, s);
    return prof ? launch_k<kSoftmax, true>(a, lds, s) : launch_k<kSoftmax, false>(a, lds, s);
}

}  // namespace ssgd
