// Two-layer ReLU network with a softmax output (the AdaSync experiment's model
// class, Sec. 6 / Algorithm 1 runs K-async SGD with a changing K): per-worker
// mini-batch gradients at possibly stale parameters, the K-gradient aggregate and
// the parameter-server update (Sec. 2.2, Eq. (3)).
//
// A worker's gradient is linear in two small factors, so what is kept per worker
// from the moment it starts (at the parameters it read) until an update consumes
// it is: its mini-batch rows in bf16, in both orientations; delta1 = back-propagated
// error of the hidden layer, scaled by 1/m and rounded to bf16, transposed; and
// the small second-layer gradients.  The first-layer gradient of an update,
//     sum over the K consumed workers of  delta1_l^T X_l    (hidden x d),
// is then one bf16 MFMA contraction over K*m rows whose epilogue applies it to the
// fp32 master weights and refreshes their bf16 copy; no first-layer gradient is ever
// stored.  Per update v:
//   gather    rows of the workers that start at version v -> bf16 (row-major and transposed)
//   forward   Z1 = X W1^T + b1 on the MFMA units (bf16 in, fp32 accumulate), H = relu(Z1) in fp32
//   layer 2   Z2 = H W2^T + b2, softmax, delta2, loss, delta1 = (W2^T delta2) * [H > 0] in fp32
//   consume   W1 -= lr/K * sum_l delta1_l^T X_l (MFMA), then b1, W2, b2 and the loss record
#include "mlp.hpp"

#include <hip/hip_ext.h>

#include <algorithm>
#include <atomic>
#include <thread>
#include <cmath>
#include <cstring>
#include <type_traits>
#include <vector>

namespace ssgd {
namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef unsigned short u16x8 __attribute__((ext_vector_type(8)));
typedef float f32x8 __attribute__((ext_vector_type(8)));

constexpr int MP = 64;         // rows kept per worker (m <= 64; the rest is zero)
constexpr int KT = 64;         // contraction depth per stage
constexpr int LDT = KT + 8;    // padded LDS row (bf16 elements): 144 bytes, keeps 16-byte reads conflict-poor
constexpr int kSmallRec = 32;  // most records per update that take the few-record path

// round to nearest even, as a 16-bit pattern; infinities and NaNs are truncated
__device__ __forceinline__ unsigned short bf16_bits(float x) {
    uint32_t b = __float_as_uint(x);
    if ((b & 0x7F800000u) != 0x7F800000u) b += 0x7FFFu + ((b >> 16) & 1u);
    return (unsigned short)(b >> 16);
}
__device__ __forceinline__ float bf16_round(float x) { return __uint_as_float((uint32_t)bf16_bits(x) << 16); }

struct MlpArgs {
    int32_t d, H, C, P, m, variant, Kcap;
    const float* X;
    const int32_t* y;
    uint32_t N;
    uint64_t seed;
    uint32_t rep;              // replica: a field of the counters of its delays and sample ids
    Trace tr;                  // this replica's rows
    int64_t v;
    int32_t nrec, Kv;
    float lr;
    float* params;             // W1[H][d], b1[H], W2[C][H], b2[C]
    unsigned short* w1r;       // bf16 copy of W1
    float* w2r;                // W2 rounded to bf16, kept as fp32
    const unsigned short* Xb;  // [N + 1][d] the sample matrix rounded to bf16 (taken when the context is made); row N is zero
    // The lists of the update when the host has them at hand and they are short: a kernel that finds them in its
    // arguments is spared a first load that everything else would wait for.
    int32_t n_cons_inline;     // > 0: cons_inline holds the slots of the Kv consumed gradients (K-async)
    int32_t n_rec_inline;      // > 0: rec_inline holds the workers of the nrec mini-batches that start (K-async)
    int16_t cons_inline[32];
    int16_t rec_inline[32];
    float* b1r;                // nullable: a copy of b1 (read by the layer-2 kernel, written by the small update) ...
    float* b2r;                // ... and of b2, when updates overlap and every version of the parameters has copies of its own
    unsigned short* xb;        // [S][MP][d]   bf16 rows of the slot's mini-batch
    unsigned short* xbt;       // [S][d][MP]   the same, transposed
    float* hbuf;               // [S][MP][H]   hidden activations
    unsigned short* d1t;       // [S][H][MP]   delta1 / m in bf16, transposed
    // The second-layer gradients and the loss have room for one record per quarter of the mini-batch (rows 16 q ..
    // 16 q + 15).  The few-record path fills all four (its workgroups take a quarter each and need not meet) and sets the
    // slot's flag; the other path adds the quarters itself, fills the first and clears the flag.  Whoever consumes a slot
    // adds what the flag says, in order.
    float* gb1;                // [S][4][H]    sum over the quarter of delta1
    float* gw2;                // [S][4][C][H] sum of delta2 (x) h
    float* gb2;                // [S][4][16]   sum of delta2
    float* d2;                 // [S][MP][16]  delta2 of every row
    float* loss;               // [S][4]       sum of the sample losses
    int32_t* quartered;        // [S]          1: four quarter records, 0: one record in the first quarter
    int32_t* ylab;             // [S][MP]      labels (-1: no sample)
    float* agg_out;            // nullable
    float* dw_part;            // [nsplit][H][d] partial first-layer gradient sums when the slots are split over workgroups;
                               // also [fsplit][nrec][MP][H] partial hidden-layer sums of the few-record forward pass
    int32_t nsplit;
    int32_t fsplit;            // shares of the depth d in the forward contraction of few records
    int64_t eval_base;         // >= 0: objective evaluation; record r holds data rows eval_base + 64 r .. + 63 in slot r
    int32_t* plan;             // K-batch-async: slot bookkeeping and the lists of the current update (layout: PlanView)
    int32_t S;                 // slots
};

// K-batch-async keeps P mini-batches in flight and consumes up to K per update, some of them started during the
// same update by a worker whose older mini-batch that update also consumes: slots are handed out from a free list,
// one per started mini-batch, and return to it at the start of the next update's plan.
struct PlanView {
    int32_t* meta;         // [0] free slots, [1] slots to free at the next plan, [2] set if the free list ran dry
    int32_t* wslot;        // [P]         slot of the worker's mini-batch in flight
    int32_t* freel;        // [S]         stack of free slots
    int32_t* pending;      // [Kcap]      slots consumed by the last planned update
    int32_t* rec_worker;   // [S]         mini-batches that start at the planned version, in event order
    int32_t* rec_ord;      // [S]
    int32_t* rec_slot;     // [S]
    int32_t* cons_slot;    // [Kcap]      slots of the K gradients of the update, in arrival order
    __host__ __device__ PlanView(int32_t* p, int P, int S, int Kcap) {
        meta = p; wslot = meta + 4; freel = wslot + P; pending = freel + S; rec_worker = pending + Kcap;
        rec_ord = rec_worker + S; rec_slot = rec_ord + S; cons_slot = rec_slot + S;
    }
    static size_t words(int P, int S, int Kcap) { return 4 + (size_t)P + 4 * (size_t)S + 2 * (size_t)Kcap; }
};

// worker and mini-batch ordinal of record r of the compute list of version v, and its slot
__device__ __forceinline__ void record_of(const MlpArgs& a, int r, int& worker, int& ordinal, int& slot) {
    if (a.eval_base >= 0) {
        worker = 0; ordinal = 0; slot = r;
    } else if (a.variant == kBatchAsync) {
        const PlanView pl(a.plan, a.P, a.S, a.Kcap);
        worker = pl.rec_worker[r]; ordinal = pl.rec_ord[r]; slot = pl.rec_slot[r];
    } else if (a.variant == kAsync) {
        worker = a.n_rec_inline > 0 ? (int)a.rec_inline[r] : ((a.v == 0) ? r : a.tr.sel[(a.v - 1) * a.tr.Kcap + r]);
        ordinal = 0;
        slot = worker;
    } else {
        worker = a.tr.sel[a.v * a.tr.Kcap + r];
        ordinal = a.tr.ord[a.v * a.tr.Kcap + r];
        slot = r;
    }
}
__device__ __forceinline__ int consumed_slot(const MlpArgs& a, int l) {
    if (a.eval_base >= 0) return l;       // evaluation over the data set: every record of the block
    if (a.variant == kBatchAsync) return PlanView(a.plan, a.P, a.S, a.Kcap).cons_slot[l];
    if (a.n_cons_inline > 0) return (int)a.cons_inline[l];
    return a.variant == kAsync ? a.tr.sel[a.v * a.tr.Kcap + l] : l;
}

// ---- K-batch-async: the lists of update v from its trace row (Sec. 2.2: the K earliest mini-batches, whoever
// computed them).  Mini-batches that start at version v: at v = 0 every worker's first one, later the one of the
// worker whose push triggered update v - 1; then, for each of the first K - 1 pushes of update v, the next mini-batch
// of the pushing worker (ordinal: how many it has started at this version).  Sequential, a few dozen entries.
__global__ void mlp_batch_plan_kernel(MlpArgs a) {
    if (threadIdx.x != 0 || blockIdx.x != 0) return;
    const PlanView pl(a.plan, a.P, a.S, a.Kcap);
    int nfree = pl.meta[0];
    const int npend = pl.meta[1];
    for (int i = 0; i < npend; ++i) pl.freel[nfree++] = pl.pending[i];
    const int64_t v = a.v;
    const int Kc = a.tr.Kcap, K = a.Kv;
    int nrec = 0;
    bool dry = false;
    auto start = [&](int worker, int ordinal) {
        if (nfree <= 0 || nrec >= a.S) { dry = true; return; }
        const int slot = pl.freel[--nfree];
        pl.wslot[worker] = slot;
        pl.rec_worker[nrec] = worker; pl.rec_ord[nrec] = ordinal; pl.rec_slot[nrec] = slot;
        ++nrec;
    };
    if (v == 0) {
        for (int w = 0; w < a.P; ++w) start(w, 0);
    } else {
        const int Kprev = a.tr.K[v - 1];
        start(a.tr.sel[(v - 1) * Kc + Kprev - 1], 0);
    }
    for (int l = 0; l < K; ++l) {
        const int w = a.tr.sel[v * Kc + l];
        const int slot = pl.wslot[w];
        pl.cons_slot[l] = slot;
        pl.pending[l] = slot;
        if (l + 1 < K) start(w, a.tr.tau[v * Kc + l] == (int32_t)v ? a.tr.ord[v * Kc + l] + 1 : 0);
    }
    pl.meta[0] = nfree;
    pl.meta[1] = K;
    if (dry) pl.meta[2] = 1;
}

// ---- gather: one workgroup per (record, block of 128 columns) ---------------------------------
__global__ __launch_bounds__(256) void mlp_gather_kernel(MlpArgs a) {
    __shared__ unsigned short tr_tile[128][MP + 2];
    __shared__ uint32_t ids[MP];
    const int r = blockIdx.x, cb = blockIdx.y, tid = threadIdx.x;
    int worker, ordinal, slot;
    record_of(a, r, worker, ordinal, slot);
    if (tid < MP) {
        uint32_t id = 0xFFFFFFFFu;
        if (a.eval_base >= 0) {
            const int64_t row = a.eval_base + (int64_t)r * MP + tid;
            if (row < (int64_t)a.N) id = (uint32_t)row;
        } else if (tid < a.m) {
            id = batch_index(a.seed, a.rep, (uint32_t)worker, (uint32_t)ordinal, (uint32_t)a.v, (uint32_t)tid, a.N);
        }
        ids[tid] = id;
        if (cb == 0) a.ylab[slot * MP + tid] = (id == 0xFFFFFFFFu) ? -1 : a.y[id];
    }
    __syncthreads();
    // 64 rows x 128 columns: thread -> (row = tid / 4 + 64 * pass?, ...): 32 float4 per row, 8 rows per pass
    const int c4 = tid & 31, r0 = tid >> 5;
    for (int s = r0; s < MP; s += 8) {
        const uint32_t id = ids[s];
        f32x4 v = {0.f, 0.f, 0.f, 0.f};
        if (id != 0xFFFFFFFFu) v = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(a.X + (int64_t)id * a.d + cb * 128 + 4 * c4));
        unsigned short b[4] = {bf16_bits(v.x), bf16_bits(v.y), bf16_bits(v.z), bf16_bits(v.w)};
        unsigned short* dst = a.xb + ((int64_t)slot * MP + s) * a.d + cb * 128 + 4 * c4;
        *reinterpret_cast<uint2*>(dst) = make_uint2((uint32_t)b[0] | ((uint32_t)b[1] << 16), (uint32_t)b[2] | ((uint32_t)b[3] << 16));
#pragma unroll
        for (int q = 0; q < 4; ++q) tr_tile[4 * c4 + q][s] = b[q];
    }
    __syncthreads();
    if (a.xbt == nullptr) return;       // objective evaluation: no gradient contraction follows
    // transposed copy: column c of the block, 64 samples = 128 bytes; 8 threads per column, 16 bytes each
    for (int q = tid; q < 128 * 8; q += 256) {
        const int c = q >> 3, part = q & 7;
        u16x8 v;
#pragma unroll
        for (int e = 0; e < 8; ++e) v[e] = tr_tile[c][8 * part + e];
        *reinterpret_cast<u16x8*>(a.xbt + ((int64_t)slot * a.d + cb * 128 + c) * MP + 8 * part) = v;
    }
}

template <int G>
__device__ __forceinline__ void small_update_body(const MlpArgs& a, int block, int nblocks);

// ---- contraction: C[M x N] = sum over stages of A_stage[M x 64] B_stage[N x 64]^T, bf16 MFMA ----
// FWD: rows = (record, sample) of the compute list, columns = hidden units, depth = d.
// BWD: rows = hidden units, columns = input features, depth = 64 samples of every consumed slot.
// BT x BT output tile per workgroup (128: four waves of 64 x 64; 64: four waves of 32 x 32, for launches
// that would otherwise leave most CUs idle).
// SPLIT (gradient contraction only): blockIdx.z takes a share of the consumed slots and leaves its partial sum in
// dw_part; mlp_w1_update_kernel adds the shares in order and applies the update.
template <bool FWD, int BT, bool SPLIT = false>
__global__ __launch_bounds__(256, 2) void mlp_contract_kernel(MlpArgs a) {
    constexpr int WT = BT / 2;          // rows and columns per wave
    constexpr int NF = WT / 32;         // 32 x 32 MFMA tiles per wave and dimension
    constexpr int LP = BT / 32;         // 16-byte loads per thread, operand and stage
    extern __shared__ __attribute__((aligned(16))) unsigned short lds[];
    unsigned short* As = lds;                       // [2][BT][LDT]
    unsigned short* Bs = lds + 2 * BT * LDT;        // [2][BT][LDT]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int d = a.d, H = a.H;
    int bm = blockIdx.x, bn = blockIdx.y, bz = blockIdx.z;
    if constexpr (!FWD && SPLIT) {
        // One-dimensional launch.  Consecutive block ids go to different XCDs; the H / BT workgroups that read the same
        // columns of the same slots (the large operand) take consecutive places on one XCD, so that they run together
        // and those columns come from HBM once.
        const int nbm = H / BT, nbn = d / BT;
        const int xcd = blockIdx.x & 7, idx = blockIdx.x >> 3;
        const int group = (idx / nbm) * 8 + xcd;          // (column tile, share)
        bm = idx % nbm;
        if (group >= nbn * a.nsplit) return;
        bn = group % nbn;
        bz = group / nbn;
    }
    if constexpr (!FWD && !SPLIT) {
        // a launch with one more row of workgroups than there are column tiles: that row takes the small parameters of
        // the update (they do not depend on the contraction), which saves a launch per update
        if ((int)blockIdx.y == d / BT) { small_update_body<1>(a, blockIdx.x, gridDim.x); return; }
    }
    // the fused update reads its tile of the fp32 parameters now, not after the contraction that it does not depend on
    constexpr int C4 = BT / 4;           // float4 groups per row
    constexpr int NPRE = (!FWD && !SPLIT) ? BT * C4 / 256 : 1;
    f32x4 wpre[NPRE];
    if constexpr (!FWD && !SPLIT) {
#pragma unroll
        for (int j = 0; j < NPRE; ++j) {
            const int q = tid + 256 * j, row = q / C4, c4 = q % C4;
            wpre[j] = *reinterpret_cast<const f32x4*>(a.params + (int64_t)(bm * BT + row) * d + bn * BT + 4 * c4);
        }
    }
    // gradient contraction: the slots of the consumed gradients are read once, not once per stage in front of the
    // operand loads that depend on them
    __shared__ int slot_list[FWD ? 1 : 256];
    if constexpr (!FWD) {
        for (int l = tid; l < a.Kv; l += 256) slot_list[l] = consumed_slot(a, l);
        __syncthreads();
    }
    int stage0 = 0, stages = FWD ? d / KT : a.Kv;
    if constexpr (SPLIT) {
        static_assert(!FWD, "only the gradient contraction is split here");
        const int total = a.Kv, shares = a.nsplit;
        const int per = (total + shares - 1) / shares;
        stage0 = bz * per;
        stages = max(0, min(per, total - stage0));
    }

    // global -> LDS: BT rows x 8 chunks of 16 bytes per operand; thread -> chunk tid % 8 of rows tid / 8 + 32 i
    const int lchunk = tid & 7, lrow = tid >> 3;
    constexpr int RPT = BT / MP;        // records per row tile (FWD)
    int slot_of[RPT];
    if (FWD) {
#pragma unroll
        for (int q = 0; q < RPT; ++q) {
            const int r = RPT * bm + q;
            int worker = 0, ordinal = 0, slot = 0;
            if (r < a.nrec) record_of(a, r, worker, ordinal, slot);
            slot_of[q] = slot;
        }
    }
    auto a_ptr = [&](int row, int stage) -> const unsigned short* {
        if (FWD) return a.xb + ((int64_t)slot_of[row / MP] * MP + (row % MP)) * d + stage * KT;
        return a.d1t + ((int64_t)slot_list[FWD ? 0 : stage] * H + bm * BT + row) * MP;
    };
    auto b_ptr = [&](int row, int stage) -> const unsigned short* {
        if (FWD) return a.w1r + (int64_t)(bn * BT + row) * d + stage * KT;
        return a.xbt + ((int64_t)slot_list[FWD ? 0 : stage] * d + bn * BT + row) * MP;
    };
    // Operand stages travel global -> registers -> LDS.  A ring of PF register sets holds the stages that have been
    // asked for and not yet stored to LDS, so that PF stages (PF x BT x 256 bytes) are in flight per workgroup: with one
    // stage in flight a workgroup is bound by the latency of its loads, whatever the tile size.
    constexpr int PF = 3;
    constexpr bool kAlways = FWD || SPLIT;   // the loops of these are long (d / 64 stages, or a share of many slots)
    u16x8 ra[PF][LP], rb[PF][LP];
    auto fetch = [&](auto slot, int stage) {
        constexpr int Q = decltype(slot)::value;
#pragma unroll
        for (int i = 0; i < LP; ++i) {
            const int row = lrow + 32 * i;
            ra[Q][i] = *reinterpret_cast<const u16x8*>(a_ptr(row, stage) + 8 * lchunk);
            rb[Q][i] = *reinterpret_cast<const u16x8*>(b_ptr(row, stage) + 8 * lchunk);
        }
    };
    auto stash = [&](auto slot, int buf) {
        constexpr int Q = decltype(slot)::value;
#pragma unroll
        for (int i = 0; i < LP; ++i) {
            const int row = lrow + 32 * i;
            *reinterpret_cast<u16x8*>(As + (buf * BT + row) * LDT + 8 * lchunk) = ra[Q][i];
            *reinterpret_cast<u16x8*>(Bs + (buf * BT + row) * LDT + 8 * lchunk) = rb[Q][i];
        }
    };

    const int wm = wave >> 1, wn = wave & 1;
    f32x16 acc[NF][NF];
#pragma unroll
    for (int i = 0; i < NF; ++i)
#pragma unroll
        for (int j = 0; j < NF; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;

    using I0 = std::integral_constant<int, 0>;
    using I1 = std::integral_constant<int, 1>;
    using I2 = std::integral_constant<int, 2>;
    if (stages > 0) fetch(I0{}, stage0);
    if (stages > 1) fetch(I1{}, stage0 + 1);
    if (stages > 2) fetch(I2{}, stage0 + 2);
    if (stages > 0) stash(I0{}, 0);
    __syncthreads();
    // stage st is in LDS buffer st & 1 and came from ring slot st % PF, which is free again
    auto one_stage = [&](auto cur, auto nxt, int st) {
        const int buf = st & 1;
        // (long loops: always issued, the last stages over again at the end.  Behind a branch the compiler no longer knows
        // how many loads are in flight and makes the stores to LDS below wait for all of them, these new ones included.)
        if constexpr (kAlways) {
            fetch(cur, stage0 + min(st + PF, stages - 1));
            // the loads go out before anything else of the stage: moved down between the MFMAs, their registers get
            // shared with the operand fragments, and every stage then starts by waiting for all loads in flight
            __builtin_amdgcn_sched_barrier(0);
        } else if (st + PF < stages) fetch(cur, stage0 + st + PF);
#pragma unroll
        for (int kk = 0; kk < KT / 16; ++kk) {
            bf16x8 fa[NF], fb[NF];
            // operand layout of the 32x32x16 MFMA: lane -> row lane % 32, depth 8 (lane / 32) .. + 7
#pragma unroll
            for (int i = 0; i < NF; ++i)
                fa[i] = *reinterpret_cast<const bf16x8*>(As + (buf * BT + wm * WT + i * 32 + (lane & 31)) * LDT + kk * 16 + 8 * (lane >> 5));
#pragma unroll
            for (int j = 0; j < NF; ++j)
                fb[j] = *reinterpret_cast<const bf16x8*>(Bs + (buf * BT + wn * WT + j * 32 + (lane & 31)) * LDT + kk * 16 + 8 * (lane >> 5));
#pragma unroll
            for (int i = 0; i < NF; ++i)
#pragma unroll
                for (int j = 0; j < NF; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
        }
        // (long loops: also after the last stage, whose other buffer nobody reads any more -- no branch, see above)
        if constexpr (kAlways) stash(nxt, buf ^ 1);
        else if (st + 1 < stages) stash(nxt, buf ^ 1);
        __syncthreads();
    };
    if constexpr (kAlways) {
        // whole rounds of the ring without a branch inside, then what is left
        int st = 0;
        for (; st + PF <= stages; st += PF) {
            one_stage(I0{}, I1{}, st);
            one_stage(I1{}, I2{}, st + 1);
            one_stage(I2{}, I0{}, st + 2);
        }
        if (st < stages) one_stage(I0{}, I1{}, st);
        if (st + 1 < stages) one_stage(I1{}, I2{}, st + 1);
    } else {
        for (int st = 0; st < stages; st += PF) {
            one_stage(I0{}, I1{}, st);
            if (st + 1 < stages) one_stage(I1{}, I2{}, st + 1);
            if (st + 2 < stages) one_stage(I2{}, I0{}, st + 2);
        }
    }

    // The result goes through LDS so that the global accesses of the epilogue run along rows.
    // result layout: element e of lane -> row 8 (e / 4) + 4 (lane / 32) + e % 4, column lane % 32
    constexpr int LDC = BT + 4;
    float* Cs = reinterpret_cast<float*>(lds);      // [BT][LDC], fits in the operand buffers
#pragma unroll
    for (int i = 0; i < NF; ++i)
#pragma unroll
        for (int j = 0; j < NF; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int row = wm * WT + i * 32 + 8 * (e >> 2) + 4 * (lane >> 5) + (e & 3);
                const int col = wn * WT + j * 32 + (lane & 31);
                Cs[row * LDC + col] = acc[i][j][e];
            }
    __syncthreads();
    const float scale = a.lr / (float)a.Kv, invK = 1.0f / (float)a.Kv;
#pragma unroll
    for (int j = 0; j < BT * C4 / 256; ++j) {
        const int q = tid + 256 * j;
        const int row = q / C4, c4 = q % C4;
        const f32x4 v = *reinterpret_cast<const f32x4*>(Cs + row * LDC + 4 * c4);
        if (FWD) {
            const int r = RPT * bm + row / MP;
            if (r < a.nrec) {
                const int n = bn * BT + 4 * c4;
                const f32x4 b1 = *reinterpret_cast<const f32x4*>(a.params + (int64_t)H * d + n);
                f32x4 h;
#pragma unroll
                for (int c = 0; c < 4; ++c) { const float z = v[c] + b1[c]; h[c] = z > 0.0f ? z : 0.0f; }
                *reinterpret_cast<f32x4*>(a.hbuf + ((int64_t)slot_of[row / MP] * MP + (row % MP)) * H + n) = h;
            }
        } else if constexpr (SPLIT) {
            const int64_t p = (int64_t)(bm * BT + row) * d + bn * BT + 4 * c4;
            *reinterpret_cast<f32x4*>(a.dw_part + (int64_t)bz * H * d + p) = v;
        } else {
            const int64_t p = (int64_t)(bm * BT + row) * d + bn * BT + 4 * c4;
            f32x4 w = wpre[NPRE == 1 ? 0 : j];
            unsigned short wb[4];
#pragma unroll
            for (int c = 0; c < 4; ++c) { w[c] -= scale * v[c]; wb[c] = bf16_bits(w[c]); }
            *reinterpret_cast<f32x4*>(a.params + p) = w;
            *reinterpret_cast<uint2*>(a.w1r + p) = make_uint2((uint32_t)wb[0] | ((uint32_t)wb[1] << 16), (uint32_t)wb[2] | ((uint32_t)wb[3] << 16));
            if (a.agg_out) *reinterpret_cast<f32x4*>(a.agg_out + p) = v * invK;
        }
    }
}

// ---- Few records (small K): the forward pass straight from the sample matrix --------------------------------
// One launch does what the gather kernel, the split forward contraction and its finishing kernel do otherwise:
// workgroup (record r, 64 hidden units bn, share z of the depth d) draws the sample ids of the record, reads its rows
// from the bf16 copy of X and leaves its partial sums of Z1 in dw_part; the workgroups
// with bn = 0 also write the rows' transposed bf16 copy, which the first-layer gradient contraction of a later update
// reads.  (Workgroups of one launch do not hand results to each other: making one workgroup's stores visible to
// another on a different XCD costs a write-back of the L2, far more than the launch it would save.)  A launch of this
// kind is a chain of load latencies, so three stages per operand are in flight in registers.
template <int BT, bool SPLIT>
__global__ __launch_bounds__(256, 2) void mlp_fwd_gather_kernel(MlpArgs a) {
    constexpr int LP = BT / 32;         // row chunks per thread, operand and stage
    constexpr int PF = BT == 64 ? 3 : 2;
    constexpr bool kAlways = !SPLIT;         // d / 64 stages; a share of them when the depth is split
    constexpr int RPT = BT / MP;        // records per workgroup
    constexpr int WT = BT / 2, NF = WT / 32;
    extern __shared__ __attribute__((aligned(16))) unsigned short lds[];
    unsigned short* As = lds;                       // [2][BT][LDT]
    unsigned short* Bs = lds + 2 * BT * LDT;        // [2][BT][LDT]
    __shared__ uint32_t ids[BT];
    __shared__ int slot_s[RPT];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int bm = blockIdx.x, bn = blockIdx.y;
    const int d = a.d, H = a.H;
    if (tid < BT) {
        const int r = RPT * bm + tid / MP, row = tid % MP;
        uint32_t id = 0xFFFFFFFFu;
        if (r < a.nrec) {
            int worker, ordinal, slot;
            record_of(a, r, worker, ordinal, slot);
            if (row < a.m) id = batch_index(a.seed, a.rep, (uint32_t)worker, (uint32_t)ordinal, (uint32_t)a.v, (uint32_t)row, a.N);
            if (bn == 0 && blockIdx.z == 0) a.ylab[slot * MP + row] = (id == 0xFFFFFFFFu) ? -1 : a.y[id];
            if (row == 0) slot_s[tid / MP] = slot;
        } else if (row == 0) slot_s[tid / MP] = -1;
        ids[tid] = id;
    }
    __syncthreads();
    int stage0 = 0, stages = d / KT;
    if constexpr (SPLIT) {
        const int total = d / KT, per = (total + a.fsplit - 1) / a.fsplit;
        stage0 = blockIdx.z * per;
        stages = max(0, min(per, total - stage0));
    }
    const int lchunk = tid & 7, lrow = tid >> 3;
    // (rows from the bf16 copy of the sample matrix; row N of it is all zero and stands for the rows a record lacks)
    const unsigned short* xrow[LP];
#pragma unroll
    for (int i = 0; i < LP; ++i) {
        const uint32_t id = ids[lrow + 32 * i];
        xrow[i] = a.Xb + (int64_t)(id != 0xFFFFFFFFu ? id : a.N) * d + 8 * lchunk;
    }
    const unsigned short* wrow = a.w1r + (int64_t)(bn * BT + lrow) * d + 8 * lchunk;
    u16x8 ra[PF][LP];
    u16x8 rb[PF][LP];
    auto fetch = [&](auto ring, int stage) {
        constexpr int Q = decltype(ring)::value;
#pragma unroll
        for (int i = 0; i < LP; ++i) {
            ra[Q][i] = *reinterpret_cast<const u16x8*>(xrow[i] + stage * KT);
            rb[Q][i] = *reinterpret_cast<const u16x8*>(wrow + (int64_t)32 * i * d + stage * KT);
        }
    };
    auto stash = [&](auto ring, int buf) {
        constexpr int Q = decltype(ring)::value;
#pragma unroll
        for (int i = 0; i < LP; ++i) {
            const int row = lrow + 32 * i;
            *reinterpret_cast<u16x8*>(As + (buf * BT + row) * LDT + 8 * lchunk) = ra[Q][i];
            *reinterpret_cast<u16x8*>(Bs + (buf * BT + row) * LDT + 8 * lchunk) = rb[Q][i];
        }
    };
    const int wm = wave >> 1, wn = wave & 1;
    f32x16 acc[NF][NF];
#pragma unroll
    for (int i = 0; i < NF; ++i)
#pragma unroll
        for (int j = 0; j < NF; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;
    // The transposed bf16 copy of the rows (read by the gradient contraction of a later update) is written by the
    // workgroups with bn = 0.  (Sharing it out between the workgroups that read the same rows was measured slower: the
    // 2-byte LDS reads of the transposition then delay the operand reads of every workgroup, not of a quarter of them.
    // Likewise the thread mapping below: eight samples per thread instead of sixteen was slower by a third.)
    using I0 = std::integral_constant<int, 0>;
    using I1 = std::integral_constant<int, 1>;
    using I2 = std::integral_constant<int, PF == 3 ? 2 : 0>;
    if (stages > 0) fetch(I0{}, stage0);
    if (stages > 1) fetch(I1{}, stage0 + 1);
    if (PF == 3 && stages > 2) fetch(I2{}, stage0 + 2);
    if (stages > 0) stash(I0{}, 0);
    __syncthreads();
    auto one_stage = [&](auto cur, auto nxt, int st) {
        const int buf = st & 1;
        // (long loops: always issued, the last stages over again at the end.  Behind a branch the compiler no longer knows
        // how many loads are in flight and makes the stores to LDS below wait for all of them, these new ones included.)
        if constexpr (kAlways) {
            fetch(cur, stage0 + min(st + PF, stages - 1));
            // the loads go out before anything else of the stage: moved down between the MFMAs, their registers get
            // shared with the operand fragments, and every stage then starts by waiting for all loads in flight
            __builtin_amdgcn_sched_barrier(0);
        } else if (st + PF < stages) fetch(cur, stage0 + st + PF);
#pragma unroll
        for (int kk = 0; kk < KT / 16; ++kk) {
            bf16x8 fa[NF], fb[NF];
#pragma unroll
            for (int i = 0; i < NF; ++i)
                fa[i] = *reinterpret_cast<const bf16x8*>(As + (buf * BT + wm * WT + i * 32 + (lane & 31)) * LDT + kk * 16 + 8 * (lane >> 5));
#pragma unroll
            for (int j = 0; j < NF; ++j)
                fb[j] = *reinterpret_cast<const bf16x8*>(Bs + (buf * BT + wn * WT + j * 32 + (lane & 31)) * LDT + kk * 16 + 8 * (lane >> 5));
#pragma unroll
            for (int i = 0; i < NF; ++i)
#pragma unroll
                for (int j = 0; j < NF; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
        }
        if (bn == 0) {
            // transposed copy of this stage's rows: thread -> feature tid / 4, samples 16 (tid % 4) .. + 15 of every record
            const int k = tid >> 2, part = tid & 3;
#pragma unroll
            for (int q = 0; q < RPT; ++q) {
                const int slot = slot_s[q];
                if (slot >= 0) {
                    u16x8 v0, v1;
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        v0[e] = As[(buf * BT + q * MP + 16 * part + e) * LDT + k];
                        v1[e] = As[(buf * BT + q * MP + 16 * part + 8 + e) * LDT + k];
                    }
                    unsigned short* dst = a.xbt + ((int64_t)slot * d + (int64_t)(stage0 + st) * KT + k) * MP + 16 * part;
                    *reinterpret_cast<u16x8*>(dst) = v0;
                    *reinterpret_cast<u16x8*>(dst + 8) = v1;
                }
            }
        }
        // (long loops: also after the last stage, whose other buffer nobody reads any more -- no branch, see above)
        if constexpr (kAlways) stash(nxt, buf ^ 1);
        else if (st + 1 < stages) stash(nxt, buf ^ 1);
        __syncthreads();
    };
    if constexpr (kAlways && PF == 3) {
        // whole rounds of the ring without a branch inside, then what is left
        int st = 0;
        for (; st + 3 <= stages; st += 3) {
            one_stage(I0{}, I1{}, st);
            one_stage(I1{}, I2{}, st + 1);
            one_stage(I2{}, I0{}, st + 2);
        }
        if (st < stages) one_stage(I0{}, I1{}, st);
        if (st + 1 < stages) one_stage(I1{}, I2{}, st + 1);
    } else if constexpr (kAlways) {
        int st = 0;
        for (; st + 2 <= stages; st += 2) {
            one_stage(I0{}, I1{}, st);
            one_stage(I1{}, I0{}, st + 1);
        }
        if (st < stages) one_stage(I0{}, I1{}, st);
    } else if constexpr (PF == 3) {
        for (int st = 0; st < stages; st += 3) {
            one_stage(I0{}, I1{}, st);
            if (st + 1 < stages) one_stage(I1{}, I2{}, st + 1);
            if (st + 2 < stages) one_stage(I2{}, I0{}, st + 2);
        }
    } else {
        for (int st = 0; st < stages; st += 2) {
            one_stage(I0{}, I1{}, st);
            if (st + 1 < stages) one_stage(I1{}, I0{}, st + 1);
        }
    }
    // result: element e of lane -> row 8 (e / 4) + 4 (lane / 32) + e % 4, column lane % 32 of a 32 x 32 block
#pragma unroll
    for (int i = 0; i < NF; ++i)
#pragma unroll
        for (int j = 0; j < NF; ++j) {
            const int col = bn * BT + wn * WT + j * 32 + (lane & 31);
            const float b1 = SPLIT ? 0.0f : (a.b1r ? a.b1r[col] : a.params[(int64_t)H * d + col]);
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int row = wm * WT + i * 32 + 8 * (e >> 2) + 4 * (lane >> 5) + (e & 3);
                const int q = row / MP, r = RPT * bm + q;
                if (r < a.nrec) {
                    if constexpr (SPLIT) {
                        a.dw_part[(((int64_t)blockIdx.z * a.nrec + r) * MP + (row % MP)) * H + col] = acc[i][j][e];
                    } else {
                        const float z = acc[i][j][e] + b1;
                        a.hbuf[((int64_t)slot_s[q] * MP + (row % MP)) * H + col] = z > 0.0f ? z : 0.0f;
                    }
                }
            }
        }
}

// ---- Few records: everything between the two contractions in one launch ---------------------------------------
// Workgroup (record r, quarter q) takes rows 16 q .. 16 q + 15 of the record: hidden activations from the partial sums
// of the split forward pass (shares added in order, bias, ReLU; kept in LDS), layer 2 on the fp32 MFMA units (wave w
// takes a quarter of the hidden units, the four partial results are added in order), softmax, delta2, loss,
// delta1 = (W2^T delta2) * [h > 0] (bf16, transposed, for the gradient contraction) and the quarter's second-layer
// gradients.
__global__ __launch_bounds__(256) void mlp_mid_kernel(MlpArgs a) {
    extern __shared__ __attribute__((aligned(16))) float mid_lds[];
    const int H = a.H, C = a.C, m = a.m;
    const int HS = H + 4;
    float* hs = mid_lds;                       // [16][H + 4]
    float* zp = hs + 16 * HS;                  // [4][16][16] partial logits
    float* d2s = zp + 4 * 256;                 // [16][16]
    float* red = d2s + 256;                    // [4] loss of the waves
    const int r = blockIdx.x >> 2, q = blockIdx.x & 3, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    int worker, ordinal, slot;
    record_of(a, r, worker, ordinal, slot);
    // ---- hidden activations of the 16 rows: every share of every position is asked for before the first is used
    {
        const int h4 = H / 4;                  // 16-byte groups per row; 16 rows = 16 h4 groups, 16 h4 / 256 per thread
        const float* src = a.dw_part + ((int64_t)r * MP + 16 * q) * H;
        const int64_t zs = (int64_t)a.nrec * MP * H;
        const float* b1 = a.b1r ? a.b1r : a.params + (int64_t)H * a.d;
        for (int p0 = tid; p0 < 16 * h4; p0 += 4 * 256) {
            f32x4 v[4][8];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int p = min(p0 + 256 * u, 16 * h4 - 1);
#pragma unroll
                for (int z = 0; z < 8; ++z)
                    if (z < a.fsplit) v[u][z] = *reinterpret_cast<const f32x4*>(src + z * zs + (int64_t)4 * p);
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int p = p0 + 256 * u;
                if (p < 16 * h4) {
                    f32x4 t = v[u][0];
#pragma unroll
                    for (int z = 1; z < 8; ++z)
                        if (z < a.fsplit) t += v[u][z];
                    const int n = 4 * (p % h4);
                    const f32x4 bb = *reinterpret_cast<const f32x4*>(b1 + n);
                    f32x4 h;
#pragma unroll
                    for (int c = 0; c < 4; ++c) { const float zc = t[c] + bb[c]; h[c] = zc > 0.0f ? zc : 0.0f; }
                    *reinterpret_cast<f32x4*>(hs + (p / h4) * HS + n) = h;
                }
            }
        }
    }
    const int cls = lane & 15, kq = lane >> 4;
    const float b2 = a.b2r ? a.b2r[min(cls, C - 1)] : a.params[(int64_t)H * a.d + H + (int64_t)C * H + min(cls, C - 1)];
    __syncthreads();
    // ---- layer 2: wave w sums over its quarter of the hidden units
    {
        const int kw = H / 4;                  // hidden units per wave, a multiple of 32
        const float* hp = hs + (lane & 15) * HS + wave * kw + 4 * kq;
        const float* wp = a.w2r + (int64_t)min(cls, C - 1) * H + wave * kw + 4 * kq;
        f32x4 acc0 = {0.f, 0.f, 0.f, 0.f}, acc1 = {0.f, 0.f, 0.f, 0.f};
        for (int k0 = 0; k0 < kw / 16; k0 += 8) {
            f32x4 hv[8], wv[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int kb = min(k0 + u, kw / 16 - 1);
                hv[u] = *reinterpret_cast<const f32x4*>(hp + 16 * kb);
                wv[u] = *reinterpret_cast<const f32x4*>(wp + 16 * kb);
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                if (k0 + u < kw / 16) {
                    acc0 = __builtin_amdgcn_mfma_f32_16x16x4f32(hv[u].x, wv[u].x, acc0, 0, 0, 0);
                    acc1 = __builtin_amdgcn_mfma_f32_16x16x4f32(hv[u].y, wv[u].y, acc1, 0, 0, 0);
                    acc0 = __builtin_amdgcn_mfma_f32_16x16x4f32(hv[u].z, wv[u].z, acc0, 0, 0, 0);
                    acc1 = __builtin_amdgcn_mfma_f32_16x16x4f32(hv[u].w, wv[u].w, acc1, 0, 0, 0);
                }
            }
        }
        const f32x4 acc = acc0 + acc1;         // class lane % 16 of rows 4 (lane / 16) + e
#pragma unroll
        for (int e = 0; e < 4; ++e) zp[wave * 256 + (4 * kq + e) * 16 + cls] = acc[e];
    }
    // second-layer weights of this thread's hidden units (delta1 below), asked for before the softmax
    float w2c[2][16];
#pragma unroll
    for (int u = 0; u < 2; ++u)
#pragma unroll
        for (int c = 0; c < 16; ++c) w2c[u][c] = (c < C && tid + 256 * u < H) ? a.w2r[c * H + tid + 256 * u] : 0.0f;
    __syncthreads();
    // ---- softmax, delta2, loss: thread -> (row tid / 16, class tid % 16)
    {
        const int row = tid >> 4, c = tid & 15;   // c == lane % 16: b2 is this lane's own class
        const int s = 16 * q + row;
        const int lab = a.ylab[slot * MP + s];
        const bool ok = s < m && lab >= 0;
        const float z = ((zp[row * 16 + c] + zp[256 + row * 16 + c]) + zp[512 + row * 16 + c]) + zp[768 + row * 16 + c] + b2;
        float zmax = c < C ? z : -3.0e38f;
#pragma unroll
        for (int o = 8; o >= 1; o >>= 1) zmax = fmaxf(zmax, __shfl_xor(zmax, o, 64));
        const float ex = c < C ? expf(z - zmax) : 0.0f;
        float den = ex;
#pragma unroll
        for (int o = 8; o >= 1; o >>= 1) den += __shfl_xor(den, o, 64);
        float dv = 0.0f, ls = 0.0f;
        if (c < C && ok) {
            dv = ex / den - (c == lab ? 1.0f : 0.0f);
            if (c == lab) ls = -(z - zmax - logf(den));
        }
        d2s[row * 16 + c] = dv;
        a.d2[(slot * MP + s) * 16 + c] = dv;
#pragma unroll
        for (int o = 32; o >= 1; o >>= 1) ls += __shfl_xor(ls, o, 64);
        if (lane == 0) red[wave] = ls;
    }
    __syncthreads();
    // ---- delta1 and the quarter's sums: thread -> hidden units tid and tid + 256
    const float inv_m = 1.0f / (float)m;
#pragma unroll
    for (int u = 0; u < 2; ++u) {
        const int j = tid + 256 * u;
        if (j < H) {
            float gw[16];
#pragma unroll
            for (int c = 0; c < 16; ++c) gw[c] = 0.0f;
            float g1 = 0.0f;
            u16x8 pack[2];
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const float h = hs[e * HS + j];
                float d1 = 0.0f;
#pragma unroll
                for (int c = 0; c < 16; ++c) {
                    const float dv = d2s[e * 16 + c];
                    d1 += w2c[u][c] * dv;
                    gw[c] += dv * h;
                }
                if (!(h > 0.0f)) d1 = 0.0f;
                g1 += d1;
                pack[e >> 3][e & 7] = bf16_bits(d1 * inv_m);
            }
            unsigned short* dst = a.d1t + ((int64_t)slot * H + j) * MP + 16 * q;
            *reinterpret_cast<u16x8*>(dst) = pack[0];
            *reinterpret_cast<u16x8*>(dst + 8) = pack[1];
            a.gb1[(slot * 4 + q) * H + j] = g1;
#pragma unroll
            for (int c = 0; c < 16; ++c)
                if (c < C) a.gw2[((int64_t)(slot * 4 + q) * C + c) * H + j] = gw[c];
        }
    }
    if (tid < 16) {
        float sum = 0.0f;
        for (int e = 0; e < 16; ++e) sum += d2s[e * 16 + tid];
        a.gb2[(slot * 4 + q) * 16 + tid] = sum;
    }
    if (tid == 16) a.loss[slot * 4 + q] = (red[0] + red[1]) + (red[2] + red[3]);
    if (tid == 17 && q == 0) a.quartered[slot] = 1;
}

// ---- layer 2 and softmax: one workgroup per record; wave w takes rows 16 w .. 16 w + 15 -------------
// Z2 = H W2^T is a 16 x 16 x H contraction per wave on the fp32 MFMA units (H is not rounded, so this
// layer runs in fp32): operand lane -> (row or class lane % 16, 4 hidden units starting at 16 kk + 4 (lane / 16)).
// With one workgroup per record the kernel is a chain of load latencies: what the epilogue needs from memory is
// asked for first, and eight 16-unit blocks of h and W2 are in flight at a time.  (Staging W2 in LDS, or sixteen
// waves per record with the hidden units split four ways, did not shorten it.)
__global__ __launch_bounds__(256) void mlp_output_kernel(MlpArgs a) {
    __shared__ float wsum[4];
    const int r = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int H = a.H, C = a.C, m = a.m;
    int worker, ordinal, slot;
    record_of(a, r, worker, ordinal, slot);
    const int cls = lane & 15, kq = lane >> 4;
    const float* hp = a.hbuf + ((int64_t)slot * MP + 16 * wave + (lane & 15)) * H + 4 * kq;
    const float* wp = a.w2r + (int64_t)min(cls, C - 1) * H + 4 * kq;
    const float b2 = a.b2r ? a.b2r[min(cls, C - 1)] : a.params[(int64_t)H * a.d + H + (int64_t)C * H + min(cls, C - 1)];
    int labs[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) labs[e] = a.ylab[slot * MP + 16 * wave + 4 * kq + e];
    f32x4 acc0 = {0.f, 0.f, 0.f, 0.f}, acc1 = {0.f, 0.f, 0.f, 0.f};
    for (int k0 = 0; k0 < H / 16; k0 += 8) {        // H is a multiple of 128
        f32x4 hv[8], wv[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            hv[u] = *reinterpret_cast<const f32x4*>(hp + 16 * (k0 + u));
            wv[u] = *reinterpret_cast<const f32x4*>(wp + 16 * (k0 + u));
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            acc0 = __builtin_amdgcn_mfma_f32_16x16x4f32(hv[u].x, wv[u].x, acc0, 0, 0, 0);
            acc1 = __builtin_amdgcn_mfma_f32_16x16x4f32(hv[u].y, wv[u].y, acc1, 0, 0, 0);
            acc0 = __builtin_amdgcn_mfma_f32_16x16x4f32(hv[u].z, wv[u].z, acc0, 0, 0, 0);
            acc1 = __builtin_amdgcn_mfma_f32_16x16x4f32(hv[u].w, wv[u].w, acc1, 0, 0, 0);
        }
    }
    const f32x4 acc = acc0 + acc1;
    // result: lane holds class lane % 16 of rows 4 (lane / 16) + e, e < 4 (classes past C repeat class C-1: unused)
    float lsum = 0.0f;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const int s = 16 * wave + 4 * kq + e;
        const int lab = labs[e];
        const bool ok = s < m && lab >= 0;
        const float z = acc[e] + b2;
        float zmax = cls < C ? z : -3.0e38f;
#pragma unroll
        for (int o = 8; o >= 1; o >>= 1) zmax = fmaxf(zmax, __shfl_xor(zmax, o, 64));
        const float ex = cls < C ? expf(z - zmax) : 0.0f;
        float den = ex;
#pragma unroll
        for (int o = 8; o >= 1; o >>= 1) den += __shfl_xor(den, o, 64);
        float dv = 0.0f;
        if (cls < C && ok) {
            dv = ex / den - (cls == lab ? 1.0f : 0.0f);
            if (cls == lab) lsum += -(z - zmax - logf(den));
        }
        a.d2[(slot * MP + s) * 16 + cls] = dv;       // zero past C and for rows without a sample
    }
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) lsum += __shfl_xor(lsum, o, 64);
    if (lane == 0) wsum[wave] = lsum;
    __syncthreads();
    if (tid == 0) a.loss[slot * 4] = (wsum[0] + wsum[1]) + (wsum[2] + wsum[3]);
}

// ---- delta1 = (W2^T delta2) * [H > 0], second-layer gradient: workgroup = (record, 64 hidden units) ----
// thread -> hidden unit jb * 64 + tid % 64, rows 16 (tid / 64) .. + 15
__global__ __launch_bounds__(256) void mlp_delta1_kernel(MlpArgs a) {
    __shared__ float d2s[MP][16];
    __shared__ float part[3][64][17];
    const int r = blockIdx.x, jb = blockIdx.y, tid = threadIdx.x;
    const int H = a.H, C = a.C;
    int worker, ordinal, slot;
    record_of(a, r, worker, ordinal, slot);
    for (int q = tid; q < MP * 16; q += 256) d2s[q >> 4][q & 15] = a.d2[slot * MP * 16 + q];
    const int jl = tid & 63, rq = tid >> 6, j = jb * 64 + jl;
    const float* hrow = a.hbuf + ((int64_t)slot * MP + 16 * rq) * H + j;
    float h[16];
#pragma unroll
    for (int e = 0; e < 16; ++e) h[e] = hrow[(int64_t)e * H];
    const float inv_m = 1.0f / (float)a.m;
    float w2c[16], gw[16];
#pragma unroll
    for (int c = 0; c < 16; ++c) { w2c[c] = (c < C) ? a.w2r[c * H + j] : 0.0f; gw[c] = 0.0f; }
    __syncthreads();
    float g1 = 0.0f;
    u16x8 pack[2];
#pragma unroll
    for (int e = 0; e < 16; ++e) {
        const int s = 16 * rq + e;
        float d1 = 0.0f;
#pragma unroll
        for (int c = 0; c < 16; ++c) {
            const float dv = d2s[s][c];          // zero past C
            d1 += w2c[c] * dv;
            gw[c] += dv * h[e];
        }
        if (!(h[e] > 0.0f)) d1 = 0.0f;
        g1 += d1;
        pack[e >> 3][e & 7] = bf16_bits(d1 * inv_m);
    }
    unsigned short* dst = a.d1t + ((int64_t)slot * H + j) * MP + 16 * rq;
    *reinterpret_cast<u16x8*>(dst) = pack[0];
    *reinterpret_cast<u16x8*>(dst + 8) = pack[1];
    // the four row quarters are added in a fixed order; the sum is the slot's only record
    if (rq > 0) {
        part[rq - 1][jl][16] = g1;
#pragma unroll
        for (int c = 0; c < 16; ++c) part[rq - 1][jl][c] = gw[c];
    }
    __syncthreads();
    if (rq == 0) {
        a.gb1[slot * 4 * H + j] = ((g1 + part[0][jl][16]) + part[1][jl][16]) + part[2][jl][16];
#pragma unroll
        for (int c = 0; c < 16; ++c)
            if (c < C) a.gw2[((int64_t)slot * 4 * C + c) * H + j] = ((gw[c] + part[0][jl][c]) + part[1][jl][c]) + part[2][jl][c];
    }
    if (jb == 0 && tid < 16) {
        float sum = 0.0f;
        for (int s = 0; s < MP; ++s) sum += d2s[s][tid];
        a.gb2[slot * 4 * 16 + tid] = sum;
    }
    if (jb == 0 && tid == 16) a.quartered[slot] = 0;
}

// ---- the small parameters of update v, and its loss record ------------------------------------
// Element q of the per-slot record [gb1 | gw2 | gb2 | loss] is summed over the consumed slots by a group of G lanes
// (G a power of two, at most 16): lane g of the group takes the slots g, g + G, ... in list order, the G partial sums are
// added in a fixed butterfly order.  (block `block` of `nblocks` blocks of 256 threads)
template <int G>
__device__ __forceinline__ void small_update_body(const MlpArgs& a, int block, int nblocks) {
    const int H = a.H, C = a.C, d = a.d;
    const float invKm = 1.0f / ((float)a.Kv * (float)a.m);
    float* small = a.params + (int64_t)H * d;          // [b1 | W2 | b2]
    const int total = H + C * H + C + 1;
    // G == 1 (few slots, a kernel that is all latency): the flag of a slot is loaded beside its record, all four
    // quarters of it.  Larger G (many slots): the flags first, so that whole records are read once, not four times.
    constexpr bool kBeside = G == 1;
    __shared__ int slots[256];
    __shared__ int nquart[kBeside ? 1 : 256];
    for (int l = threadIdx.x; l < a.Kv; l += blockDim.x) {
        const int sl = consumed_slot(a, l);
        slots[l] = sl;
        if constexpr (!kBeside) nquart[l] = a.quartered[sl];
    }
    __syncthreads();
    const int g = threadIdx.x % G;
    const int per_block = blockDim.x / G;
    const int rounds = (total + nblocks * per_block - 1) / (nblocks * per_block);
    for (int it = 0; it < rounds; ++it) {
        const int q = (it * nblocks + block) * per_block + threadIdx.x / G;
        const bool live = q < total;
        const float* base = a.loss;
        int stride = 1;             // between the quarters of a slot; four times that between slots
        if (live) {
            if (q < H) { base = a.gb1 + q; stride = H; }
            else if (q < H + C * H) { base = a.gw2 + (q - H); stride = C * H; }
            else if (q < H + C * H + C) { base = a.gb2 + (q - H - C * H); stride = 16; }
        }
        // Everything the element needs is asked for at once: its old value, and of every slot the flag and all four
        // quarters of the record (the quarters a whole record does not have are there in memory and are dropped by the
        // select), so that the kernel is one round trip to memory deep, not three.
        const float oldv = (live && g == 0 && q < total - 1) ? small[q] : 0.0f;
        float sum = 0.0f;
        if (live) {
            int l = g;
            for (; l + 3 * G < a.Kv; l += 4 * G) {
                float v[4][4];
                int nq[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int sl = slots[l + u * G];
                    if constexpr (kBeside) nq[u] = a.quartered[sl]; else nq[u] = nquart[l + u * G];
                    v[u][0] = base[(int64_t)sl * 4 * stride];
#pragma unroll
                    for (int qq = 1; qq < 4; ++qq) v[u][qq] = (kBeside || nq[u] != 0) ? base[((int64_t)sl * 4 + qq) * stride] : 0.0f;
                }
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const bool four = nq[u] != 0;
                    sum += ((v[u][0] + (four ? v[u][1] : 0.0f)) + (four ? v[u][2] : 0.0f)) + (four ? v[u][3] : 0.0f);
                }
            }
            for (; l < a.Kv; l += G) {
                const int sl = slots[l];
                int nq1;
                if constexpr (kBeside) nq1 = a.quartered[sl]; else nq1 = nquart[l];
                const bool four = nq1 != 0;
                float v[4];
                v[0] = base[(int64_t)sl * 4 * stride];
#pragma unroll
                for (int qq = 1; qq < 4; ++qq) v[qq] = (kBeside || four) ? base[((int64_t)sl * 4 + qq) * stride] : 0.0f;
                sum += ((v[0] + (four ? v[1] : 0.0f)) + (four ? v[2] : 0.0f)) + (four ? v[3] : 0.0f);
            }
        }
#pragma unroll
        for (int o = 1; o < G; o <<= 1) sum += __shfl_xor(sum, o, 64);
        if (live && g == 0) {
            const float gr = sum * invKm;
            if (q == total - 1) {
                a.tr.loss[a.v] = gr;
            } else {
                const float nv = oldv - a.lr * gr;
                small[q] = nv;
                if (q < H) { if (a.b1r) a.b1r[q] = nv; }
                else if (q < H + C * H) a.w2r[q - H] = bf16_round(nv);
                else if (a.b2r) a.b2r[q - H - C * H] = nv;
                if (a.agg_out) a.agg_out[(int64_t)H * d + q] = gr;
            }
        }
    }
}
// ---- first-layer update from the partial sums of a split gradient contraction: shares added in order; the
// first kSmallBlocks16 workgroups take the small parameters of the update instead, which need nothing from the others
// (first, because theirs is the longer chain of loads)
constexpr int kW1Blocks = 1024, kSmallBlocks16 = 360;
__global__ __launch_bounds__(256) void mlp_w1_update_kernel(MlpArgs a) {
    if ((int)blockIdx.x < kSmallBlocks16) { small_update_body<16>(a, blockIdx.x, kSmallBlocks16); return; }
    const int block = blockIdx.x - kSmallBlocks16;
    const int64_t n4 = (int64_t)a.H * a.d / 4;
    const float scale = a.lr / (float)a.Kv, invK = 1.0f / (float)a.Kv;
    for (int64_t q = (int64_t)block * blockDim.x + threadIdx.x; q < n4; q += (int64_t)kW1Blocks * blockDim.x) {
        const int64_t p = 4 * q;
        f32x4 v = *reinterpret_cast<const f32x4*>(a.dw_part + p);
        for (int sp = 1; sp < a.nsplit; ++sp) v += *reinterpret_cast<const f32x4*>(a.dw_part + (int64_t)sp * a.H * a.d + p);
        f32x4 w = *reinterpret_cast<const f32x4*>(a.params + p);
        unsigned short wb[4];
#pragma unroll
        for (int c = 0; c < 4; ++c) { w[c] -= scale * v[c]; wb[c] = bf16_bits(w[c]); }
        *reinterpret_cast<f32x4*>(a.params + p) = w;
        *reinterpret_cast<uint2*>(a.w1r + p) = make_uint2((uint32_t)wb[0] | ((uint32_t)wb[1] << 16), (uint32_t)wb[2] | ((uint32_t)wb[3] << 16));
        if (a.agg_out) *reinterpret_cast<f32x4*>(a.agg_out + p) = v * invK;
    }
}

__global__ void mlp_refresh_kernel(const float* params, unsigned short* w1r, float* w2r, int64_t n1, int64_t off2, int64_t n2) {
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t q = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; q < n1; q += stride) w1r[q] = bf16_bits(params[q]);
    for (int64_t q = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; q < n2; q += stride) w2r[q] = bf16_round(params[off2 + q]);
}

// the sample matrix in bf16 (round to nearest even, eight values per thread and pass), and a row of zeros behind it
__global__ void mlp_rows_bf16_kernel(const float* X, unsigned short* Xb, int64_t n8, int64_t zero8) {
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t q = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; q < n8 + zero8; q += stride) {
        f32x8 w;
#pragma unroll
        for (int e = 0; e < 8; ++e) w[e] = 0.0f;
        if (q < n8) {
            const f32x4 lo = *reinterpret_cast<const f32x4*>(X + 8 * q), hi = *reinterpret_cast<const f32x4*>(X + 8 * q + 4);
#pragma unroll
            for (int e = 0; e < 4; ++e) { w[e] = lo[e]; w[4 + e] = hi[e]; }
        }
        *reinterpret_cast<bf16x8*>(Xb + 8 * q) = __builtin_convertvector(w, bf16x8);
    }
}

// W1, W2 uniform on (-1/sqrt(fan_in), 1/sqrt(fan_in)) from the INIT stream, biases zero
__global__ void mlp_init_kernel(float* params, uint64_t seed, int64_t nw, int64_t n1, int64_t off2, int64_t n2, float bound1, float bound2) {
#pragma clang fp contract(off)
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t q = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; q < nw; q += stride) {
        float w = 0.0f;
        const bool in1 = q < n1, in2 = q >= off2 && q < off2 + n2;
        if (in1 || in2) {
            const u32x4 b = draw(seed, kInit, (uint32_t)((q >> 2) >> 32), 0u, 0u, 0u, (uint32_t)(q >> 2));
            const uint32_t word = (q & 2) ? ((q & 1) ? b.w : b.z) : ((q & 1) ? b.y : b.x);
            const float u = uniform_open(word);
            float v = u + u;
            v = v - 1.0f;
            w = v * (in1 ? bound1 : bound2);
        }
        params[q] = w;
    }
}

// operand double buffer; the epilogue's fp32 tile [BT][BT + 4] fits inside it
size_t contract_lds(int bt) { return (size_t)4 * bt * LDT * 2; }
// Forward streams of the overlapped updates.  With the caller's stream and the stream of the schedule they are four:
// a process has four hardware queues here, and streams that share one run their kernels one after the other (a long
// schedule kernel in front of a forward kernel, say).
constexpr int kFwdStreams = 2;
constexpr int kVer = 8;          // versions of the operand copies of the parameters when updates overlap
constexpr int kMaxSplit = 8;     // shares of the consumed slots in the split gradient contraction
size_t mid_lds_bytes(int H) { return sizeof(float) * (16 * (size_t)(H + 4) + 4 * 256 + 256 + 4); }

struct DevMem {
    void* p = nullptr;
    size_t bytes = 0;
    hipError_t alloc(size_t n) { bytes = n; return hipMalloc(&p, n ? n : 16); }
    void release() { if (p) (void)hipFree(p); p = nullptr; }
};

}  // namespace

struct MlpState {
    MlpArgs a{};
    int S = 0;
    int64_t nw = 0;
    int prevK = 0;          // size of the consume list of the last update run (records of the next K-async step)
    int replica = 0;
    hipStream_t own = nullptr;   // replicas beyond the first run on streams of their own, beside each other
    // overlapped updates (few records, one replica): kVer versions of the operand copies of the parameters, three
    // streams for the forward halves of consecutive updates, a pool of events
    DevMem xb16;                 // the first replica's bf16 copy of the sample matrix; the others use it too
    DevMem w1v, w2v, b1v, b2v, fwd_part;   // allocated by the first segment that overlaps
    hipStream_t fwd_stream[kFwdStreams] = {};
    std::vector<hipEvent_t> ev_pool;
    DevMem params, w1r, w2r, xb, xbt, hbuf, d1t, gb1, gw2, gb2, d2, loss, ylab, dw_part, plan, quartered;
    hipStream_t stream = nullptr;
};

hipError_t mlp_create(MlpState** out, const ssgd_model& model, int P, int m, int variant, int Kcap, double lr,
                      uint64_t seed, int replica, const MlpState* first, hipStream_t stream, std::string* msg) {
    auto fail = [&](hipError_t e, const char* what) { if (msg) *msg = what; return e; };
    if (!model.bf16) return fail(hipErrorInvalidValue, "the MLP runs with bf16 operands only (model.bf16 = 1)");
    if (m > MP) return fail(hipErrorInvalidValue, "the MLP keeps at most 64 rows per mini-batch");
    if (model.hidden % 128 || model.d % 128) return fail(hipErrorInvalidValue, "the MLP needs hidden % 128 == 0 and d % 128 == 0");
    if (model.classes > 16) return fail(hipErrorInvalidValue, "at most 16 classes");
    MlpState* s = new MlpState();
    s->stream = stream;
    s->replica = replica;
    MlpArgs& a = s->a;
    a.rep = (uint32_t)replica;
    a.d = model.d; a.H = model.hidden; a.C = model.classes; a.P = P; a.m = m; a.variant = variant; a.Kcap = Kcap;
    a.X = model.X; a.y = (const int32_t*)model.y; a.N = (uint32_t)model.N; a.seed = seed; a.lr = (float)lr;
    s->S = (variant == kAsync) ? P : (variant == kBatchAsync ? P + Kcap : Kcap);
    a.S = s->S;
    const int64_t n1 = (int64_t)a.H * a.d, off2 = n1 + a.H, n2 = (int64_t)a.C * a.H;
    s->nw = off2 + n2 + a.C;
    const size_t S = (size_t)s->S;
    hipError_t e;
#define TRY(x) do { e = (x); if (e != hipSuccess) { mlp_destroy(s); return fail(e, #x); } } while (0)
    TRY(s->params.alloc(sizeof(float) * s->nw));
    TRY(s->w1r.alloc(2 * (size_t)n1));
    TRY(s->w2r.alloc(sizeof(float) * n2));
    TRY(s->xb.alloc(2 * S * MP * a.d));
    TRY(s->xbt.alloc(2 * S * MP * a.d));
    TRY(s->hbuf.alloc(sizeof(float) * S * MP * a.H));
    TRY(s->d1t.alloc(2 * S * MP * a.H));
    TRY(s->gb1.alloc(sizeof(float) * S * 4 * a.H));
    TRY(s->gw2.alloc(sizeof(float) * S * 4 * a.C * a.H));
    TRY(s->gb2.alloc(sizeof(float) * S * 4 * 16));
    TRY(s->d2.alloc(sizeof(float) * S * MP * 16));
    TRY(s->loss.alloc(sizeof(float) * S * 4));
    TRY(s->ylab.alloc(sizeof(int32_t) * S * MP));
    TRY(s->quartered.alloc(sizeof(int32_t) * S));
    TRY(hipMemsetAsync(s->quartered.p, 0, sizeof(int32_t) * S, stream));
    TRY(s->dw_part.alloc(sizeof(float) * kMaxSplit * (size_t)n1));
    if (first != nullptr) {
        a.Xb = first->a.Xb;
    } else {
        TRY(s->xb16.alloc(2 * ((size_t)model.N + 1) * a.d));
        a.Xb = (const unsigned short*)s->xb16.p;
        hipLaunchKernelGGL(mlp_rows_bf16_kernel, dim3(2048), dim3(256), 0, stream, model.X, (unsigned short*)s->xb16.p,
                           (int64_t)model.N * a.d / 8, (int64_t)a.d / 8);
        TRY(hipGetLastError());
    }
    {
        // every slot free (popped in the order 0, 1, ...), no worker has a mini-batch yet
        std::vector<int32_t> h(PlanView::words(P, s->S, Kcap), 0);
        TRY(s->plan.alloc(sizeof(int32_t) * h.size()));
        PlanView pl(h.data(), P, s->S, Kcap);
        pl.meta[0] = s->S;
        for (int i = 0; i < P; ++i) pl.wslot[i] = -1;
        for (int i = 0; i < s->S; ++i) pl.freel[i] = s->S - 1 - i;
        TRY(hipMemcpy(s->plan.p, h.data(), sizeof(int32_t) * h.size(), hipMemcpyHostToDevice));
        a.plan = (int32_t*)s->plan.p;
    }
    TRY(hipMemsetAsync(s->xb.p, 0, 2 * S * MP * a.d, stream));
    TRY(hipMemsetAsync(s->xbt.p, 0, 2 * S * MP * a.d, stream));
    TRY(hipMemsetAsync(s->hbuf.p, 0, sizeof(float) * S * MP * a.H, stream));
    TRY(hipMemsetAsync(s->d1t.p, 0, 2 * S * MP * a.H, stream));
    TRY(hipMemsetAsync(s->gb1.p, 0, sizeof(float) * S * 4 * a.H, stream));
    TRY(hipMemsetAsync(s->gw2.p, 0, sizeof(float) * S * 4 * a.C * a.H, stream));
    TRY(hipMemsetAsync(s->gb2.p, 0, sizeof(float) * S * 4 * 16, stream));
    TRY(hipMemsetAsync(s->loss.p, 0, sizeof(float) * S * 4, stream));
    TRY(hipMemsetAsync(s->ylab.p, 0xFF, sizeof(int32_t) * S * MP, stream));
    a.params = (float*)s->params.p; a.w1r = (unsigned short*)s->w1r.p; a.w2r = (float*)s->w2r.p;
    a.xb = (unsigned short*)s->xb.p; a.xbt = (unsigned short*)s->xbt.p; a.hbuf = (float*)s->hbuf.p;
    a.d1t = (unsigned short*)s->d1t.p; a.gb1 = (float*)s->gb1.p; a.gw2 = (float*)s->gw2.p; a.gb2 = (float*)s->gb2.p;
    a.loss = (float*)s->loss.p; a.ylab = (int32_t*)s->ylab.p; a.d2 = (float*)s->d2.p; a.quartered = (int32_t*)s->quartered.p;
    a.dw_part = (float*)s->dw_part.p; a.nsplit = 1; a.fsplit = 1; a.eval_base = -1;
    a.b1r = nullptr; a.b2r = nullptr; a.n_cons_inline = 0; a.n_rec_inline = 0;

    const float bound1 = (float)(1.0 / sqrt((double)a.d)), bound2 = (float)(1.0 / sqrt((double)a.H));
    hipLaunchKernelGGL(mlp_init_kernel, dim3(1024), dim3(256), 0, stream, a.params, seed, s->nw, n1, off2, n2, bound1, bound2);
    TRY(hipGetLastError());
    TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(mlp_contract_kernel<true, 128>), hipFuncAttributeMaxDynamicSharedMemorySize, (int)contract_lds(128)));
    TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(mlp_contract_kernel<true, 64>), hipFuncAttributeMaxDynamicSharedMemorySize, (int)contract_lds(64)));
    TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(mlp_contract_kernel<false, 64>), hipFuncAttributeMaxDynamicSharedMemorySize, (int)contract_lds(64)));
    TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(mlp_contract_kernel<false, 128, true>), hipFuncAttributeMaxDynamicSharedMemorySize, (int)contract_lds(128)));
    TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(mlp_mid_kernel), hipFuncAttributeMaxDynamicSharedMemorySize, (int)mid_lds_bytes(1024)));
    TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(mlp_fwd_gather_kernel<128, false>), hipFuncAttributeMaxDynamicSharedMemorySize, (int)contract_lds(128)));
    TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(mlp_fwd_gather_kernel<64, true>), hipFuncAttributeMaxDynamicSharedMemorySize, (int)contract_lds(64)));
    TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(mlp_fwd_gather_kernel<64, false>), hipFuncAttributeMaxDynamicSharedMemorySize, (int)contract_lds(64)));
#undef TRY
    *out = s;
    return hipSuccess;
}

namespace {

// this replica's rows of the trace
Trace trace_of(const Trace& tr, int r) {
    Trace t = tr;
    t.t += (int64_t)r * tr.cap; t.loss += (int64_t)r * tr.cap; t.K += (int64_t)r * tr.cap;
    t.sel += (int64_t)r * tr.cap * tr.Kcap; t.tau += (int64_t)r * tr.cap * tr.Kcap; t.ord += (int64_t)r * tr.cap * tr.Kcap;
    return t;
}

// few records start at this version: the forward pass splits the depth d over workgroups
bool few_records(const MlpArgs& a, int nrec, int regions) {
    return nrec > 0 && nrec <= kSmallRec && nrec * (a.H / 64) <= 256 && a.H <= 1024 &&
           (int64_t)regions * nrec * MP * a.H * 8 <= (int64_t)kMaxSplit * a.H * a.d;
}
int few_records_split(const MlpArgs& a, int nrec) { return std::max(2, std::min(8, 512 / (nrec * (a.H / 64)))); }

// The launches of one update (a.v, a.Kv, a.nrec set), in two halves.  Forward half: the mini-batches that start at
// version v, up to delta1 and the second-layer gradient records of their slots.
void launch_forward(MlpArgs& a, hipStream_t stream, hipEvent_t done = nullptr) {
    if (a.variant == kBatchAsync) hipLaunchKernelGGL(mlp_batch_plan_kernel, dim3(1), dim3(64), 0, stream, a);
    if (few_records(a, a.nrec, 1)) {
        // few records: two launches; the depth is split so that two workgroups share every CU and none walks all of d
        a.fsplit = few_records_split(a, a.nrec);
        hipLaunchKernelGGL((mlp_fwd_gather_kernel<64, true>), dim3(a.nrec, a.H / 64, a.fsplit), dim3(256), contract_lds(64), stream, a);
        hipExtLaunchKernelGGL(mlp_mid_kernel, dim3(a.nrec * 4), dim3(256), mid_lds_bytes(a.H), stream, nullptr, done, 0, a);
    } else if (a.nrec > 0 && ((a.nrec + 1) / 2) * (a.H / 128) >= 192) {
        // many records: large tiles, the rows again straight from the sample matrix
        hipLaunchKernelGGL((mlp_fwd_gather_kernel<128, false>), dim3((a.nrec + 1) / 2, a.H / 128), dim3(256), contract_lds(128), stream, a);
        hipLaunchKernelGGL(mlp_output_kernel, dim3(a.nrec), dim3(256), 0, stream, a);
        hipExtLaunchKernelGGL(mlp_delta1_kernel, dim3(a.nrec, a.H / 64), dim3(256), 0, stream, nullptr, done, 0, a);
    } else if (a.nrec > 0) {
        // in between: small tiles (the large ones would not fill the chip), the whole depth per workgroup
        hipLaunchKernelGGL((mlp_fwd_gather_kernel<64, false>), dim3(a.nrec, a.H / 64), dim3(256), contract_lds(64), stream, a);
        hipLaunchKernelGGL(mlp_output_kernel, dim3(a.nrec), dim3(256), 0, stream, a);
        hipExtLaunchKernelGGL(mlp_delta1_kernel, dim3(a.nrec, a.H / 64), dim3(256), 0, stream, nullptr, done, 0, a);
    }
}
// Backward half: the first-layer gradient over the consumed slots and the update of every parameter.
// (done: an event that the completion of the last launch records by itself, without an entry of its own in the stream)
void launch_backward(MlpArgs& a, hipStream_t stream, hipEvent_t done = nullptr) {
    if (a.Kv >= 32) {
        // many slots: 128 x 128 tiles (half the operand traffic of the small ones), the slots split into shares so
        // that the chip is still full; the shares are added, in order, by the update kernel
        // (as many shares as keep all workgroups resident at once, two per CU on 256 CUs: a second, partial round of
        // workgroups costs more than the shorter shares gain)
        const int tiles = (a.H / 128) * (a.d / 128);
        a.nsplit = std::max(1, std::min({kMaxSplit, a.Kv / 8, 512 / tiles}));
        hipLaunchKernelGGL((mlp_contract_kernel<false, 128, true>), dim3((a.H / 128) * 8 * (((a.d / 128) * a.nsplit + 7) / 8)), dim3(256), contract_lds(128), stream, a);
        hipExtLaunchKernelGGL(mlp_w1_update_kernel, dim3(kW1Blocks + kSmallBlocks16), dim3(256), 0, stream, nullptr, done, 0, a);
    } else {
        // small tiles: 384 workgroups instead of 96 matter more than the reuse inside a larger tile; one more row of
        // workgroups takes the small parameters
        hipExtLaunchKernelGGL((mlp_contract_kernel<false, 64>), dim3(a.H / 64, a.d / 64 + 1), dim3(256), contract_lds(64), stream, nullptr, done, 0, a);
    }
}
void launch_update(MlpArgs& a, hipStream_t stream) {
    launch_forward(a, stream);
    launch_backward(a, stream);
}

}  // namespace

// Updates [v0, v0 + n) of every replica.  The replicas are independent runs: replica r's launches go to a stream of
// its own (created here, default priority), update by update in turn, so that the latency chains of the replicas'
// small kernels overlap on the device; the streams start after everything queued on `stream` and `stream` waits for them.
hipError_t mlp_run_segment(MlpState* const* states, int R, const Trace& tr, const WorkerState& ws, int64_t v0, int64_t n,
                           float* agg_out, hipStream_t stream, double* ms_accum, int64_t* launches, std::string* msg,
                           const MlpPieces* pieces) {
    auto fail = [&](hipError_t e, const char* what) { if (msg) *msg = what; return e; };
    if (pieces != nullptr && (R != 1 || pieces->count < 1 || pieces->len < 1 || pieces->count * pieces->len < n))
        return fail(hipErrorInvalidValue, "pieces of a segment: one replica, and they cover the segment");
    std::vector<MlpArgs> args((size_t)R);
    std::vector<std::vector<int32_t>> Ks((size_t)R, std::vector<int32_t>((size_t)n));
    std::vector<int32_t> prevK((size_t)R, 0);
    hipError_t e = hipSuccess;
    for (int r = 0; r < R && e == hipSuccess; ++r) {
        MlpState* s = states[r];
        MlpArgs& a = args[(size_t)r];
        a = s->a;
        a.tr = trace_of(tr, r);
        a.agg_out = r == 0 ? agg_out : nullptr;
        const int64_t n1 = (int64_t)a.H * a.d, off2 = n1 + a.H, n2 = (int64_t)a.C * a.H;
        // the parameters may have been set from outside since the last segment
        hipLaunchKernelGGL(mlp_refresh_kernel, dim3(1024), dim3(256), 0, stream, a.params, a.w1r, a.w2r, n1, off2, n2);
        // K is constant inside a segment; it is read back once (or comes piece by piece, see below)
        if (pieces == nullptr) e = hipMemcpyAsync(Ks[(size_t)r].data(), a.tr.K + v0, sizeof(int32_t) * n, hipMemcpyDeviceToHost, stream);
        if (e == hipSuccess && a.variant == kAsync && v0 > 0)
            e = hipMemcpyAsync(&prevK[(size_t)r], a.tr.K + (v0 - 1), sizeof(int32_t), hipMemcpyDeviceToHost, stream);
        if (r > 0 && s->own == nullptr && e == hipSuccess) e = hipStreamCreateWithFlags(&s->own, hipStreamNonBlocking);
    }
    // the versions of the consumed gradients, where updates may overlap (below)
    std::vector<int32_t> tau_host, sel_host;
    int64_t sel_first = 0;
    if (pieces != nullptr) {
        tau_host.resize((size_t)(n * tr.Kcap));
        sel_host.resize((size_t)((n + 1) * tr.Kcap));
        sel_first = v0 - 1;
    } else if (R == 1 && args[0].variant == kAsync && agg_out == nullptr && e == hipSuccess) {
        tau_host.resize((size_t)(n * tr.Kcap));
        e = hipMemcpyAsync(tau_host.data(), args[0].tr.tau + v0 * tr.Kcap, sizeof(int32_t) * tau_host.size(), hipMemcpyDeviceToHost, stream);
        // ... and who they came from, one row more in front (the mini-batches that start at v0 are those of update v0 - 1)
        const int64_t first = v0 > 0 ? v0 - 1 : 0;
        sel_host.resize((size_t)((v0 + n - first) * tr.Kcap));
        sel_first = first;
        if (e == hipSuccess)
            e = hipMemcpyAsync(sel_host.data(), args[0].tr.sel + first * tr.Kcap, sizeof(int32_t) * sel_host.size(), hipMemcpyDeviceToHost, stream);
    }
    if (e == hipSuccess) e = hipStreamSynchronize(stream);
    if (e != hipSuccess) return fail(e, "reading K of the segment");
    hipEvent_t e0 = nullptr, e1 = nullptr, fork = nullptr;
    (void)hipEventCreate(&e0); (void)hipEventCreate(&e1);
    (void)hipEventCreateWithFlags(&fork, hipEventDisableTiming);
    auto drop = [&]() { (void)hipEventDestroy(e0); (void)hipEventDestroy(e1); (void)hipEventDestroy(fork); };
    (void)hipEventRecord(e0, stream);
    (void)hipEventRecord(fork, stream);
    for (int r = 1; r < R; ++r) (void)hipStreamWaitEvent(states[r]->own, fork, 0);
    // the K of every update is checked before anything of it is launched
    auto valid_K = [&](int r, int64_t qa, int64_t qb) {
        const MlpArgs& a = args[(size_t)r];
        const std::vector<int32_t>& K = Ks[(size_t)r];
        for (int64_t q = qa; q < qb; ++q) {
            const int64_t v = v0 + q;
            int nrec = (a.variant == kAsync) ? (v == 0 ? a.P : (q == 0 ? prevK[(size_t)r] : K[(size_t)q - 1])) : K[(size_t)q];
            if (a.variant == kBatchAsync) nrec = (v == 0 ? a.P : 1) + K[(size_t)q] - 1;
            if (K[(size_t)q] < 1 || K[(size_t)q] > a.Kcap || nrec < 0 || nrec > states[r]->S) return false;
        }
        return true;
    };
    // Pieces: the rows of piece k are taken from the pinned copies once its event has happened.  avail = number of
    // updates of the segment whose rows are here (all of them without pieces).
    int64_t avail = pieces ? 0 : n;
    int pieces_taken = 0;
    int nrec_cap = 0;            // set by the overlapped path: the most records its forward buffers hold
    auto take_piece = [&]() -> hipError_t {
        const int k = pieces_taken;
        const hipError_t pe = hipEventSynchronize(pieces->ready[k]);
        if (pe != hipSuccess) return pe;
        const int64_t qa = (int64_t)k * pieces->len, qb = std::min<int64_t>(n, qa + pieces->len);
        const size_t W = (size_t)tr.Kcap;
        std::memcpy(Ks[0].data() + qa, pieces->K + qa, sizeof(int32_t) * (size_t)(qb - qa));
        std::memcpy(tau_host.data() + (size_t)qa * W, pieces->tau + (size_t)qa * W, sizeof(int32_t) * (size_t)(qb - qa) * W);
        const int64_t ra = k == 0 ? 0 : qa + 1;     // rows of the copy of sel: one in front
        std::memcpy(sel_host.data() + (size_t)ra * W, pieces->sel + (size_t)ra * W, sizeof(int32_t) * (size_t)(qb + 1 - ra) * W);
        if (!valid_K(0, qa, qb)) return hipErrorInvalidValue;
        if (nrec_cap > 0)
            for (int64_t q = qa; q < qb; ++q) {
                const int nr = (v0 + q == 0) ? args[0].P : (q == 0 ? prevK[0] : Ks[0][(size_t)q - 1]);
                if (args[0].variant == kAsync && few_records(args[0], nr, 1) && nr > nrec_cap) return hipErrorInvalidValue;
            }
        ++pieces_taken;
        avail = qb;
        return hipSuccess;
    };
    if (pieces) {
        const hipError_t pe = take_piece();
        if (pe != hipSuccess) { drop(); return fail(pe, "the first piece of the schedule"); }
    } else {
        for (int r = 0; r < R; ++r)
            if (!valid_K(r, 0, n)) { drop(); return fail(hipErrorInvalidValue, "inconsistent K in the trace"); }
    }
    auto nrec_of = [&](int r, int64_t q) {
        const MlpArgs& a = args[(size_t)r];
        const std::vector<int32_t>& K = Ks[(size_t)r];
        if (a.variant == kBatchAsync) return (v0 + q == 0 ? a.P : 1) + K[(size_t)q] - 1;
        if (a.variant == kAsync) return v0 + q == 0 ? a.P : (q == 0 ? prevK[(size_t)r] : K[(size_t)q - 1]);
        return K[(size_t)q];
    };
    // One K-async run: the two halves of an update overlap with those of its neighbours.  The gradients that update v
    // consumes were computed at versions tau <= v (Sec. 2.2), with few gradients per update many updates ago, so the
    // backward half of v (which gives w_{v+1}) needs the backward half of v - 1 and the forward halves of the versions in
    // its list, not the forward half of v itself unless the list names it; that one needs w_v only.  The backward halves
    // follow each other on `stream`; the forward halves of consecutive versions go to kFwdStreams streams in turn, each fed
    // by a host thread of its own (the host's calls, not the device, would otherwise set the pace).
    // The operand copies of the parameters (bf16 W1, rounded W2, the biases) and the partial sums of the split forward
    // pass exist kVer times, indexed by version modulo kVer: the update of v writes the copies of v + 1 after the
    // forward half of v + 1 - kVer, their last reader, has ended.  (With K near P most lists name the version itself and
    // the halves run one after the other as they would on one stream.)
    // (worth it where at most a quarter of the lists of the segment name their own version)
    int64_t q0 = n;
    if (tau_host.size() == (size_t)(n * tr.Kcap) && n >= 4 && args[0].variant == kAsync && agg_out == nullptr) {
        int64_t own = 0;
        for (int64_t q = 0; q < avail; ++q) {
            bool names_itself = false;
            for (int l = 0; l < Ks[0][(size_t)q]; ++l) names_itself |= tau_host[(size_t)(q * tr.Kcap + l)] >= (int32_t)(v0 + q);
            own += names_itself ? 1 : 0;
        }
        if (4 * own <= avail) q0 = 0;
    }
    if (q0 < n) {
        // the updates before q0
        for (int64_t q = 0; q < q0; ++q) {
            MlpArgs& a = args[0];
            a.v = v0 + q; a.Kv = Ks[0][(size_t)q]; a.nrec = nrec_of(0, q);
            launch_update(a, stream);
        }
        MlpState* s = states[0];
        const MlpArgs& base = args[0];
        const int64_t n1 = (int64_t)base.H * base.d, off2 = n1 + base.H, n2 = (int64_t)base.C * base.H;
        int nrec_max = 1;
        // (K does not change inside a segment: the pieces still to come start no more records than these)
        for (int64_t q = q0; q < avail; ++q)
            if (few_records(base, nrec_of(0, q), 1)) nrec_max = std::max(nrec_max, nrec_of(0, q));
        nrec_cap = nrec_max;
        const int64_t region = (int64_t)8 * nrec_max * MP * base.H;
        hipError_t oe = hipSuccess;
        for (hipStream_t& f : s->fwd_stream)
            if (f == nullptr && oe == hipSuccess) oe = hipStreamCreateWithFlags(&f, hipStreamNonBlocking);
        constexpr int kRing = 32;
        while (s->ev_pool.size() < 2 * kRing + 1 && oe == hipSuccess) {
            hipEvent_t ev = nullptr;
            oe = hipEventCreateWithFlags(&ev, hipEventDisableTiming);
            if (oe == hipSuccess) s->ev_pool.push_back(ev);
        }
        if (s->w1v.p == nullptr && oe == hipSuccess) {
            oe = s->w1v.alloc(2 * kVer * (size_t)n1);
            if (oe == hipSuccess) oe = s->w2v.alloc(sizeof(float) * kVer * (size_t)n2);
            if (oe == hipSuccess) oe = s->b1v.alloc(sizeof(float) * kVer * (size_t)base.H);
            if (oe == hipSuccess) oe = s->b2v.alloc(sizeof(float) * kVer * 16);
        }
        if (s->fwd_part.bytes < sizeof(float) * kVer * (size_t)region && oe == hipSuccess) {
            // (nothing of an earlier segment still uses the smaller one: every segment ends with a wait for its streams)
            s->fwd_part.release();
            oe = s->fwd_part.alloc(sizeof(float) * kVer * (size_t)region);
        }
        int dev = 0;
        if (oe == hipSuccess) oe = hipGetDevice(&dev);
        if (oe != hipSuccess) { drop(); return fail(oe, "streams, events and buffers of the overlapped updates"); }
        auto ev_upd = [&](int64_t v) { return s->ev_pool[(size_t)(v % kRing)]; };            // contraction and update of v done
        auto ev_fwd = [&](int64_t v) { return s->ev_pool[(size_t)(kRing + v % kRing)]; };    // forward half of v done
        auto versioned = [&](MlpArgs& a, int64_t ver) {
            const int k = (int)(ver % kVer);
            a.w1r = (unsigned short*)s->w1v.p + (int64_t)k * n1;
            a.w2r = (float*)s->w2v.p + (int64_t)k * n2;
            a.b1r = (float*)s->b1v.p + (int64_t)k * base.H;
            a.b2r = (float*)s->b2v.p + (int64_t)k * 16;
        };
        const int64_t vs = v0 + q0;  // the first overlapped update
        // short lists travel in the kernel arguments
        auto inline_lists = [&](MlpArgs& a, int64_t v, int Kv, int nrec) {
            a.n_cons_inline = 0; a.n_rec_inline = 0;
            if (Kv <= 32) {
                a.n_cons_inline = Kv;
                for (int l = 0; l < Kv; ++l) a.cons_inline[l] = (int16_t)sel_host[(size_t)((v - sel_first) * tr.Kcap + l)];
            }
            if (v >= 1 && nrec <= 32) {
                a.n_rec_inline = nrec;
                for (int r = 0; r < nrec; ++r) a.rec_inline[r] = (int16_t)sel_host[(size_t)((v - 1 - sel_first) * tr.Kcap + r)];
            }
        };
        // the copies of version vs
        {
            MlpArgs a = base;
            versioned(a, vs);
            hipLaunchKernelGGL(mlp_refresh_kernel, dim3(1024), dim3(256), 0, stream, a.params, a.w1r, a.w2r, n1, off2, n2);
            (void)hipMemcpyAsync(a.b1r, a.params + n1, sizeof(float) * base.H, hipMemcpyDeviceToDevice, stream);
            (void)hipMemcpyAsync(a.b2r, a.params + off2 + n2, sizeof(float) * base.C, hipMemcpyDeviceToDevice, stream);
        }
        hipEvent_t start = s->ev_pool[2 * kRing];
        (void)hipEventRecord(start, stream);
        // what the host threads tell each other: an event may be waited for only after the call that records it
        std::atomic<int64_t> upd_recorded{vs - 1};                 // ev_upd of every version up to here has been recorded
        std::atomic<int64_t> fwd_recorded[kFwdStreams];                      // per forward stream: its newest version with ev_fwd recorded
        for (auto& f : fwd_recorded) f.store(-1);
        std::atomic<int> thread_error{0};
        auto forward_half = [&](int k) {
            if (hipSetDevice(dev) != hipSuccess) { thread_error.store((int)hipErrorInvalidDevice); return; }
            hipStream_t fs = s->fwd_stream[k];
            for (int64_t q = q0; q < n; ++q) {
                const int64_t v = v0 + q;
                if ((int)(v % kFwdStreams) != k) continue;
                while (upd_recorded.load(std::memory_order_acquire) < v - 1) {
                    if (thread_error.load(std::memory_order_relaxed) != 0) return;
                }
                MlpArgs f = base;
                f.v = v; f.Kv = Ks[0][(size_t)q]; f.nrec = nrec_of(0, q);
                versioned(f, v);
                f.dw_part = (float*)s->fwd_part.p + (v % kVer) * region;
                inline_lists(f, v, f.Kv, f.nrec);
                // (asked for on the host until it has happened: making the stream wait for an event that has not happened yet
                // is the most expensive call there is here, 12 us, and a waiting entry holds up the kernels of the other
                // streams that share its hardware queue)
                for (;;) {
                    const hipError_t qe = hipEventQuery(q == q0 ? start : ev_upd(v - 1));
                    if (qe == hipSuccess) break;
                    (void)hipGetLastError();
                    // anything but "not ready" is an error of the device: nobody waits for an event that will not come
                    if (qe != hipErrorNotReady) { thread_error.store((int)qe); return; }
                    if (thread_error.load(std::memory_order_relaxed) != 0) return;
                }
                launch_forward(f, fs, f.nrec > 0 ? ev_fwd(v) : nullptr);
                const hipError_t fe = f.nrec > 0 ? hipSuccess : hipEventRecord(ev_fwd(v), fs);
                const hipError_t le = hipGetLastError();
                if (fe != hipSuccess || le != hipSuccess) { thread_error.store((int)(fe != hipSuccess ? fe : le)); return; }
                fwd_recorded[k].store(v, std::memory_order_release);
            }
        };
        std::thread feeders[kFwdStreams];
        // (a thread that cannot be started must not throw through the C boundary above: the ones that run are told to stop)
        try {
            for (int k = 0; k < kFwdStreams; ++k) feeders[k] = std::thread(forward_half, k);
        } catch (...) {
            thread_error.store((int)hipErrorOutOfMemory);
        }
        int64_t waited = vs - 1;     // the contractions have waited for the forward halves of every version up to here
        auto wait_forward = [&](int64_t t) {
            while (fwd_recorded[t % kFwdStreams].load(std::memory_order_acquire) < t)
                if (thread_error.load(std::memory_order_relaxed) != 0) return;
            // (an event that has already happened needs no entry in the stream)
            if (hipEventQuery(ev_fwd(t)) != hipSuccess) {
                (void)hipGetLastError();   // "not ready" is no error of this thread's launches, which are checked one by one
                (void)hipStreamWaitEvent(stream, ev_fwd(t), 0);
            }
        };
        for (int64_t q = q0; q < n && thread_error.load() == 0; ++q) {
            const int64_t v = v0 + q;
            const int Kv = Ks[0][(size_t)q];
            // contraction and update of v: after the forward halves of every version in its list, and of v + 1 - kVer
            int64_t need = v + 1 - kVer;
            for (int l = 0; l < Kv; ++l) need = std::max<int64_t>(need, tau_host[(size_t)(q * tr.Kcap + l)]);
            need = std::min(need, v);
            for (int64_t t = std::max(waited + 1, vs); t <= need; ++t) wait_forward(t);
            waited = std::max(waited, need);
            MlpArgs u = base;
            u.v = v; u.Kv = Kv; u.nrec = nrec_of(0, q);
            versioned(u, v + 1);
            inline_lists(u, v, u.Kv, u.nrec);
            launch_backward(u, stream, ev_upd(v));
            const hipError_t le = hipGetLastError();
            const hipError_t re = hipSuccess;
            if (le != hipSuccess || re != hipSuccess) { thread_error.store((int)(le != hipSuccess ? le : re)); break; }
            // the rows of the next update are here before anybody is told that this one has been launched
            if (q + 1 < n && q + 1 >= avail) {
                const hipError_t pe = take_piece();
                if (pe != hipSuccess) { thread_error.store((int)pe); break; }
            }
            upd_recorded.store(v, std::memory_order_release);
        }
        for (std::thread& f : feeders) if (f.joinable()) f.join();
        if (thread_error.load() == 0)
            for (int64_t t = std::max(waited + 1, vs); t < v0 + n; ++t) (void)hipStreamWaitEvent(stream, ev_fwd(t), 0);
        if (thread_error.load() != 0) {
            for (hipStream_t f : s->fwd_stream) (void)hipStreamSynchronize(f);
            (void)hipStreamSynchronize(stream);
            drop();
            return fail((hipError_t)thread_error.load(), "launching the overlapped updates");
        }
    }
    // update by update, the replicas in turn: nothing in one replica's launches depends on another's.  (Launching every
    // replica from a host thread of its own gave the same rate: the device, not the host, is what limits it.)
    for (int64_t q = 0; q < n && q0 == n; ++q) {
        if (q >= avail) {
            const hipError_t pe = take_piece();
            if (pe != hipSuccess) {
                (void)hipStreamSynchronize(stream);
                drop();
                return fail(pe, "a piece of the schedule");
            }
        }
        for (int r = 0; r < R; ++r) {
            MlpArgs& a = args[(size_t)r];
            const std::vector<int32_t>& K = Ks[(size_t)r];
            a.v = v0 + q;
            a.Kv = K[(size_t)q];
            a.nrec = (a.variant == kAsync) ? (a.v == 0 ? a.P : (q == 0 ? prevK[(size_t)r] : K[(size_t)q - 1])) : a.Kv;
            if (a.variant == kBatchAsync) a.nrec = (a.v == 0 ? a.P : 1) + a.Kv - 1;
            launch_update(a, r == 0 ? stream : states[r]->own);
        }
    }
    if (launches) *launches += n;
    // the first replica's stream waits for the others
    for (int r = 1; r < R; ++r) {
        hipEvent_t done = nullptr;
        if (hipEventCreateWithFlags(&done, hipEventDisableTiming) == hipSuccess) {
            (void)hipEventRecord(done, states[r]->own);
            (void)hipStreamWaitEvent(stream, done, 0);
            (void)hipEventDestroy(done);
        }
    }
    (void)hipEventRecord(e1, stream);
    e = hipStreamSynchronize(stream);
    float ms = 0.0f;
    if (e == hipSuccess && hipEventElapsedTime(&ms, e0, e1) == hipSuccess && ms_accum) *ms_accum += ms;
    drop();
    if (e != hipSuccess) return fail(e, "running the segment");
    e = hipGetLastError();
    if (e != hipSuccess) return fail(e, "launching the segment");
    for (int r = 0; r < R; ++r) {
        if (args[(size_t)r].variant != kBatchAsync) continue;
        int32_t meta[4] = {0, 0, 0, 0};
        e = hipMemcpy(meta, args[(size_t)r].plan, sizeof(meta), hipMemcpyDeviceToHost);
        if (e != hipSuccess) return fail(e, "reading the slot plan");
        if (meta[2] != 0) return fail(hipErrorInvalidValue, "the slot pool of K-batch-async ran dry: inconsistent trace");
    }
    (void)ws;
    return hipSuccess;
}

// Objective over the whole data set with the forward pass of the trainer (bf16 operands in the first contraction,
// W2 at its bf16 values, fp32 accumulation): the data set goes through the gather, forward and output kernels in
// blocks of 64 rows per slot, into buffers of its own so that the mini-batches in flight are untouched; the
// per-slot sums are added on the host in fp64, in row order.
hipError_t mlp_full_loss(MlpState* s, double* out, hipStream_t stream, std::string* msg) {
    auto fail = [&](hipError_t e, const char* what) { if (msg) *msg = what; return e; };
    MlpArgs a = s->a;
    const int64_t N = (int64_t)a.N, nslot = (N + MP - 1) / MP;
    const int E = (int)std::min<int64_t>(nslot, 256);
    DevMem xb, hbuf, d2, loss, ylab;
    auto release = [&]() { xb.release(); hbuf.release(); d2.release(); loss.release(); ylab.release(); };
    hipError_t e = hipSuccess;
    if (e == hipSuccess) e = xb.alloc(2 * (size_t)E * MP * a.d);
    if (e == hipSuccess) e = hbuf.alloc(sizeof(float) * (size_t)E * MP * a.H);
    if (e == hipSuccess) e = d2.alloc(sizeof(float) * (size_t)E * MP * 16);
    if (e == hipSuccess) e = loss.alloc(sizeof(float) * (size_t)E * 4);
    if (e == hipSuccess) e = ylab.alloc(sizeof(int32_t) * (size_t)E * MP);
    if (e != hipSuccess) { release(); return fail(e, "allocating the evaluation buffers"); }
    a.xb = (unsigned short*)xb.p; a.xbt = nullptr; a.hbuf = (float*)hbuf.p; a.d2 = (float*)d2.p;
    a.loss = (float*)loss.p; a.ylab = (int32_t*)ylab.p;
    a.d1t = nullptr; a.gb1 = nullptr; a.gw2 = nullptr; a.gb2 = nullptr; a.agg_out = nullptr;
    a.m = MP; a.v = 0; a.Kv = 1;
    const int64_t n1 = (int64_t)a.H * a.d, off2 = n1 + a.H, n2 = (int64_t)a.C * a.H;
    hipLaunchKernelGGL(mlp_refresh_kernel, dim3(1024), dim3(256), 0, stream, a.params, a.w1r, a.w2r, n1, off2, n2);
    std::vector<float> h((size_t)E * 4);
    double total = 0.0;
    for (int64_t s0 = 0; s0 < nslot && e == hipSuccess; s0 += E) {
        a.eval_base = s0 * MP;
        a.nrec = (int)std::min<int64_t>(E, nslot - s0);
        hipLaunchKernelGGL(mlp_gather_kernel, dim3(a.nrec, a.d / 128), dim3(256), 0, stream, a);
        if (((a.nrec + 1) / 2) * (a.H / 128) >= 192)
            hipLaunchKernelGGL((mlp_contract_kernel<true, 128>), dim3((a.nrec + 1) / 2, a.H / 128), dim3(256), contract_lds(128), stream, a);
        else
            hipLaunchKernelGGL((mlp_contract_kernel<true, 64>), dim3(a.nrec, a.H / 64), dim3(256), contract_lds(64), stream, a);
        hipLaunchKernelGGL(mlp_output_kernel, dim3(a.nrec), dim3(256), 0, stream, a);
        e = hipGetLastError();
        if (e == hipSuccess) e = hipMemcpyAsync(h.data(), a.loss, sizeof(float) * a.nrec * 4, hipMemcpyDeviceToHost, stream);
        if (e == hipSuccess) e = hipStreamSynchronize(stream);
        if (e == hipSuccess) for (int q = 0; q < a.nrec; ++q) total += (double)h[(size_t)q * 4];
    }
    release();
    if (e != hipSuccess) return fail(e, "evaluating the objective");
    *out = total / (double)N;
    return hipSuccess;
}


// Gradient of the objective over the whole data set, with the arithmetic of the trainer's gradients (bf16 operands in
// the two large contractions, fp32 accumulation): the data set goes through the training kernels in blocks of up to
// 256 slots of 64 rows, each block as one "update" that consumes all its slots with a step size of zero, so that the
// parameters keep their values and the block's averaged gradient lands in a device buffer; the blocks are added on the
// host in fp64; rows left over after the last whole slot form a mini-batch of their own size.  Buffers of its own, so
// that the mini-batches in flight stay untouched.
hipError_t mlp_full_gradient(MlpState* s, float* grad_out_host, hipStream_t stream, std::string* msg) {
    auto fail = [&](hipError_t e, const char* what) { if (msg) *msg = what; return e; };
    MlpArgs a = s->a;
    const int64_t N = (int64_t)a.N, nslot = (N + MP - 1) / MP;
    const size_t E = (size_t)std::min<int64_t>(nslot, 256);
    DevMem xb, xbt, hbuf, d1t, gb1, gw2, gb2, d2, loss, ylab, quart, agg, tloss;
    DevMem* all[] = {&xb, &xbt, &hbuf, &d1t, &gb1, &gw2, &gb2, &d2, &loss, &ylab, &quart, &agg, &tloss};
    auto release = [&]() { for (DevMem* b : all) b->release(); };
    const size_t sizes[] = {2 * E * MP * a.d, 2 * E * MP * a.d, sizeof(float) * E * MP * a.H, 2 * E * MP * a.H,
                            sizeof(float) * E * 4 * a.H, sizeof(float) * E * 4 * a.C * a.H, sizeof(float) * E * 4 * 16,
                            sizeof(float) * E * MP * 16, sizeof(float) * E * 4, sizeof(int32_t) * E * MP, sizeof(int32_t) * E,
                            sizeof(float) * (size_t)s->nw, sizeof(float) * 16};
    hipError_t e = hipSuccess;
    for (size_t q = 0; q < sizeof(all) / sizeof(all[0]) && e == hipSuccess; ++q) e = all[q]->alloc(sizes[q]);
    if (e != hipSuccess) { release(); return fail(e, "allocating the evaluation buffers"); }
    a.xb = (unsigned short*)xb.p; a.xbt = (unsigned short*)xbt.p; a.hbuf = (float*)hbuf.p; a.d1t = (unsigned short*)d1t.p;
    a.gb1 = (float*)gb1.p; a.gw2 = (float*)gw2.p; a.gb2 = (float*)gb2.p; a.d2 = (float*)d2.p; a.loss = (float*)loss.p;
    a.ylab = (int32_t*)ylab.p; a.quartered = (int32_t*)quart.p; a.agg_out = (float*)agg.p;
    a.tr.loss = (float*)tloss.p;       // the loss record of the pretended update goes nowhere
    a.m = MP; a.v = 0; a.lr = 0.0f; a.variant = kSync; a.S = (int32_t)E;
    const int64_t n1 = (int64_t)a.H * a.d, off2 = n1 + a.H, n2 = (int64_t)a.C * a.H;
    hipLaunchKernelGGL(mlp_refresh_kernel, dim3(1024), dim3(256), 0, stream, a.params, a.w1r, a.w2r, n1, off2, n2);
    std::vector<float> h((size_t)s->nw);
    std::vector<double> total((size_t)s->nw, 0.0);
    // whole slots in blocks; the rows that are left over (fewer than 64) as a mini-batch of their own size, so that
    // delta1 is scaled and rounded as in a mini-batch of that size
    const int64_t nfull = N / MP;
    struct Block { int64_t slot0; int nrec, m; };
    std::vector<Block> blocks;
    for (int64_t s0 = 0; s0 < nfull; s0 += (int64_t)E) blocks.push_back({s0, (int)std::min<int64_t>((int64_t)E, nfull - s0), MP});
    if (nfull * MP < N) blocks.push_back({nfull, 1, (int)(N - nfull * MP)});
    for (const Block& blk : blocks) {
        if (e != hipSuccess) break;
        a.eval_base = blk.slot0 * MP;
        a.nrec = blk.nrec;
        a.m = blk.m;
        a.Kv = a.nrec;
        hipLaunchKernelGGL(mlp_gather_kernel, dim3(a.nrec, a.d / 128), dim3(256), 0, stream, a);
        if (((a.nrec + 1) / 2) * (a.H / 128) >= 192)
            hipLaunchKernelGGL((mlp_contract_kernel<true, 128>), dim3((a.nrec + 1) / 2, a.H / 128), dim3(256), contract_lds(128), stream, a);
        else
            hipLaunchKernelGGL((mlp_contract_kernel<true, 64>), dim3(a.nrec, a.H / 64), dim3(256), contract_lds(64), stream, a);
        hipLaunchKernelGGL(mlp_output_kernel, dim3(a.nrec), dim3(256), 0, stream, a);
        hipLaunchKernelGGL(mlp_delta1_kernel, dim3(a.nrec, a.H / 64), dim3(256), 0, stream, a);
        if (a.Kv >= 32) {
            const int tiles = (a.H / 128) * (a.d / 128);
            a.nsplit = std::max(1, std::min({kMaxSplit, a.Kv / 8, 512 / tiles}));
            hipLaunchKernelGGL((mlp_contract_kernel<false, 128, true>), dim3((a.H / 128) * 8 * (((a.d / 128) * a.nsplit + 7) / 8)), dim3(256), contract_lds(128), stream, a);
            hipLaunchKernelGGL(mlp_w1_update_kernel, dim3(kW1Blocks + kSmallBlocks16), dim3(256), 0, stream, a);
        } else {
            hipLaunchKernelGGL((mlp_contract_kernel<false, 64>), dim3(a.H / 64, a.d / 64 + 1), dim3(256), contract_lds(64), stream, a);
        }
        e = hipGetLastError();
        if (e == hipSuccess) e = hipMemcpyAsync(h.data(), a.agg_out, sizeof(float) * (size_t)s->nw, hipMemcpyDeviceToHost, stream);
        if (e == hipSuccess) e = hipStreamSynchronize(stream);
        // the block's gradient is the mean over its Kv slots of the slots' means over their rows
        const double wgt = (double)a.Kv * (double)a.m;
        if (e == hipSuccess) for (size_t q = 0; q < h.size(); ++q) total[q] += (double)h[q] * wgt;
    }
    release();
    if (e != hipSuccess) return fail(e, "evaluating the gradient of the objective");
    for (size_t q = 0; q < h.size(); ++q) grad_out_host[q] = (float)(total[q] / (double)N);
    return hipSuccess;
}

// Everything a later update depends on: parameters (fp32 master and operand copies) and the factors of the
// mini-batches in flight, slot by slot.
static std::vector<DevMem*> mlp_state_buffers(MlpState* s) {
    return {&s->params, &s->w1r, &s->w2r, &s->xb, &s->xbt, &s->hbuf, &s->d1t, &s->gb1, &s->gw2, &s->gb2, &s->d2, &s->loss,
            &s->ylab, &s->plan, &s->quartered};
}

int64_t mlp_state_bytes(MlpState* s) {
    int64_t n = 8;
    for (DevMem* b : mlp_state_buffers(s)) n += (int64_t)b->bytes;
    return n;
}

hipError_t mlp_get_state(MlpState* s, unsigned char* host) {
    const int64_t k = s->prevK;
    memcpy(host, &k, 8);
    size_t off = 8;
    for (DevMem* b : mlp_state_buffers(s)) {
        hipError_t e = hipMemcpy(host + off, b->p, b->bytes, hipMemcpyDeviceToHost);
        if (e != hipSuccess) return e;
        off += b->bytes;
    }
    return hipSuccess;
}

hipError_t mlp_set_state(MlpState* s, const unsigned char* host) {
    int64_t k = 0;
    memcpy(&k, host, 8);
    s->prevK = (int)k;
    size_t off = 8;
    for (DevMem* b : mlp_state_buffers(s)) {
        hipError_t e = hipMemcpy(b->p, host + off, b->bytes, hipMemcpyHostToDevice);
        if (e != hipSuccess) return e;
        off += b->bytes;
    }
    return hipSuccess;
}

float* mlp_params(MlpState* s) { return s ? (float*)s->params.p : nullptr; }

void mlp_destroy(MlpState* s) {
    if (!s) return;
    if (s->own) { (void)hipStreamSynchronize(s->own); (void)hipStreamDestroy(s->own); }
    for (hipStream_t& f : s->fwd_stream) if (f) { (void)hipStreamSynchronize(f); (void)hipStreamDestroy(f); }
    for (hipEvent_t ev : s->ev_pool) (void)hipEventDestroy(ev);
    DevMem* bufs[] = {&s->params, &s->w1r, &s->w2r, &s->xb, &s->xbt, &s->hbuf, &s->d1t, &s->gb1, &s->gw2, &s->gb2, &s->d2, &s->loss, &s->ylab,
                      &s->dw_part, &s->plan, &s->quartered, &s->w1v, &s->w2v, &s->b1v, &s->b2v, &s->fwd_part, &s->xb16};
    for (DevMem* b : bufs) b->release();
    delete s;
}

}  // namespace ssgd
