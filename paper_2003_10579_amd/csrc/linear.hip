// Mini-batch gradients of the linear models at possibly stale parameters, the
// K-gradient aggregate and the parameter-server update (Sec. 2.2, Eq. (2), Eq. (3)).
//
// One persistent launch runs a whole segment of updates.  Each replica is a
// "cluster" of G workgroups; workgroup s owns the column slice [s*SL, (s+1)*SL) of
// the sample matrix, of the weights and of every parked gradient, so the update
// and the staleness bookkeeping never leave the workgroup.  Per step v:
//   1. compute list of v (the mini-batches that start at parameter version v): gather
//      the rows into LDS, partial logits X_slice W_slice^T on the fp32 MFMA units;
//   2. one exchange of partial logits inside the cluster (arrival counter in HBM);
//   3. residual / softmax, then the gradient slice delta^T X_slice (MFMA) from the same
//      LDS tile, parked per slot (a K-async worker keeps it until it is selected);
//   4. update v: w -= (lr/K) sum over the consume list of update v.
// The schedule (who starts, who is consumed, K) was written by the schedule kernel.
#include "common.hpp"

namespace ssgd {
namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int ROWS = 64;   // rows of one LDS tile

struct ChunkMap {
    int n_rec, n_chunks, rpc, spr;
};

__device__ __forceinline__ ChunkMap chunk_map(int n_rec, int mp) {
    ChunkMap c;
    c.n_rec = n_rec;
    if (mp <= ROWS) { c.rpc = ROWS / mp; c.spr = 1; c.n_chunks = (n_rec + c.rpc - 1) / c.rpc; }
    else { c.rpc = 1; c.spr = (mp + ROWS - 1) / ROWS; c.n_chunks = n_rec * c.spr; }
    return c;
}

// The mini-batches that start at parameter version v, and the slot their gradient is parked in.
struct StepLists {
    int n_rec;        // compute list length
    int K;            // consume list length of update v
};

template <int NBW>
__global__ __launch_bounds__(64 * NBW) void linear_cluster_kernel(LinArgs a) {
    constexpr int SL = 64 * NBW;        // columns per workgroup
    constexpr int NT = 64 * NBW;        // threads
    constexpr int CPR = SL / 4;         // float4 chunks per tile row
    constexpr int RB = 4 / NBW;         // 16-row blocks per wave in the forward pass
    constexpr int LOADS = ROWS * CPR / NT;   // float4 loads per thread per tile (= 16)

    // cluster id / slice id from the block id: consecutive block ids go to different XCDs, so
    // all slices of one cluster take block ids that are congruent modulo 8 and share one L2.
    const int xcd = blockIdx.x & 7, slot_in_xcd = blockIdx.x >> 3;
    const int cluster = (slot_in_xcd / a.G) * 8 + xcd;
    const int slice = slot_in_xcd % a.G;
    if (cluster >= a.replicas) return;
    const int rep = a.replica0 + cluster;

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int d = a.d, C = a.C, m = a.m, mp = a.mp, P = a.P, S = a.S, G = a.G;
    const int Kcap = a.tr.Kcap;
    const int64_t cap = a.tr.cap;
    const int64_t nw = (a.kind == kLsq) ? d : (int64_t)C * d + C;
    const int col0 = slice * SL;

    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    float* tile = reinterpret_cast<float*>(smem);            // [64][SL], 16-byte chunks xor-swizzled by row
    float* wlds = tile + ROWS * SL;                          // [C][SL], same swizzle
    float* zbuf = wlds + C * SL;                             // [64][16] logits, then delta
    uint32_t* rowid = reinterpret_cast<uint32_t*>(zbuf + ROWS * 16);   // [64]
    float* ylab = reinterpret_cast<float*>(rowid + ROWS);    // [64] label (int bits) or target
    float* lossrow = ylab + ROWS;                            // [64]
    float* bias = lossrow + ROWS;                            // [16]
    float* small = bias + 16;                                // [S][17] bias gradient + loss per slot
    int* stop = reinterpret_cast<int*>(small + S * 17);      // [1] set when the cluster barrier gave up

    const int32_t* tr_K = a.tr.K + (int64_t)rep * cap;
    const int32_t* tr_sel = a.tr.sel + (int64_t)rep * cap * Kcap;
    const int32_t* tr_ord = a.tr.ord + (int64_t)rep * cap * Kcap;
    float* tr_loss = a.tr.loss + (int64_t)rep * cap;
    float* params = a.params + (int64_t)rep * nw;
    float* park = a.park + ((int64_t)rep * G + slice) * S * 16 * NT;
    float* small_g = a.park_small + ((int64_t)rep * G + slice) * S * 17;
    float* zpart = a.zpart + (int64_t)rep * 2 * G * a.maxrows * 16;
    unsigned long long* arrive = a.arrive + rep;
    const float inv_m = 1.0f / (float)m;
    const bool vec_ok = (d % 4) == 0;

    // ---- parameters owned by this thread: class 4*(lane/16)+v, column col0 + 64*wave + 4*(lane%16) + c
    float W[16];
    const int own_col = col0 + 64 * wave + 4 * (lane & 15);
    const int own_cls = 4 * (lane >> 4);
#pragma unroll
    for (int v = 0; v < 4; ++v)
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const int cls = own_cls + v, col = own_col + c;
            W[v * 4 + c] = (cls < C && col < d) ? params[(int64_t)cls * d + col] : 0.0f;
        }
    if (tid < 16) bias[tid] = (a.kind == kSoftmax && tid < C) ? params[(int64_t)C * d + tid] : 0.0f;
    for (int q = tid; q < S * 17; q += NT) small[q] = small_g[q];

    auto publish_weights = [&]() {
        // thread-owned values -> LDS in the layout the forward MFMA reads (class-major, swizzled)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int cls = own_cls + v;
            if (cls < C) {
                const int ch = 16 * wave + (lane & 15);
                f32x4 val = {W[v * 4 + 0], W[v * 4 + 1], W[v * 4 + 2], W[v * 4 + 3]};
                *reinterpret_cast<f32x4*>(wlds + cls * SL + ((ch ^ (cls & 15)) << 2)) = val;
            }
        }
    };
    publish_weights();
    if (tid == 0) *stop = __hip_atomic_load(a.abort_flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __syncthreads();
    if (*stop != 0) return;

    for (int64_t step = 0; step < a.nsteps; ++step) {
        const int64_t v = a.v0 + step;
        const int par = (int)((a.arrive_base + (unsigned long long)step) & 1ull);
        float* zp_mine = zpart + ((int64_t)par * G + slice) * a.maxrows * 16;
        const float* zp_all = zpart + (int64_t)par * G * a.maxrows * 16;

        // ---- lists of step v
        const int Kv = tr_K[v];
        int n_rec;
        if (a.variant == kAsync) n_rec = (v == 0) ? P : tr_K[v - 1];
        else n_rec = Kv;
        const ChunkMap cm = chunk_map(n_rec, mp);

        // record r of the compute list -> (worker, ordinal, slot)
        auto rec_worker = [&](int r) -> int {
            if (a.variant == kAsync) return (v == 0) ? r : tr_sel[(v - 1) * Kcap + r];
            return tr_sel[v * Kcap + r];
        };
        auto rec_ord = [&](int r) -> int { return (a.variant == kAsync) ? 0 : tr_ord[v * Kcap + r]; };
        auto rec_slot = [&](int r) -> int { return (a.variant == kAsync) ? rec_worker(r) : r; };

        auto stage_rows = [&](int chunk) {
            // sample id and label of every tile row (one thread per row)
            if (tid < ROWS) {
                int r, s;
                bool ok;
                if (mp <= ROWS) { r = chunk * cm.rpc + tid / mp; s = tid % mp; ok = tid < cm.rpc * mp && r < n_rec && s < m; }
                else { r = chunk / cm.spr; s = ROWS * (chunk % cm.spr) + tid; ok = s < m; }
                uint32_t id = 0xFFFFFFFFu;
                float lab = 0.0f;
                if (ok) {
                    id = batch_index(a.seed, (uint32_t)rep, (uint32_t)rec_worker(r), (uint32_t)rec_ord(r), (uint32_t)v,
                                     (uint32_t)s, a.N);
                    lab = (a.kind == kLsq) ? reinterpret_cast<const float*>(a.y)[id]
                                           : __int_as_float(reinterpret_cast<const int32_t*>(a.y)[id]);
                }
                rowid[tid] = id;
                ylab[tid] = lab;
            }
        };

        auto load_tile = [&]() {
            f32x4 buf[LOADS];
#pragma unroll
            for (int i = 0; i < LOADS; ++i) {
                const int e = tid + NT * i, row = e / CPR, ch = e % CPR;
                const uint32_t id = rowid[row];
                const int col = col0 + 4 * ch;
                f32x4 val = {0.0f, 0.0f, 0.0f, 0.0f};
                if (id != 0xFFFFFFFFu) {
                    const float* src = a.X + (int64_t)id * d + col;
                    if (vec_ok && col + 3 < d) val = *reinterpret_cast<const f32x4*>(src);
                    else {
                        if (col + 0 < d) val.x = src[0];
                        if (col + 1 < d) val.y = src[1];
                        if (col + 2 < d) val.z = src[2];
                        if (col + 3 < d) val.w = src[3];
                    }
                }
                buf[i] = val;
            }
#pragma unroll
            for (int i = 0; i < LOADS; ++i) {
                const int e = tid + NT * i, row = e / CPR, ch = e % CPR;
                *reinterpret_cast<f32x4*>(tile + row * SL + ((ch ^ (row & 15)) << 2)) = buf[i];
            }
        };

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
                *reinterpret_cast<f32x4*>(zp_mine + ((int64_t)chunk * ROWS + row) * 16 + 4 * (lane >> 4)) = out;
            }
        };

        // ---- phase 1: partial logits of every chunk
        for (int chunk = 0; chunk < cm.n_chunks; ++chunk) {
            stage_rows(chunk);
            __syncthreads();
            load_tile();
            __syncthreads();
            forward(chunk);
            if (chunk + 1 < cm.n_chunks) __syncthreads();
        }

        // ---- phase 2: exchange inside the cluster
        if (G > 1) {
            __syncthreads();
            if (tid == 0) {
                __hip_atomic_fetch_add(arrive, 1ull, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
                const unsigned long long target = (a.arrive_base + (unsigned long long)step + 1ull) * (unsigned long long)G;
                uint32_t spins = 0;
                while (__hip_atomic_load(arrive, __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_AGENT) < target) {
                    __builtin_amdgcn_s_sleep(2);
                    if (++spins > a.spin_limit ||
                        __hip_atomic_load(a.abort_flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0) {
                        __hip_atomic_store(a.abort_flag, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                        *stop = 1;
                        break;
                    }
                }
            }
            __syncthreads();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
            if (*stop != 0) return;   // uniform: every thread reads the same LDS word
        } else {
            __syncthreads();
        }

        // ---- phase 3: residual / softmax and the gradient slices
        for (int chunk = 0; chunk < cm.n_chunks; ++chunk) {
            if (cm.n_chunks > 1) {
                __syncthreads();
                stage_rows(chunk);
                __syncthreads();
                load_tile();
            }
            // full logits of the 64 rows: sum of the G partials in slice order
            for (int q = tid; q < ROWS * 4; q += NT) {
                f32x4 z = {0.f, 0.f, 0.f, 0.f};
                for (int g = 0; g < G; ++g)
                    z += *reinterpret_cast<const f32x4*>(zp_all + ((int64_t)g * a.maxrows + (int64_t)chunk * ROWS) * 16 + 4 * q);
                *reinterpret_cast<f32x4*>(zbuf + 4 * q) = z;
            }
            __syncthreads();
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
            __syncthreads();

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
                const int slot = rec_slot(r);
                if (tid < 17) {
                    float sacc = 0.0f;
                    if (tid < 16) { for (int row = row_lo; row < row_hi; ++row) sacc += zbuf[row * 16 + tid]; }
                    else { for (int row = row_lo; row < row_hi; ++row) sacc += lossrow[row]; }
                    small[slot * 17 + tid] = first ? sacc : small[slot * 17 + tid] + sacc;
                }
                if (wave < NBW) {
                    f32x4 acc[4];
#pragma unroll
                    for (int c = 0; c < 4; ++c) acc[c] = f32x4{0.f, 0.f, 0.f, 0.f};
                    for (int ks = row_lo / 4; ks < row_hi / 4; ++ks) {
                        const int row = 4 * ks + (lane >> 4);
                        const float dv = zbuf[row * 16 + (lane & 15)];
                        const int ch = 16 * wave + (lane & 15);
                        const f32x4 xv = *reinterpret_cast<const f32x4*>(tile + row * SL + ((ch ^ (row & 15)) << 2));
                        acc[0] = __builtin_amdgcn_mfma_f32_16x16x4f32(dv, xv.x, acc[0], 0, 0, 0);
                        acc[1] = __builtin_amdgcn_mfma_f32_16x16x4f32(dv, xv.y, acc[1], 0, 0, 0);
                        acc[2] = __builtin_amdgcn_mfma_f32_16x16x4f32(dv, xv.z, acc[2], 0, 0, 0);
                        acc[3] = __builtin_amdgcn_mfma_f32_16x16x4f32(dv, xv.w, acc[3], 0, 0, 0);
                    }
                    float* pk = park + (int64_t)slot * 16 * NT + tid;
#pragma unroll
                    for (int vv = 0; vv < 4; ++vv)
#pragma unroll
                        for (int c = 0; c < 4; ++c) {
                            if (own_cls + vv < C) {
                                float g = acc[c][vv];
                                if (!first) g += pk[(vv * 4 + c) * NT];
                                pk[(vv * 4 + c) * NT] = g;
                            }
                        }
                }
            }
        }
        __syncthreads();

        // ---- phase 4: update v
        {
            const float scale = (float)((double)a.lr / (double)Kv);
            float sum[16];
#pragma unroll
            for (int e = 0; e < 16; ++e) sum[e] = 0.0f;
            float bsum = 0.0f;
            for (int l = 0; l < Kv; ++l) {
                const int slot = (a.variant == kAsync) ? tr_sel[v * Kcap + l] : l;
                const float* pk = park + (int64_t)slot * 16 * NT + tid;
#pragma unroll
                for (int vv = 0; vv < 4; ++vv)
#pragma unroll
                    for (int c = 0; c < 4; ++c)
                        if (own_cls + vv < C) sum[vv * 4 + c] += pk[(vv * 4 + c) * NT];
                if (tid < 17) bsum += small[slot * 17 + tid];
            }
#pragma unroll
            for (int e = 0; e < 16; ++e) W[e] -= scale * sum[e];
            if (a.kind == kSoftmax && tid < C) bias[tid] -= scale * bsum;
            if (tid == 16 && slice == 0) tr_loss[v] = bsum / (float)Kv;
            if (a.agg_out != nullptr && rep == 0) {
                const float invK = 1.0f / (float)Kv;
#pragma unroll
                for (int vv = 0; vv < 4; ++vv)
#pragma unroll
                    for (int c = 0; c < 4; ++c) {
                        const int cls = own_cls + vv, col = own_col + c;
                        if (cls < C && col < d) a.agg_out[(int64_t)cls * d + col] = sum[vv * 4 + c] * invK;
                    }
                if (a.kind == kSoftmax && slice == 0 && tid < C) a.agg_out[(int64_t)C * d + tid] = bsum * invK;
            }
            publish_weights();
        }
        __syncthreads();
    }

    // ---- leave the state in HBM for the next launch
#pragma unroll
    for (int vv = 0; vv < 4; ++vv)
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const int cls = own_cls + vv, col = own_col + c;
            if (cls < C && col < d) params[(int64_t)cls * d + col] = W[vv * 4 + c];
        }
    if (a.kind == kSoftmax && slice == 0 && tid < C) params[(int64_t)C * d + tid] = bias[tid];
    for (int q = tid; q < S * 17; q += NT) small_g[q] = small[q];
}

template <int NBW>
hipError_t launch_t(const LinArgs& a, hipStream_t s) {
    const size_t lds = linear_lds_bytes(NBW, a.C, a.S);
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(linear_cluster_kernel<NBW>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    const int groups = (a.replicas + 7) / 8;
    hipLaunchKernelGGL(linear_cluster_kernel<NBW>, dim3(groups * 8 * a.G), dim3(64 * NBW), lds, s, a);
    return hipGetLastError();
}

}  // namespace

size_t linear_lds_bytes(int nbw, int C, int S) {
    const size_t SL = 64 * (size_t)nbw;
    return sizeof(float) * (ROWS * SL + (size_t)C * SL + ROWS * 16 + 3 * ROWS + 16 + (size_t)S * 17 + 4);
}

int linear_max_resident_groups(int nbw, size_t lds_bytes) {
    int per_cu = 0, dev = 0;
    hipDeviceProp_t prop;
    if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess) return 0;
    hipError_t e;
    if (nbw == 1) {
        hipFuncSetAttribute(reinterpret_cast<const void*>(linear_cluster_kernel<1>), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
        e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, linear_cluster_kernel<1>, 64, lds_bytes);
    } else if (nbw == 2) {
        hipFuncSetAttribute(reinterpret_cast<const void*>(linear_cluster_kernel<2>), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
        e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, linear_cluster_kernel<2>, 128, lds_bytes);
    } else {
        hipFuncSetAttribute(reinterpret_cast<const void*>(linear_cluster_kernel<4>), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
        e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, linear_cluster_kernel<4>, 256, lds_bytes);
    }
    if (e != hipSuccess) return 0;
    return per_cu * prop.multiProcessorCount;
}

hipError_t launch_linear(const LinArgs& a, int nbw, hipStream_t s) {
    if (nbw == 1) return launch_t<1>(a, s);
    if (nbw == 2) return launch_t<2>(a, s);
    return launch_t<4>(a, s);
}

}  // namespace ssgd
