// The objective F(w) = (1/N) sum_n f(w, xi_n) over the whole data set (Eq. (1)) for the linear models:
// one streaming pass over the sample matrix, which is what bounds it (HBM).
//
// A workgroup of 16 waves keeps the weights in LDS (rows padded so that the 16 classes of one
// operand fetch fall into different banks) and takes 16 samples at a time; wave w covers the
// columns of its sixteenth of the row, so the workgroup reads 16 whole rows together and the
// chip streams 16 rows per CU at a time (with a row block per wave instead, every wave walked
// 16 rows 64 bytes at a time, 50 000 interleaved streams, and the pass ran at a third of the
// rate).  The partial logits W x come from fp32 MFMA 16x16x4 steps whose class operand is read
// from LDS and whose sample operand is loaded straight from global memory, 16 bytes per lane
// (lane = row + 16 * quarter: columns 16 s + 4 quarter .. + 3 of its row; the four MFMA steps
// of a 16-column block take one of those four columns each, and the weights are fetched in the
// same order, so the k index of a step is a permutation of the columns, which a dot product
// does not mind).  The loads of the next 16 samples are issued while the current ones are
// multiplied.  The 16 partial results meet in LDS (two buffers, one barrier per 16 samples)
// and one wave, a different one each time, adds them in wave order and takes the residual or
// the softmax loss in fp32.  Sums of losses in fp64: per lane, then per wave, then per
// workgroup in a fixed order; the host adds the workgroups' partial sums in order.
#include "common.hpp"

namespace ssgd {
namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int FL_WAVES = 16;
constexpr int FL_DEPTH = 12;     // 16-column blocks held per lane: a wave's share of a row up to d = 3072

struct FullLossArgs {
    const float* X;
    const void* y;
    const float* w;      // parameters of one replica, standard layout
    int64_t N;
    int32_t d, C, kind;
    int32_t stride;      // words per weight row in LDS
    double* partial;     // [gridDim.x]
};

template <int KIND, bool WHOLE>
__global__ __launch_bounds__(64 * FL_WAVES) void full_loss_kernel(FullLossArgs a) {
    extern __shared__ __attribute__((aligned(16))) float smem[];
    __shared__ double wave_sum[FL_WAVES];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int d = a.d, C = a.C, stride = a.stride;
    float* wl = smem;                                                    // [C][stride], zero past column d
    f32x4* part = reinterpret_cast<f32x4*>(smem + (size_t)C * stride);   // [2][FL_WAVES][64]
    for (int q = tid; q < C * stride; q += 64 * FL_WAVES) {
        const int c = q / stride, col = q - c * stride;
        wl[q] = (col < d) ? a.w[(int64_t)c * d + col] : 0.0f;
    }
    __syncthreads();

    const int j = lane & 15, quarter = lane >> 4;
    const float* wrow = wl + min(j, C - 1) * stride + 4 * quarter;   // classes past C read the last one; never used
    float bias[4] = {0.f, 0.f, 0.f, 0.f};
    if (KIND == kSoftmax)
        for (int v = 0; v < 4; ++v)
            if (4 * quarter + v < C) bias[v] = a.w[(int64_t)C * d + 4 * quarter + v];
    const int nblk16 = (d + 15) / 16;                    // 16-column blocks of a row
    const int per_wave = (nblk16 + FL_WAVES - 1) / FL_WAVES;
    const int s_lo = wave * per_wave, s_hi = min(s_lo + per_wave, nblk16);   // this wave's blocks
    const int64_t nrb = (a.N + 15) / 16;                 // blocks of 16 rows
    double lane_sum = 0.0;

    // block s of the rows of row block rb: columns 16 s + 4 quarter .. + 3 (d is a multiple of 4: wholly inside the row
    // or wholly outside)
    auto fetch = [&](int64_t rb, int s) -> f32x4 {
        const int64_t row = rb * 16 + j;
        if (row < a.N && s < s_hi && 16 * s + 4 * quarter < d)
            return __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(a.X + row * (int64_t)d + 16 * s + 4 * quarter));
        return f32x4{0.f, 0.f, 0.f, 0.f};
    };
    auto mac = [&](int s, const f32x4& xv, f32x4& acc0, f32x4& acc1) {
        const f32x4 wv = *reinterpret_cast<const f32x4*>(wrow + 16 * s);
        acc0 = __builtin_amdgcn_mfma_f32_16x16x4f32(wv.x, xv.x, acc0, 0, 0, 0);
        acc1 = __builtin_amdgcn_mfma_f32_16x16x4f32(wv.y, xv.y, acc1, 0, 0, 0);
        acc0 = __builtin_amdgcn_mfma_f32_16x16x4f32(wv.z, xv.z, acc0, 0, 0, 0);
        acc1 = __builtin_amdgcn_mfma_f32_16x16x4f32(wv.w, xv.w, acc1, 0, 0, 0);
    };

    // WHOLE: the queue holds a wave's whole share of a row block (d <= 3072) and is refilled with the next 16 samples
    // while the current ones are multiplied; otherwise the share is walked four blocks at a time.
    f32x4 xq[WHOLE ? FL_DEPTH : 4];
    // WHOLE: one buffer descriptor per block of 16 rows (rows past the end of the data read as zeros), one byte
    // offset per lane, the 16-column blocks of the share at constant distances from it; blocks that are not part of
    // the share or lie past the end of the row are sent out of range
    const uint32_t row_bytes = (uint32_t)d * 4u;
    const int lane_off = (int)(j * row_bytes) + (16 * s_lo + 4 * quarter) * 4;
    uint32_t in_share = 0;
#pragma unroll
    for (int u = 0; u < FL_DEPTH; ++u)
        if (s_lo + u < s_hi && 16 * (s_lo + u) + 4 * quarter < d) in_share |= 1u << u;
    auto fetch_block = [&](int64_t rb, f32x4 (&q)[WHOLE ? FL_DEPTH : 4]) {
        if constexpr (WHOLE) {
            const int64_t first = rb * 16;
            const int64_t rows = (first < a.N) ? ((a.N - first < 16) ? a.N - first : 16) : 0;
            const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(
                const_cast<float*>(a.X + (rows > 0 ? first : 0) * (int64_t)d), 0, (int)(rows * row_bytes), 0x00020000);
#pragma unroll
            for (int u = 0; u < FL_DEPTH; ++u) {
                const int off = ((in_share >> u) & 1u) ? lane_off : (int)0x80000000;
                q[u] = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(rs, off + 64 * u, 0, 0));
            }
        }
    };
    fetch_block(blockIdx.x, xq);
    int it = 0;
    for (int64_t rb = blockIdx.x; rb < nrb; rb += gridDim.x, ++it) {
        f32x4 acc0 = {0.f, 0.f, 0.f, 0.f}, acc1 = {0.f, 0.f, 0.f, 0.f};
        if constexpr (WHOLE) {
            // each block's registers are refilled with the next 16 samples as soon as its MFMA steps have been issued
            const int64_t nfirst = (rb + gridDim.x) * 16;
            const int64_t nrows = (nfirst < a.N) ? ((a.N - nfirst < 16) ? a.N - nfirst : 16) : 0;
            const __amdgpu_buffer_rsrc_t nrs = __builtin_amdgcn_make_buffer_rsrc(
                const_cast<float*>(a.X + (nrows > 0 ? nfirst : 0) * (int64_t)d), 0, (int)(nrows * row_bytes), 0x00020000);
#pragma unroll
            for (int u = 0; u < FL_DEPTH; ++u) {
                if (s_lo + u < s_hi) mac(s_lo + u, xq[u], acc0, acc1);
                __builtin_amdgcn_sched_barrier(0);
                const int off = ((in_share >> u) & 1u) ? lane_off : (int)0x80000000;
                xq[u] = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(nrs, off + 64 * u, 0, 0));
                __builtin_amdgcn_sched_barrier(0);
            }
        } else {
            for (int s0 = s_lo; s0 < s_hi; s0 += 4) {
#pragma unroll
                for (int u = 0; u < 4; ++u) xq[u] = fetch(rb, s0 + u);
#pragma unroll
                for (int u = 0; u < 4; ++u)
                    if (s0 + u < s_hi) mac(s0 + u, xq[u], acc0, acc1);
            }
        }
        const int buf = it & 1;
        part[(buf * FL_WAVES + wave) * 64 + lane] = acc0 + acc1;
        __syncthreads();
        if (wave == (it & (FL_WAVES - 1))) {
            // this lane: classes 4 quarter .. + 3 of row j, summed over the column shares in wave order
            f32x4 z4 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll 1
            for (int w0 = 0; w0 < FL_WAVES; w0 += 4) {      // four reads in flight: the sample registers stay where they are
                f32x4 p4[4];
#pragma unroll
                for (int w = 0; w < 4; ++w) p4[w] = part[(buf * FL_WAVES + w0 + w) * 64 + lane];
#pragma unroll
                for (int w = 0; w < 4; ++w) z4 += p4[w];
            }
            const int64_t row = rb * 16 + j;
            const bool valid = row < a.N;
            float loss = 0.0f;
            if constexpr (KIND == kLsq) {
                const float r = z4.x - (valid ? reinterpret_cast<const float*>(a.y)[row] : 0.0f);
                loss = (valid && quarter == 0) ? 0.5f * r * r : 0.0f;
            } else {
                const int lab = valid ? reinterpret_cast<const int32_t*>(a.y)[row] : 0;
                float z[4], zmax = -3.0e38f;
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    z[v] = z4[v] + bias[v];
                    if (4 * quarter + v < C) zmax = fmaxf(zmax, z[v]);
                }
                zmax = fmaxf(zmax, __shfl_xor(zmax, 16, 64));
                zmax = fmaxf(zmax, __shfl_xor(zmax, 32, 64));
                float den = 0.0f, zl = 0.0f;
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    if (4 * quarter + v < C) den += expf(z[v] - zmax);
                    if (4 * quarter + v == lab) zl = z[v] - zmax;
                }
                den += __shfl_xor(den, 16, 64);
                den += __shfl_xor(den, 32, 64);
                zl += __shfl_xor(zl, 16, 64);
                zl += __shfl_xor(zl, 32, 64);
                loss = (valid && quarter == 0) ? logf(den) - zl : 0.0f;
            }
            lane_sum += (double)loss;
        }
    }

    // fixed-order sums: lanes of a wave (butterfly), waves of the workgroup (serial)
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) lane_sum += __shfl_xor(lane_sum, off, 64);
    if (lane == 0) wave_sum[wave] = lane_sum;
    __syncthreads();
    if (tid == 0) {
        double s = 0.0;
        for (int q = 0; q < FL_WAVES; ++q) s += wave_sum[q];
        a.partial[blockIdx.x] = s;
    }
}

}  // namespace

int full_loss_stride(int d) {
    const int dpad = (d + 15) / 16 * 16;
    return dpad + ((4 - dpad % 64 + 64) % 64);     // stride % 64 == 4: the 16 class rows of a fetch hit 16 different bank groups
}

bool full_loss_supports(int kind, int d, int C) {
    if (kind != kLsq && kind != kSoftmax) return false;
    if (d % 4 != 0 || C > 16) return false;
    return sizeof(float) * (size_t)C * full_loss_stride(d) + 2 * FL_WAVES * 64 * sizeof(f32x4) <= 158 * 1024;
}

hipError_t launch_full_loss(int kind, const float* X, const void* y, int64_t N, int d, int C, const float* w, double* partial,
                            int blocks, hipStream_t s) {
    FullLossArgs a{};
    a.X = X; a.y = y; a.w = w; a.N = N; a.d = d; a.C = C; a.kind = kind; a.stride = full_loss_stride(d); a.partial = partial;
    const size_t lds = sizeof(float) * (size_t)C * a.stride + 2 * FL_WAVES * 64 * sizeof(f32x4);
    const bool whole = ((d + 15) / 16 + FL_WAVES - 1) / FL_WAVES <= FL_DEPTH;
    const void* fn = kind == kLsq ? (whole ? (const void*)full_loss_kernel<kLsq, true> : (const void*)full_loss_kernel<kLsq, false>)
                                  : (whole ? (const void*)full_loss_kernel<kSoftmax, true> : (const void*)full_loss_kernel<kSoftmax, false>);
    hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    if (kind == kLsq) {
        if (whole) hipLaunchKernelGGL((full_loss_kernel<kLsq, true>), dim3(blocks), dim3(64 * FL_WAVES), lds, s, a);
        else hipLaunchKernelGGL((full_loss_kernel<kLsq, false>), dim3(blocks), dim3(64 * FL_WAVES), lds, s, a);
    } else {
        if (whole) hipLaunchKernelGGL((full_loss_kernel<kSoftmax, true>), dim3(blocks), dim3(64 * FL_WAVES), lds, s, a);
        else hipLaunchKernelGGL((full_loss_kernel<kSoftmax, false>), dim3(blocks), dim3(64 * FL_WAVES), lds, s, a);
    }
    return hipGetLastError();
}

}  // namespace ssgd
