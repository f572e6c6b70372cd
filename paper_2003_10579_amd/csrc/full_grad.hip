// Gradient of the objective over the whole data set, grad F(w) = (1/N) sum_n grad f(w, xi_n) (Eq. (1)), for the
// linear models: the quantity in which the staleness bound (fifth assumption of Sec. 4.1) is stated
// (E||grad F(w_j) - grad F(w_tau)||^2 <= gamma E||grad F(w_j)||^2).  Two streaming passes over the sample matrix:
//   1. delta[n][c] = softmax(W x_n + b)_c - [y_n = c]  (least squares: x_n . w - y_n), 16 floats per sample;
//   2. G[c][col] = sum_n delta[n][c] X[n][col], a thread per column (the bias is one more column of ones), the
//      samples split into chunks whose partial sums (fp32 within a chunk) are added in chunk order in fp64.
// A statistic for drivers, not part of an update: plain FMA code, bound by the two reads of X.
#include <mutex>

#include "common.hpp"

namespace ssgd {
namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));

// Scratch memory of the entry point that allocates nothing: every GPU the library runs on holds one copy of this
// array for the life of the process (16 MiB).  In host code the name stands for the symbol, not for a device
// address: the address on the current device comes from hipGetSymbolAddress, once per device, and only that pointer
// is handed to kernels.
constexpr int64_t kStaticScratchFloats = 4ll << 20;
static __device__ __align__(256) float scratch[kStaticScratchFloats];
constexpr int kMaxDevices = 64;
float* g_scratch_ptr[kMaxDevices] = {};
std::mutex g_scratch_mutex;

struct FullGradArgs {
    const float* X;
    const void* y;
    const float* w;      // parameters of one replica, standard layout
    int64_t N;
    int32_t d, C, kind;
    int32_t chunks;      // the samples are split into this many runs of chunk_rows rows
    int64_t chunk_rows;
    float* delta;        // [N][16]
    float* partial;      // [chunks][C][d + 1]
    float* out;          // [C * d (+ C)]
};

// 16 samples per workgroup and turn; thread -> (sample tid / 16, columns 4 (tid % 16) + 64 k .. + 3)
template <int KIND>
__global__ __launch_bounds__(256) void full_grad_delta_kernel(FullGradArgs a) {
    const int tid = threadIdx.x, part = tid & 15, rl = tid >> 4;
    const int d = a.d, C = a.C;
    for (int64_t n0 = (int64_t)blockIdx.x * 16; n0 < a.N; n0 += (int64_t)gridDim.x * 16) {
        const int64_t n = n0 + rl;
        const bool have = n < a.N;
        float z[16];
#pragma unroll
        for (int c = 0; c < 16; ++c) z[c] = 0.0f;
        if (have) {
            const float* xr = a.X + n * d;
            for (int col = 4 * part; col < d; col += 64) {
                const f32x4 xv = *reinterpret_cast<const f32x4*>(xr + col);
#pragma unroll
                for (int c = 0; c < 16; ++c) {
                    if (c < C) {
                        const float* wp = a.w + (int64_t)c * d + col;      // a replica's parameters need not be 16-byte aligned
                        z[c] += (xv.x * wp[0] + xv.y * wp[1]) + (xv.z * wp[2] + xv.w * wp[3]);
                    }
                }
            }
        }
        // the 16 parts of a sample sit in 16 neighbouring lanes
#pragma unroll
        for (int c = 0; c < 16; ++c)
#pragma unroll
            for (int o = 8; o >= 1; o >>= 1) z[c] += __shfl_xor(z[c], o, 64);
        if (have && part == 0) {
            float dl[16];
#pragma unroll
            for (int c = 0; c < 16; ++c) dl[c] = 0.0f;
            if (KIND == kLsq) {
                dl[0] = z[0] - reinterpret_cast<const float*>(a.y)[n];
            } else {
                const int lab = reinterpret_cast<const int32_t*>(a.y)[n];
                float zmax = -3.0e38f;
#pragma unroll
                for (int c = 0; c < 16; ++c)
                    if (c < C) { z[c] += a.w[(int64_t)C * d + c]; zmax = fmaxf(zmax, z[c]); }
                float den = 0.0f;
#pragma unroll
                for (int c = 0; c < 16; ++c)
                    if (c < C) { dl[c] = expf(z[c] - zmax); den += dl[c]; }
                const float inv = 1.0f / den;
#pragma unroll
                for (int c = 0; c < 16; ++c)
                    if (c < C) dl[c] = dl[c] * inv - (c == lab ? 1.0f : 0.0f);
            }
            f32x4* dst = reinterpret_cast<f32x4*>(a.delta + n * 16);
#pragma unroll
            for (int q = 0; q < 4; ++q) dst[q] = f32x4{dl[4 * q], dl[4 * q + 1], dl[4 * q + 2], dl[4 * q + 3]};
        }
    }
}

// workgroup = (block of 256 columns, chunk of samples); column d is the bias column (x = 1)
__global__ __launch_bounds__(256) void full_grad_partial_kernel(FullGradArgs a) {
    __shared__ float ds[64][16];
    const int tid = threadIdx.x;
    const int col = blockIdx.x * 256 + tid;
    const int d = a.d, C = a.C;
    const int64_t r0 = (int64_t)blockIdx.y * a.chunk_rows, r1 = min(a.N, r0 + a.chunk_rows);
    float acc[16];
#pragma unroll
    for (int c = 0; c < 16; ++c) acc[c] = 0.0f;
    for (int64_t b0 = r0; b0 < r1; b0 += 64) {
        const int cnt = (int)min<int64_t>(64, r1 - b0);
        __syncthreads();
        for (int q = tid; q < cnt * 16; q += 256) ds[q >> 4][q & 15] = a.delta[b0 * 16 + q];
        __syncthreads();
        if (col <= d) {
            for (int s = 0; s < cnt; ++s) {
                const float x = (col < d) ? a.X[(b0 + s) * d + col] : 1.0f;
#pragma unroll
                for (int c = 0; c < 16; ++c) acc[c] += ds[s][c] * x;
            }
        }
    }
    if (col <= d)
        for (int c = 0; c < C; ++c) a.partial[((int64_t)blockIdx.y * C + c) * (d + 1) + col] = acc[c];
}

__global__ __launch_bounds__(256) void full_grad_reduce_kernel(FullGradArgs a) {
    const int d = a.d, C = a.C;
    const int64_t total = (int64_t)C * (d + 1);
    for (int64_t q = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; q < total; q += (int64_t)gridDim.x * blockDim.x) {
        const int c = (int)(q / (d + 1)), col = (int)(q - (int64_t)c * (d + 1));
        double sum = 0.0;
        for (int ch = 0; ch < a.chunks; ++ch) sum += (double)a.partial[((int64_t)ch * C + c) * (d + 1) + col];
        const float g = (float)(sum / (double)a.N);
        if (col < d) a.out[(int64_t)c * d + col] = g;
        else if (a.kind == kSoftmax) a.out[(int64_t)C * d + c] = g;
    }
}

}  // namespace

bool full_grad_supports(int kind, int d, int C) {
    return (kind == kLsq || kind == kSoftmax) && d % 4 == 0 && C >= 1 && C <= 16;
}

int64_t full_grad_scratch_floats(int64_t N, int d, int C, int* chunks_out) {
    const int chunks = (int)std::max<int64_t>(1, std::min<int64_t>(64, (N + 255) / 256));
    if (chunks_out) *chunks_out = chunks;
    return N * 16 + (int64_t)chunks * C * (d + 1);
}

int64_t full_grad_static_scratch_floats() { return kStaticScratchFloats; }

// Looks up, once per device, where that device keeps its copy of the static scratch array.  Called with the device
// current (ssgd_create does, for every context of a linear model), so that the entry point itself only reads the table.
hipError_t full_grad_static_scratch_prepare() {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (g_scratch_ptr[dev] != nullptr) return hipSuccess;
    float* p = nullptr;
    e = hipGetSymbolAddress(reinterpret_cast<void**>(&p), HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (p == nullptr) return hipErrorInvalidSymbol;
    g_scratch_ptr[dev] = p;
    return hipSuccess;
}

// The current device's copy of the static scratch array, nullptr before full_grad_static_scratch_prepare ran there.
float* full_grad_static_scratch() {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    return g_scratch_ptr[dev];
}

// `work`: full_grad_scratch_floats floats of device memory; `out`: |w| floats of device memory
hipError_t launch_full_grad(int kind, const float* X, const void* y, int64_t N, int d, int C, const float* w,
                            float* work, float* out, int cus, hipStream_t s) {
    FullGradArgs a{};
    a.X = X; a.y = y; a.w = w; a.N = N; a.d = d; a.C = C; a.kind = kind;
    (void)full_grad_scratch_floats(N, d, C, &a.chunks);
    a.chunk_rows = ((N + a.chunks - 1) / a.chunks + 63) / 64 * 64;
    a.delta = work; a.partial = work + N * 16; a.out = out;
    const int blocks = (int)std::min<int64_t>((N + 15) / 16, (int64_t)std::max(1, cus) * 8);
    if (kind == kLsq) hipLaunchKernelGGL(full_grad_delta_kernel<kLsq>, dim3(blocks), dim3(256), 0, s, a);
    else hipLaunchKernelGGL(full_grad_delta_kernel<kSoftmax>, dim3(blocks), dim3(256), 0, s, a);
    hipLaunchKernelGGL(full_grad_partial_kernel, dim3((d + 1 + 255) / 256, a.chunks), dim3(256), 0, s, a);
    hipLaunchKernelGGL(full_grad_reduce_kernel, dim3(64), dim3(256), 0, s, a);
    return hipGetLastError();
}

}  // namespace ssgd
