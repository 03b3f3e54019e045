// Pointwise helpers of the widened entry points.
//
// Phase modulation for the phased kernel
//   P_ij = exp(-|a_i - b_j|) cos(phi_i - psi_j)          (Sec. 3, "Phased Laplace kernels").
// With cos(phi - psi) = cos phi cos psi + sin phi sin psi a phased product is two plain ones on a
// doubled batch:  P x = cos(phi) * L (x cos psi) + sin(phi) * L (x sin psi),  and the same identity
// carries every gradient.  The two kernels here split a matrix into its cosine and sine halves
// (before the scans) and merge two halves back (after them), one wavefront per row; the merge also
// forms the phase gradient of the row, a fixed-order reduction over the batch.
#include "laplex_internal.h"

namespace laplex {

namespace {

// dst[r][t] = src[r][t] cos(phase_r),  dst[r][batch + t] = src[r][t] sin(phase_r);  dst rows are 2 * batch wide
__global__ void __launch_bounds__(256)
k_phase_split(const float* __restrict__ src, int64_t ld_src, const float* __restrict__ phase,
              int64_t rows, int64_t batch, float* __restrict__ dst)
{
    const int lane = threadIdx.x & 63;
    const int64_t wave = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
    const int64_t nwaves = ((int64_t)gridDim.x * blockDim.x) >> 6;
    for (int64_t r = wave; r < rows; r += nwaves) {
        float s, c;
        sincosf(phase[r], &s, &c);
        const float* in = src + r * ld_src;
        float* out = dst + r * 2 * batch;
        for (int64_t t = lane; t < batch; t += 64) {
            const float v = in[t];
            out[t] = v * c;
            out[batch + t] = v * s;
        }
    }
}

// dst[r][t] = cos(phase_r) src2[r][t] + sin(phase_r) src2[r][batch + t]                      (dst may be null)
// gphase[r] = sum_t other[r][t] (cos(phase_r) src2[r][batch + t] - sin(phase_r) src2[r][t])  (gphase may be null)
__global__ void __launch_bounds__(256)
k_phase_merge(const float* __restrict__ src2, const float* __restrict__ phase, int64_t rows, int64_t batch,
              float* __restrict__ dst, int64_t ld_dst, const float* __restrict__ other, int64_t ld_other,
              float* __restrict__ gphase)
{
    const int lane = threadIdx.x & 63;
    const int64_t wave = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
    const int64_t nwaves = ((int64_t)gridDim.x * blockDim.x) >> 6;
    for (int64_t r = wave; r < rows; r += nwaves) {
        float s, c;
        sincosf(phase[r], &s, &c);
        const float* in = src2 + r * 2 * batch;
        float acc = 0.0f;
        for (int64_t t = lane; t < batch; t += 64) {
            const float u = in[t], v = in[batch + t];
            if (dst) dst[r * ld_dst + t] = c * u + s * v;
            if (gphase) acc += other[r * ld_other + t] * (c * v - s * u);
        }
        if (gphase) {
#pragma unroll
            for (int m = 32; m >= 1; m >>= 1) acc += __shfl_xor(acc, m);
            if (lane == 0) gphase[r] = acc;
        }
    }
}


// ---------------------------------------------------------------------------
// Inverse temperature tau (App. A: the temperature-scaled kernel exp(-|a_i - b_j| / t), tau = 1/t).
// The scans work on the scaled anchors tau a, tau b and return the gradients ga', gb' with respect to
// those; the chain rule gives  d/d tau = sum_i a_i ga'_i + sum_j b_j gb'_j  and  ga = tau ga', gb = tau gb'.
// Two launches with a fixed summation order (partials per workgroup, then one workgroup over them).
__global__ void __launch_bounds__(256)
k_tau_partial(const float* __restrict__ a, const float* __restrict__ ga, int64_t k,
              const float* __restrict__ b, const float* __restrict__ gb, int64_t n, float* __restrict__ partial)
{
    __shared__ float red[256];
    const int64_t total = k + n;
    const int64_t per = (total + gridDim.x - 1) / gridDim.x;
    const int64_t lo = per * blockIdx.x, hi = lo + per < total ? lo + per : total;
    float acc = 0.0f;
    for (int64_t i = lo + threadIdx.x; i < hi; i += 256) acc += i < k ? a[i] * ga[i] : b[i - k] * gb[i - k];
    red[threadIdx.x] = acc;
    __syncthreads();
    for (int s = 128; s >= 1; s >>= 1) {
        if ((int)threadIdx.x < s) red[threadIdx.x] += red[threadIdx.x + s];
        __syncthreads();
    }
    if (threadIdx.x == 0) partial[blockIdx.x] = red[0];
}

__global__ void __launch_bounds__(256)
k_tau_final(const float* __restrict__ partial, int count, float* __restrict__ gtau)
{
    __shared__ float red[256];
    float acc = 0.0f;
    for (int i = threadIdx.x; i < count; i += 256) acc += partial[i];
    red[threadIdx.x] = acc;
    __syncthreads();
    for (int s = 128; s >= 1; s >>= 1) {
        if ((int)threadIdx.x < s) red[threadIdx.x] += red[threadIdx.x + s];
        __syncthreads();
    }
    if (threadIdx.x == 0) gtau[0] = red[0];
}

__global__ void __launch_bounds__(256)
k_scale(float* __restrict__ p, int64_t count, float f)
{
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < count; i += stride) p[i] *= f;
}

inline unsigned rows_grid(int64_t rows)
{
    int64_t g = (rows + 3) / 4;          // four wavefronts (rows) per workgroup
    if (g < 1) g = 1;
    if (g > 65536) g = 65536;
    return (unsigned)g;
}

}  // namespace

hipError_t launch_phase_split(const float* src, int64_t ld_src, const float* phase, int64_t rows, int64_t batch,
                              float* dst, hipStream_t st)
{
    if (rows <= 0 || batch <= 0) return hipSuccess;
    LAPLEX_TIMED("phase", st, hipLaunchKernelGGL(k_phase_split, dim3(rows_grid(rows)), dim3(256), 0, st,
                                                 src, ld_src, phase, rows, batch, dst));
    return hipGetLastError();
}

hipError_t launch_phase_merge(const float* src2, const float* phase, int64_t rows, int64_t batch,
                              float* dst, int64_t ld_dst, const float* other, int64_t ld_other, float* gphase,
                              hipStream_t st)
{
    if (rows <= 0) return hipSuccess;
    LAPLEX_TIMED("phase", st, hipLaunchKernelGGL(k_phase_merge, dim3(rows_grid(rows)), dim3(256), 0, st,
                                                 src2, phase, rows, batch, dst, ld_dst, other, ld_other, gphase));
    return hipGetLastError();
}

hipError_t launch_tau_grad(const float* a, const float* ga, int64_t k, const float* b, const float* gb, int64_t n,
                           float* partial, float* gtau, hipStream_t st)
{
    int64_t groups = (k + n + 8191) / 8192;
    if (groups < 1) groups = 1;
    if (groups > kTauPartials) groups = kTauPartials;
    LAPLEX_TIMED("tau", st, hipLaunchKernelGGL(k_tau_partial, dim3((unsigned)groups), dim3(256), 0, st, a, ga, k, b, gb, n, partial));
    LAPLEX_TIMED("tau", st, hipLaunchKernelGGL(k_tau_final, dim3(1), dim3(256), 0, st, (const float*)partial, (int)groups, gtau));
    return hipGetLastError();
}

hipError_t launch_scale(float* p, int64_t count, float f, hipStream_t st)
{
    if (count <= 0) return hipSuccess;
    int64_t g = (count + 255) / 256;
    if (g > 65536) g = 65536;
    LAPLEX_TIMED("tau", st, hipLaunchKernelGGL(k_scale, dim3((unsigned)g), dim3(256), 0, st, p, count, f));
    return hipGetLastError();
}

}  // namespace laplex
