// Pointwise phase modulation for the phased kernel
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

}  // namespace laplex
