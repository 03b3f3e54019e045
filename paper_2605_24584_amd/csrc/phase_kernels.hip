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
__global__ void k_set_word(uint32_t* __restrict__ p, uint32_t v)
{
    if (threadIdx.x == 0) *p = v;
}

// `whole` (may be null) records whether dst holds every row: the pass sets it to 1; with `unless_whole` it first looks at the
// word and does nothing if the rows are all there already (a pass that wrote only some of them had set it to 0).
__global__ void __launch_bounds__(256)
k_phase_split(const float* __restrict__ src, int64_t ld_src, const float* __restrict__ phase,
              int64_t rows, int64_t batch, float* __restrict__ dst, uint32_t* __restrict__ whole, int unless_whole)
{
    if (whole != nullptr && unless_whole && *whole == 1u) return;
    // (set by a later launch when this one decided by the word: other workgroups may still have to read it)
    if (whole != nullptr && !unless_whole && blockIdx.x == 0 && threadIdx.x == 0) *whole = 1u;
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


// ---------------------------------------------------------------------------
// LAPLEX^(r) = sum_q w_q L(a_q, b_q)  (Sec. 7 "Learned anchor geometry in neural heads"): r plain operators
// with independent anchor pairs and scalar mixing weights w (device memory: they are trained).  The products
// of the r operators are combined in a fixed order; the gradient of w_q is the inner product <gy, L_q x>.
// y[i][t] = sum_q w[q] parts[q][i][t]    (parts: r contiguous (rows, batch) matrices; w == null: plain sum)
__global__ void __launch_bounds__(256)
k_mix_combine(const float* __restrict__ parts, const float* __restrict__ w, int64_t r, int64_t rows, int64_t batch,
              float* __restrict__ y, int64_t ldy)
{
    const int64_t total = rows * batch;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < total; e += stride) {
        float acc = 0.0f;
        for (int64_t q = 0; q < r; ++q) acc += (w ? w[q] : 1.0f) * parts[q * total + e];
        y[(e / batch) * ldy + (e % batch)] = acc;
    }
}

// dst[i][t] (contiguous) = scale[0] * src[i*ld_src + t]
__global__ void __launch_bounds__(256)
k_scale_by_device_scalar(const float* __restrict__ src, int64_t ld_src, const float* __restrict__ scale,
                         int64_t rows, int64_t batch, float* __restrict__ dst)
{
    const float f = scale[0];
    const int64_t total = rows * batch;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < total; e += stride)
        dst[e] = f * src[(e / batch) * ld_src + (e % batch)];
}

// dst[i*ld_dst + t] = (first ? 0 : dst[...]) + src[i][t] (src contiguous)
__global__ void __launch_bounds__(256)
k_accumulate(const float* __restrict__ src, int64_t rows, int64_t batch, float* __restrict__ dst, int64_t ld_dst, int first)
{
    const int64_t total = rows * batch;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < total; e += stride) {
        float* p = dst + (e / batch) * ld_dst + (e % batch);
        *p = first ? src[e] : *p + src[e];
    }
}

// partial[g] = sum over workgroup g's share of u[i*ldu + t] * v[i][t] (v contiguous); k_tau_final adds the partials
__global__ void __launch_bounds__(256)
k_dot_partial(const float* __restrict__ u, int64_t ldu, const float* __restrict__ v, int64_t rows, int64_t batch,
              float* __restrict__ partial)
{
    __shared__ float red[256];
    const int64_t total = rows * batch;
    const int64_t per = (total + gridDim.x - 1) / gridDim.x;
    const int64_t lo = per * blockIdx.x, hi = lo + per < total ? lo + per : total;
    float acc = 0.0f;
    for (int64_t e = lo + threadIdx.x; e < hi; e += 256) acc += u[(e / batch) * ldu + (e % batch)] * v[e];
    red[threadIdx.x] = acc;
    __syncthreads();
    for (int s = 128; s >= 1; s >>= 1) {
        if ((int)threadIdx.x < s) red[threadIdx.x] += red[threadIdx.x + s];
        __syncthreads();
    }
    if (threadIdx.x == 0) partial[blockIdx.x] = red[0];
}

// dst[q][i][t] = w[q] * src[i*ld_src + t] for the r operators (blockIdx.y)
__global__ void __launch_bounds__(256)
k_scale_ops(const float* __restrict__ src, int64_t ld_src, const float* __restrict__ w, int64_t rows, int64_t batch,
            float* __restrict__ dst)
{
    const float f = w[blockIdx.y];
    const int64_t total = rows * batch;
    float* out = dst + (int64_t)blockIdx.y * total;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < total; e += stride)
        out[e] = f * src[(e / batch) * ld_src + (e % batch)];
}

// partial[q][g] = workgroup g's share of sum u .* v[q]; then out[q] = sum_g partial[q][g]   (blockIdx.y = q)
__global__ void __launch_bounds__(256)
k_dot_ops_partial(const float* __restrict__ u, int64_t ldu, const float* __restrict__ v, int64_t rows, int64_t batch,
                  float* __restrict__ partial)
{
    __shared__ float red[256];
    const int64_t total = rows * batch;
    const float* vq = v + (int64_t)blockIdx.y * total;
    const int64_t per = (total + gridDim.x - 1) / gridDim.x;
    const int64_t lo = per * blockIdx.x, hi = lo + per < total ? lo + per : total;
    float acc = 0.0f;
    for (int64_t e = lo + threadIdx.x; e < hi; e += 256) acc += u[(e / batch) * ldu + (e % batch)] * vq[e];
    red[threadIdx.x] = acc;
    __syncthreads();
    for (int s = 128; s >= 1; s >>= 1) {
        if ((int)threadIdx.x < s) red[threadIdx.x] += red[threadIdx.x + s];
        __syncthreads();
    }
    if (threadIdx.x == 0) partial[(int64_t)blockIdx.y * gridDim.x + blockIdx.x] = red[0];
}

__global__ void __launch_bounds__(64)
k_dot_ops_final(const float* __restrict__ partial, int groups, float* __restrict__ out)
{
    float acc = 0.0f;
    for (int g = threadIdx.x; g < groups; g += 64) acc += partial[(int64_t)blockIdx.x * groups + g];
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) acc += __shfl_xor(acc, m);
    if (threadIdx.x == 0) out[blockIdx.x] = acc;
}

inline unsigned flat_grid(int64_t total)
{
    int64_t g = (total + 255) / 256;
    if (g < 1) g = 1;
    if (g > 65536) g = 65536;
    return (unsigned)g;
}

inline unsigned rows_grid(int64_t rows)
{
    int64_t g = (rows + 3) / 4;          // four wavefronts (rows) per workgroup
    if (g < 1) g = 1;
    if (g > 65536) g = 65536;
    return (unsigned)g;
}

}  // namespace

hipError_t launch_set_word(uint32_t* p, uint32_t v, hipStream_t st)
{
    LAPLEX_TIMED("phase", st, hipLaunchKernelGGL(k_set_word, dim3(1), dim3(64), 0, st, p, v));
    return hipGetLastError();
}

hipError_t launch_phase_split(const float* src, int64_t ld_src, const float* phase, int64_t rows, int64_t batch,
                              float* dst, hipStream_t st, uint32_t* whole, bool unless_whole)
{
    if (rows <= 0 || batch <= 0) return hipSuccess;
    LAPLEX_TIMED("phase", st, hipLaunchKernelGGL(k_phase_split, dim3(rows_grid(rows)), dim3(256), 0, st,
                                                 src, ld_src, phase, rows, batch, dst, whole, unless_whole ? 1 : 0));
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

hipError_t launch_mix_combine(const float* parts, const float* w, int64_t r, int64_t rows, int64_t batch,
                              float* y, int64_t ldy, hipStream_t st)
{
    LAPLEX_TIMED("mix", st, hipLaunchKernelGGL(k_mix_combine, dim3(flat_grid(rows * batch)), dim3(256), 0, st,
                                               parts, w, r, rows, batch, y, ldy));
    return hipGetLastError();
}

hipError_t launch_scale_by_device_scalar(const float* src, int64_t ld_src, const float* scale, int64_t rows, int64_t batch,
                                         float* dst, hipStream_t st)
{
    LAPLEX_TIMED("mix", st, hipLaunchKernelGGL(k_scale_by_device_scalar, dim3(flat_grid(rows * batch)), dim3(256), 0, st,
                                               src, ld_src, scale, rows, batch, dst));
    return hipGetLastError();
}

hipError_t launch_accumulate(const float* src, int64_t rows, int64_t batch, float* dst, int64_t ld_dst, bool first,
                             hipStream_t st)
{
    LAPLEX_TIMED("mix", st, hipLaunchKernelGGL(k_accumulate, dim3(flat_grid(rows * batch)), dim3(256), 0, st,
                                               src, rows, batch, dst, ld_dst, first ? 1 : 0));
    return hipGetLastError();
}

hipError_t launch_dot(const float* u, int64_t ldu, const float* v, int64_t rows, int64_t batch,
                      float* partial, float* out, hipStream_t st)
{
    int64_t groups = (rows * batch + 8191) / 8192;
    if (groups < 1) groups = 1;
    if (groups > kTauPartials) groups = kTauPartials;
    LAPLEX_TIMED("mix", st, hipLaunchKernelGGL(k_dot_partial, dim3((unsigned)groups), dim3(256), 0, st, u, ldu, v, rows, batch, partial));
    LAPLEX_TIMED("mix", st, hipLaunchKernelGGL(k_tau_final, dim3(1), dim3(256), 0, st, (const float*)partial, (int)groups, out));
    return hipGetLastError();
}

hipError_t launch_scale_ops(const float* src, int64_t ld_src, const float* w, int64_t r, int64_t rows, int64_t batch,
                            float* dst, hipStream_t st)
{
    unsigned g = flat_grid(rows * batch);
    if (g > 1024) g = 1024;
    LAPLEX_TIMED("mix", st, hipLaunchKernelGGL(k_scale_ops, dim3(g, (unsigned)r), dim3(256), 0, st, src, ld_src, w, rows, batch, dst));
    return hipGetLastError();
}

hipError_t launch_dot_ops(const float* u, int64_t ldu, const float* v, int64_t r, int64_t rows, int64_t batch,
                          float* partial, float* out, hipStream_t st)
{
    int64_t groups = (rows * batch + 2047) / 2048;
    if (groups < 1) groups = 1;
    if (groups > kDotGroups) groups = kDotGroups;
    LAPLEX_TIMED("mix", st, hipLaunchKernelGGL(k_dot_ops_partial, dim3((unsigned)groups, (unsigned)r), dim3(256), 0, st,
                                               u, ldu, v, rows, batch, partial));
    LAPLEX_TIMED("mix", st, hipLaunchKernelGGL(k_dot_ops_final, dim3((unsigned)r), dim3(64), 0, st, (const float*)partial, (int)groups, out));
    return hipGetLastError();
}


// ---------------------------------------------------------------------------
// Diagnostics: move whole rows at scattered positions (the access pattern of the heavy scan kernels at wide
// batches) and nothing else: the measured ceiling a benchmark puts beside the nominal HBM peak.
// One wavefront per row, eight rows in flight per wavefront, nontemporal 16-byte accesses.
// ---------------------------------------------------------------------------
namespace {

typedef float diag_v4f __attribute__((ext_vector_type(4)));

template <bool WRITE>
__global__ void __launch_bounds__(256)
k_diag_move_rows(const float* __restrict__ src, float* __restrict__ dst, const uint32_t* __restrict__ row_ids,
                 int64_t rows, int64_t cols)
{
    constexpr int CH = 8;
    const int lane = threadIdx.x & 63;
    const int64_t wave = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
    const int64_t waves = ((int64_t)gridDim.x * blockDim.x) >> 6;
    diag_v4f acc = {0.0f, 0.0f, 0.0f, 0.0f};
    for (int64_t r0 = wave * CH; r0 < rows; r0 += waves * CH) {
        for (int64_t c0 = 4 * (int64_t)lane; c0 < cols; c0 += 256) {
            diag_v4f buf[CH];
            int64_t at[CH];
#pragma unroll
            for (int i = 0; i < CH; ++i) {
                const int64_t r = r0 + i < rows ? r0 + i : rows - 1;
                at[i] = (int64_t)row_ids[r] * cols + c0;
                buf[i] = __builtin_nontemporal_load(reinterpret_cast<const diag_v4f*>(src + at[i]));
            }
#pragma unroll
            for (int i = 0; i < CH; ++i) {
                if (WRITE) { if (r0 + i < rows) __builtin_nontemporal_store(buf[i], reinterpret_cast<diag_v4f*>(dst + at[i])); }
                else acc += buf[i];
            }
        }
    }
    // read only: the sums are "used" by an empty statement, so that the loads stay, and go nowhere
    if (!WRITE) asm volatile("" :: "v"(acc.x), "v"(acc.y), "v"(acc.z), "v"(acc.w));
}

}  // namespace

hipError_t launch_diag_move_rows(const float* src, float* dst, const uint32_t* row_ids, int64_t rows, int64_t cols, hipStream_t st)
{
    if (rows <= 0 || cols <= 0) return hipSuccess;
    int64_t grid = (rows + 31) / 32;            // four wavefronts a workgroup, eight rows a wavefront
    if (grid > 16384) grid = 16384;
    if (dst) hipLaunchKernelGGL(k_diag_move_rows<true>, dim3((unsigned)grid), dim3(256), 0, st, src, dst, row_ids, rows, cols);
    else hipLaunchKernelGGL(k_diag_move_rows<false>, dim3((unsigned)grid), dim3(256), 0, st, src, dst, row_ids, rows, cols);
    return hipGetLastError();
}

}  // namespace laplex
