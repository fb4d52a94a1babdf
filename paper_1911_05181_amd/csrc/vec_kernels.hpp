// Vector kernels of the optimiser step (section 4.2, last paragraph): dot products, the Polak-Ribiere
// coefficient, direction and weight updates over the parameter vector (1.73 M floats for 400-480-3203).
// All of them stream through HBM once; sums are taken in double, per workgroup and then by one workgroup in a
// fixed order, so results do not depend on scheduling.
#pragma once

#include <hip/hip_runtime.h>

namespace ulsnn {

constexpr int VEC_MAX_BLOCKS = 1024;   // partial sums a workspace must hold per quantity

__device__ __forceinline__ double block_sum_256(double s, double *red)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) s += __shfl_xor(s, o, 64);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = s;
    __syncthreads();
    const double t = red[0] + red[1] + red[2] + red[3];
    __syncthreads();
    return t;
}

// partial[b] = sum over this workgroup's elements of x*y.
// PR = true: x = g_new, y = g_old: partial[b] = sum x*(x - y), partial[gridDim.x + b] = sum y*y.
template <bool PR>
__global__ __launch_bounds__(256) void dot_partial_kernel(size_t n, const float *__restrict__ x,
                                                          const float *__restrict__ y, double *__restrict__ partial)
{
    __shared__ double red[4];
    double a = 0.0, b = 0.0;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) {
        const double xv = x[i], yv = y[i];
        if (PR) {
            a += xv * (xv - yv);
            b += yv * yv;
        } else {
            a += xv * yv;
        }
    }
    a = block_sum_256(a, red);
    if (PR) b = block_sum_256(b, red);
    if (threadIdx.x == 0) {
        partial[blockIdx.x] = a;
        if (PR) partial[gridDim.x + blockIdx.x] = b;
    }
}

// One workgroup adds the partial sums in index order.  PR = false: *out = sum.  PR = true: *out = a / b (0 if b = 0).
template <bool PR>
__global__ __launch_bounds__(256) void dot_final_kernel(const double *__restrict__ partial, int nb,
                                                        float *__restrict__ out)
{
    __shared__ double red[4];
    double a = 0.0, b = 0.0;
    for (int i = threadIdx.x; i < nb; i += 256) {
        a += partial[i];
        if (PR) b += partial[nb + i];
    }
    a = block_sum_256(a, red);
    if (PR) b = block_sum_256(b, red);
    if (threadIdx.x == 0) *out = PR ? (b != 0.0 ? (float)(a / b) : 0.f) : (float)a;
}

// d = -g + beta d  (beta read from device memory; beta == nullptr: d = -g, d is not read).
__global__ __launch_bounds__(256) void cg_update_kernel(size_t n, const float *__restrict__ g,
                                                        float *__restrict__ d, const float *__restrict__ beta)
{
    const float bv = beta ? *beta : 0.f;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256)
        d[i] = beta ? -g[i] + bv * d[i] : -g[i];
}

// out = w + alpha x  (out may be w itself: y += alpha x).
__global__ __launch_bounds__(256) void add_scaled_kernel(size_t n, const float *w, float alpha,
                                                         const float *__restrict__ x, float *out)
{
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256)
        out[i] = w[i] + alpha * x[i];
}

// Measurement aid: one wavefront reads the shader cycle counter and the constant-rate wall clock until
// `wall_ticks` ticks of the latter have passed (or `max_iterations` readings, so that it always ends), and writes
// out[0] = shader cycles, out[1] = wall-clock ticks that elapsed in between.  Launched beside a workload, the
// quotient is the shader clock the chip ran at under that workload.
__global__ __launch_bounds__(64) void clock_probe_kernel(unsigned long long wall_ticks, unsigned int max_iterations,
                                                         unsigned long long *__restrict__ out)
{
    const unsigned long long t0 = wall_clock64();
    const unsigned long long c0 = clock64();
    unsigned long long t1 = t0, c1 = c0;
    for (unsigned int it = 0; it < max_iterations && t1 - t0 < wall_ticks; ++it) {
        __builtin_amdgcn_s_sleep(32);
        c1 = clock64();
        t1 = wall_clock64();
    }
    if (threadIdx.x == 0) {
        out[0] = c1 - c0;
        out[1] = t1 - t0;
    }
}

}  // namespace ulsnn
