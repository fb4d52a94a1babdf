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

// Two-segment forms for the line search, whose parameter vector is the pair (W1, W2): one launch instead of two.
// out = w + alpha x on both segments; alpha comes from device memory when alpha_dev is not null (a step the device
// itself chose), else from the argument.
__global__ __launch_bounds__(256) void add_scaled2_kernel(size_t n1, const float *w1, const float *__restrict__ x1,
                                                          float *o1, size_t n2, const float *w2,
                                                          const float *__restrict__ x2, float *o2, float alpha,
                                                          const float *__restrict__ alpha_dev)
{
    const float a = alpha_dev ? *alpha_dev : alpha;
    if (a == 0.f && o1 == w1 && o2 == w2) return;      // in-place update by a zero step: nothing changes
    const size_t n = n1 + n2;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) {
        if (i < n1) o1[i] = w1[i] + a * x1[i];
        else o2[i - n1] = w2[i - n1] + a * x2[i - n1];
    }
}

// partial[b] = this workgroup's share of x1.y1 + x2.y2 (double); dot_final_kernel<false> adds the shares.
__global__ __launch_bounds__(256) void dot2_partial_kernel(size_t n1, const float *__restrict__ x1,
                                                           const float *__restrict__ y1, size_t n2,
                                                           const float *__restrict__ x2, const float *__restrict__ y2,
                                                           double *__restrict__ partial)
{
    __shared__ double red[4];
    double a = 0.0;
    const size_t n = n1 + n2;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256)
        a += i < n1 ? (double)x1[i] * (double)y1[i] : (double)x2[i - n1] * (double)y2[i - n1];
    a = block_sum_256(a, red);
    if (threadIdx.x == 0) partial[blockIdx.x] = a;
}

// Decisions of the line search taken on the device, so that the host need not read the errors one by one.
// E[0] = E(W), E[1..3] = E at lo, mid, hi (E[1] unused when lo == 0), E[4] = E at the vertex.
struct LineSearchScalars {
    float E[5];
    float q;            // vertex of the parabola through (lo, mid, hi), clamped to the bracket; mid if not convex
    int convex;
    float alpha, loss;  // the step chosen and the error there
    float slope[16];    // slopes of one group of bracketing steps
};

__global__ void ls_vertex_kernel(LineSearchScalars *s, int lo_is_zero, float lo_f, float hi_f)
{
    const double lo = lo_f, hi = hi_f, mid = 0.5 * (lo + hi);
    const double e_lo = lo_is_zero ? s->E[0] : s->E[1], e_mid = s->E[2], e_hi = s->E[3];
    const double curv = e_lo - 2.0 * e_mid + e_hi;
    double q = mid;
    if (curv > 0.0) {
        const double h = 0.5 * (hi - lo);
        q = mid - h * (e_hi - e_lo) / (2.0 * curv);
        q = q < lo ? lo : (q > hi ? hi : q);
    }
    s->q = (float)q;
    s->convex = curv > 0.0 ? 1 : 0;
}

__global__ void ls_pick_kernel(LineSearchScalars *s, int lo_is_zero, float lo_f, float hi_f)
{
    const double lo = lo_f, hi = hi_f, mid = 0.5 * (lo + hi);
    double best_a = lo, best_e = lo_is_zero ? s->E[0] : s->E[1];
    if ((double)s->E[2] < best_e) { best_a = mid; best_e = s->E[2]; }
    if ((double)s->E[3] < best_e) { best_a = hi; best_e = s->E[3]; }
    if (s->convex && (double)s->E[4] < best_e) { best_a = s->q; best_e = s->E[4]; }
    s->alpha = (float)best_a;
    s->loss = (float)best_e;
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
