// Row softmax + cross-entropy + output delta, split-k reduction, column sums and the loss reduction.
// These stages move data and do no matrix products: they are bound by HBM traffic, so each reads its input
// once with coalesced accesses and reduces inside wavefronts.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace ulsnn {

__device__ __forceinline__ float wave_max(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}

__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

template <int THREADS>
__device__ __forceinline__ float block_max(float v, float *red)
{
    v = wave_max(v);
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    __syncthreads();                       // red may still be read from a previous reduction
    if (lane == 0) red[wave] = v;
    __syncthreads();
    float r = red[0];
#pragma unroll
    for (int w = 1; w < THREADS / 64; ++w) r = fmaxf(r, red[w]);
    return r;
}

template <int THREADS>
__device__ __forceinline__ float block_sum(float v, float *red)
{
    v = wave_sum(v);
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    __syncthreads();
    if (lane == 0) red[wave] = v;
    __syncthreads();
    float r = red[0];
#pragma unroll
    for (int w = 1; w < THREADS / 64; ++w) r += red[w];   // fixed order: deterministic
    return r;
}

// One workgroup per pattern (row of Z, n columns, row stride ldz).  In place:
//     m = max_c z_c,  s = sum_c exp(z_c - m),  p_c = exp(z_c - m) / s
//     z_c <- p_c - [c == label]            (the output delta; zero row if the label is out of range)
//     row_loss[r] = m + ln s - z_label     (0 if the label is out of range)
// The row is read from HBM once into registers (PER values per thread), so Z is read once and written once.
template <int THREADS, int PER>
__global__ __launch_bounds__(THREADS) void softmax_ce_kernel(float *__restrict__ Z, int ldz, int n,
                                                             const int32_t *__restrict__ labels,
                                                             float *__restrict__ row_loss)
{
    __shared__ float red[THREADS / 64];
    const int r = blockIdx.x;
    float *z = Z + (size_t)r * ldz;
    const int y = labels[r];
    const bool labelled = (y >= 0 && y < n);

    float v[PER];
    float m = -INFINITY;
#pragma unroll
    for (int e = 0; e < PER; ++e) {
        const int c = threadIdx.x + e * THREADS;
        v[e] = c < n ? z[c] : -INFINITY;
        m = fmaxf(m, v[e]);
    }
    m = block_max<THREADS>(m, red);
    float s = 0.f;
#pragma unroll
    for (int e = 0; e < PER; ++e) {
        v[e] = __expf(v[e] - m);         // exp(-inf) = 0 for the padding lanes
        s += v[e];
    }
    s = block_sum<THREADS>(s, red);
    const float inv = 1.0f / s;
    if (threadIdx.x == 0) row_loss[r] = labelled ? (m + __logf(s)) - z[y] : 0.f;
    __syncthreads();                       // z[y] is read before any thread overwrites it
#pragma unroll
    for (int e = 0; e < PER; ++e) {
        const int c = threadIdx.x + e * THREADS;
        if (c < n) z[c] = labelled ? v[e] * inv - (c == y ? 1.0f : 0.0f) : 0.0f;
    }
}

// Same operation for rows too long for registers: three passes over the row (the re-reads hit in cache).
template <int THREADS>
__global__ __launch_bounds__(THREADS) void softmax_ce_long_kernel(float *__restrict__ Z, int ldz, int n,
                                                                  const int32_t *__restrict__ labels,
                                                                  float *__restrict__ row_loss)
{
    __shared__ float red[THREADS / 64];
    const int r = blockIdx.x;
    float *z = Z + (size_t)r * ldz;
    const int y = labels[r];
    const bool labelled = (y >= 0 && y < n);
    float m = -INFINITY;
    for (int c = threadIdx.x; c < n; c += THREADS) m = fmaxf(m, z[c]);
    m = block_max<THREADS>(m, red);
    float s = 0.f;
    for (int c = threadIdx.x; c < n; c += THREADS) s += __expf(z[c] - m);
    s = block_sum<THREADS>(s, red);
    const float inv = 1.0f / s;
    if (threadIdx.x == 0) row_loss[r] = labelled ? (m + __logf(s)) - z[y] : 0.f;
    __syncthreads();
    for (int c = threadIdx.x; c < n; c += THREADS)
        z[c] = labelled ? __expf(z[c] - m) * inv - (c == y ? 1.0f : 0.0f) : 0.0f;
}

// out = alpha * sum_z partial[z] + beta * out over an M x N matrix (partials dense, ld = N; out with ldc).
// With MUL_TANHGRAD the sum is multiplied by (1 - aux^2) first (hidden delta after a split-k product).
template <bool MUL_TANHGRAD>
__global__ __launch_bounds__(256) void splitk_reduce_kernel(const float *__restrict__ partial, size_t stride,
                                                            int splits, float *__restrict__ out, int M, int N,
                                                            int ldc, float alpha, float beta,
                                                            const float *__restrict__ aux, int ldaux)
{
    const size_t total = (size_t)M * N;
    for (size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x; idx < total; idx += (size_t)gridDim.x * 256) {
        float s = 0.f;
        for (int zz = 0; zz < splits; ++zz) s += partial[(size_t)zz * stride + idx];   // fixed order
        const int i = (int)(idx / N), j = (int)(idx % N);
        if (MUL_TANHGRAD) {
            const float hv = aux[(size_t)i * ldaux + j];
            s *= (1.0f - hv * hv);
        }
        float *dst = out + (size_t)i * ldc + j;
        float o = alpha * s;
        if (beta != 0.f) o += beta * *dst;
        *dst = o;
    }
}

// out[c] = beta*out[c] + sum_r D[r][c] for an R x N matrix: 64 columns per workgroup, 4 row phases.
__global__ __launch_bounds__(256) void column_sum_kernel(const float *__restrict__ D, int ld, int R, int N,
                                                         float *__restrict__ out, float beta)
{
    __shared__ float red[4][64];
    const int c = blockIdx.x * 64 + (threadIdx.x & 63);
    const int phase = threadIdx.x >> 6;
    float s = 0.f;
    if (c < N)
        for (int r = phase; r < R; r += 4) s += D[(size_t)r * ld + c];
    red[phase][threadIdx.x & 63] = s;
    __syncthreads();
    if (phase == 0 && c < N) {
        const float t = ((red[0][threadIdx.x] + red[1][threadIdx.x]) + red[2][threadIdx.x]) + red[3][threadIdx.x];
        out[c] = (beta != 0.f ? beta * out[c] : 0.f) + t;
    }
}

// loss = beta*loss + sum_r row_loss[r], summed in double by one workgroup in a fixed order.
__global__ __launch_bounds__(1024) void loss_reduce_kernel(const float *__restrict__ row_loss, long long n,
                                                           float *__restrict__ loss, float beta)
{
    __shared__ double red[16];
    double s = 0.0;
    for (long long r = threadIdx.x; r < n; r += 1024) s += (double)row_loss[r];
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) s += __shfl_xor(s, o, 64);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = s;
    __syncthreads();
    if (threadIdx.x == 0) {
        double t = 0.0;
        for (int w = 0; w < 16; ++w) t += red[w];
        *loss = (beta != 0.f ? beta * *loss : 0.f) + (float)t;
    }
}

// Fill n floats with zero (used instead of a memset so that the call can be captured in a HIP graph).
__global__ __launch_bounds__(256) void zero_kernel(float *__restrict__ p, size_t n)
{
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) p[i] = 0.f;
}

// C = beta * C over an m x n matrix with row stride ldc (SGEMM with k == 0 or alpha == 0).
__global__ __launch_bounds__(256) void scale_kernel(float *__restrict__ C, int m, int n, int ldc, float beta)
{
    const size_t total = (size_t)m * n;
    for (size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x; idx < total; idx += (size_t)gridDim.x * 256) {
        float *dst = C + (idx / n) * (size_t)ldc + (idx % n);
        *dst = (beta == 0.f) ? 0.f : beta * *dst;
    }
}

}  // namespace ulsnn
