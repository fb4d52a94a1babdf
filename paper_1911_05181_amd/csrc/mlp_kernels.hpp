// Row softmax + cross-entropy + output delta, split-k reduction, column sums and the loss reduction.
// These stages move data and do no matrix products: they are bound by HBM traffic, so each reads its input
// once with coalesced accesses and reduces inside wavefronts.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "gemm_bf16.hpp"   // u16, bf16_to_f32, f32_to_bf16

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
// With WRITE_DELTA = false only the row loss is produced (error-only evaluation): Z is read and nothing else written.
template <int THREADS, int PER, bool WRITE_DELTA = true>
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
    if (!WRITE_DELTA) return;
    __syncthreads();                       // z[y] is read before any thread overwrites it
#pragma unroll
    for (int e = 0; e < PER; ++e) {
        const int c = threadIdx.x + e * THREADS;
        if (c < n) {
            z[c] = labelled ? v[e] * inv - (c == y ? 1.0f : 0.0f) : 0.0f;
        }
    }
}

// Same operation for rows too long for registers: three passes over the row (the re-reads hit in cache).
template <int THREADS, bool WRITE_DELTA = true>
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
    if (!WRITE_DELTA) return;
    __syncthreads();
    for (int c = threadIdx.x; c < n; c += THREADS) {
        z[c] = labelled ? __expf(z[c] - m) * inv - (c == y ? 1.0f : 0.0f) : 0.0f;
    }
}

// Output stage of the bf16-operand path, after an output-layer product that left, for each of `groups` column
// groups, (max, sum of exp(z - max)) of the fp32 logits of every row (stats[group * stat_stride + row]) and the
// fp32 logit of the label.  A workgroup joins the groups of 64 patterns: wavefront q takes groups q, q+4, ... of
// each (consecutive lanes read consecutive rows), the four partial pairs meet in LDS in the order q = 0..3:
//     lse = ln sum_c exp(z_c);  row_loss[r] = lse - z_label  (0 if the label is out of range)
//     row_lse[r] = lse (+inf for an ignored pattern: exp(z - inf) = 0 gives its zero delta)
__global__ __launch_bounds__(256) void softmax16_finish_kernel(int n, int rows, const float2 *__restrict__ stats,
                                                               size_t stat_stride, int groups,
                                                               const float *__restrict__ label_logit,
                                                               const int32_t *__restrict__ labels,
                                                               float *__restrict__ row_loss,
                                                               float *__restrict__ row_lse)
{
    __shared__ float2 part[4][64];
    const int lr = threadIdx.x & 63, q = threadIdx.x >> 6;
    const int r = blockIdx.x * 64 + lr;
    float m = -INFINITY, s = 0.f;
    if (r < rows) {
#pragma unroll 4
        for (int gI = q; gI < groups; gI += 4) {
            const float2 p = stats[(size_t)gI * stat_stride + r];
            softmax_merge(m, s, p.x, p.y);
        }
    }
    part[q][lr] = make_float2(m, s);
    __syncthreads();
    if (q != 0 || r >= rows) return;
#pragma unroll
    for (int k = 1; k < 4; ++k) softmax_merge(m, s, part[k][lr].x, part[k][lr].y);
    const int y = labels[r];
    const bool labelled = (y >= 0 && y < n);
    const float lse = m + __logf(s);
    row_loss[r] = labelled ? lse - label_logit[r] : 0.f;
    if (row_lse) row_lse[r] = labelled ? lse : INFINITY;
}

// Squared-error form of the bf16-operand path: the output layer's epilogue left, per row and column group, the sum
// of (y - t)^2 in stats[group * stat_stride + row].x.  row_loss[r] = their sum, taken as above (wavefront q sums
// groups q, q+4, ...; the four partial sums are added in the order q = 0..3).
__global__ __launch_bounds__(256) void mse16_finish_kernel(int rows, const float2 *__restrict__ stats,
                                                           size_t stat_stride, int groups,
                                                           float *__restrict__ row_loss)
{
    __shared__ float part[4][64];
    const int lr = threadIdx.x & 63, q = threadIdx.x >> 6;
    const int r = blockIdx.x * 64 + lr;
    float s = 0.f;
    if (r < rows) {
#pragma unroll 4
        for (int gI = q; gI < groups; gI += 4) s += stats[(size_t)gI * stat_stride + r].x;
    }
    part[q][lr] = s;
    __syncthreads();
    if (q != 0 || r >= rows) return;
    row_loss[r] = ((s + part[1][lr]) + part[2][lr]) + part[3][lr];
}

// Output stage of the paper's own form (tanh outputs, summed squared error against dense targets): one workgroup
// per pattern; Y holds the outputs y = tanh(z) (written by the output-layer product's epilogue).
//     row_loss[r] = sum_c (y_c - t_c)^2,   y_c <- 2 (y_c - t_c) (1 - y_c^2)   (in place, if WRITE_DELTA)
template <int THREADS, bool WRITE_DELTA>
__global__ __launch_bounds__(THREADS) void mse_delta_kernel(float *__restrict__ Y, int ldy, int n,
                                                            const float *__restrict__ T, int ldt,
                                                            float *__restrict__ row_loss)
{
    __shared__ float red[THREADS / 64];
    const int r = blockIdx.x;
    float *y = Y + (size_t)r * ldy;
    const float *t = T + (size_t)r * ldt;
    float e = 0.f;
    for (int c = threadIdx.x; c < n; c += THREADS) {
        const float yv = y[c];
        const float diff = yv - t[c];
        e += diff * diff;
        if (WRITE_DELTA) y[c] = 2.0f * diff * (1.0f - yv * yv);
    }
    e = block_sum<THREADS>(e, red);
    if (threadIdx.x == 0) row_loss[r] = e;
}

// out = alpha * sum_z partial[z] + beta * out over an M x N matrix (partials dense, ld = N; out with ldc).
// With MUL_TANHGRAD the sum is multiplied by (1 - aux^2) first (hidden delta after a split-k product); with BF16
// (hidden delta of the bf16-operand path) aux and out are bf16 and the result is rounded to nearest-even.
template <bool MUL_TANHGRAD, bool BF16 = false>
__global__ __launch_bounds__(256) void splitk_reduce_kernel(const float *__restrict__ partial, size_t stride,
                                                            int splits, void *__restrict__ out_v, int M, int N,
                                                            int ldc, float alpha, float beta,
                                                            const void *__restrict__ aux_v, int ldaux)
{
    float *out = (float *)out_v;
    const float *aux = (const float *)aux_v;
    const size_t total = (size_t)M * N;
    for (size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x; idx < total; idx += (size_t)gridDim.x * 256) {
        float s = 0.f;
        int zz = 0;
        for (; zz + 3 < splits; zz += 4) {   // four loads in flight; the additions keep the split order
            const float *q = partial + (size_t)zz * stride + idx;
            const float p0 = q[0], p1 = q[stride], p2 = q[2 * stride], p3 = q[3 * stride];
            s = (((s + p0) + p1) + p2) + p3;
        }
        for (; zz < splits; ++zz) s += partial[(size_t)zz * stride + idx];
        const int i = (int)(idx / N), j = (int)(idx % N);
        if (MUL_TANHGRAD) {
            const float hv = BF16 ? bf16_to_f32(((const u16 *)aux_v)[(size_t)i * ldaux + j]) : aux[(size_t)i * ldaux + j];
            s *= (1.0f - hv * hv);
        }
        if (BF16) {
            ((u16 *)out_v)[(size_t)i * ldc + j] = f32_to_bf16(alpha * s);
        } else {
            float *dst = out + (size_t)i * ldc + j;
            float o = alpha * s;
            if (beta != 0.f) o += beta * *dst;
            *dst = o;
        }
    }
}

// dst[r][0..cols) = src[r][0..cols) for 2-byte elements with different row strides (repack to aligned rows).
__global__ __launch_bounds__(256) void repack16_kernel(const u16 *__restrict__ src, int ld_src, u16 *__restrict__ dst,
                                                       int ld_dst, int rows, int cols)
{
    const size_t total = (size_t)rows * cols;
    for (size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x; idx < total; idx += (size_t)gridDim.x * 256) {
        const size_t r = idx / cols, c = idx % cols;
        dst[r * ld_dst + c] = src[r * ld_src + c];
    }
}

// out[c] = beta*out[c] + sum_r D[r][c] for a bf16 R x N matrix (bias gradients of the bf16-operand path).
__global__ __launch_bounds__(256) void column_sum16_kernel(const u16 *__restrict__ D, int ld, int R, int N,
                                                           float *__restrict__ out, float beta)
{
    __shared__ float red[4][64];
    const int c = blockIdx.x * 64 + (threadIdx.x & 63);
    const int phase = threadIdx.x >> 6;
    float s = 0.f;
    if (c < N)
        for (int r = phase; r < R; r += 4) s += bf16_to_f32(D[(size_t)r * ld + c]);
    red[phase][threadIdx.x & 63] = s;
    __syncthreads();
    if (phase == 0 && c < N) {
        const float t = ((red[0][threadIdx.x] + red[1][threadIdx.x]) + red[2][threadIdx.x]) + red[3][threadIdx.x];
        out[c] = (beta != 0.f ? beta * out[c] : 0.f) + t;
    }
}

// The same sum over the output delta of the softmax form, which the bf16-operand path never stores: D[r][c] =
// exp(z[r][c] - row_lse[r]) - [c == labels[r]] from the bf16 logits Z (row_lse = +inf: an ignored pattern, zero row).
__global__ __launch_bounds__(256) void column_sum16_delta_kernel(const u16 *__restrict__ Z, int ld, int R, int N,
                                                                 const float *__restrict__ row_lse,
                                                                 const int32_t *__restrict__ labels,
                                                                 float *__restrict__ out, float beta)
{
    __shared__ float red[4][64];
    const int c = blockIdx.x * 64 + (threadIdx.x & 63);
    const int phase = threadIdx.x >> 6;
    float s = 0.f;
    if (c < N)
        for (int r = phase; r < R; r += 4)
            s += __expf(bf16_to_f32(Z[(size_t)r * ld + c]) - row_lse[r]) - (labels[r] == c ? 1.0f : 0.0f);
    red[phase][threadIdx.x & 63] = s;
    __syncthreads();
    if (phase == 0 && c < N) {
        const float t = ((red[0][threadIdx.x] + red[1][threadIdx.x]) + red[2][threadIdx.x]) + red[3][threadIdx.x];
        out[c] = (beta != 0.f ? beta * out[c] : 0.f) + t;
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
    long long r = threadIdx.x;
    for (; r + 7 * 1024 < n; r += 8 * 1024) {   // eight loads in flight; the additions keep the order of r
        float v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = row_loss[r + u * 1024];
#pragma unroll
        for (int u = 0; u < 8; ++u) s += (double)v[u];
    }
    for (; r < n; r += 1024) s += (double)row_loss[r];
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

// *count = number of labels outside [0, n_out): the patterns the output stage ignores.  One workgroup.
__global__ __launch_bounds__(1024) void count_ignored_labels_kernel(const int32_t *__restrict__ labels, long long n,
                                                                    int n_out, long long *__restrict__ count)
{
    __shared__ long long red[16];
    long long c = 0;
    for (long long r = threadIdx.x; r < n; r += 1024) {
        const int y = labels[r];
        c += (y < 0 || y >= n_out) ? 1 : 0;
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) c += __shfl_xor(c, o, 64);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = c;
    __syncthreads();
    if (threadIdx.x == 0) {
        long long t = 0;
        for (int w = 0; w < 16; ++w) t += red[w];
        *count = t;
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
