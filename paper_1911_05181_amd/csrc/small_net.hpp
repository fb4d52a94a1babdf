// Gradient of a SMALL network in two launches.  For nets like 64-32-10 at a few hundred patterns the whole
// problem is a few MFLOP: the general path's nine launches are pure launch latency.  Here one workgroup takes
// SMALL_ROWS patterns through all steps of section 4.2 (forward, output stage, the three backward products)
// with the weights staged in LDS and plain fp32 FMAs, and writes its share of the sums; a second launch adds the
// shares in workgroup order (deterministic) with the accumulate rule.  Both output stages exist: softmax /
// cross-entropy against labels, and the paper's tanh outputs with squared error against dense targets.
// (Letting the workgroup that finishes last add the shares, found with a ticket counter, saves the second launch
// but was slower: 21.1 against 20.0 us per call for 64-32-10 at 256 patterns; one workgroup's loads after a
// device-wide fence cost more than the launch.)
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "gemm.hpp"   // tanh_f32

namespace ulsnn {

constexpr int SMALL_ROWS = 16;        // patterns per workgroup
constexpr int SMALL_MAX_IN = 128;     // limits of the small-net path (LDS footprint below 64 KB)
constexpr int SMALL_MAX_HID = 64;
constexpr int SMALL_MAX_OUT = 64;
constexpr int SMALL_MAX_BATCH = 4096;

struct SmallReduceArgs {
    const float *partial;
    int stride, groups;
    int n1, n2, n_hid, n_out;
    float *dW1, *dW2, *db1, *db2, *loss;   // db* may be null; dW* null for a loss-only call
    float beta;
};

struct SmallNetArgs {
    int n_in, n_hid, n_out, batch;
    const float *W1, *W2, *b1, *b2;   // biases may be null
    const float *X;
    const int32_t *labels;            // softmax / cross-entropy form
    const float *targets;             // squared-error form (labels == nullptr): dense T[batch x n_out]
    float *partial;                   // [workgroups][stride]: dW1 | dW2 | db1 | db2 | loss
    int stride;
    int backward;                     // 0: loss only
};

// dest = beta*dest + sum over workgroup shares, added in workgroup order, for the groups of four consecutive sums
// number first, first + step, ...  (the share stride is a multiple of 4 floats and the shares are 16-byte
// aligned).  The 16-byte loads of up to eight shares are issued together.
__device__ __forceinline__ void small_reduce_elements(const SmallReduceArgs &a, int first, int step)
{
    typedef float f4 __attribute__((ext_vector_type(4)));
    const int total = a.n1 + a.n2 + a.n_hid + a.n_out + 1;
    const int begin = a.dW1 ? 0 : (total - 1) / 4;   // loss only: just the group holding the last element
    for (int q = begin + first; q * 4 < total; q += step) {
        f4 s = {0.f, 0.f, 0.f, 0.f};
        const float *src = a.partial + (size_t)q * 4;
        int g = 0;
        for (; g + 8 <= a.groups; g += 8) {
            f4 v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) v[u] = *reinterpret_cast<const f4 *>(src + (size_t)(g + u) * a.stride);
#pragma unroll
            for (int u = 0; u < 8; ++u) s += v[u];
        }
        for (; g < a.groups; ++g) s += *reinterpret_cast<const f4 *>(src + (size_t)g * a.stride);
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const int e = q * 4 + c;
            if (e >= total) break;
            float *dst;
            if (e < a.n1) dst = a.dW1;
            else if (e < a.n1 + a.n2) dst = a.dW2 ? a.dW2 + (e - a.n1) : nullptr;
            else if (e < a.n1 + a.n2 + a.n_hid) dst = a.db1 ? a.db1 + (e - a.n1 - a.n2) : nullptr;
            else if (e < total - 1) dst = a.db2 ? a.db2 + (e - a.n1 - a.n2 - a.n_hid) : nullptr;
            else dst = a.loss;
            if (e < a.n1 && dst) dst += e;
            if (!dst) continue;
            *dst = a.beta != 0.f ? s[c] + a.beta * *dst : s[c];
        }
    }
}

// Floats of LDS the kernel needs.
__host__ __device__ inline int small_net_lds_floats(int n_in, int n_hid, int n_out)
{
    return n_in * n_hid + n_hid * n_out + n_hid + n_out + SMALL_ROWS * (n_in + 2 * n_hid + n_out) + SMALL_ROWS;
}

// The three backward products of one workgroup's patterns, written to its share `out`.
__device__ __forceinline__ void small_net_backward(const SmallNetArgs &a, float *out, const float *x, const float *h,
                                                   float *p, float *da, const float *w2, const int tid)
{
    const int n_in = a.n_in, n_hid = a.n_hid, n_out = a.n_out;
    const int n1 = n_in * n_hid, n2 = n_hid * n_out;
    // dW2 share = H^T dO, db2 share = 1^T dO
    for (int o = tid; o < n2; o += 256) {
        const int j = o / n_out, c = o % n_out;
        float s = 0.f;
#pragma unroll
        for (int r = 0; r < SMALL_ROWS; ++r) s += h[r * n_hid + j] * p[r * n_out + c];
        out[n1 + o] = s;
    }
    for (int c = tid; c < n_out; c += 256) {
        float s = 0.f;
#pragma unroll
        for (int r = 0; r < SMALL_ROWS; ++r) s += p[r * n_out + c];
        out[n1 + n2 + n_hid + c] = s;
    }
    // dA1 = (dO W2^T) * (1 - H*H)
    for (int o = tid; o < SMALL_ROWS * n_hid; o += 256) {
        const int r = o / n_hid, j = o % n_hid;
        float s = 0.f;
        for (int c = 0; c < n_out; ++c) s += p[r * n_out + c] * w2[j * n_out + c];
        const float hv = h[o];
        da[o] = s * (1.0f - hv * hv);
    }
    __syncthreads();
    // dW1 share = X^T dA1, db1 share = 1^T dA1
    for (int o = tid; o < n1; o += 256) {
        const int i = o / n_hid, j = o % n_hid;
        float s = 0.f;
#pragma unroll
        for (int r = 0; r < SMALL_ROWS; ++r) s += x[r * n_in + i] * da[r * n_hid + j];
        out[o] = s;
    }
    for (int j = tid; j < n_hid; j += 256) {
        float s = 0.f;
#pragma unroll
        for (int r = 0; r < SMALL_ROWS; ++r) s += da[r * n_hid + j];
        out[n1 + n2 + j] = s;
    }
}

__global__ __launch_bounds__(256) void small_net_kernel(const SmallNetArgs a)
{
    extern __shared__ __attribute__((aligned(16))) float sm[];
    const int n_in = a.n_in, n_hid = a.n_hid, n_out = a.n_out;
    float *w1 = sm;                              // [n_in][n_hid]
    float *w2 = w1 + n_in * n_hid;               // [n_hid][n_out]
    float *bb1 = w2 + n_hid * n_out;             // [n_hid]
    float *bb2 = bb1 + n_hid;                    // [n_out]
    float *x = bb2 + n_out;                      // [ROWS][n_in]
    float *h = x + SMALL_ROWS * n_in;            // [ROWS][n_hid]
    float *p = h + SMALL_ROWS * n_hid;           // [ROWS][n_out]  logits, then the output delta
    float *da = p + SMALL_ROWS * n_out;          // [ROWS][n_hid]  hidden delta
    float *rl = da + SMALL_ROWS * n_hid;         // [ROWS]         row losses
    const int tid = threadIdx.x;
    const int r0 = blockIdx.x * SMALL_ROWS;
    const int rows = min(SMALL_ROWS, a.batch - r0);

    for (int i = tid; i < n_in * n_hid; i += 256) w1[i] = a.W1[i];
    for (int i = tid; i < n_hid * n_out; i += 256) w2[i] = a.W2[i];
    for (int i = tid; i < n_hid; i += 256) bb1[i] = a.b1 ? a.b1[i] : 0.f;
    for (int i = tid; i < n_out; i += 256) bb2[i] = a.b2 ? a.b2[i] : 0.f;
    for (int i = tid; i < SMALL_ROWS * n_in; i += 256)
        x[i] = (i / n_in) < rows ? a.X[(size_t)r0 * n_in + i] : 0.f;       // rows beyond the batch: zeros
    __syncthreads();

    // H = tanh(X W1 + b1)
    for (int o = tid; o < SMALL_ROWS * n_hid; o += 256) {
        const int r = o / n_hid, j = o % n_hid;
        float s = bb1[j];
        for (int i = 0; i < n_in; ++i) s += x[r * n_in + i] * w1[i * n_hid + j];
        h[o] = tanh_f32(s);
    }
    __syncthreads();
    // Z = H W2 + b2
    for (int o = tid; o < SMALL_ROWS * n_out; o += 256) {
        const int r = o / n_out, c = o % n_out;
        float s = bb2[c];
        for (int j = 0; j < n_hid; ++j) s += h[r * n_hid + j] * w2[j * n_out + c];
        p[o] = s;
    }
    __syncthreads();
    if (a.labels) {
        // softmax, cross-entropy and the output delta: one wavefront per row, four rows per wavefront (n_out <= 64)
        const int lane = tid & 63, wave = tid >> 6;
        for (int r = wave; r < SMALL_ROWS; r += 4) {
            const bool live = r < rows;
            const int y = live ? a.labels[r0 + r] : -1;
            const bool labelled = y >= 0 && y < n_out;
            const float z = lane < n_out ? p[r * n_out + lane] : -INFINITY;
            float m = z;
#pragma unroll
            for (int o = 32; o > 0; o >>= 1) m = fmaxf(m, __shfl_xor(m, o, 64));
            const float e = __expf(z - m);
            float s = e;
#pragma unroll
            for (int o = 32; o > 0; o >>= 1) s += __shfl_xor(s, o, 64);
            const float zy = __shfl(z, labelled ? y : 0, 64);
            if (lane == 0) rl[r] = labelled ? (m + __logf(s)) - zy : 0.f;
            if (lane < n_out) p[r * n_out + lane] = labelled ? e / s - (lane == y ? 1.0f : 0.0f) : 0.0f;
        }
    } else {
        // the paper's output stage: y = tanh(z), row error sum (y - t)^2, delta 2 (y - t)(1 - y^2)
        const int lane = tid & 63, wave = tid >> 6;
        for (int r = wave; r < SMALL_ROWS; r += 4) {
            const bool live = r < rows;
            float e = 0.f;
            if (lane < n_out) {
                const float yv = tanh_f32(p[r * n_out + lane]);
                const float diff = live ? yv - a.targets[(size_t)(r0 + r) * n_out + lane] : 0.f;
                e = diff * diff;
                p[r * n_out + lane] = 2.0f * diff * (1.0f - yv * yv);
            }
#pragma unroll
            for (int o = 32; o > 0; o >>= 1) e += __shfl_xor(e, o, 64);
            if (lane == 0) rl[r] = e;
        }
    }
    __syncthreads();
    float *out = a.partial + (size_t)blockIdx.x * a.stride;
    const int n1 = n_in * n_hid, n2 = n_hid * n_out;
    if (tid == 0) {
        float s = 0.f;
        for (int r = 0; r < SMALL_ROWS; ++r) s += rl[r];
        out[n1 + n2 + n_hid + n_out] = s;
    }
    if (a.backward) small_net_backward(a, out, x, h, p, da, w2, tid);
}

// dest = beta*dest + sum over workgroup shares, added in workgroup order (the second launch).
__global__ __launch_bounds__(256) void small_reduce_kernel(const SmallReduceArgs a)
{
    small_reduce_elements(a, blockIdx.x * 256 + threadIdx.x, gridDim.x * 256);   // groups of four sums
}

}  // namespace ulsnn
