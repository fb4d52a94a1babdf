// Host side of the C ABI declared in include/ulsnn.h: argument checks, choice of tile shape and k split,
// workspace layout, and the stream-ordered launches.  No device memory is allocated here.
#include "../../include/ulsnn.h"

#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstdio>
#include <mutex>

#include "gemm.hpp"
#include "gemm_bf16.hpp"
#include "mlp_kernels.hpp"
#include "small_net.hpp"
#include "vec_kernels.hpp"

using namespace ulsnn;

// Built-in scratch of ulsnn_mlp_grad_static (callers that cannot allocate a workspace).  In host code this name is
// only a handle for hipGetSymbolAddress: the device address, one per GPU, is resolved by static_scratch() below.
static __device__ __align__(256) unsigned char scratch[ULSNN_STATIC_SCRATCH_BYTES];

namespace {

// Compute units of the current device (MI355X: 8 XCDs x 32 = 256), read from the runtime once; the planner's
// cost model and the grid sizes of the streaming kernels use it.  Without a device (host-only plan queries) the
// MI355X figure is assumed.
int query_num_cu()
{
    int dev = 0, n = 0;
    if (hipGetDevice(&dev) == hipSuccess &&
        hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && n > 0)
        return n;
    (void)hipGetLastError();   // no device: not an error of a later launch
    return 256;
}
inline int num_cu()
{
    static const int n = query_num_cu();
    return n;
}
constexpr int SLAB_ROWS = 65536;     // patterns processed per internal pass of the MLP gradient

inline bool is_n(char t) { return t == 'N' || t == 'n'; }
inline bool is_t(char t) { return t == 'T' || t == 't' || t == 'C' || t == 'c'; }
inline size_t round_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// ---------------------------------------------------------------------------------------------------------
// GEMM dispatch: tile shapes, the cost model that picks one (and a k split), and the launchers
// ---------------------------------------------------------------------------------------------------------

// Tile shapes.  The sixth template argument is the number of wavefronts per SIMD the register allocation must
// allow, chosen so that LDS and registers admit the same number of workgroups per compute unit; the seventh
// (default 1) the number of wavefront groups that share every k step.
using Cfg256x128 = TileCfg<256, 128, 16, 4, 2, 4>;   // 512 threads, 2 workgroups / CU: large problems
using Cfg128w8 = TileCfg<128, 128, 16, 4, 2, 6>;     // 512 threads, 3 workgroups / CU
using Cfg128 = TileCfg<128, 128, 16, 2, 2, 4>;       // 256 threads, 4 workgroups / CU
using Cfg128x64 = TileCfg<128, 64, 16, 2, 2, 5>;     // 256 threads, 5 workgroups / CU
using Cfg64x128 = TileCfg<64, 128, 16, 2, 2, 5>;     // 256 threads, 5 workgroups / CU
using Cfg64 = TileCfg<64, 64, 16, 2, 2, 8>;          // 256 threads, 8 workgroups / CU: small problems
// The same tile with a k step of 64 and eight wavefronts, two groups of four that each take half of every step:
// a launch that cannot fill the chip (one or two workgroups per CU) is bound by the latency of its chain of k
// steps, not by the matrix cores; four times fewer, larger steps shorten it, and the second group of wavefronts
// gives every SIMD something to run while the first waits (1024^3: 34.5 us with the plain 64x64 tile, 29.0 with
// the k step of 64, 26.9 with the two groups).
using Cfg64k64 = TileCfg<64, 64, 64, 2, 2, 4, 2>;
// k step 32, two groups of wavefronts, 4 workgroups / CU: for launches of at most four 64x64 workgroups per CU.
using Cfg64k32 = TileCfg<64, 64, 32, 2, 2, 4, 2>;
// 160 rows = 5 accumulator blocks per wavefront (sub-tile 160 x 32): three tiles cover a dimension of 480 without
// padding, where 128-row tiles compute 512.  Measured on dW2 = H^T dO at 32768 patterns: 946 -> 865 us.
using Cfg160x128 = TileCfg<160, 128, 16, 1, 4, 3>;   // 256 threads, 3 workgroups / CU

enum CfgId { CFG_256x128 = 0, CFG_128W8, CFG_128, CFG_128x64, CFG_64x128, CFG_64, CFG_64K64, CFG_160x128, CFG_64K32, CFG_COUNT };

struct CfgInfo {
    int bm, bn, bk, threads, occ;   // occ = resident workgroups per compute unit
    double eff;                     // matrix-core efficiency of the steady state relative to the best shape
    const char *name;
};

constexpr CfgInfo CFG_INFO[CFG_COUNT] = {
    {256, 128, 16, 512, 2, 1.00, "256x128"}, {128, 128, 16, 512, 3, 0.98, "128x128w8"},
    {128, 128, 16, 256, 4, 0.97, "128x128"}, {128, 64, 16, 256, 5, 0.93, "128x64"},
    {64, 128, 16, 256, 5, 0.93, "64x128"},   {64, 64, 16, 256, 8, 0.86, "64x64"},
    {64, 64, 64, 512, 2, 0.86, "64x64k64"},
    {160, 128, 16, 256, 3, 1.06, "160x128"},   // (1.06 x the 3-wavefront utilisation = what it sustains: 116 TFLOP/s)
    {64, 64, 32, 512, 4, 0.86, "64x64k32"},
};

struct GemmPlan {
    CfgId cfg;
    int tiles_m, tiles_n;
    int splits, kchunk;
    double est_us;
};

// Fraction of the matrix-core rate a SIMD reaches with w resident wavefronts (measured: one wavefront cannot
// hide its own LDS, barrier and global-load latency; four can).
inline double simd_utilisation(double w)
{
    static const double u[5] = {0.0, 0.60, 0.78, 0.86, 0.90};
    if (w >= 4.0) return u[4];
    if (w <= 1.0) return u[1];
    const int lo = (int)w;
    return u[lo] + (u[lo + 1] - u[lo]) * (w - lo);
}

// Estimated run time of one launch (+ the split-k reduction), in microseconds.  Not a simulator: a consistent
// way to trade tile efficiency against how evenly the workgroups fill 256 compute units.
double model_us(const CfgInfo &c, bool a_kc, bool b_kc, int m, int n, int k, int splits, int *kchunk_out,
                int *splits_out, double peak_flops = 155.0e12)
{
    const int chunk = (int)round_up((size_t)(k + splits - 1) / splits, c.bk);
    const int sp = (k + chunk - 1) / chunk;
    *kchunk_out = chunk;
    *splits_out = sp;
    const long tiles = (long)((m + c.bm - 1) / c.bm) * ((n + c.bn - 1) / c.bn);
    const long wgs = tiles * sp;
    const double layout = (!a_kc && !b_kc) ? 0.92 : (a_kc && b_kc) ? 1.0 : 0.97;   // 4-byte LDS reads cost more
    const double cu_rate = peak_flops / 256.0 * c.eff * layout;   // flop/s of one compute unit (peak is for 256 of them)
    const double flops_wg = 2.0 * c.bm * c.bn * (double)chunk;
    const double wps = c.threads / 256.0;                                          // wavefronts per SIMD per WG
    const long slots = (long)num_cu() * c.occ;
    const long full = wgs / slots, rem = wgs % slots;
    double t = full * c.occ * flops_wg / (cu_rate * simd_utilisation(c.occ * wps));
    if (rem) {
        const double per_cu = std::ceil((double)rem / num_cu());
        t += per_cu * flops_wg / (cu_rate * simd_utilisation(per_cu * wps));
    }
    t += 3.0e-6 + (double)m * n * sp * 4.0 / 4.0e12;                               // ramp-up and the store burst
    if (sp > 1) t += 3.0e-6 + (double)m * n * (sp + 1.0) * 4.0 / 5.0e12;            // reduction pass
    return t * 1e6;
}

// Choose tile shape and k split (at most `split_limit` slices; 1 = no split).  `cfg_mask` restricts the shapes
// (bit i = CfgId i).
GemmPlan plan_gemm(int m, int n, int k, bool a_kc, bool b_kc, int split_limit, unsigned cfg_mask)
{
    GemmPlan best{};
    best.est_us = 1e30;
    for (int ci = 0; ci < CFG_COUNT; ++ci) {
        if (!(cfg_mask >> ci & 1) || ci == CFG_64K64 || ci == CFG_64K32) continue;
        const CfgInfo &c = CFG_INFO[ci];
        // the 160-row shape exists to avoid padding: only where it computes fewer rows than 128-row tiles would
        if (ci == CFG_160x128 && round_up((size_t)m, 160) >= round_up((size_t)m, 128)) continue;
        const int max_splits = std::max(1, std::min(std::min(64, split_limit), k / (8 * c.bk)));
        for (int s = 1; s <= max_splits; ++s) {
            int chunk, sp;
            const double us = model_us(c, a_kc, b_kc, m, n, std::max(k, 1), s, &chunk, &sp);
            if (sp != s) continue;   // this s collapses onto a smaller split count already seen
            if (us < best.est_us) {
                best.cfg = (CfgId)ci;
                best.tiles_m = (m + c.bm - 1) / c.bm;
                best.tiles_n = (n + c.bn - 1) / c.bn;
                best.splits = sp;
                best.kchunk = chunk;
                best.est_us = us;
            }
        }
    }
    // Unsplit 64x64 launches that cannot fill the chip take the eight-wavefront variants of the tile.  Up to four
    // workgroups per compute unit: k step 32 (2048^3 161 -> 155 us; with more workgroups than that the plain tile's
    // eight small workgroups per CU do better: output layer at 4096 patterns 120 against 124.5 us).  At most one
    // workgroup per compute unit: k step 64; the launch is bound by the latency of its chain of k steps
    // (1024^3 34.5 -> 26.9 us, 512^3 17.8 -> 14.4 us).
    if (best.cfg == CFG_64 && best.splits == 1) {
        const long tiles = (long)best.tiles_m * best.tiles_n;
        CfgId alt = CFG_64;
        if ((cfg_mask >> CFG_64K32 & 1) && tiles <= 4 * num_cu() && k >= 4 * CFG_INFO[CFG_64K32].bk &&
            k % CFG_INFO[CFG_64K32].bk == 0)   // (a partial last step would eat the gain: hidden layer, k = 400)
            alt = CFG_64K32;
        if ((cfg_mask >> CFG_64K64 & 1) && tiles <= num_cu() && k >= 4 * CFG_INFO[CFG_64K64].bk) alt = CFG_64K64;
        if (alt != CFG_64) {
            best.cfg = alt;
            best.kchunk = (int)round_up((size_t)k, CFG_INFO[alt].bk);
        }
    }
    return best;
}

constexpr unsigned ALL_CFGS = (1u << CFG_COUNT) - 1;
constexpr unsigned CFGS_256_THREADS =
    (1u << CFG_128) | (1u << CFG_128x64) | (1u << CFG_64x128) | (1u << CFG_64) | (1u << CFG_160x128);
constexpr unsigned CFGS_PAIRABLE = (1u << CFG_128) | (1u << CFG_128x64) | (1u << CFG_64x128) | (1u << CFG_160x128);

template <class F>
hipError_t with_cfg(CfgId id, F &&f)
{
    switch (id) {
        case CFG_256x128: return f(Cfg256x128{});
        case CFG_128W8: return f(Cfg128w8{});
        case CFG_128: return f(Cfg128{});
        case CFG_128x64: return f(Cfg128x64{});
        case CFG_64x128: return f(Cfg64x128{});
        case CFG_64K64: return f(Cfg64k64{});
        case CFG_160x128: return f(Cfg160x128{});
        case CFG_64K32: return f(Cfg64k32{});
        default: return f(Cfg64{});
    }
}

template <class Cfg, bool A_KC, bool B_KC, int EPI>
hipError_t launch_one(const GemmArgs &a, int splits, hipStream_t s)
{
    const dim3 grid((unsigned)(a.tiles_m * a.tiles_n), (unsigned)splits);
    hipLaunchKernelGGL((gemm_kernel<Cfg, A_KC, B_KC, EPI>), grid, dim3(Cfg::THREADS), 0, s, a);
    return hipGetLastError();
}

template <class Cfg, int EPI>
hipError_t launch_layout(bool a_kc, bool b_kc, const GemmArgs &a, int splits, hipStream_t s)
{
    if (a_kc && !b_kc) return launch_one<Cfg, true, false, EPI>(a, splits, s);    // NN
    if (a_kc && b_kc) return launch_one<Cfg, true, true, EPI>(a, splits, s);       // NT
    if (!a_kc && !b_kc) return launch_one<Cfg, false, false, EPI>(a, splits, s);   // TN
    return launch_one<Cfg, false, true, EPI>(a, splits, s);                        // TT
}

// Which (shape, layout, epilogue) combinations exist is decided here; the planner's masks match it.
hipError_t launch_gemm(const GemmPlan &p, bool a_kc, bool b_kc, int epi, GemmArgs a, hipStream_t s)
{
    a.tiles_m = p.tiles_m;
    a.tiles_n = p.tiles_n;
    a.kchunk = p.kchunk;
    const int splits = p.splits;
    return with_cfg(p.cfg, [&](auto cfg) -> hipError_t {
        using Cfg = decltype(cfg);
        switch (epi) {
            case EPI_AXPBY: return launch_layout<Cfg, EPI_AXPBY>(a_kc, b_kc, a, splits, s);
            case EPI_PARTIAL: return launch_layout<Cfg, EPI_PARTIAL>(a_kc, b_kc, a, splits, s);
            case EPI_BIAS_TANH: return launch_one<Cfg, true, false, EPI_BIAS_TANH>(a, splits, s);   // NN only
            case EPI_BIAS: return launch_one<Cfg, true, false, EPI_BIAS>(a, splits, s);             // NN only
            default: return launch_one<Cfg, true, true, EPI_TANHGRAD>(a, splits, s);                // NT only
        }
    });
}

// Hidden-delta product (NT, plan p4) and output-weight-gradient product (TN, plan p3) as ONE launch of split-k
// partial products: the longer-running workgroups (p4's) are numbered first.
hipError_t launch_pair_partial(const GemmPlan &p4, GemmArgs a4, const GemmPlan &p3, GemmArgs a3, hipStream_t s)
{
    a4.tiles_m = p4.tiles_m; a4.tiles_n = p4.tiles_n; a4.kchunk = p4.kchunk;
    a3.tiles_m = p3.tiles_m; a3.tiles_n = p3.tiles_n; a3.kchunk = p3.kchunk;
    const int n4 = p4.tiles_m * p4.tiles_n * p4.splits, n3 = p3.tiles_m * p3.tiles_n * p3.splits;
    auto second = [&](auto c4) -> hipError_t {
        using C4 = decltype(c4);
        auto go = [&](auto c3) -> hipError_t {
            using C3 = decltype(c3);
            hipLaunchKernelGGL((gemm_pair_kernel<C4, true, true, EPI_PARTIAL, C3, false, false, EPI_PARTIAL>),
                               dim3((unsigned)(n4 + n3)), dim3(256), 0, s, a4, a3, n4);
            return hipGetLastError();
        };
        switch (p3.cfg) {
            case CFG_128: return go(Cfg128{});
            case CFG_128x64: return go(Cfg128x64{});
            case CFG_64x128: return go(Cfg64x128{});
            case CFG_160x128: return go(Cfg160x128{});
            default: return hipErrorInvalidValue;
        }
    };
    switch (p4.cfg) {
        case CFG_128: return second(Cfg128{});
        case CFG_128x64: return second(Cfg128x64{});
        case CFG_64x128: return second(Cfg64x128{});
        case CFG_160x128: return second(Cfg160x128{});
        default: return hipErrorInvalidValue;
    }
}

inline unsigned grid_for(size_t elems)
{
    return (unsigned)std::min<size_t>((elems + 255) / 256, (size_t)num_cu() * 8);
}

// The reduction that follows a split-k launch: out = epilogue(sum of partials).
hipError_t launch_reduce(int splits, int epi, const GemmArgs &a, const float *partial, hipStream_t s)
{
    const size_t total = (size_t)a.M * a.N;
    if (epi == EPI_TANHGRAD) {
        hipLaunchKernelGGL(splitk_reduce_kernel<true>, dim3(grid_for(total)), dim3(256), 0, s, partial, total, splits,
                           a.C, a.M, a.N, a.ldc, 1.0f, 0.0f, a.aux, a.ldaux);
    } else {
        hipLaunchKernelGGL(splitk_reduce_kernel<false>, dim3(grid_for(total)), dim3(256), 0, s, partial, total,
                           splits, a.C, a.M, a.N, a.ldc, a.alpha, a.beta, (const float *)nullptr, 0);
    }
    return hipGetLastError();
}

// Work that rides along with the launch of the dW1 product when the batch is small: the reduction of the dW2
// partial products (HBM-bound, independent of dW1) fills compute units the short dW1 product leaves idle, and the
// sum of the row losses needs no launch of its own.
struct TailWork {
    const float *partial;    // dW2 split-k partials, dense M x N each, `stride` elements apart
    size_t stride;
    int splits;
    float *out;              // dW2
    int M, N, ldc;
    float beta;
    int reduce_blocks;       // workgroups that share the reduction
    const float *row_loss;   // one loss per pattern
    long long rows;
    float *loss;
    float loss_beta;
};

// Workgroups [0, n_gemm): split-k partial products of g (TN);  [n_gemm, n_gemm + reduce_blocks): dW2 reduction;
// the last workgroup: loss = loss_beta*loss + sum of the row losses (double, fixed order).
template <class Cfg>
__global__ __launch_bounds__(256, Cfg::WAVES_PER_SIMD) void dw1_with_tail_kernel(const GemmArgs g, const int n_gemm,
                                                                                 const TailWork t)
{
    static_assert(Cfg::THREADS == 256, "tail work is written for 256 threads");
    __shared__ __attribute__((aligned(16))) float lds[gemm_lds_floats<Cfg, false, false>()];
    const int id = blockIdx.x;
    if (id < n_gemm) {
        gemm_tile<Cfg, false, false, EPI_PARTIAL>(g, id, n_gemm / (g.tiles_m * g.tiles_n), lds);
    } else if (id < n_gemm + t.reduce_blocks) {
        const size_t total = (size_t)t.M * t.N;
        for (size_t idx = (size_t)(id - n_gemm) * 256 + threadIdx.x; idx < total; idx += (size_t)t.reduce_blocks * 256) {
            float sum = 0.f;
            int z = 0;
            for (; z + 3 < t.splits; z += 4) {   // four loads in flight; the additions keep the split order
                const float *q = t.partial + (size_t)z * t.stride + idx;
                const float p0 = q[0], p1 = q[t.stride], p2 = q[2 * t.stride], p3 = q[3 * t.stride];
                sum = (((sum + p0) + p1) + p2) + p3;
            }
            for (; z < t.splits; ++z) sum += t.partial[(size_t)z * t.stride + idx];
            float *dst = t.out + (idx / t.N) * (size_t)t.ldc + (idx % t.N);
            *dst = t.beta != 0.f ? sum + t.beta * *dst : sum;
        }
    } else {
        double *red = reinterpret_cast<double *>(lds);
        double sum = 0.0;
        for (long long r = threadIdx.x; r < t.rows; r += 256) sum += (double)t.row_loss[r];
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) sum += __shfl_xor(sum, o, 64);
        if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = sum;
        __syncthreads();
        if (threadIdx.x == 0)
            *t.loss = (t.loss_beta != 0.f ? t.loss_beta * *t.loss : 0.f) + (float)(red[0] + red[1] + red[2] + red[3]);
    }
}

hipError_t launch_dw1_with_tail(const GemmPlan &p, GemmArgs a, const TailWork &t, hipStream_t s)
{
    a.tiles_m = p.tiles_m;
    a.tiles_n = p.tiles_n;
    a.kchunk = p.kchunk;
    const int n_gemm = p.tiles_m * p.tiles_n * p.splits;
    const dim3 grid((unsigned)(n_gemm + t.reduce_blocks + 1));
    switch (p.cfg) {
        case CFG_128: hipLaunchKernelGGL(dw1_with_tail_kernel<Cfg128>, grid, dim3(256), 0, s, a, n_gemm, t); break;
        case CFG_128x64: hipLaunchKernelGGL(dw1_with_tail_kernel<Cfg128x64>, grid, dim3(256), 0, s, a, n_gemm, t); break;
        case CFG_64x128: hipLaunchKernelGGL(dw1_with_tail_kernel<Cfg64x128>, grid, dim3(256), 0, s, a, n_gemm, t); break;
        case CFG_64: hipLaunchKernelGGL(dw1_with_tail_kernel<Cfg64>, grid, dim3(256), 0, s, a, n_gemm, t); break;
        case CFG_160x128: hipLaunchKernelGGL(dw1_with_tail_kernel<Cfg160x128>, grid, dim3(256), 0, s, a, n_gemm, t); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------------------
// bf16-operand GEMM dispatch (fp32 accumulation): two tile shapes, same cost model with the measured bf16 rate
// ---------------------------------------------------------------------------------------------------------

using T16_128 = Tile16<128, 128, 2, 2, 4, 1>;   // 256 threads, 4 workgroups / CU (LDS 39 KB each)
using T16_64 = Tile16<64, 64, 2, 2, 8, 1>;      // 256 threads, 8 workgroups / CU
// Wavefront sub-tile 128 x 64: a third fewer LDS bytes per matrix instruction than 64 x 64 (the 128x128 shape is
// bound by LDS reads).  Two workgroups per CU, so the epilogue's stores are poorly hidden: long-k products only.
using T16_256 = Tile16<256, 128, 2, 2, 2, 2>;
// 256 x 256 with eight wavefronts (sub-tile 64 x 128), one workgroup per CU: a third less operand traffic per
// product again.  Measured on the hidden-delta product (both operands k-contiguous): 164 -> 140 us at 32768 patterns;
// on the dW2 product (both m-contiguous) at 65536 patterns: backward products 645 -> 618 us.
using T16_256x256 = Tile16<256, 256, 4, 2, 2, 2>;

enum Cfg16Id { CFG16_128 = 0, CFG16_64, CFG16_256, CFG16_256x256, CFG16_COUNT };
constexpr int CFG16_256_MIN_K = 1024;

constexpr CfgInfo CFG16_INFO[CFG16_COUNT] = {
    {128, 128, 32, 256, 4, 1.00, "bf16 128x128"},
    {64, 64, 32, 256, 8, 0.70, "bf16 64x64"},
    {256, 128, 32, 256, 2, 1.30, "bf16 256x128"},
    {256, 256, 32, 512, 1, 1.55, "bf16 256x256"},
};
constexpr double BF16_SUSTAINED_FLOPS = 800.0e12;   // what the 128x128 bf16 tile sustains on large problems

struct Gemm16Plan {
    Cfg16Id cfg;
    int tiles_m, tiles_n;
    int splits, kchunk;
    double est_us;
};

Gemm16Plan plan_gemm16(int m, int n, int k, bool a_kc, bool b_kc, bool allow_split, size_t max_partial_floats)
{
    Gemm16Plan best{};
    best.est_us = 1e30;
    for (int ci = 0; ci < CFG16_COUNT; ++ci) {
        const CfgInfo &c = CFG16_INFO[ci];
        if (ci == CFG16_256 && k < CFG16_256_MIN_K) continue;
        if (ci == CFG16_256x256 && !(a_kc == b_kc && k >= CFG16_256_MIN_K)) continue;   // NT and TN long-k products
        int max_splits = allow_split ? std::max(1, std::min(64, k / (8 * c.bk))) : 1;
        if ((size_t)m * n > 0) max_splits = (int)std::min<size_t>(max_splits, std::max<size_t>(1, max_partial_floats / ((size_t)m * n)));
        for (int s = 1; s <= max_splits; ++s) {
            int chunk, sp;
            const double us = model_us(c, a_kc, b_kc, m, n, std::max(k, 1), s, &chunk, &sp, BF16_SUSTAINED_FLOPS);
            if (sp != s) continue;
            if (us < best.est_us) {
                best.cfg = (Cfg16Id)ci;
                best.tiles_m = (m + c.bm - 1) / c.bm;
                best.tiles_n = (n + c.bn - 1) / c.bn;
                best.splits = sp;
                best.kchunk = chunk;
                best.est_us = us;
            }
        }
    }
    return best;
}

template <class Cfg, bool A_KC, bool B_KC, int EPI, int DELTA = 0>
hipError_t launch16_one(const Gemm16Args &a, int splits, hipStream_t s)
{
    const dim3 grid((unsigned)(a.tiles_m * a.tiles_n), (unsigned)splits);
    hipLaunchKernelGGL((gemm16_kernel<Cfg, A_KC, B_KC, EPI, DELTA>), grid, dim3(Cfg::THREADS), 0, s, a);
    return hipGetLastError();
}

inline bool rows_16b_aligned(const void *p, int ld) { return ((uintptr_t)p & 15) == 0 && (ld & 7) == 0; }

// Columns of C one statistics group of the output-layer epilogue covers: the wavefront sub-tile width of the shape.
inline int stat_group_width(Cfg16Id id)
{
    switch (id) {
        case CFG16_128: return T16_128::WTN;
        case CFG16_256: return T16_256::WTN;
        case CFG16_256x256: return T16_256x256::WTN;
        default: return T16_64::WTN;
    }
}

// The combinations the MLP gradient needs: NN with bias+tanh / bias / bias + softmax statistics, NT with the tanh'
// mask, NT and TN partials, TN with alpha/beta.
hipError_t launch_gemm16(const Gemm16Plan &p, bool a_kc, bool b_kc, int epi, Gemm16Args a, hipStream_t s)
{
    a.tiles_m = p.tiles_m;
    a.tiles_n = p.tiles_n;
    a.kchunk = p.kchunk;
    a.aligned = rows_16b_aligned(a.A, a.lda) && rows_16b_aligned(a.B, a.ldb);
    const bool c_bf16 = epi == EPI_BIAS_TANH || epi == EPI_TANHGRAD || epi == EPI_BIAS_STATS || epi == EPI_TANH_MSE;
    a.c_vec = ((uintptr_t)a.C & 15) == 0 && (a.ldc % (c_bf16 ? 8 : 4)) == 0;
    a.aux_vec = a.aux != nullptr && rows_16b_aligned(a.aux, a.ldaux);
    auto go = [&](auto cfg) -> hipError_t {
        using Cfg = decltype(cfg);
        if (epi == EPI_BIAS_TANH && a_kc && !b_kc) return launch16_one<Cfg, true, false, EPI_BIAS_TANH>(a, p.splits, s);
        if (epi == EPI_BIAS && a_kc && !b_kc) return launch16_one<Cfg, true, false, EPI_BIAS>(a, p.splits, s);
        if ((epi == EPI_BIAS_STATS || epi == EPI_STATS_ONLY) && a_kc && !b_kc) {
            // one statistics group per wavefront column; the logits' rows must be 16-byte aligned
            if (a.stat_groups != (a.N + Cfg::WTN - 1) / Cfg::WTN || a.stat_stride < (size_t)a.M || !a.stats || !a.label_logit || !a.labels ||
                (epi == EPI_BIAS_STATS && !a.c_vec))
                return hipErrorInvalidValue;
            return epi == EPI_BIAS_STATS ? launch16_one<Cfg, true, false, EPI_BIAS_STATS>(a, p.splits, s)
                                         : launch16_one<Cfg, true, false, EPI_STATS_ONLY>(a, p.splits, s);
        }
        if ((epi == EPI_TANH_MSE || epi == EPI_MSE_ONLY) && a_kc && !b_kc) {
            if (a.stat_groups != (a.N + Cfg::WTN - 1) / Cfg::WTN || a.stat_stride < (size_t)a.M || !a.stats || !a.targets || a.ldt < a.N ||
                (epi == EPI_TANH_MSE && !a.c_vec))
                return hipErrorInvalidValue;
            return epi == EPI_TANH_MSE ? launch16_one<Cfg, true, false, EPI_TANH_MSE>(a, p.splits, s)
                                       : launch16_one<Cfg, true, false, EPI_MSE_ONLY>(a, p.splits, s);
        }
        if (a.row_lse) {   // a product that forms the output delta from the logits while loading them
            if (!a.aligned || !a.labels) return hipErrorInvalidValue;
            if (a_kc && b_kc && epi == EPI_TANHGRAD) return launch16_one<Cfg, true, true, EPI_TANHGRAD, 1>(a, p.splits, s);
            if (a_kc && b_kc && epi == EPI_PARTIAL) return launch16_one<Cfg, true, true, EPI_PARTIAL, 1>(a, p.splits, s);
            if (!a_kc && !b_kc && epi == EPI_PARTIAL) return launch16_one<Cfg, false, false, EPI_PARTIAL, 2>(a, p.splits, s);
            if (!a_kc && !b_kc && epi == EPI_AXPBY) return launch16_one<Cfg, false, false, EPI_AXPBY, 2>(a, p.splits, s);
            return hipErrorInvalidValue;
        }
        if (epi == EPI_TANHGRAD && a_kc && b_kc) return launch16_one<Cfg, true, true, EPI_TANHGRAD>(a, p.splits, s);
        if (epi == EPI_PARTIAL && a_kc && b_kc) return launch16_one<Cfg, true, true, EPI_PARTIAL>(a, p.splits, s);
        if (epi == EPI_PARTIAL && !a_kc && !b_kc) return launch16_one<Cfg, false, false, EPI_PARTIAL>(a, p.splits, s);
        if (epi == EPI_AXPBY && !a_kc && !b_kc) return launch16_one<Cfg, false, false, EPI_AXPBY>(a, p.splits, s);
        return hipErrorInvalidValue;
    };
    return p.cfg == CFG16_128 ? go(T16_128{}) : p.cfg == CFG16_256 ? go(T16_256{})
         : p.cfg == CFG16_256x256 ? go(T16_256x256{}) : go(T16_64{});
}

// ---------------------------------------------------------------------------------------------------------
// MLP gradient: plans and workspace layout for one slab of patterns
// ---------------------------------------------------------------------------------------------------------

constexpr size_t PARTIAL_CAP_FLOATS = (size_t)32 << 20;   // at most 128 MiB of split-k partials per product

struct MlpLayout {
    int slab;                       // rows per pass
    int ldh, ldz;                   // row strides (elements) of H / dA1 and of Z / dO
    int ldw1p, ldw2p;               // bf16 path: row strides of the 16-byte aligned copies of W1 and W2
    size_t floats_pa, floats_pb;    // split-k partial regions: A (dW2, then dW1) and B (hidden delta)
    size_t off_h, off_z, off_da1, off_rowloss, off_pa, off_pb, bytes;
    size_t off_do16, off_w1p, off_w2p, off_zlab, off_lse;   // bf16 path only
};

struct SlabPlans {
    GemmPlan g1, g2, g3, g4, g5;
    bool paired;                    // g4 and g3 run as one launch of partial products
};

bool desc_ok(const ulsnn_mlp_desc *d)
{
    return d && d->n_in >= 1 && d->n_hid >= 1 && d->n_out >= 1;
}

// Sizes depend on the network and on min(batch, SLAB_ROWS) only, and do not decrease with the batch, so a
// workspace sized for a batch also serves every smaller one.
// Small networks at small batches take a two-launch path (small_net.hpp).  Its scratch: one share of every sum
// per workgroup of SMALL_ROWS patterns.
inline int small_net_stride(const ulsnn_mlp_desc *d)
{
    return (int)round_up((size_t)d->n_in * d->n_hid + (size_t)d->n_hid * d->n_out + d->n_hid + d->n_out + 1, 4);
}
inline bool small_net_shape(const ulsnn_mlp_desc *d, long long batch)
{
    return d->operand_dtype == 0 && d->n_in <= SMALL_MAX_IN && d->n_hid <= SMALL_MAX_HID &&
           d->n_out <= SMALL_MAX_OUT && batch >= 1 && batch <= SMALL_MAX_BATCH &&
           (size_t)small_net_lds_floats(d->n_in, d->n_hid, d->n_out) * sizeof(float) <= 64 * 1024;
}
inline size_t small_net_bytes(const ulsnn_mlp_desc *d, long long batch)
{
    if (!small_net_shape(d, batch)) return 0;
    const size_t groups = (size_t)(batch + SMALL_ROWS - 1) / SMALL_ROWS;
    return round_up(groups * small_net_stride(d) * sizeof(float), 256);
}

MlpLayout mlp_layout(const ulsnn_mlp_desc *d, int batch)
{
    MlpLayout L{};
    const bool bf16 = d->operand_dtype == 1;
    const size_t act = bf16 ? 2 : 4;               // bytes per stored activation (H, dA1)
    L.slab = std::max(1, std::min(batch, SLAB_ROWS));
    L.ldh = (int)round_up((size_t)d->n_hid, 32);
    L.ldz = (int)round_up((size_t)d->n_out, 32);
    L.ldw1p = (int)round_up((size_t)d->n_hid, 8);
    L.ldw2p = (int)round_up((size_t)d->n_out, 8);
    const size_t mn3 = (size_t)d->n_hid * d->n_out, mn5 = (size_t)d->n_in * d->n_hid;
    const size_t mn4 = (size_t)L.slab * d->n_hid;
    L.floats_pa = std::max(std::max(mn3, mn5), std::min(PARTIAL_CAP_FLOATS, 64 * std::max(mn3, mn5)));
    L.floats_pb = std::max(mn4, std::min(PARTIAL_CAP_FLOATS, 16 * mn4));
    size_t off = 0;
    L.off_h = off;        off += round_up((size_t)L.slab * L.ldh * act, 256);
    // fp32: the logits / output delta.  bf16: the softmax statistics of the output layer's epilogue, one
    // (max, sum) pair per row and group of at least 32 columns (the logits themselves live at off_do16)
    L.off_z = off;        off += round_up(bf16 ? (size_t)L.slab * (L.ldz / 32) * sizeof(float2) : (size_t)L.slab * L.ldz * 4, 256);
    L.off_da1 = off;      off += round_up((size_t)L.slab * L.ldh * act, 256);
    L.off_rowloss = off;  off += round_up((size_t)L.slab * 4, 256);
    L.off_pa = off;       off += round_up(L.floats_pa * 4, 256);
    L.off_pb = off;       off += round_up(L.floats_pb * 4, 256);
    if (bf16) {
        L.off_do16 = off; off += round_up((size_t)L.slab * L.ldz * 2, 256);
        L.off_w1p = off;  off += round_up((size_t)d->n_in * L.ldw1p * 2, 256);
        L.off_w2p = off;  off += round_up((size_t)d->n_hid * L.ldw2p * 2, 256);
        L.off_zlab = off; off += round_up((size_t)L.slab * 4, 256);
        L.off_lse = off;  off += round_up((size_t)L.slab * 4, 256);
    }
    L.bytes = std::max(off, small_net_bytes(d, batch));
    return L;
}

// Plans of the five products for `rows` patterns.  A split count is limited by the partial region it writes.
SlabPlans plan_slab(const MlpLayout &L, int n_in, int n_hid, int n_out, int rows)
{
    SlabPlans s;
    auto slices = [](size_t region, int m, int n) { return (int)std::min<size_t>(64, region / ((size_t)m * n)); };
    s.g1 = plan_gemm(rows, n_hid, n_in, true, false, 1, ALL_CFGS);
    s.g2 = plan_gemm(rows, n_out, n_hid, true, false, 1, ALL_CFGS);
    s.g3 = plan_gemm(n_hid, n_out, rows, false, false, slices(L.floats_pa, n_hid, n_out), CFGS_256_THREADS);
    s.g4 = plan_gemm(rows, n_hid, n_out, true, true, slices(L.floats_pb, rows, n_hid), CFGS_256_THREADS);
    s.g5 = plan_gemm(n_in, n_hid, rows, false, false, slices(L.floats_pa, n_in, n_hid), CFGS_256_THREADS);
    // the 256-thread restriction serves the paired launch; an unsplit hidden-delta product runs alone and may take
    // any shape (32768 patterns: 256x128 instead of 128x128, 20 us of 870)
    if (s.g4.splits == 1) {
        const GemmPlan any = plan_gemm(rows, n_hid, n_out, true, true, 1, ALL_CFGS);
        if (any.est_us < s.g4.est_us) s.g4 = any;
    }
    s.paired = s.g3.splits > 1 && s.g4.splits > 1 && (CFGS_PAIRABLE >> s.g3.cfg & 1) && (CFGS_PAIRABLE >> s.g4.cfg & 1);
    return s;
}

int check_mlp_args(const ulsnn_mlp_desc *d, const void *W1, const void *W2, const void *X, const void *targets,
                   long long batch, const float *dW1, const float *dW2, const float *loss, bool backward)
{
    if (!d) return ULSNN_ERR_NULL;
    if (d->n_in < 1 || d->n_hid < 1 || d->n_out < 1 || batch < 0) return ULSNN_ERR_DIM;
    if (d->n_in > ULSNN_MAX_LD || d->n_hid > ULSNN_MAX_LD || d->n_out > ULSNN_MAX_LD) return ULSNN_ERR_UNSUPPORTED;
    if (!W1 || !W2 || !loss) return ULSNN_ERR_NULL;
    if (backward && (!dW1 || !dW2)) return ULSNN_ERR_NULL;
    if (batch > 0 && (!X || !targets)) return ULSNN_ERR_NULL;
    const int nb = (d->b1 != nullptr) + (d->b2 != nullptr) + (d->db1 != nullptr) + (d->db2 != nullptr);
    if (backward ? (nb != 0 && nb != 4) : ((d->b1 != nullptr) != (d->b2 != nullptr))) return ULSNN_ERR_NULL;
    if (d->accumulate != 0 && d->accumulate != 1) return ULSNN_ERR_UNSUPPORTED;
    if (d->operand_dtype != 0 && d->operand_dtype != 1) return ULSNN_ERR_UNSUPPORTED;
    return ULSNN_OK;
}

#define HIP_TRY(expr)                                   \
    do {                                                \
        if ((expr) != hipSuccess) return ULSNN_ERR_HIP; \
    } while (0)
#define MARK(stage)                                       \
    do {                                                  \
        if (ev) HIP_TRY(hipEventRecord(ev[stage], s));    \
    } while (0)

// `ev`, if not null, is an array of ULSNN_MLP_STAGES + 1 events recorded at the stage boundaries.
// What one call computes beyond the forward pass.
struct MlpTask {
    const int32_t *labels;   // softmax / cross-entropy output stage (targets == nullptr)
    const float *targets;    // tanh / squared-error output stage of the paper: dense T[batch x n_out]
    bool backward;           // false: loss only (error evaluation), dW1 / dW2 untouched
};

int mlp_grad_impl16(const ulsnn_mlp_desc *d, const u16 *W1, const u16 *W2, const u16 *X, const MlpTask &task,
                    int batch, float *dW1, float *dW2, float *loss, bool accumulate, hipEvent_t *ev);

// W1v, W2v, Xv point at fp32 (operand_dtype 0) or bf16 (operand_dtype 1) data.
int mlp_grad_impl(const ulsnn_mlp_desc *d, const void *W1v, const void *W2v, const void *Xv,
                  const MlpTask &task, int batch, float *dW1, float *dW2, float *loss, bool accumulate,
                  hipEvent_t *ev = nullptr)
{
    hipStream_t s = (hipStream_t)d->hip_stream;
    const int n_in = d->n_in, n_hid = d->n_hid, n_out = d->n_out;
    const bool biases = d->b1 != nullptr;

    if (batch == 0) {
        if (!accumulate) {
            hipLaunchKernelGGL(zero_kernel, dim3(1), dim3(256), 0, s, loss, (size_t)1);
            if (task.backward) {
                hipLaunchKernelGGL(zero_kernel, dim3(grid_for((size_t)n_in * n_hid)), dim3(256), 0, s, dW1,
                                   (size_t)n_in * n_hid);
                hipLaunchKernelGGL(zero_kernel, dim3(grid_for((size_t)n_hid * n_out)), dim3(256), 0, s, dW2,
                                   (size_t)n_hid * n_out);
            }
            if (biases && task.backward) {
                hipLaunchKernelGGL(zero_kernel, dim3(grid_for(n_hid)), dim3(256), 0, s, d->db1, (size_t)n_hid);
                hipLaunchKernelGGL(zero_kernel, dim3(grid_for(n_out)), dim3(256), 0, s, d->db2, (size_t)n_out);
            }
            HIP_TRY(hipGetLastError());
        }
        return ULSNN_OK;
    }

    if (d->operand_dtype == 1)
        return mlp_grad_impl16(d, (const u16 *)W1v, (const u16 *)W2v, (const u16 *)Xv, task, batch, dW1, dW2, loss,
                               accumulate, ev);
    const float *W1 = (const float *)W1v, *W2 = (const float *)W2v, *X = (const float *)Xv;

    // small network, small batch, no stage timing asked for: two launches instead of nine
    if (!ev && small_net_shape(d, batch)) {
        const size_t need = mlp_layout(d, batch).bytes;
        if (!d->workspace || ((uintptr_t)d->workspace & 255) || d->workspace_bytes < need) return ULSNN_ERR_WORKSPACE;
        SmallNetArgs a{};
        a.n_in = n_in; a.n_hid = n_hid; a.n_out = n_out; a.batch = batch;
        a.W1 = W1; a.W2 = W2; a.b1 = d->b1; a.b2 = d->b2; a.X = X; a.labels = task.labels; a.targets = task.targets;
        a.partial = (float *)d->workspace; a.stride = small_net_stride(d); a.backward = task.backward ? 1 : 0;
        const int groups = (batch + SMALL_ROWS - 1) / SMALL_ROWS;
        const size_t lds = (size_t)small_net_lds_floats(n_in, n_hid, n_out) * sizeof(float);
        SmallReduceArgs r{};
        r.partial = a.partial; r.stride = a.stride; r.groups = groups;
        r.n1 = n_in * n_hid; r.n2 = n_hid * n_out; r.n_hid = n_hid; r.n_out = n_out;
        r.dW1 = task.backward ? dW1 : nullptr; r.dW2 = task.backward ? dW2 : nullptr;
        r.db1 = task.backward ? d->db1 : nullptr; r.db2 = task.backward ? d->db2 : nullptr;
        r.loss = loss; r.beta = accumulate ? 1.0f : 0.0f;
        const int total = task.backward ? r.n1 + r.n2 + n_hid + n_out + 1 : 1;
        hipLaunchKernelGGL(small_net_kernel, dim3(groups), dim3(256), lds, s, a);
        hipLaunchKernelGGL(small_reduce_kernel, dim3((total / 4 + 256) / 256), dim3(256), 0, s, r);
        HIP_TRY(hipGetLastError());
        return ULSNN_OK;
    }

    const MlpLayout L = mlp_layout(d, batch);
    if (!d->workspace || ((uintptr_t)d->workspace & 255) || d->workspace_bytes < L.bytes)
        return ULSNN_ERR_WORKSPACE;
    char *ws = (char *)d->workspace;
    float *H = (float *)(ws + L.off_h);
    float *Z = (float *)(ws + L.off_z);
    float *dA1 = (float *)(ws + L.off_da1);
    float *row_loss = (float *)(ws + L.off_rowloss);
    float *part_a = (float *)(ws + L.off_pa);
    float *part_b = (float *)(ws + L.off_pb);

    for (int r0 = 0; r0 < batch; r0 += L.slab) {
        const int rows = std::min(L.slab, batch - r0);
        const SlabPlans P = plan_slab(L, n_in, n_hid, n_out, rows);
        const float beta = (r0 > 0 || accumulate) ? 1.0f : 0.0f;
        const float *Xs = X + (size_t)r0 * n_in;
        const int32_t *ys = task.labels ? task.labels + r0 : nullptr;
        const float *ts = task.targets ? task.targets + (size_t)r0 * n_out : nullptr;
        GemmArgs a{};
        MARK(0);

        // H = tanh(Xs W1 + b1)
        a = GemmArgs{};
        a.A = Xs; a.lda = n_in; a.B = W1; a.ldb = n_hid; a.C = H; a.ldc = L.ldh;
        a.M = rows; a.N = n_hid; a.K = n_in; a.alpha = 1.f; a.beta = 0.f; a.bias = d->b1;
        HIP_TRY(launch_gemm(P.g1, true, false, EPI_BIAS_TANH, a, s));
        MARK(1);

        // Z = H W2 + b2   (softmax form)   or   Y = tanh(H W2 + b2)   (the paper's form)
        a = GemmArgs{};
        a.A = H; a.lda = L.ldh; a.B = W2; a.ldb = n_out; a.C = Z; a.ldc = L.ldz;
        a.M = rows; a.N = n_out; a.K = n_hid; a.alpha = 1.f; a.beta = 0.f; a.bias = d->b2;
        HIP_TRY(launch_gemm(P.g2, true, false, ts ? EPI_BIAS_TANH : EPI_BIAS, a, s));
        MARK(2);

        // output stage: row losses and, for a gradient, the output delta in place of Z; loss (+)= their sum
        if (ts) {
            if (task.backward)
                hipLaunchKernelGGL((mse_delta_kernel<256, true>), dim3(rows), dim3(256), 0, s, Z, L.ldz, n_out, ts,
                                   n_out, row_loss);
            else
                hipLaunchKernelGGL((mse_delta_kernel<256, false>), dim3(rows), dim3(256), 0, s, Z, L.ldz, n_out, ts,
                                   n_out, row_loss);
        } else if (n_out <= 256 * 16) {
            if (task.backward)
                hipLaunchKernelGGL((softmax_ce_kernel<256, 16>), dim3(rows), dim3(256), 0, s, Z, L.ldz, n_out, ys,
                                   row_loss);
            else
                hipLaunchKernelGGL((softmax_ce_kernel<256, 16, false>), dim3(rows), dim3(256), 0, s, Z, L.ldz,
                                   n_out, ys, row_loss);
        } else {
            if (task.backward)
                hipLaunchKernelGGL((softmax_ce_long_kernel<256>), dim3(rows), dim3(256), 0, s, Z, L.ldz, n_out, ys,
                                   row_loss);
            else
                hipLaunchKernelGGL((softmax_ce_long_kernel<256, false>), dim3(rows), dim3(256), 0, s, Z, L.ldz,
                                   n_out, ys, row_loss);
        }
        // Small batches: the dW2 reduction and the loss sum ride along with the dW1 product's launch (whose
        // partials then go to the hidden-delta region, free by then).
        const bool fuse_tail = task.backward && P.paired && P.g5.splits > 1 &&
                               (CFGS_256_THREADS >> P.g5.cfg & 1) != 0 &&
                               (size_t)P.g5.splits * n_in * n_hid <= L.floats_pb;
        if (!fuse_tail)
            hipLaunchKernelGGL(loss_reduce_kernel, dim3(1), dim3(1024), 0, s, row_loss, (long long)rows, loss, beta);
        HIP_TRY(hipGetLastError());
        MARK(3);
        if (!task.backward) {
            MARK(4); MARK(5); MARK(6); MARK(7); MARK(8);
            continue;
        }

        // dW2 (+)= H^T dO   and   dA1 = (dO W2^T) * (1 - H*H): independent of each other
        GemmArgs a3{}, a4{};
        a3.A = H; a3.lda = L.ldh; a3.B = Z; a3.ldb = L.ldz; a3.C = dW2; a3.ldc = n_out;
        a3.M = n_hid; a3.N = n_out; a3.K = rows; a3.alpha = 1.f; a3.beta = beta;
        a4.A = Z; a4.lda = L.ldz; a4.B = W2; a4.ldb = n_out; a4.C = dA1; a4.ldc = L.ldh;
        a4.M = rows; a4.N = n_hid; a4.K = n_out; a4.alpha = 1.f; a4.beta = 0.f; a4.aux = H; a4.ldaux = L.ldh;
        if (P.paired) {
            GemmArgs p3 = a3, p4 = a4;
            p3.C = part_a; p3.partial_stride = (size_t)a3.M * a3.N;
            p4.C = part_b; p4.partial_stride = (size_t)a4.M * a4.N;
            HIP_TRY(launch_pair_partial(P.g4, p4, P.g3, p3, s));
            MARK(4);
            HIP_TRY(launch_reduce(P.g4.splits, EPI_TANHGRAD, a4, part_b, s));
            if (!fuse_tail) HIP_TRY(launch_reduce(P.g3.splits, EPI_AXPBY, a3, part_a, s));
        } else {
            GemmArgs p3 = a3, p4 = a4;
            if (P.g4.splits > 1) { p4.C = part_b; p4.partial_stride = (size_t)a4.M * a4.N; }
            if (P.g3.splits > 1) { p3.C = part_a; p3.partial_stride = (size_t)a3.M * a3.N; }
            HIP_TRY(launch_gemm(P.g4, true, true, P.g4.splits > 1 ? EPI_PARTIAL : EPI_TANHGRAD, p4, s));
            HIP_TRY(launch_gemm(P.g3, false, false, P.g3.splits > 1 ? EPI_PARTIAL : EPI_AXPBY, p3, s));
            MARK(4);
            if (P.g4.splits > 1) HIP_TRY(launch_reduce(P.g4.splits, EPI_TANHGRAD, a4, part_b, s));
            if (P.g3.splits > 1 && !fuse_tail) HIP_TRY(launch_reduce(P.g3.splits, EPI_AXPBY, a3, part_a, s));
        }
        MARK(5);

        // dW1 (+)= Xs^T dA1
        a = GemmArgs{};
        a.A = Xs; a.lda = n_in; a.B = dA1; a.ldb = L.ldh; a.C = dW1; a.ldc = n_hid;
        a.M = n_in; a.N = n_hid; a.K = rows; a.alpha = 1.f; a.beta = beta;
        if (fuse_tail) {
            GemmArgs p5 = a;
            p5.C = part_b; p5.partial_stride = (size_t)a.M * a.N;
            TailWork t{};
            t.partial = part_a; t.stride = (size_t)a3.M * a3.N; t.splits = P.g3.splits;
            t.out = dW2; t.M = a3.M; t.N = a3.N; t.ldc = a3.ldc; t.beta = beta;
            t.reduce_blocks = (int)grid_for(t.stride);
            t.row_loss = row_loss; t.rows = rows; t.loss = loss; t.loss_beta = beta;
            HIP_TRY(launch_dw1_with_tail(P.g5, p5, t, s));
            MARK(6);
            HIP_TRY(launch_reduce(P.g5.splits, EPI_AXPBY, a, part_b, s));
        } else if (P.g5.splits > 1) {
            GemmArgs p5 = a;
            p5.C = part_a; p5.partial_stride = (size_t)a.M * a.N;
            HIP_TRY(launch_gemm(P.g5, false, false, EPI_PARTIAL, p5, s));
            MARK(6);
            HIP_TRY(launch_reduce(P.g5.splits, EPI_AXPBY, a, part_a, s));
        } else {
            HIP_TRY(launch_gemm(P.g5, false, false, EPI_AXPBY, a, s));
            MARK(6);
        }
        MARK(7);

        // db2 (+)= 1^T dO,  db1 (+)= 1^T dA1
        if (biases) {
            hipLaunchKernelGGL(column_sum_kernel, dim3((n_out + 63) / 64), dim3(256), 0, s, Z, L.ldz, rows, n_out,
                               d->db2, beta);
            hipLaunchKernelGGL(column_sum_kernel, dim3((n_hid + 63) / 64), dim3(256), 0, s, dA1, L.ldh, rows,
                               n_hid, d->db1, beta);
            HIP_TRY(hipGetLastError());
        }
        MARK(8);
    }
    return ULSNN_OK;
}

// The same gradient with X, W1, W2 stored as bf16 (operand_dtype 1): H, the logits and dA1 are kept in bf16 and fed
// to the bf16 matrix instructions, every product accumulates in fp32; the softmax statistics and the loss come from
// the fp32 accumulators of the output layer, the output delta exists only in registers (formed from the bf16 logits
// inside the two products that consume it), and the weight gradients are fp32.
int mlp_grad_impl16(const ulsnn_mlp_desc *d, const u16 *W1, const u16 *W2, const u16 *X, const MlpTask &task,
                    int batch, float *dW1, float *dW2, float *loss, bool accumulate, hipEvent_t *ev)
{
    hipStream_t s = (hipStream_t)d->hip_stream;
    const int n_in = d->n_in, n_hid = d->n_hid, n_out = d->n_out;
    const bool biases = d->b1 != nullptr;
    const MlpLayout L = mlp_layout(d, batch);
    if (!d->workspace || ((uintptr_t)d->workspace & 255) || d->workspace_bytes < L.bytes)
        return ULSNN_ERR_WORKSPACE;
    char *ws = (char *)d->workspace;
    u16 *H = (u16 *)(ws + L.off_h);
    float2 *stats = (float2 *)(ws + L.off_z);
    // one rows x ldz bf16 array: the logits (softmax form; the delta is formed from them inside the backward
    // products and never stored) or the output delta (squared-error form, written by the output layer's epilogue)
    u16 *dO = (u16 *)(ws + L.off_do16);
    u16 *Z16 = dO;
    float *zlab = (float *)(ws + L.off_zlab);
    float *row_lse = (float *)(ws + L.off_lse);
    u16 *dA1 = (u16 *)(ws + L.off_da1);
    float *row_loss = (float *)(ws + L.off_rowloss);
    float *part_a = (float *)(ws + L.off_pa);
    float *part_b = (float *)(ws + L.off_pb);

    // weights whose rows are not 16-byte aligned (n_out = 3203) are copied once into aligned rows
    int ldw1 = n_hid, ldw2 = n_out;
    if (!rows_16b_aligned(W1, ldw1)) {
        u16 *W1p = (u16 *)(ws + L.off_w1p);
        hipLaunchKernelGGL(repack16_kernel, dim3(grid_for((size_t)n_in * n_hid)), dim3(256), 0, s, W1, ldw1, W1p,
                           L.ldw1p, n_in, n_hid);
        W1 = W1p;
        ldw1 = L.ldw1p;
    }
    if (!rows_16b_aligned(W2, ldw2)) {
        u16 *W2p = (u16 *)(ws + L.off_w2p);
        hipLaunchKernelGGL(repack16_kernel, dim3(grid_for((size_t)n_hid * n_out)), dim3(256), 0, s, W2, ldw2, W2p,
                           L.ldw2p, n_hid, n_out);
        W2 = W2p;
        ldw2 = L.ldw2p;
    }
    HIP_TRY(hipGetLastError());

    for (int r0 = 0; r0 < batch; r0 += L.slab) {
        const int rows = std::min(L.slab, batch - r0);
        const float beta = (r0 > 0 || accumulate) ? 1.0f : 0.0f;
        const u16 *Xs = X + (size_t)r0 * n_in;
        const int32_t *ys = task.labels ? task.labels + r0 : nullptr;
        const float *ts = task.targets ? task.targets + (size_t)r0 * n_out : nullptr;
        const Gemm16Plan p1 = plan_gemm16(rows, n_hid, n_in, true, false, false, 0);
        const Gemm16Plan p2 = plan_gemm16(rows, n_out, n_hid, true, false, false, 0);
        const Gemm16Plan p3 = plan_gemm16(n_hid, n_out, rows, false, false, true, L.floats_pa);
        const Gemm16Plan p4 = plan_gemm16(rows, n_hid, n_out, true, true, true, L.floats_pb);
        const Gemm16Plan p5 = plan_gemm16(n_in, n_hid, rows, false, false, true, L.floats_pa);
        Gemm16Args a{};
        MARK(0);

        // H = tanh(Xs W1 + b1), stored bf16
        a = Gemm16Args{};
        a.A = Xs; a.lda = n_in; a.B = W1; a.ldb = ldw1; a.C = H; a.ldc = L.ldh;
        a.M = rows; a.N = n_hid; a.K = n_in; a.alpha = 1.f; a.bias = d->b1;
        HIP_TRY(launch_gemm16(p1, true, false, EPI_BIAS_TANH, a, s));
        MARK(1);

        // Z = H W2 + b2 rounded to bf16, with the softmax statistics of every row taken from the fp32 accumulators
        // in the product's epilogue (an error-only call writes the statistics alone)
        a = Gemm16Args{};
        a.A = H; a.lda = L.ldh; a.B = W2; a.ldb = ldw2; a.C = ts ? dO : Z16; a.ldc = L.ldz;
        a.M = rows; a.N = n_out; a.K = n_hid; a.alpha = 1.f; a.bias = d->b2;
        a.stats = stats; a.label_logit = zlab; a.labels = ys; a.targets = ts; a.ldt = n_out;
        const int sgw = stat_group_width(p2.cfg);
        a.stat_groups = (n_out + sgw - 1) / sgw;
        a.stat_stride = (size_t)rows;
        if (ts)   // the paper's output stage (tanh, squared error, delta) entirely in the epilogue
            HIP_TRY(launch_gemm16(p2, true, false, task.backward ? EPI_TANH_MSE : EPI_MSE_ONLY, a, s));
        else
            HIP_TRY(launch_gemm16(p2, true, false, task.backward ? EPI_BIAS_STATS : EPI_STATS_ONLY, a, s));
        MARK(2);

        // row losses (and, softmax form, each row's log-sum-exp for the delta); loss (+)= their sum
        if (ts)
            hipLaunchKernelGGL(mse16_finish_kernel, dim3((rows + 63) / 64), dim3(256), 0, s, rows,
                               (const float2 *)stats, a.stat_stride, a.stat_groups, row_loss);
        else
            hipLaunchKernelGGL(softmax16_finish_kernel, dim3((rows + 63) / 64), dim3(256), 0, s, n_out, rows,
                               (const float2 *)stats, a.stat_stride, a.stat_groups, (const float *)zlab, ys, row_loss,
                               row_lse);
        hipLaunchKernelGGL(loss_reduce_kernel, dim3(1), dim3(1024), 0, s, row_loss, (long long)rows, loss, beta);
        HIP_TRY(hipGetLastError());
        MARK(3);
        if (!task.backward) {
            MARK(4); MARK(5); MARK(6); MARK(7); MARK(8);
            continue;
        }

        // dA1 = (dO W2^T) * (1 - H*H), stored bf16, and dW2 (+)= H^T dO.  Softmax form: both products read the
        // LOGITS and form dO = softmax - onehot on the way into LDS; the delta is never stored (no pass over the
        // 2 x batch x n_out bytes of logits and delta, and no write of the delta, which cost the hidden-delta
        // product a third of its time).  Squared-error form: the delta came out of the output layer's epilogue.
        Gemm16Args a4{};
        a4.A = ts ? dO : Z16; a4.lda = L.ldz; a4.B = W2; a4.ldb = ldw2; a4.C = dA1; a4.ldc = L.ldh;
        a4.M = rows; a4.N = n_hid; a4.K = n_out; a4.alpha = 1.f; a4.aux = H; a4.ldaux = L.ldh;
        Gemm16Args a3{};
        a3.A = H; a3.lda = L.ldh; a3.B = ts ? dO : Z16; a3.ldb = L.ldz; a3.C = dW2; a3.ldc = n_out;
        a3.M = n_hid; a3.N = n_out; a3.K = rows; a3.alpha = 1.f; a3.beta = beta;
        if (!ts) {
            a4.row_lse = row_lse; a4.labels = ys;
            a3.row_lse = row_lse; a3.labels = ys;
        }
        {
            Gemm16Args q4 = a4, q3 = a3;
            if (p4.splits > 1) { q4.C = part_b; q4.partial_stride = (size_t)a4.M * a4.N; }
            if (p3.splits > 1) { q3.C = part_a; q3.partial_stride = (size_t)a3.M * a3.N; }
            HIP_TRY(launch_gemm16(p4, true, true, p4.splits > 1 ? EPI_PARTIAL : EPI_TANHGRAD, q4, s));
            HIP_TRY(launch_gemm16(p3, false, false, p3.splits > 1 ? EPI_PARTIAL : EPI_AXPBY, q3, s));
        }
        MARK(4);
        if (p4.splits > 1) {
            const size_t total = (size_t)a4.M * a4.N;
            hipLaunchKernelGGL((splitk_reduce_kernel<true, true>), dim3(grid_for(total)), dim3(256), 0, s, part_b, total,
                               p4.splits, (void *)dA1, a4.M, a4.N, a4.ldc, 1.0f, 0.0f, (const void *)H, L.ldh);
        }
        if (p3.splits > 1) {
            const size_t total = (size_t)a3.M * a3.N;
            hipLaunchKernelGGL((splitk_reduce_kernel<false, false>), dim3(grid_for(total)), dim3(256), 0, s, part_a,
                               total, p3.splits, (void *)dW2, a3.M, a3.N, a3.ldc, 1.0f, beta, (const void *)nullptr, 0);
        }
        HIP_TRY(hipGetLastError());
        MARK(5);

        // dW1 (+)= Xs^T dA1
        a = Gemm16Args{};
        a.A = Xs; a.lda = n_in; a.B = dA1; a.ldb = L.ldh; a.C = dW1; a.ldc = n_hid;
        a.M = n_in; a.N = n_hid; a.K = rows; a.alpha = 1.f; a.beta = beta;
        if (p5.splits > 1) {
            Gemm16Args q5 = a;
            q5.C = part_a; q5.partial_stride = (size_t)a.M * a.N;
            HIP_TRY(launch_gemm16(p5, false, false, EPI_PARTIAL, q5, s));
            MARK(6);
            const size_t total = (size_t)a.M * a.N;
            hipLaunchKernelGGL((splitk_reduce_kernel<false, false>), dim3(grid_for(total)), dim3(256), 0, s, part_a,
                               total, p5.splits, (void *)dW1, a.M, a.N, a.ldc, 1.0f, beta, (const void *)nullptr, 0);
            HIP_TRY(hipGetLastError());
        } else {
            HIP_TRY(launch_gemm16(p5, false, false, EPI_AXPBY, a, s));
            MARK(6);
        }
        MARK(7);

        if (biases) {
            if (ts)
                hipLaunchKernelGGL(column_sum16_kernel, dim3((n_out + 63) / 64), dim3(256), 0, s, dO, L.ldz, rows, n_out,
                                   d->db2, beta);
            else
                hipLaunchKernelGGL(column_sum16_delta_kernel, dim3((n_out + 63) / 64), dim3(256), 0, s, Z16, L.ldz, rows,
                                   n_out, (const float *)row_lse, ys, d->db2, beta);
            hipLaunchKernelGGL(column_sum16_kernel, dim3((n_hid + 63) / 64), dim3(256), 0, s, dA1, L.ldh, rows, n_hid,
                               d->db1, beta);
            HIP_TRY(hipGetLastError());
        }
        MARK(8);
    }
    return ULSNN_OK;
}

}  // namespace

// ---------------------------------------------------------------------------------------------------------
// C ABI
// ---------------------------------------------------------------------------------------------------------

extern "C" {

int ulsnn_sgemm(char transa, char transb, int m, int n, int k, float alpha, const float *A, int lda,
                const float *B, int ldb, float beta, float *C, int ldc, void *hip_stream)
{
    if (!(is_n(transa) || is_t(transa)) || !(is_n(transb) || is_t(transb))) return ULSNN_ERR_TRANS;
    if (m < 0 || n < 0 || k < 0) return ULSNN_ERR_DIM;
    const int cols_a = is_n(transa) ? k : m;
    const int cols_b = is_n(transb) ? n : k;
    if (lda < std::max(1, cols_a) || ldb < std::max(1, cols_b) || ldc < std::max(1, n)) return ULSNN_ERR_LD;
    if (lda > ULSNN_MAX_LD || ldb > ULSNN_MAX_LD) return ULSNN_ERR_UNSUPPORTED;   // 32-bit offsets inside a tile
    if (m == 0 || n == 0) return ULSNN_OK;
    if (!C) return ULSNN_ERR_NULL;
    hipStream_t s = (hipStream_t)hip_stream;
    if (k == 0 || alpha == 0.0f) {
        if (beta == 1.0f) return ULSNN_OK;
        hipLaunchKernelGGL(scale_kernel, dim3(grid_for((size_t)m * n)), dim3(256), 0, s, C, m, n, ldc, beta);
        return hipGetLastError() == hipSuccess ? ULSNN_OK : ULSNN_ERR_HIP;
    }
    if (!A || !B) return ULSNN_ERR_NULL;
    const GemmPlan p = plan_gemm(m, n, k, is_n(transa), is_t(transb), 1, ALL_CFGS);
    GemmArgs a{};
    a.A = A; a.B = B; a.C = C; a.M = m; a.N = n; a.K = k; a.lda = lda; a.ldb = ldb; a.ldc = ldc;
    a.alpha = alpha; a.beta = beta;
    return launch_gemm(p, is_n(transa), is_t(transb), EPI_AXPBY, a, s) == hipSuccess ? ULSNN_OK : ULSNN_ERR_HIP;
}

// Plan of a product that may cut k into at most `slices` slices.  A split plan costs a second launch (the
// reduction), and two launches back to back take at least 12.6 us, which the cost model prices a little low
// (measured, split against unsplit: 256^3 13 against 10 us, 512^3 12.6 against 15.7, 1024^3 TN 33 against 27,
// 2048^3 TN 158 against 168).  So a split plan is taken only where the model promises at least a fifth less time:
// the products that cannot fill the chip without it (512^3, small outputs with a long k), not the close calls.
GemmPlan plan_sgemm_ws(int m, int n, int k, bool a_kc, bool b_kc, size_t slices)
{
    const GemmPlan one = plan_gemm(m, n, k, a_kc, b_kc, 1, ALL_CFGS);
    if (slices < 2) return one;
    const GemmPlan cut = plan_gemm(m, n, k, a_kc, b_kc, (int)std::min<size_t>(64, slices), ALL_CFGS);
    return (cut.splits > 1 && cut.est_us < 0.8 * one.est_us) ? cut : one;
}

int ulsnn_sgemm_ws(char transa, char transb, int m, int n, int k, float alpha, const float *A, int lda,
                   const float *B, int ldb, float beta, float *C, int ldc, void *workspace, size_t workspace_bytes,
                   void *hip_stream)
{
    if (!(is_n(transa) || is_t(transa)) || !(is_n(transb) || is_t(transb))) return ULSNN_ERR_TRANS;
    if (m < 0 || n < 0 || k < 0) return ULSNN_ERR_DIM;
    const int cols_a = is_n(transa) ? k : m;
    const int cols_b = is_n(transb) ? n : k;
    if (lda < std::max(1, cols_a) || ldb < std::max(1, cols_b) || ldc < std::max(1, n)) return ULSNN_ERR_LD;
    if (lda > ULSNN_MAX_LD || ldb > ULSNN_MAX_LD) return ULSNN_ERR_UNSUPPORTED;
    if (workspace_bytes > 0 && (!workspace || ((uintptr_t)workspace & 255) != 0)) return ULSNN_ERR_WORKSPACE;
    if (m == 0 || n == 0 || k == 0 || alpha == 0.0f)
        return ulsnn_sgemm(transa, transb, m, n, k, alpha, A, lda, B, ldb, beta, C, ldc, hip_stream);
    if (!C || !A || !B) return ULSNN_ERR_NULL;
    // as many k slices as the planner likes and the workspace can hold partial products for
    const size_t slices = workspace_bytes / ((size_t)m * n * sizeof(float));
    const GemmPlan p = plan_sgemm_ws(m, n, k, is_n(transa), is_t(transb), slices);
    hipStream_t s = (hipStream_t)hip_stream;
    GemmArgs a{};
    a.A = A; a.B = B; a.C = C; a.M = m; a.N = n; a.K = k; a.lda = lda; a.ldb = ldb; a.ldc = ldc;
    a.alpha = alpha; a.beta = beta;
    if (p.splits == 1)
        return launch_gemm(p, is_n(transa), is_t(transb), EPI_AXPBY, a, s) == hipSuccess ? ULSNN_OK : ULSNN_ERR_HIP;
    GemmArgs q = a;
    q.C = (float *)workspace;
    q.partial_stride = (size_t)m * n;
    if (launch_gemm(p, is_n(transa), is_t(transb), EPI_PARTIAL, q, s) != hipSuccess) return ULSNN_ERR_HIP;
    return launch_reduce(p.splits, EPI_AXPBY, a, (const float *)workspace, s) == hipSuccess ? ULSNN_OK : ULSNN_ERR_HIP;
}

size_t ulsnn_mlp_grad_workspace_bytes(const ulsnn_mlp_desc *desc, int batch)
{
    if (!desc_ok(desc) || batch < 0) return 0;
    if (batch == 0) return 0;
    return mlp_layout(desc, batch).bytes;
}

int ulsnn_mlp_grad(const ulsnn_mlp_desc *desc, const void *W1, const void *W2, const void *X,
                   const int32_t *labels, int batch, float *dW1, float *dW2, float *loss)
{
    const int rc = check_mlp_args(desc, W1, W2, X, labels, batch, dW1, dW2, loss, true);
    if (rc != ULSNN_OK) return rc;
    return mlp_grad_impl(desc, W1, W2, X, MlpTask{labels, nullptr, true}, batch, dW1, dW2, loss,
                         desc->accumulate != 0);
}

// Device address of `scratch` on the current device, resolved once per device.
static int static_scratch(void **out)
{
    constexpr int MAX_DEVICES = 64;
    static std::mutex mu;
    static void *address[MAX_DEVICES] = {};
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) return ULSNN_ERR_HIP;
    std::lock_guard<std::mutex> lock(mu);
    if (!address[dev]) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return ULSNN_ERR_HIP;
        address[dev] = p;
    }
    *out = address[dev];
    return ULSNN_OK;
}

size_t ulsnn_static_scratch_bytes(void) { return (size_t)ULSNN_STATIC_SCRATCH_BYTES; }

int ulsnn_static_scratch_init(void)
{
    void *p = nullptr;
    return static_scratch(&p);
}

int ulsnn_mlp_grad_static(const ulsnn_mlp_desc *desc, const void *W1, const void *W2, const void *X,
                          const int32_t *labels, int batch, float *dW1, float *dW2, float *loss)
{
    const int rc = check_mlp_args(desc, W1, W2, X, labels, batch, dW1, dW2, loss, true);
    if (rc != ULSNN_OK) return rc;
    if (batch > 0 && mlp_layout(desc, batch).bytes > (size_t)ULSNN_STATIC_SCRATCH_BYTES) return ULSNN_ERR_WORKSPACE;
    ulsnn_mlp_desc d = *desc;
    const int rs = static_scratch(&d.workspace);
    if (rs != ULSNN_OK) return rs;
    d.workspace_bytes = (size_t)ULSNN_STATIC_SCRATCH_BYTES;
    return mlp_grad_impl(&d, W1, W2, X, MlpTask{labels, nullptr, true}, batch, dW1, dW2, loss, d.accumulate != 0);
}

int ulsnn_check_labels(const int32_t *labels, int64_t batch, int n_out, int64_t *count, void *hip_stream)
{
    if (batch < 0 || n_out < 1) return ULSNN_ERR_DIM;
    if (!count || (batch > 0 && !labels)) return ULSNN_ERR_NULL;
    hipLaunchKernelGGL(count_ignored_labels_kernel, dim3(1), dim3(1024), 0, (hipStream_t)hip_stream, labels,
                       (long long)batch, n_out, (long long *)count);
    return hipGetLastError() == hipSuccess ? ULSNN_OK : ULSNN_ERR_HIP;
}

int ulsnn_mlp_loss(const ulsnn_mlp_desc *desc, const void *W1, const void *W2, const void *X,
                   const int32_t *labels, int batch, float *loss)
{
    const int rc = check_mlp_args(desc, W1, W2, X, labels, batch, nullptr, nullptr, loss, false);
    if (rc != ULSNN_OK) return rc;
    return mlp_grad_impl(desc, W1, W2, X, MlpTask{labels, nullptr, false}, batch, nullptr, nullptr, loss,
                         desc->accumulate != 0);
}

int ulsnn_mlp_grad_mse(const ulsnn_mlp_desc *desc, const void *W1, const void *W2, const void *X, const float *T,
                       int batch, float *dW1, float *dW2, float *loss)
{
    const int rc = check_mlp_args(desc, W1, W2, X, T, batch, dW1, dW2, loss, true);
    if (rc != ULSNN_OK) return rc;
    return mlp_grad_impl(desc, W1, W2, X, MlpTask{nullptr, T, true}, batch, dW1, dW2, loss, desc->accumulate != 0);
}

int ulsnn_mlp_mse(const ulsnn_mlp_desc *desc, const void *W1, const void *W2, const void *X, const float *T,
                  int batch, float *loss)
{
    const int rc = check_mlp_args(desc, W1, W2, X, T, batch, nullptr, nullptr, loss, false);
    if (rc != ULSNN_OK) return rc;
    return mlp_grad_impl(desc, W1, W2, X, MlpTask{nullptr, T, false}, batch, nullptr, nullptr, loss,
                         desc->accumulate != 0);
}

int ulsnn_mlp_grad_epoch(const ulsnn_mlp_desc *desc, const void *W1, const void *W2, const void *X,
                         const int32_t *labels, int64_t n_patterns, int chunk, float *dW1, float *dW2,
                         float *loss)
{
    const int rc = check_mlp_args(desc, W1, W2, X, labels, (long long)n_patterns, dW1, dW2, loss, true);
    if (rc != ULSNN_OK) return rc;
    if (chunk < 1) return ULSNN_ERR_DIM;
    if (n_patterns == 0)
        return mlp_grad_impl(desc, W1, W2, nullptr, MlpTask{nullptr, nullptr, true}, 0, dW1, dW2, loss,
                             desc->accumulate != 0);
    const int first = (int)std::min<int64_t>(chunk, n_patterns);
    if (!desc->workspace || ((uintptr_t)desc->workspace & 255) ||
        desc->workspace_bytes < ulsnn_mlp_grad_workspace_bytes(desc, first))
        return ULSNN_ERR_WORKSPACE;
    const size_t elem = desc->operand_dtype == 1 ? 2 : 4;
    for (int64_t p0 = 0; p0 < n_patterns; p0 += chunk) {
        const int rows = (int)std::min<int64_t>(chunk, n_patterns - p0);
        const int r = mlp_grad_impl(desc, W1, W2, (const char *)X + (size_t)p0 * desc->n_in * elem,
                                    MlpTask{labels + p0, nullptr, true}, rows, dW1, dW2, loss,
                                    p0 > 0 || desc->accumulate != 0);
        if (r != ULSNN_OK) return r;
    }
    return ULSNN_OK;
}

int ulsnn_mlp_grad_timed(const ulsnn_mlp_desc *desc, const void *W1, const void *W2, const void *X,
                         const int32_t *labels, int batch, float *dW1, float *dW2, float *loss, float *stage_ms)
{
    const int rc = check_mlp_args(desc, W1, W2, X, labels, batch, dW1, dW2, loss, true);
    if (rc != ULSNN_OK) return rc;
    if (!stage_ms) return ULSNN_ERR_NULL;
    if (batch < 1 || batch > SLAB_ROWS) return ULSNN_ERR_UNSUPPORTED;   // one internal pass only
    hipEvent_t ev[ULSNN_MLP_STAGES + 1];
    int made = 0, out = ULSNN_OK;
    for (; made <= ULSNN_MLP_STAGES; ++made)
        if (hipEventCreate(&ev[made]) != hipSuccess) { out = ULSNN_ERR_HIP; break; }
    if (out == ULSNN_OK)
        out = mlp_grad_impl(desc, W1, W2, X, MlpTask{labels, nullptr, true}, batch, dW1, dW2, loss,
                            desc->accumulate != 0, ev);
    if (out == ULSNN_OK && hipEventSynchronize(ev[ULSNN_MLP_STAGES]) != hipSuccess) out = ULSNN_ERR_HIP;
    if (out == ULSNN_OK)
        for (int i = 0; i < ULSNN_MLP_STAGES; ++i)
            if (hipEventElapsedTime(&stage_ms[i], ev[i], ev[i + 1]) != hipSuccess) out = ULSNN_ERR_HIP;
    for (int i = 0; i < made; ++i) (void)hipEventDestroy(ev[i]);
    return out;
}

// ---------------------------------------------------------------------------------------------------------
// Optimiser step (section 4.2, last paragraph): vector primitives, Polak-Ribiere direction, line search
// ---------------------------------------------------------------------------------------------------------

namespace {

inline unsigned vec_grid(size_t n) { return (unsigned)std::min<size_t>((n + 255) / 256, (size_t)VEC_MAX_BLOCKS); }

inline bool vec_ws_ok(const void *ws, size_t bytes)
{
    return ws && ((uintptr_t)ws & 255) == 0 && bytes >= (size_t)ULSNN_VEC_WORKSPACE_BYTES;
}

// *out (device) = x . y
hipError_t launch_dot(size_t n, const float *x, const float *y, float *out, double *partial, hipStream_t s)
{
    const unsigned nb = vec_grid(n);
    hipLaunchKernelGGL(dot_partial_kernel<false>, dim3(nb), dim3(256), 0, s, n, x, y, partial);
    hipLaunchKernelGGL(dot_final_kernel<false>, dim3(1), dim3(256), 0, s, (const double *)partial, (int)nb, out);
    return hipGetLastError();
}

struct LsLayout {
    size_t mlp_bytes, n1, n2;
    size_t off_w1, off_w2, off_g1, off_g2, off_vec, off_scalars, bytes;
};

LsLayout ls_layout(const ulsnn_mlp_desc *d, int batch)
{
    LsLayout L{};
    L.mlp_bytes = round_up(mlp_layout(d, batch).bytes, 256);
    L.n1 = (size_t)d->n_in * d->n_hid;
    L.n2 = (size_t)d->n_hid * d->n_out;
    size_t off = L.mlp_bytes;
    L.off_w1 = off; off += round_up(L.n1 * 4, 256);
    L.off_w2 = off; off += round_up(L.n2 * 4, 256);
    L.off_g1 = off; off += round_up(L.n1 * 4, 256);
    L.off_g2 = off; off += round_up(L.n2 * 4, 256);
    L.off_vec = off; off += round_up((size_t)ULSNN_VEC_WORKSPACE_BYTES, 256);
    L.off_scalars = off; off += 256;
    L.bytes = off;
    return L;
}

}  // namespace

int ulsnn_dot(int64_t n, const float *x, const float *y, float *result, void *workspace, size_t workspace_bytes,
              void *hip_stream)
{
    if (n < 0) return ULSNN_ERR_DIM;
    if (!result || (n > 0 && (!x || !y))) return ULSNN_ERR_NULL;
    if (!vec_ws_ok(workspace, workspace_bytes)) return ULSNN_ERR_WORKSPACE;
    hipStream_t s = (hipStream_t)hip_stream;
    if (n == 0) {
        hipLaunchKernelGGL(zero_kernel, dim3(1), dim3(256), 0, s, result, (size_t)1);
        return hipGetLastError() == hipSuccess ? ULSNN_OK : ULSNN_ERR_HIP;
    }
    return launch_dot((size_t)n, x, y, result, (double *)workspace, s) == hipSuccess ? ULSNN_OK : ULSNN_ERR_HIP;
}

int ulsnn_axpy(int64_t n, float alpha, const float *x, float *y, void *hip_stream)
{
    if (n < 0) return ULSNN_ERR_DIM;
    if (n == 0) return ULSNN_OK;
    if (!x || !y) return ULSNN_ERR_NULL;
    hipLaunchKernelGGL(add_scaled_kernel, dim3(grid_for((size_t)n)), dim3(256), 0, (hipStream_t)hip_stream, (size_t)n,
                       (const float *)y, alpha, x, y);
    return hipGetLastError() == hipSuccess ? ULSNN_OK : ULSNN_ERR_HIP;
}

int ulsnn_cg_direction(int64_t n, const float *g_new, const float *g_old, float *d, float *beta, void *workspace,
                       size_t workspace_bytes, void *hip_stream)
{
    if (n < 0) return ULSNN_ERR_DIM;
    if (n > 0 && (!g_new || !d)) return ULSNN_ERR_NULL;
    if (!vec_ws_ok(workspace, workspace_bytes)) return ULSNN_ERR_WORKSPACE;
    hipStream_t s = (hipStream_t)hip_stream;
    double *partial = (double *)workspace;
    float *bdev = beta ? beta : (float *)((char *)workspace + 2 * VEC_MAX_BLOCKS * sizeof(double));
    if (n == 0 || !g_old) {
        if (beta) hipLaunchKernelGGL(zero_kernel, dim3(1), dim3(256), 0, s, beta, (size_t)1);
        if (n > 0)
            hipLaunchKernelGGL(cg_update_kernel, dim3(grid_for((size_t)n)), dim3(256), 0, s, (size_t)n, g_new, d,
                               (const float *)nullptr);
        return hipGetLastError() == hipSuccess ? ULSNN_OK : ULSNN_ERR_HIP;
    }
    const unsigned nb = vec_grid((size_t)n);
    hipLaunchKernelGGL(dot_partial_kernel<true>, dim3(nb), dim3(256), 0, s, (size_t)n, g_new, g_old, partial);
    hipLaunchKernelGGL(dot_final_kernel<true>, dim3(1), dim3(256), 0, s, (const double *)partial, (int)nb, bdev);
    hipLaunchKernelGGL(cg_update_kernel, dim3(grid_for((size_t)n)), dim3(256), 0, s, (size_t)n, g_new, d,
                       (const float *)bdev);
    return hipGetLastError() == hipSuccess ? ULSNN_OK : ULSNN_ERR_HIP;
}

size_t ulsnn_mlp_line_search_workspace_bytes(const ulsnn_mlp_desc *desc, int batch)
{
    if (!desc_ok(desc) || batch < 1) return 0;
    return ls_layout(desc, batch).bytes;
}

int ulsnn_mlp_line_search(const ulsnn_mlp_desc *desc, float *W1, float *W2, const float *d1, const float *d2,
                          const float *X, const int32_t *labels, int batch, int bracket_batch, float alpha0,
                          int max_doublings, ulsnn_line_search_result *result)
{
    if (!desc || !result) return ULSNN_ERR_NULL;
    if (!desc_ok(desc) || batch < 1 || bracket_batch < 1 || max_doublings < 0 || max_doublings > 60 ||
        !(alpha0 > 0.0f) || !std::isfinite(alpha0))
        return ULSNN_ERR_DIM;
    if (!W1 || !W2 || !d1 || !d2 || !X || !labels) return ULSNN_ERR_NULL;
    if (desc->b1 || desc->b2 || desc->db1 || desc->db2 || desc->operand_dtype != 0) return ULSNN_ERR_UNSUPPORTED;
    const LsLayout L = ls_layout(desc, batch);
    if (!desc->workspace || ((uintptr_t)desc->workspace & 255) != 0 || desc->workspace_bytes < L.bytes)
        return ULSNN_ERR_WORKSPACE;
    char *base = (char *)desc->workspace;
    float *T1 = (float *)(base + L.off_w1), *T2 = (float *)(base + L.off_w2);
    float *G1 = (float *)(base + L.off_g1), *G2 = (float *)(base + L.off_g2);
    double *partial = (double *)(base + L.off_vec);
    static_assert(sizeof(LineSearchScalars) <= 256, "scalars fit their workspace slot");
    LineSearchScalars *scal = (LineSearchScalars *)(base + L.off_scalars);
    hipStream_t s = (hipStream_t)desc->hip_stream;
    ulsnn_mlp_desc sub = *desc;
    sub.workspace = base;
    sub.workspace_bytes = L.mlp_bytes;
    sub.accumulate = 0;
    const int nsub = std::min(bracket_batch, batch);
    const unsigned wgrid = grid_for(L.n1 + L.n2);

    // weights at step alpha: the caller's own for alpha == 0, else T = W + alpha d (alpha from the host, or, with
    // alpha_dev, a step the device chose)
    auto weights_at = [&](double alpha, const float *alpha_dev, const float *&w1, const float *&w2) -> hipError_t {
        if (!alpha_dev && alpha == 0.0) {
            w1 = W1; w2 = W2;
            return hipSuccess;
        }
        hipLaunchKernelGGL(add_scaled2_kernel, dim3(wgrid), dim3(256), 0, s, L.n1, (const float *)W1, d1, T1, L.n2,
                           (const float *)W2, d2, T2, (float)alpha, alpha_dev);
        w1 = T1; w2 = T2;
        return hipGetLastError();
    };
    // E(W + alpha d) over all `batch` patterns (one error evaluation, section 6.2), left in *out on the device
    auto error_at = [&](double alpha, const float *alpha_dev, float *out) -> int {
        const float *w1, *w2;
        HIP_TRY(weights_at(alpha, alpha_dev, w1, w2));
        return mlp_grad_impl(&sub, w1, w2, X, MlpTask{labels, nullptr, false}, batch, nullptr, nullptr, out, false);
    };
    // grad E_sub(W + alpha d) . d on the first nsub patterns, left in *out on the device: only its sign is used
    auto slope_at = [&](double alpha, float *out) -> int {
        const float *w1, *w2;
        HIP_TRY(weights_at(alpha, nullptr, w1, w2));
        const int rc = mlp_grad_impl(&sub, w1, w2, X, MlpTask{labels, nullptr, true}, nsub, G1, G2, &scal->E[4], false);
        if (rc != ULSNN_OK) return rc;
        const unsigned nb = vec_grid(L.n1 + L.n2);
        hipLaunchKernelGGL(dot2_partial_kernel, dim3(nb), dim3(256), 0, s, L.n1, (const float *)G1, d1, L.n2,
                           (const float *)G2, d2, partial);
        hipLaunchKernelGGL(dot_final_kernel<false>, dim3(1), dim3(256), 0, s, (const double *)partial, (int)nb, out);
        HIP_TRY(hipGetLastError());
        return ULSNN_OK;
    };

    // The host reads device scalars only where it must decide what to launch next: once per group of GROUP
    // bracketing steps (the steps of a group are evaluated whether or not an earlier one of the group already
    // closed the bracket: a few spare evaluations on the small subset instead of a round trip each), and once at
    // the end.  Vertex, comparison of the errors and the weight update use steps the device computes.
    constexpr int GROUP = 8;                          // largest group; the first two hold 2 and 4 steps
    int rc;
    if ((rc = error_at(0.0, nullptr, &scal->E[0])) != ULSNN_OK) return rc;
    double lo = 0.0, hi = alpha0, prev = 0.0;
    int n_grad = 0;
    bool closed = false;
    int size = 2;
    for (int k0 = 0; k0 <= max_doublings && !closed; k0 += size, size = std::min(2 * size, GROUP)) {
        const int cnt = std::min(size, max_doublings + 1 - k0);
        for (int j = 0; j < cnt; ++j)
            if ((rc = slope_at((double)alpha0 * std::ldexp(1.0, k0 + j), &scal->slope[j])) != ULSNN_OK) return rc;
        float h[GROUP] = {};
        HIP_TRY(hipMemcpyAsync(h, scal->slope, cnt * sizeof(float), hipMemcpyDeviceToHost, s));
        HIP_TRY(hipStreamSynchronize(s));
        for (int j = 0; j < cnt; ++j) {
            hi = (double)alpha0 * std::ldexp(1.0, k0 + j);
            lo = prev;
            ++n_grad;
            if (h[j] >= 0.0f) { closed = true; break; }
            prev = hi;
        }
    }
    const bool lo_zero = lo == 0.0;
    const double mid = 0.5 * (lo + hi);
    if (!lo_zero && (rc = error_at(lo, nullptr, &scal->E[1])) != ULSNN_OK) return rc;
    if ((rc = error_at(mid, nullptr, &scal->E[2])) != ULSNN_OK) return rc;
    if ((rc = error_at(hi, nullptr, &scal->E[3])) != ULSNN_OK) return rc;
    hipLaunchKernelGGL(ls_vertex_kernel, dim3(1), dim3(1), 0, s, scal, (int)lo_zero, (float)lo, (float)hi);
    HIP_TRY(hipGetLastError());
    if ((rc = error_at(0.0, &scal->q, &scal->E[4])) != ULSNN_OK) return rc;   // at the vertex (at mid again if not convex)
    hipLaunchKernelGGL(ls_pick_kernel, dim3(1), dim3(1), 0, s, scal, (int)lo_zero, (float)lo, (float)hi);
    hipLaunchKernelGGL(add_scaled2_kernel, dim3(wgrid), dim3(256), 0, s, L.n1, (const float *)W1, d1, W1, L.n2,
                       (const float *)W2, d2, W2, 0.0f, (const float *)&scal->alpha);
    HIP_TRY(hipGetLastError());
    LineSearchScalars host{};
    HIP_TRY(hipMemcpyAsync(&host, scal, sizeof(host), hipMemcpyDeviceToHost, s));
    HIP_TRY(hipStreamSynchronize(s));
    result->alpha = host.alpha;
    result->loss = host.loss;
    result->loss0 = host.E[0];
    result->bracket_lo = (float)lo;
    result->bracket_hi = (float)hi;
    result->error_evaluations = 1 + (lo_zero ? 0 : 1) + 2 + (host.convex ? 1 : 0);   // the algorithm's own count
    result->gradient_evaluations = n_grad;
    return ULSNN_OK;
}

int ulsnn_mlp_grad_describe_plan(const ulsnn_mlp_desc *desc, int batch, char *buf, size_t buf_bytes)
{
    if (!desc || !buf) return ULSNN_ERR_NULL;
    if (!desc_ok(desc) || batch < 1 || buf_bytes < 1) return ULSNN_ERR_DIM;
    const MlpLayout L = mlp_layout(desc, batch);
    const char *what[5] = {"hidden_layer", "output_layer", "dW2", "hidden_delta", "dW1"};
    size_t used = 0;
    auto add = [&](int n) {
        if (n > 0) used = std::min(used + (size_t)n, buf_bytes - 1);
    };
    auto five_lines = [&](const SlabPlans &P) {
        const GemmPlan *g[5] = {&P.g1, &P.g2, &P.g3, &P.g4, &P.g5};
        for (int i = 0; i < 5 && used + 1 < buf_bytes; ++i)
            add(snprintf(buf + used, buf_bytes - used, "%s: tile=%s tiles=%dx%d splits=%d kchunk=%d model_us=%.1f\n",
                         what[i], CFG_INFO[g[i]->cfg].name, g[i]->tiles_m, g[i]->tiles_n, g[i]->splits, g[i]->kchunk,
                         g[i]->est_us));
    };
    const SlabPlans P = plan_slab(L, desc->n_in, desc->n_hid, desc->n_out, L.slab);
    add(snprintf(buf, buf_bytes, "rows_per_pass=%d paired_backward=%d workspace_bytes=%zu small_network_path=%d\n",
                 L.slab, (int)P.paired, L.bytes, (int)small_net_shape(desc, batch)));
    five_lines(P);
    const int tail = batch % L.slab;
    if (tail != 0 && used + 1 < buf_bytes) {
        const SlabPlans T = plan_slab(L, desc->n_in, desc->n_hid, desc->n_out, tail);
        add(snprintf(buf + used, buf_bytes - used, "tail_rows=%d paired_backward=%d\n", tail, (int)T.paired));
        five_lines(T);
    }
    return ULSNN_OK;
}

int ulsnn_sgemm_describe_plan(char transa, char transb, int m, int n, int k, char *buf, size_t buf_bytes)
{
    if (!buf) return ULSNN_ERR_NULL;
    if (!(is_n(transa) || is_t(transa)) || !(is_n(transb) || is_t(transb))) return ULSNN_ERR_TRANS;
    if (m < 1 || n < 1 || k < 1 || buf_bytes < 1) return ULSNN_ERR_DIM;
    const GemmPlan p = plan_gemm(m, n, k, is_n(transa), is_t(transb), 1, ALL_CFGS);
    snprintf(buf, buf_bytes, "tile=%s tiles=%dx%d splits=%d kchunk=%d model_us=%.1f\n", CFG_INFO[p.cfg].name,
             p.tiles_m, p.tiles_n, p.splits, p.kchunk, p.est_us);
    return ULSNN_OK;
}

int ulsnn_sgemm_ws_describe_plan(char transa, char transb, int m, int n, int k, size_t workspace_bytes, char *buf,
                                 size_t buf_bytes)
{
    if (!buf) return ULSNN_ERR_NULL;
    if (!(is_n(transa) || is_t(transa)) || !(is_n(transb) || is_t(transb))) return ULSNN_ERR_TRANS;
    if (m < 1 || n < 1 || k < 1 || buf_bytes < 1) return ULSNN_ERR_DIM;
    const size_t slices = workspace_bytes / ((size_t)m * n * sizeof(float));
    const GemmPlan p = plan_sgemm_ws(m, n, k, is_n(transa), is_t(transb), slices);
    const GemmPlan cut = plan_gemm(m, n, k, is_n(transa), is_t(transb), (int)std::min<size_t>(64, std::max<size_t>(1, slices)), ALL_CFGS);
    snprintf(buf, buf_bytes, "tile=%s tiles=%dx%d splits=%d kchunk=%d model_us=%.1f (best split plan: %d slices, %.1f us)\n",
             CFG_INFO[p.cfg].name, p.tiles_m, p.tiles_n, p.splits, p.kchunk, p.est_us, cut.splits, cut.est_us);
    return ULSNN_OK;
}

int ulsnn_sgemm_planned(int tile_shape, int k_splits, char transa, char transb, int m, int n, int k, float alpha,
                        const float *A, int lda, const float *B, int ldb, float beta, float *C, int ldc,
                        void *workspace, size_t workspace_bytes, void *hip_stream)
{
    if (!(is_n(transa) || is_t(transa)) || !(is_n(transb) || is_t(transb))) return ULSNN_ERR_TRANS;
    if (tile_shape < 0 || tile_shape >= CFG_COUNT || k_splits < 1 || m < 0 || n < 0 || k < 0) return ULSNN_ERR_DIM;
    const int cols_a = is_n(transa) ? k : m;
    const int cols_b = is_n(transb) ? n : k;
    if (lda < std::max(1, cols_a) || ldb < std::max(1, cols_b) || ldc < std::max(1, n)) return ULSNN_ERR_LD;
    if (lda > ULSNN_MAX_LD || ldb > ULSNN_MAX_LD) return ULSNN_ERR_UNSUPPORTED;
    if (m == 0 || n == 0) return ULSNN_OK;
    if (!C) return ULSNN_ERR_NULL;
    hipStream_t s = (hipStream_t)hip_stream;
    if (k == 0 || alpha == 0.0f)
        return ulsnn_sgemm(transa, transb, m, n, k, alpha, A, lda, B, ldb, beta, C, ldc, hip_stream);
    if (!A || !B) return ULSNN_ERR_NULL;
    const CfgInfo &c = CFG_INFO[tile_shape];
    GemmPlan p{};
    p.cfg = (CfgId)tile_shape;
    p.tiles_m = (m + c.bm - 1) / c.bm;
    p.tiles_n = (n + c.bn - 1) / c.bn;
    p.kchunk = (int)round_up((size_t)(k + k_splits - 1) / k_splits, c.bk);
    p.splits = (k + p.kchunk - 1) / p.kchunk;
    GemmArgs a{};
    a.A = A; a.B = B; a.C = C; a.M = m; a.N = n; a.K = k; a.lda = lda; a.ldb = ldb; a.ldc = ldc;
    a.alpha = alpha; a.beta = beta;
    if (p.splits == 1)
        return launch_gemm(p, is_n(transa), is_t(transb), EPI_AXPBY, a, s) == hipSuccess ? ULSNN_OK : ULSNN_ERR_HIP;
    const size_t need = (size_t)p.splits * m * n * sizeof(float);
    if (!workspace || ((uintptr_t)workspace & 255) != 0 || workspace_bytes < need) return ULSNN_ERR_WORKSPACE;
    GemmArgs q = a;
    q.C = (float *)workspace;
    q.partial_stride = (size_t)m * n;
    if (launch_gemm(p, is_n(transa), is_t(transb), EPI_PARTIAL, q, s) != hipSuccess) return ULSNN_ERR_HIP;
    return launch_reduce(p.splits, EPI_AXPBY, a, (const float *)workspace, s) == hipSuccess ? ULSNN_OK : ULSNN_ERR_HIP;
}

int ulsnn_device_info(int *compute_units, int *max_shader_clock_khz, int *wall_clock_khz)
{
    int dev = 0, cu = 0, sclk = 0, wall = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&cu, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess ||
        hipDeviceGetAttribute(&sclk, hipDeviceAttributeClockRate, dev) != hipSuccess ||
        hipDeviceGetAttribute(&wall, hipDeviceAttributeWallClockRate, dev) != hipSuccess) {
        (void)hipGetLastError();
        return ULSNN_ERR_HIP;
    }
    if (compute_units) *compute_units = cu;
    if (max_shader_clock_khz) *max_shader_clock_khz = sclk;
    if (wall_clock_khz) *wall_clock_khz = wall;
    return ULSNN_OK;
}

int ulsnn_clock_probe(double window_ms, unsigned long long *cycles_and_ticks, void *hip_stream)
{
    if (!cycles_and_ticks) return ULSNN_ERR_NULL;
    if (!(window_ms > 0.0) || window_ms > 1000.0) return ULSNN_ERR_DIM;
    int wall_khz = 0;
    const int rc = ulsnn_device_info(nullptr, nullptr, &wall_khz);
    if (rc != ULSNN_OK) return rc;
    if (wall_khz <= 0) return ULSNN_ERR_UNSUPPORTED;
    const unsigned long long ticks = (unsigned long long)(window_ms * (double)wall_khz);
    // one reading takes well over 100 ns (the sleep alone is 32 x 64 cycles): the cap only guards the exit
    const unsigned int max_iterations = (unsigned int)std::min(1.0e8, window_ms * 2.0e4 + 1000.0);
    hipLaunchKernelGGL(clock_probe_kernel, dim3(1), dim3(64), 0, (hipStream_t)hip_stream, ticks, max_iterations,
                       cycles_and_ticks);
    return hipGetLastError() == hipSuccess ? ULSNN_OK : ULSNN_ERR_HIP;
}

double ulsnn_sgemm_flops(int m, int n, int k) { return 2.0 * (double)m * (double)n * (double)k; }

double ulsnn_mlp_loss_flops(int n_in, int n_hid, int n_out, int64_t batch)
{
    return 2.0 * (double)batch * ((double)n_in + n_out) * n_hid;
}

double ulsnn_mlp_grad_flops(int n_in, int n_hid, int n_out, int64_t batch)
{
    return (double)batch * (4.0 * (double)n_in * n_hid + 6.0 * (double)n_hid * n_out);
}

const char *ulsnn_status_string(int status)
{
    switch (status) {
        case ULSNN_OK: return "ok";
        case ULSNN_ERR_NULL: return "null pointer";
        case ULSNN_ERR_TRANS: return "bad transpose flag";
        case ULSNN_ERR_DIM: return "bad dimension";
        case ULSNN_ERR_LD: return "leading dimension too small";
        case ULSNN_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
        case ULSNN_ERR_UNSUPPORTED: return "option not supported by this build";
        case ULSNN_ERR_HIP: return "HIP launch failed";
        default: return "unknown status";
    }
}

int ulsnn_version(void) { return 100; }

}  // extern "C"
