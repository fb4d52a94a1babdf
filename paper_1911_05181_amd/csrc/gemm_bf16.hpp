// GEMM with bf16 operands and fp32 accumulation on the gfx950 matrix cores: C = epilogue(op(A) * op(B)).
//
// Same structure as the fp32 kernel (gemm.hpp): a BM x BN tile per workgroup, 32 x 32 accumulator blocks, a k loop
// over two LDS stages with register prefetch of the next panels.  What differs:
//   * the instruction is v_mfma_f32_32x32x16_bf16: each lane supplies EIGHT consecutive k of its row
//     (k = 8*(lane/32) .. +7), so a step is BK = 32 deep and holds two such instructions per accumulator block;
//   * an operand whose k is contiguous in memory ("KC") is kept row-major in LDS and read with one 16-byte read;
//     an operand whose row/column index is contiguous ("MC") is kept k-major in LDS, exactly as it arrives, and
//     read with the LDS transpose read (ds_read_b64_tr_b16), which hands each lane four consecutive k of its own
//     row: transposition again costs no extra pass;
//   * C is fp32 (logits, split-k partials, weight gradients) or bf16 rounded to nearest-even (hidden
//     activations, hidden delta).
// The fast global fetch needs 16-byte aligned rows (pointer and leading dimension multiples of 8 elements); the
// host checks this and otherwise selects the element-wise checked fetch for every step (slow, but correct for any
// 2-byte aligned operand).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>


#include "gemm.hpp"

namespace ulsnn {

typedef unsigned short u16;
typedef u16 u16x8 __attribute__((ext_vector_type(8)));
typedef short shortx4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

__device__ __forceinline__ float bf16_to_f32(u16 v) { return __uint_as_float((unsigned)v << 16); }

// round to nearest, ties to even; NaN stays NaN: the conversion instruction of gfx950 (v_cvt_pk_bf16_f32)
typedef float floatx2_t __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ u16 f32_to_bf16(float x) { return __builtin_bit_cast(u16, (__bf16)x); }
__device__ __forceinline__ unsigned f32x2_to_bf16x2(float lo, float hi)
{
    const floatx2_t v = {lo, hi};
    return __builtin_bit_cast(unsigned, __builtin_convertvector(v, bf16x2_t));
}
typedef unsigned uintx4_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ u16x8 f32x8_to_bf16x8(const float (&v)[8])
{
    const uintx4_t p = {f32x2_to_bf16x2(v[0], v[1]), f32x2_to_bf16x2(v[2], v[3]), f32x2_to_bf16x2(v[4], v[5]),
                        f32x2_to_bf16x2(v[6], v[7])};
    return __builtin_bit_cast(u16x8, p);
}

struct Gemm16Args {
    const u16 *A, *B;
    void *C;               // float* or u16* (bf16), by epilogue
    int M, N, K;
    int lda, ldb, ldc;
    float alpha, beta;
    const float *bias;     // EPI_BIAS_TANH / EPI_BIAS, may be null
    const u16 *aux;        // EPI_TANHGRAD: the tanh outputs (bf16), same shape as C
    int ldaux;
    int kchunk;            // k range per split (multiple of 32)
    int tiles_m, tiles_n;
    size_t partial_stride; // EPI_PARTIAL: elements between consecutive partial results
    // EPI_BIAS_STATS / EPI_STATS_ONLY: softmax statistics of the logits, from the fp32 values before rounding.
    // stats[(tile_n * WN + wn) * stat_stride + i] = (max, sum of exp(z - max)) over the columns of row i that the
    // wavefront column (tile_n, wn) covers; label_logit[i] = z[i][labels[i]] where the label is in range.  Group-major,
    // so that the 16 rows a wavefront finishes together leave as one 128-byte store and the kernel that joins the
    // groups reads consecutive rows with consecutive lanes (row-major, every 8-byte pair was a partial line write:
    // the output layer at 65536 patterns wrote 543 MB where 447 MB are due).
    float2 *stats;
    int stat_groups;       // tiles_n * WN of the launch's tile shape
    size_t stat_stride;    // pairs between consecutive groups (>= M)
    float *label_logit;
    const int32_t *labels;
    // EPI_TANH_MSE / EPI_MSE_ONLY: dense fp32 targets t[i][j] (row stride ldt, 4-byte aligned); stats[..].x receives
    // the group's sum of (y - t)^2
    const float *targets;
    int ldt;
    // DELTA kernels: one operand holds the bf16 LOGITS z[pattern][class] and the product uses the output delta
    //     exp(z - row_lse[pattern]) - [class == labels[pattern]]   (rounded to bf16)
    // instead, formed in registers on the way from global memory to LDS; row_lse = +inf gives a zero row.  DELTA 1:
    // the operand is A of an NT product (patterns = rows of A, classes = k: the hidden delta); DELTA 2: it is B of a TN
    // product (patterns = k, classes = columns of B: the dW2 product).  The delta itself is never stored.
    const float *row_lse;
    int aligned;           // 1: A and B rows are 16-byte aligned (fast vector fetch allowed)
    int c_vec;             // 1: rows of C are 16-byte aligned (pointer and ldc): row-wise vector epilogue
    int aux_vec;           // 1: rows of aux are 16-byte aligned
};

// PREFETCH_ = k steps kept in flight in registers.  A bf16 step is eight times shorter on the matrix cores than an
// fp32 one, so a single step of products does not cover the latency of the next step's global loads.
template <int BM_, int BN_, int WM_, int WN_, int WAVES_PER_SIMD_ = 1, int PREFETCH_ = 1>
struct Tile16 {
    static constexpr int BM = BM_, BN = BN_, BK = 32, WM = WM_, WN = WN_, WAVES_PER_SIMD = WAVES_PER_SIMD_;
    static constexpr int PREFETCH = PREFETCH_;
    static_assert(PREFETCH_ >= 1, "prefetch depth");
    static constexpr int THREADS = WM * WN * 64;
    static constexpr int WTM = BM / WM, WTN = BN / WN;
    static constexpr int TM = WTM / 32, TN = WTN / 32;
    static_assert(WTM % 32 == 0 && WTN % 32 == 0, "tile shape");
};

// LDS footprint (bf16 elements) of one stage of one operand panel; row lengths keep 16-byte (KC) / 8-byte (MC)
// alignment of every read
template <bool KC, int R>
struct Panel16 {
    // KC: rows of 32 + 8 elements.  MC: k rows 8 banks (32 B) apart modulo the 32 banks, so the four k rows a
    // 16-lane group of the transpose read touches cover all banks once (R + 8 gave 2-way conflicts).
    static constexpr int LD = KC ? (32 + 8) : (R + 16);
    static constexpr int SIZE = KC ? R * LD : 32 * LD;
};

__device__ __forceinline__ u16x8 load8_aligned(const u16 *p) { return *reinterpret_cast<const u16x8 *>(p); }

// Checked fetch of this thread's share of a panel (rows r0.., k from k0, valid k < kend), zero filled.  With VEC and
// 16-byte aligned rows (`aligned`: pointer and leading dimension multiples of 8 elements) a vector that lies wholly
// inside the k range is one 16-byte load (an m-contiguous vector that starts inside the matrix stays inside its row,
// see FastFetch16); everything else goes element by element.  VEC is for the forward products, whose k is a layer
// width and often no multiple of 32 (n_in = 400: the hidden layer at 65536 patterns 60 -> 54 us); in the long-k
// backward kernels the extra code cost more than the one partial step it speeds up.
template <bool KC, int R, int THREADS, int NV, bool VEC>
__device__ __forceinline__ void panel16_fetch_checked(u16x8 (&reg)[NV], const u16 *__restrict__ P, int ld, int r0,
                                                      int rmax, int k0, int kend, int tid, bool aligned)
{
    constexpr int TOTAL = R * 32 / 8;
#pragma unroll
    for (int v = 0; v < NV; ++v) {
        const int f = tid + v * THREADS;
        u16x8 val = {0, 0, 0, 0, 0, 0, 0, 0};
        if (TOTAL % THREADS == 0 || f < TOTAL) {
            if (KC) {
                const int row = f / 4, kq = (f % 4) * 8;
                const int gr = r0 + row, gk = k0 + kq;
                if (gr < rmax) {
                    const u16 *src = P + (size_t)gr * ld + gk;
                    if (VEC && aligned && gk + 7 < kend) {
                        val = load8_aligned(src);
                    } else {
#pragma unroll
                        for (int e = 0; e < 8; ++e)
                            if (gk + e < kend) val[e] = src[e];
                    }
                }
            } else {
                const int krow = f / (R / 8), rq = (f % (R / 8)) * 8;
                const int gk = k0 + krow, gr = r0 + rq;
                if (gk < kend) {
                    const u16 *src = P + (size_t)gk * ld + gr;
                    if (VEC && aligned && gr < rmax) {
                        val = load8_aligned(src);
                    } else {
#pragma unroll
                        for (int e = 0; e < 8; ++e)
                            if (gr + e < rmax) val[e] = src[e];
                    }
                }
            }
        }
        reg[v] = val;
    }
}

template <bool KC, int R, int THREADS, int NV>
__device__ __forceinline__ void panel16_store(u16 *lds, const u16x8 (&reg)[NV], int tid)
{
    constexpr int TOTAL = R * 32 / 8;
    constexpr int LD = Panel16<KC, R>::LD;
#pragma unroll
    for (int v = 0; v < NV; ++v) {
        const int f = tid + v * THREADS;
        if (TOTAL % THREADS == 0 || f < TOTAL) {
            const int off = KC ? (f / 4) * LD + (f % 4) * 8 : (f / (R / 8)) * LD + (f % (R / 8)) * 8;
            *reinterpret_cast<u16x8 *>(lds + off) = reg[v];
        }
    }
}

// Unchecked 16-byte fetch for full k steps of aligned operands (pointer and leading dimension multiples of 8
// elements).  Offsets are fixed per thread as in FastFetch (gemm.hpp).  A vector that lies wholly beyond the
// matrix edge is redirected to a valid address (row clamped for KC, first column of the tile for MC).  An MC
// vector that straddles the edge needs no guard: it starts at a multiple of 8 below the width N and the row
// stride is a multiple of 8 not smaller than N, so its 8 elements stay inside the row; the elements beyond N
// only reach accumulators that are never stored.
template <bool KC, int R, int THREADS, int NV>
struct FastFetch16 {
    unsigned off[NV];
    int valid;

    __device__ __forceinline__ void init(int ld, int r0, int rmax, int tid)
    {
        constexpr int TOTAL = R * 32 / 8;
        valid = rmax - r0;
#pragma unroll
        for (int v = 0; v < NV; ++v) {
            int f = tid + v * THREADS;
            if (TOTAL % THREADS != 0 && f >= TOTAL) f = 0;
            if (KC) {
                int row = f / 4;
                const int kq = (f % 4) * 8;
                row = row < valid ? row : valid - 1;
                off[v] = (unsigned)row * (unsigned)ld + (unsigned)kq;
            } else {
                const int krow = f / (R / 8);
                int rq = (f % (R / 8)) * 8;
                if (rq >= valid) rq = 0;
                off[v] = (unsigned)krow * (unsigned)ld + (unsigned)rq;
            }
        }
    }

    __device__ __forceinline__ void fetch(u16x8 (&reg)[NV], const u16 *__restrict__ base, int tid) const
    {
        (void)tid;
#pragma unroll
        for (int v = 0; v < NV; ++v) reg[v] = load8_aligned(base + off[v]);
    }
};

// The eight consecutive k (k = 16*ks + 8*(lane/32) .. +7) of row `row + lane%32` for one 32x32x16 instruction.
template <bool KC, int R>
__device__ __forceinline__ bf16x8 panel16_read(const u16 *lds, int row, int ks, int lane)
{
    constexpr int LD = Panel16<KC, R>::LD;
    const int l32 = lane & 31, h = lane >> 5;
    u16x8 raw;
    if (KC) {
        raw = *reinterpret_cast<const u16x8 *>(lds + (row + l32) * LD + ks * 16 + h * 8);
    } else {
        // Transpose read: within each group of 16 lanes, lane s supplies the address of a chunk of four
        // consecutive rows at ONE k, and receives element s%4 of the chunks supplied by lanes s/4 + 4e, e = 0..3.
        // With lane s pointing at (k0 + s/4, rows 4*(s%4)..+3), lane j ends up with row j at k0 .. k0+3.
        const int s = lane & 15, g = (lane >> 4) & 1;
        const u16 *p = lds + (ks * 16 + h * 8 + (s >> 2)) * LD + row + 16 * g + 4 * (s & 3);
        typedef __attribute__((address_space(3))) shortx4 lds_shortx4;
        const shortx4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_shortx4 *)(p));
        const shortx4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_shortx4 *)(p + 4 * LD));
        raw = u16x8{(u16)lo.x, (u16)lo.y, (u16)lo.z, (u16)lo.w, (u16)hi.x, (u16)hi.y, (u16)hi.z, (u16)hi.w};
    }
    return __builtin_bit_cast(bf16x8, raw);
}

template <class Cfg, bool A_KC, bool B_KC>
constexpr int gemm16_lds_elems()
{
    return 2 * (Panel16<A_KC, Cfg::BM>::SIZE + Panel16<B_KC, Cfg::BN>::SIZE);
}

// tanh for a result that is rounded to bf16 straight away: tanh|x| = (1 - t) / (1 + t) with t = exp(-2|x|), one
// exponential and one reciprocal, no case distinction.  Absolute error about 1e-7 (the cancellation in 1 - t), i.e.
// relative error below the bf16 rounding (2^-9) for |x| > 3e-5 and an absolute error far below any bf16 quantum that
// matters for smaller ones.  (tanh_f32, which the fp32 results use, keeps full relative accuracy with a series for
// small arguments, at about twice the instructions.)
__device__ __forceinline__ float tanh_for_bf16(float x)
{
    const float t = __builtin_amdgcn_exp2f(-2.8853900817779268f * fabsf(x));      // 2 log2(e)
    return copysignf((1.0f - t) * __builtin_amdgcn_rcpf(1.0f + t), x);
}

// Merge two (max, sum of exp(. - max)) pairs of disjoint column sets; a pair of an empty set is (-inf, 0).
__device__ __forceinline__ void softmax_merge(float &m, float &s, float om, float os)
{
    const float nm = fmaxf(m, om);
    s = (m == nm ? s : s * __expf(m - nm)) + (om == nm ? os : os * __expf(om - nm));
    m = nm;
}

// Epilogue of one tile: the accumulators of this wavefront's sub-tile (rows i0 + wrow.., columns j0 + wcol..) leave
// through `scratch`, EPILOGUE_SCRATCH_FLOATS floats of LDS private to the wavefront, wherever rows of C are 16-byte
// aligned.  Every thread of the workgroup must call this (it starts with a workgroup barrier: the operand panels,
// whose LDS the scratch may reuse, are dead after it).
constexpr int EPILOGUE_SCRATCH_FLOATS = 32 * 36;
template <class Cfg, int EPI>
__device__ __forceinline__ void gemm16_epilogue(const Gemm16Args &g, floatx16 (&acc)[Cfg::TM][Cfg::TN],
                                                float *scratch, const int i0, const int j0, const int z,
                                                const int tile_n)
{
    constexpr int TM = Cfg::TM, TN = Cfg::TN;
    constexpr bool OUT_BF16 = (EPI == EPI_BIAS_TANH || EPI == EPI_TANHGRAD || EPI == EPI_BIAS_STATS || EPI == EPI_TANH_MSE);
    constexpr bool MSE = (EPI == EPI_TANH_MSE || EPI == EPI_MSE_ONLY);
    constexpr bool STATS = (EPI == EPI_BIAS_STATS || EPI == EPI_STATS_ONLY || MSE);
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, h = lane >> 5;
    const int wm = wave / Cfg::WN, wn = wave % Cfg::WN;
    const int wrow = wm * Cfg::WTM, wcol = wn * Cfg::WTN;
    (void)wm;
    // Epilogue.  Accumulator register r of a block holds row 8*(r/4) + 4*h + r%4, column lane%32: a lane owns a
    // COLUMN of the block, so stores straight from the accumulators are one element per lane and instruction
    // (2 bytes for bf16 results).  With 16-byte aligned rows of C (and of aux) each block instead goes through a
    // wavefront-private LDS scratch and leaves as rows: every lane handles 8 consecutive columns of one row with
    // 16-byte loads and stores, an eighth of the memory instructions.
    float *Cf = (float *)g.C;
    u16 *Ch = (u16 *)g.C;
    int ldc = g.ldc;
    if (EPI == EPI_PARTIAL) {
        Cf += (size_t)z * g.partial_stride;
        ldc = g.N;
    }
    if constexpr (STATS) {
        // Output layer with softmax statistics.  Blocks leave through the wavefront-private scratch as rows (as
        // below): a lane then holds 8 consecutive logits of ONE row, the same row for every block y of its
        // wavefront's sub-tile, so the row's running (max, sum of exp) stays in registers across y and is joined
        // over the 4 lanes that share the row with two shuffles.  C (bf16, 16-byte aligned rows: the caller's
        // workspace) is written unless only the statistics are wanted.
        constexpr int SLD = 36;
        __syncthreads();
        float *scr = scratch;
        const int srow = lane >> 2, scol = (lane & 3) * 8;
        const int group = tile_n * Cfg::WN + wn;
#pragma unroll
        for (int x = 0; x < TM; ++x) {
            float rm[2] = {-INFINITY, -INFINITY}, rs[2] = {0.f, 0.f};
            int lab[2];
#pragma unroll
            for (int pass = 0; pass < 2; ++pass) {
                const int i = i0 + wrow + x * 32 + pass * 16 + srow;
                lab[pass] = (!MSE && i < g.M) ? g.labels[i] : -1;
            }
#pragma unroll
            for (int y = 0; y < TN; ++y) {
#pragma unroll
                for (int r = 0; r < 16; ++r) scr[(8 * (r / 4) + 4 * h + (r % 4)) * SLD + l32] = acc[x][y][r];
                __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
                __builtin_amdgcn_wave_barrier();
#pragma unroll
                for (int pass = 0; pass < 2; ++pass) {
                    const int row = pass * 16 + srow;
                    const floatx4 lo = *reinterpret_cast<const floatx4 *>(scr + row * SLD + scol);
                    const floatx4 hi = *reinterpret_cast<const floatx4 *>(scr + row * SLD + scol + 4);
                    if (pass == 1) {
                        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
                        __builtin_amdgcn_wave_barrier();
                    }
                    float v[8] = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
                    const int i = i0 + wrow + x * 32 + row;
                    const int j = j0 + wcol + y * 32 + scol;
                    if (i >= g.M || j >= g.N) continue;
                    if (MSE) {
                        // the paper's output stage on the spot: no row-wide quantity is needed for the delta
                        const float *tp = g.targets + (size_t)i * g.ldt + j;
                        float t[8];
                        if (j + 7 < g.N) {                       // two 16-byte loads (rows are only 4-byte aligned)
                            const floatx4 t0 = load4_any_align(tp), t1 = load4_any_align(tp + 4);
                            t[0] = t0.x; t[1] = t0.y; t[2] = t0.z; t[3] = t0.w;
                            t[4] = t1.x; t[5] = t1.y; t[6] = t1.z; t[7] = t1.w;
                        } else {
#pragma unroll
                            for (int e = 0; e < 8; ++e) t[e] = j + e < g.N ? tp[e] : 0.f;
                        }
                        const bool whole = j + 7 < g.N;
                        if (g.bias) {
#pragma unroll
                            for (int e = 0; e < 8; ++e) v[e] += (whole || j + e < g.N) ? g.bias[j + e] : 0.f;
                        }
                        float err = 0.f;
#pragma unroll
                        for (int e = 0; e < 8; ++e) {
                            // (the delta is rounded to bf16; the error is summed from y with an absolute error of 1e-7)
                            const float yv = tanh_for_bf16(v[e]);
                            const float diff = (whole || j + e < g.N) ? yv - t[e] : 0.f;
                            err += diff * diff;
                            v[e] = 2.0f * diff * (1.0f - yv * yv);
                        }
                        rs[pass] += err;
                    } else {
                    // (the whole vector lies inside the matrix except in the last column tile, and the label falls
                    // into this vector once per row: both cases are kept out of the per-element work)
                    const bool whole = j + 7 < g.N;
                    if (g.bias) {
#pragma unroll
                        for (int e = 0; e < 8; ++e) v[e] += (whole || j + e < g.N) ? g.bias[j + e] : 0.f;
                    }
                    if (!whole) {
#pragma unroll
                        for (int e = 1; e < 8; ++e) v[e] = j + e < g.N ? v[e] : -INFINITY;   // exp(-inf) = 0
                    }
                    const float bm = fmaxf(fmaxf(fmaxf(v[0], v[1]), fmaxf(v[2], v[3])),
                                           fmaxf(fmaxf(v[4], v[5]), fmaxf(v[6], v[7])));
                    const float nm = fmaxf(rm[pass], bm);      // finite: column j itself is inside the matrix
                    const float nml = -nm * 1.44269504088896340736f;       // exp(v - nm) = 2^(v log2e - nm log2e)
                    float bs = 0.f;
#pragma unroll
                    for (int e = 0; e < 8; ++e)
                        bs += __builtin_amdgcn_exp2f(__builtin_fmaf(v[e], 1.44269504088896340736f, nml));
                    rs[pass] = (rm[pass] == nm ? rs[pass] : rs[pass] * __expf(rm[pass] - nm)) + bs;
                    rm[pass] = nm;
                    const unsigned at_label = (unsigned)(lab[pass] - j);
                    if (at_label < 8u && lab[pass] < g.N) {
                        float zl = v[0];
#pragma unroll
                        for (int e = 1; e < 8; ++e) zl = at_label == (unsigned)e ? v[e] : zl;
                        g.label_logit[i] = zl;
                    }
                    }
                    if (EPI == EPI_BIAS_STATS || EPI == EPI_TANH_MSE) {
                        const u16x8 o = f32x8_to_bf16x8(v);
                        const size_t at = (size_t)i * g.ldc + j;
                        if (j + 7 < g.N) {
                            *reinterpret_cast<u16x8 *>(Ch + at) = o;
                        } else {
#pragma unroll
                            for (int e = 0; e < 8; ++e)
                                if (j + e < g.N) Ch[at + e] = o[e];
                        }
                    }
                }
            }
#pragma unroll
            for (int pass = 0; pass < 2; ++pass) {
#pragma unroll
                for (int o = 1; o <= 2; o <<= 1) {
                    const float om = __shfl_xor(rm[pass], o, 64), os = __shfl_xor(rs[pass], o, 64);
                    if (MSE) rs[pass] += os;
                    else softmax_merge(rm[pass], rs[pass], om, os);
                }
                const int i = i0 + wrow + x * 32 + pass * 16 + srow;
                if ((lane & 3) == 0 && i < g.M && j0 + wcol < g.N)
                    g.stats[(size_t)group * g.stat_stride + i] = MSE ? make_float2(rs[pass], 0.f) : make_float2(rm[pass], rs[pass]);
            }
        }
        return;
    }
    const bool rows_vec = (EPI == EPI_PARTIAL) ? ((g.N & 3) == 0 && (g.partial_stride & 3) == 0 && g.c_vec) : g.c_vec != 0;
    if (rows_vec) {
        constexpr int SLD = 36;                                   // scratch row stride (floats): 16-byte aligned rows
        __syncthreads();                                          // every wavefront is done reading the panels
        float *scr = scratch;
        const int srow = lane >> 2, scol = (lane & 3) * 8;        // this lane's row (of 16 per pass) and 8 columns
#pragma unroll
        for (int x = 0; x < TM; ++x) {
#pragma unroll
            for (int y = 0; y < TN; ++y) {
#pragma unroll
                for (int r = 0; r < 16; ++r) scr[(8 * (r / 4) + 4 * h + (r % 4)) * SLD + l32] = acc[x][y][r];
                // LDS operations of one wavefront complete in order; the fences keep the compiler from moving the
                // reads of other lanes' elements above these writes (and the next block's writes above the reads)
                __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
                __builtin_amdgcn_wave_barrier();
#pragma unroll
                for (int pass = 0; pass < 2; ++pass) {
                    const int row = pass * 16 + srow;
                    const floatx4 lo = *reinterpret_cast<const floatx4 *>(scr + row * SLD + scol);
                    const floatx4 hi = *reinterpret_cast<const floatx4 *>(scr + row * SLD + scol + 4);
                    if (pass == 1) {
                        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
                        __builtin_amdgcn_wave_barrier();
                    }
                    float v[8] = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
                    const int i = i0 + wrow + x * 32 + row;
                    const int j = j0 + wcol + y * 32 + scol;
                    if (i >= g.M || j >= g.N) continue;
                    const bool whole = j + 7 < g.N;
                    const size_t at = (size_t)i * ldc + j;
                    if (EPI == EPI_BIAS_TANH || EPI == EPI_BIAS) {
#pragma unroll
                        for (int e = 0; e < 8; ++e) v[e] += (g.bias && j + e < g.N) ? g.bias[j + e] : 0.f;
                    }
                    if (EPI == EPI_TANHGRAD) {
                        const u16 *ap = g.aux + (size_t)i * g.ldaux + j;
                        u16x8 hv;
                        if (whole && g.aux_vec) {
                            hv = load8_aligned(ap);
                        } else {
#pragma unroll
                            for (int e = 0; e < 8; ++e) hv[e] = j + e < g.N ? ap[e] : (u16)0;
                        }
#pragma unroll
                        for (int e = 0; e < 8; ++e) {
                            const float t = bf16_to_f32(hv[e]);
                            v[e] *= (1.0f - t * t);
                        }
                    }
                    if (EPI == EPI_BIAS_TANH) {
#pragma unroll
                        for (int e = 0; e < 8; ++e) v[e] = tanh_for_bf16(v[e]);
                    }
                    if (OUT_BF16) {
                        const u16x8 o = f32x8_to_bf16x8(v);
                        if (whole) {
                            *reinterpret_cast<u16x8 *>(Ch + at) = o;
                        } else {
#pragma unroll
                            for (int e = 0; e < 8; ++e)
                                if (j + e < g.N) Ch[at + e] = o[e];
                        }
                    } else {
                        if (EPI == EPI_AXPBY) {
#pragma unroll
                            for (int e = 0; e < 8; ++e) {
                                v[e] *= g.alpha;
                                if (g.beta != 0.f && j + e < g.N) v[e] += g.beta * Cf[at + e];
                            }
                        }
                        if (whole) {
                            *reinterpret_cast<floatx4 *>(Cf + at) = floatx4{v[0], v[1], v[2], v[3]};
                            *reinterpret_cast<floatx4 *>(Cf + at + 4) = floatx4{v[4], v[5], v[6], v[7]};
                        } else {
#pragma unroll
                            for (int e = 0; e < 8; ++e)
                                if (j + e < g.N) Cf[at + e] = v[e];
                        }
                    }
                }
            }
        }
        return;
    }
#pragma unroll
    for (int y = 0; y < TN; ++y) {
        const int j = j0 + wcol + y * 32 + l32;
        if (j >= g.N) continue;
        float bias = 0.f;
        if ((EPI == EPI_BIAS_TANH || EPI == EPI_BIAS) && g.bias) bias = g.bias[j];
#pragma unroll
        for (int x = 0; x < TM; ++x) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int i = i0 + wrow + x * 32 + 8 * (r / 4) + 4 * h + (r % 4);
                if (i >= g.M) continue;
                const float v = acc[x][y][r];
                const size_t at = (size_t)i * ldc + j;
                if (EPI == EPI_AXPBY) {
                    float out = g.alpha * v;
                    if (g.beta != 0.f) out += g.beta * Cf[at];
                    Cf[at] = out;
                } else if (EPI == EPI_PARTIAL) {
                    Cf[at] = v;
                } else if (EPI == EPI_BIAS_TANH) {
                    Ch[at] = f32_to_bf16(tanh_for_bf16(v + bias));
                } else if (EPI == EPI_BIAS) {
                    Cf[at] = v + bias;
                } else {
                    const float hv = bf16_to_f32(g.aux[(size_t)i * g.ldaux + j]);
                    Ch[at] = f32_to_bf16(v * (1.0f - hv * hv));
                }
            }
        }
    }
    (void)OUT_BF16;
}

// OUT_BF16: C is bf16 (EPI_BIAS_TANH, EPI_TANHGRAD, EPI_BIAS_STATS) else fp32.
template <class Cfg, bool A_KC, bool B_KC, int EPI, int DELTA = 0>
__device__ __forceinline__ void gemm16_tile(const Gemm16Args &g, const int hw, const int splits, u16 *lds)
{
    constexpr bool DELTA_A = DELTA == 1, DELTA_B = DELTA == 2;
    static_assert(!DELTA_A || A_KC, "the delta is formed on a k-contiguous A operand ...");
    static_assert(!DELTA_B || !B_KC, "... or on an m-contiguous B operand");
    constexpr int BM = Cfg::BM, BN = Cfg::BN, BK = 32, THREADS = Cfg::THREADS;
    constexpr int TM = Cfg::TM, TN = Cfg::TN;
    using PA = Panel16<A_KC, BM>;
    using PB = Panel16<B_KC, BN>;
    constexpr int NVA = (BM * BK / 8 + THREADS - 1) / THREADS;
    constexpr int NVB = (BN * BK / 8 + THREADS - 1) / THREADS;

    auto stage_a = [&](int st) { return lds + st * PA::SIZE; };
    auto stage_b = [&](int st) { return lds + 2 * PA::SIZE + st * PB::SIZE; };

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave / Cfg::WN, wn = wave % Cfg::WN;
    const int wrow = wm * Cfg::WTM, wcol = wn * Cfg::WTN;

    int tile_m, tile_n, z;
    work_of_workgroup(hw, g.tiles_m, g.tiles_n, splits, tile_m, tile_n, z);
    const int i0 = tile_m * BM, j0 = tile_n * BN;
    const int kbeg = z * g.kchunk;
    const int kend = (kbeg + g.kchunk < g.K) ? kbeg + g.kchunk : g.K;
    // without 16-byte aligned rows every step goes through the checked fetch
    const int nfull = g.aligned ? (kend - kbeg) / BK : 0;
    const int nkb = (kend - kbeg + BK - 1) / BK;

    floatx16 acc[TM][TN];
#pragma unroll
    for (int a = 0; a < TM; ++a)
#pragma unroll
        for (int b = 0; b < TN; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.f;

    FastFetch16<A_KC, BM, THREADS, NVA> fa;
    FastFetch16<B_KC, BN, THREADS, NVB> fb;
    fa.init(g.lda, i0, g.M, tid);
    fb.init(g.ldb, j0, g.N, tid);
    const u16 *pa = A_KC ? g.A + (size_t)i0 * g.lda + kbeg : g.A + (size_t)kbeg * g.lda + i0;
    const u16 *pb = B_KC ? g.B + (size_t)j0 * g.ldb + kbeg : g.B + (size_t)kbeg * g.ldb + j0;
    const size_t step_a = A_KC ? (size_t)BK : (size_t)BK * g.lda;
    const size_t step_b = B_KC ? (size_t)BK : (size_t)BK * g.ldb;

    constexpr int D = Cfg::PREFETCH;
    // Register slots of the fetch pipeline: while step kb is multiplied out of LDS, the loads of steps
    // kb+1 .. kb+D are in flight; step s lives in slot s % D (the loops below are unrolled so that slot numbers are
    // compile-time constants).
    u16x8 ra[D][NVA], rb[D][NVB];
#pragma unroll
    for (int u = 0; u < D; ++u) {
#pragma unroll
        for (int v = 0; v < NVA; ++v) ra[u][v] = u16x8{0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
        for (int v = 0; v < NVB; ++v) rb[u][v] = u16x8{0, 0, 0, 0, 0, 0, 0, 0};
    }

    // DELTA: the logits in the fetch registers become the output delta just before they are stored to LDS (the
    // transform is issued ahead of the matrix instructions of the step that hides it).
    constexpr float LOG2E = 1.44269504088896340736f;
    auto to_delta = [&](u16x8 &reg, const float nl, const int lab) {   // nl = -lse*log2(e); lab relative to element 0
        const uintx4_t raw = __builtin_bit_cast(uintx4_t, reg);
        float d[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const float x = __uint_as_float((e & 1) ? (raw[e >> 1] & 0xffff0000u) : (raw[e >> 1] << 16));
            const float p = __builtin_amdgcn_exp2f(__builtin_fmaf(x, LOG2E, nl));
            d[e] = p - (lab == e ? 1.0f : 0.0f);
        }
        reg = f32x8_to_bf16x8(d);
    };
    // DELTA 1 (A, k-contiguous): each thread's vectors stay on the same rows (patterns) for the whole k loop, so the
    // row's log-sum-exp and label are loaded once; the label moves BK classes down per step.
    static_assert(!DELTA_A || (BM * BK / 8) % THREADS == 0, "every thread owns whole vectors of the A panel");
    float a_nl[NVA];       // -lse * log2(e) of the vector's row
    int a_lab[NVA];        // label of that row, relative to the first k of the vector in the step about to be stored
    if constexpr (DELTA_A) {
#pragma unroll
        for (int v = 0; v < NVA; ++v) {
            const int f = tid + v * THREADS;
            int row = f / 4;
            row = row < g.M - i0 ? row : g.M - i0 - 1;
            a_nl[v] = -g.row_lse[i0 + row] * LOG2E;
            a_lab[v] = g.labels[i0 + row] - kbeg - (f % 4) * 8;
        }
    }
    auto prepare_a = [&](u16x8 (&reg)[NVA], const int k_first, const bool checked) {
        if constexpr (DELTA_A) {
#pragma unroll
            for (int v = 0; v < NVA; ++v) {
                to_delta(reg[v], a_nl[v], a_lab[v]);
                a_lab[v] -= BK;
                if (checked) {                                 // the partial last step: classes beyond K stay zero
                    const int kq = k_first + ((tid + v * THREADS) % 4) * 8;
#pragma unroll
                    for (int e = 0; e < 8; ++e)
                        if (kq + e >= kend) reg[v][e] = 0;
                }
            }
        }
    };
    // DELTA 2 (B, m-contiguous): a vector is eight classes of ONE pattern, and the pattern (the k row) changes with
    // every step, so log-sum-exp and label of a vector's pattern travel with the panel: they are loaded when the
    // panel is fetched, into the same register slot.  A k row beyond the range (partial last step, zero filled)
    // gets -inf, which keeps it zero.
    static_assert(!DELTA_B || (BN * BK / 8) % THREADS == 0, "every thread owns whole vectors of the B panel");
    // (The loaded values are kept raw until the panel is stored: arithmetic on them at fetch time would make the
    // compiler wait for the loads on the spot.)
    float b_lse[Cfg::PREFETCH][NVB];
    int b_lab[Cfg::PREFETCH][NVB];
    auto fetch_b_meta = [&](const int slot, const int k_first, const bool checked) {
        if constexpr (DELTA_B) {
#pragma unroll
            for (int v = 0; v < NVB; ++v) {
                const int k = k_first + (tid + v * THREADS) / (BN / 8);
                if (!checked || k < kend) {
                    b_lse[slot][v] = g.row_lse[k];
                    b_lab[slot][v] = g.labels[k];
                } else {
                    b_lse[slot][v] = INFINITY;
                    b_lab[slot][v] = -8;
                }
            }
        }
    };
    auto prepare_b = [&](const int slot, u16x8 (&reg)[NVB]) {
        if constexpr (DELTA_B) {
#pragma unroll
            for (int v = 0; v < NVB; ++v) {
                const int col0 = j0 + ((tid + v * THREADS) % (BN / 8)) * 8;     // class of the vector's first element
                to_delta(reg[v], -b_lse[slot][v] * LOG2E, b_lab[slot][v] - col0);
            }
        }
    };
    auto store_a = [&](u16 *stage_ptr, const u16x8 (&reg)[NVA]) {
        panel16_store<A_KC, BM, THREADS, NVA>(stage_ptr, reg, tid);
    };

    const u16 *na = pa, *nb = pb;   // where the next unchecked fetch reads ...
    int nk = kbeg;                  // ... and the k it starts at
    auto fetch_full = [&](const int slot) {
        fa.fetch(ra[slot], na, tid);
        fb.fetch(rb[slot], nb, tid);
        fetch_b_meta(slot, nk, false);
        na += step_a;
        nb += step_b;
        nk += BK;
    };
    auto fetch_checked = [&](const int slot, const int k0) {
        panel16_fetch_checked<A_KC, BM, THREADS, NVA, A_KC && !B_KC>(ra[slot], g.A, g.lda, i0, g.M, k0, kend, tid, g.aligned != 0);
        panel16_fetch_checked<B_KC, BN, THREADS, NVB, A_KC && !B_KC>(rb[slot], g.B, g.ldb, j0, g.N, k0, kend, tid, g.aligned != 0);
        fetch_b_meta(slot, k0, true);
    };
    if (nkb > 0) {
        if (nfull > 0) {
#pragma unroll
            for (int u = 0; u < D; ++u)
                if (u < nfull) fetch_full(u);
        } else {
            fetch_checked(0, kbeg);
        }
        prepare_a(ra[0], kbeg, nfull == 0);
        prepare_b(0, rb[0]);
        store_a(stage_a(0), ra[0]);
        panel16_store<B_KC, BN, THREADS, NVB>(stage_b(0), rb[0], tid);
    }
    __syncthreads();

    auto compute = [&](int cur) {
        const u16 *la = stage_a(cur), *lb = stage_b(cur);
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            bf16x8 a[TM], b[TN];
#pragma unroll
            for (int x = 0; x < TM; ++x) a[x] = panel16_read<A_KC, BM>(la, wrow + x * 32, ks, lane);
#pragma unroll
            for (int y = 0; y < TN; ++y) b[y] = panel16_read<B_KC, BN>(lb, wcol + y * 32, ks, lane);
#pragma unroll
            for (int x = 0; x < TM; ++x)
#pragma unroll
                for (int y = 0; y < TN; ++y)
                    acc[x][y] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[x], b[y], acc[x][y], 0, 0, 0);
        }
    };

    // Full steps 0 .. nfull-1.  On entry to step kb its panels are in LDS stage kb & 1 and slot kb % D is free.
    // Steady state first: while every step of a round of D still has a step D ahead to fetch, the round is
    // branch-free, so the compiler's wait for the slot being stored leaves the newer loads in flight (at a join
    // of "fetched" and "not fetched" paths it would have to wait for everything, which defeats the pipeline).
    int base = 0;
    if constexpr (D > 1) {
    for (; base + 2 * D <= nfull; base += D) {
#pragma unroll
        for (int u = 0; u < D; ++u) {
            const int cur = (base + u) & 1;
            const int un = (u + 1) % D;
            fetch_full(u);
            prepare_a(ra[un], kbeg + (base + u + 1) * BK, false);   // independent of the products below
            prepare_b(un, rb[un]);
            compute(cur);
            store_a(stage_a(cur ^ 1), ra[un]);
            panel16_store<B_KC, BN, THREADS, NVB>(stage_b(cur ^ 1), rb[un], tid);
            if constexpr (DELTA_B) {
                // The dW2 product has the least idle time of all: left to itself the compiler puts the transform in
                // one block ahead of the matrix instructions, and with every wavefront of the workgroup in step
                // (a barrier per k step) the two kinds of work then take turns instead of overlapping.  Ask for one
                // matrix instruction followed by the vector instructions that fit in its shadow (5 plain + 1
                // transcendental; 3, 4 and 6 measured slower, and on the hidden-delta product any such order was).
#pragma unroll
                for (int i = 0; i < 2 * TM * TN; ++i) {
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);   // 1 matrix instruction
                    __builtin_amdgcn_sched_group_barrier(0x002, 5, 0);   // 5 vector ALU instructions
                    __builtin_amdgcn_sched_group_barrier(0x400, 1, 0);   // 1 transcendental
                }
            }
            __syncthreads();
        }
    }
    }
    // Drain: the last rounds, where fetches run out (with a single slot: every step).
    for (; base < nfull; base += D) {
#pragma unroll
        for (int u = 0; u < D; ++u) {
            const int kb = base + u;
            if (kb < nfull) {
                const int cur = kb & 1, next = kb + 1;
                const int un = (u + 1) % D;            // slot of step kb + 1
                if (kb + D < nfull) fetch_full(u);     // refill the free slot with step kb + D
                if (next == nfull && next < nkb)       // the partial last step: checked fetch, zero filled
                    fetch_checked(un, kbeg + next * BK);
                if (next < nkb) {
                    prepare_a(ra[un], kbeg + next * BK, next == nfull);
                    prepare_b(un, rb[un]);
                }
                compute(cur);
                if (next < nkb) {
                    store_a(stage_a(cur ^ 1), ra[un]);
                    panel16_store<B_KC, BN, THREADS, NVB>(stage_b(cur ^ 1), rb[un], tid);
                }
                __syncthreads();
            }
        }
    }
    // Steps from nfull on: the one partial step after full ones (already in LDS), or every step of an operand
    // without 16-byte aligned rows (nfull == 0).
    for (int kb = nfull; kb < nkb; ++kb) {
        const int cur = kb & 1;
        const bool more = kb + 1 < nkb;
        if (more) {
            fetch_checked(0, kbeg + (kb + 1) * BK);
            prepare_a(ra[0], kbeg + (kb + 1) * BK, true);
            prepare_b(0, rb[0]);
        }
        compute(cur);
        if (more) {
            store_a(stage_a(cur ^ 1), ra[0]);
            panel16_store<B_KC, BN, THREADS, NVB>(stage_b(cur ^ 1), rb[0], tid);
        }
        __syncthreads();
    }
    static_assert(gemm16_lds_elems<Cfg, A_KC, B_KC>() * 2 >= Cfg::WM * Cfg::WN * EPILOGUE_SCRATCH_FLOATS * 4,
                  "epilogue scratch fits in the panels' LDS");
    gemm16_epilogue<Cfg, EPI>(g, acc, reinterpret_cast<float *>(lds) + wave * EPILOGUE_SCRATCH_FLOATS, i0, j0, z, tile_n);
}

template <class Cfg, bool A_KC, bool B_KC, int EPI, int DELTA = 0>
__global__ __launch_bounds__(Cfg::THREADS, Cfg::WAVES_PER_SIMD) void gemm16_kernel(const Gemm16Args g)
{
    __shared__ __attribute__((aligned(16))) u16 lds[gemm16_lds_elems<Cfg, A_KC, B_KC>()];
    gemm16_tile<Cfg, A_KC, B_KC, EPI, DELTA>(g, blockIdx.y * gridDim.x + blockIdx.x, gridDim.y, lds);
}

}  // namespace ulsnn
