// fp32 GEMM on the gfx950 matrix cores: C = epilogue(op(A) * op(B)).
//
// One workgroup computes a BM x BN tile of C.  It is WM x WN wavefronts of 64 lanes; each wavefront owns a
// (BM/WM) x (BN/WN) sub-tile built from 32 x 32 accumulator blocks of v_mfma_f32_32x32x2_f32.  The k loop runs
// in steps of BK: the next A and B panels are fetched from global memory into registers while the matrix cores
// work on the current panels in LDS (two LDS stages, one barrier per step).
//
// Operand layouts.  An operand is "KC" when k is the contiguous direction of its storage (A for op = N,
// B for op = T) and "MC" when the row/column index of C is (A for op = T, B for op = N).  Both are fetched
// with 16-byte loads along their contiguous direction and stored to LDS the same way round, so transposition
// costs nothing: it only changes which LDS addresses a lane reads.  The 32x32x2 instruction takes, per lane,
// ONE element of A (row lane%32, k = lane/32) and ONE of B (column lane%32, same k).  Because a sum over k does
// not care about the order of its terms, lane half h = lane/32 is given k = 8*s + 4*h + t in the t-th
// instruction of the s-th group of four: a KC operand then needs a single 16-byte LDS read per 32 rows per
// group, an MC operand four 4-byte reads.
//
// Edges.  Rows/columns beyond M/N are fetched from a clamped (valid) address or zero filled and never stored;
// k beyond the end of the workgroup's k range is zero filled.  Pointers need only 4-byte alignment.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>

namespace ulsnn {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx4 __attribute__((ext_vector_type(4)));

enum Epilogue {
    EPI_AXPBY = 0,      // C = alpha*acc + beta*C   (beta == 0: C not read)
    EPI_PARTIAL = 1,    // split-k partial: P[z] = acc (dense, ld = N)
    EPI_BIAS_TANH = 2,  // C = tanh(acc + bias[j])
    EPI_BIAS = 3,       // C = acc + bias[j]
    EPI_TANHGRAD = 4,   // C = acc * (1 - aux[i][j]^2)
    // bf16-operand kernel only: output layer with the softmax statistics of its rows taken in the epilogue
    EPI_BIAS_STATS = 5, // C = bf16(acc + bias[j]); per row and column group: max and sum of exp; the label's logit
    EPI_STATS_ONLY = 6, // the same statistics, C not written (error-only evaluation)
    // bf16-operand kernel only: output layer of the squared-error form, output stage taken in the epilogue
    EPI_TANH_MSE = 7,   // y = tanh(acc + bias[j]); C = bf16(2 (y - t)(1 - y^2)); per row and column group: sum (y - t)^2
    EPI_MSE_ONLY = 8    // the same sums, C not written
};

struct GemmArgs {
    const float *A, *B;
    float *C;
    int M, N, K;
    int lda, ldb, ldc;
    float alpha, beta;
    const float *bias;   // EPI_BIAS_TANH / EPI_BIAS, may be null (no bias)
    const float *aux;    // EPI_TANHGRAD: the tanh outputs, same shape as C
    int ldaux;
    int kchunk;          // k range handled per blockIdx.y (multiple of BK); >= K when there is no split
    int tiles_m, tiles_n;
    size_t partial_stride;  // EPI_PARTIAL: elements between consecutive partial results
};

// WAVES_PER_SIMD_ is the occupancy the register allocation must allow (wavefronts per SIMD).
// KW_ > 1: KW_ groups of WM x WN wavefronts share the tile; each group takes 1/KW_ of every k step and the
// groups' accumulators are added through LDS before the epilogue (in group order, so the sum is reproducible).
// It gives a launch with few workgroups per compute unit more wavefronts per SIMD to hide latency with.
template <int BM_, int BN_, int BK_, int WM_, int WN_, int WAVES_PER_SIMD_ = 1, int KW_ = 1>
struct TileCfg {
    static constexpr int BM = BM_, BN = BN_, BK = BK_, WM = WM_, WN = WN_, WAVES_PER_SIMD = WAVES_PER_SIMD_;
    static constexpr int KW = KW_;
    static constexpr int THREADS = WM * WN * KW * 64;
    static constexpr int WTM = BM / WM, WTN = BN / WN;   // wavefront sub-tile
    static constexpr int TM = WTM / 32, TN = WTN / 32;   // 32x32 accumulator blocks per wavefront
    // k-contiguous panels: dense rows with permuted 16-byte chunks (no LDS bank conflicts at all) or rows padded
    // by 4 floats (conflict-free fragment reads, two-way conflicts in the panel stores).  Measured: the permuted
    // layout takes the conflict counter to zero everywhere and is 0.6 % faster on the batch-4096 gradient (small
    // tiles), but 3 % slower on 8192^3 NT with the 256 x 128 tile, which keeps the padded rows.
    static constexpr bool PERMUTE_KC = BM < 256;
    static_assert(WTM % 32 == 0 && WTN % 32 == 0 && BK % 8 == 0 && (BK / 8) % KW == 0, "tile shape");
};

// LDS footprint (floats) of one stage of one operand panel with R rows/columns of C.
// MC panels: k rows of R + 8 floats.  KC panels, PERM: rows of BK floats, dense; the 16-byte chunk c of row r sits
// at chunk position c ^ kc_chunk_key(r), which keeps every group of 8 and of 16 consecutive rows that access the
// same chunk number on different banks, for fragment reads and panel stores alike.  KC panels, not PERM: rows
// padded to BK + 4 floats (the fragment reads are conflict free, the 16-byte stores are not: four consecutive rows
// of 16 floats overlap modulo the banks).
template <bool KC, int R, int BK, bool PERM>
struct Panel {
    static constexpr int LD = KC ? (PERM ? BK : BK + 4) : (R + 8);
    static constexpr int SIZE = KC ? R * LD : BK * LD;
};

__device__ __forceinline__ int kc_chunk_key(int r) { return (((r >> 1) ^ (r >> 3)) & 1) | (((r >> 2) & 1) << 1); }

__device__ __forceinline__ floatx4 load4_any_align(const float *p)
{
    floatx4 v;
    __builtin_memcpy(&v, p, 16);   // 4-byte aligned 16-byte load
    return v;
}

// Fetch this thread's share of a panel (rows r0.., k from k0, valid k < kend) into registers.
template <bool KC, int R, int BK, int THREADS, int NV>
__device__ __forceinline__ void panel_fetch(floatx4 (&reg)[NV], const float *__restrict__ P, int ld, int r0,
                                            int rmax, int k0, int kend, int tid)
{
    constexpr int TOTAL = R * BK / 4;
#pragma unroll
    for (int v = 0; v < NV; ++v) {
        const int f = tid + v * THREADS;
        floatx4 val = {0.f, 0.f, 0.f, 0.f};
        if (TOTAL % THREADS == 0 || f < TOTAL) {
            if (KC) {
                const int row = f / (BK / 4), kq = (f % (BK / 4)) * 4;
                int gr = r0 + row;
                gr = gr < rmax ? gr : rmax - 1;                       // clamp: value unused beyond the edge
                const int gk = k0 + kq;
                const float *src = P + (size_t)gr * ld + gk;
                if (gk + 3 < kend) {
                    val = load4_any_align(src);
                } else {
                    if (gk + 0 < kend) val.x = src[0];
                    if (gk + 1 < kend) val.y = src[1];
                    if (gk + 2 < kend) val.z = src[2];
                }
            } else {
                const int krow = f / (R / 4), rq = (f % (R / 4)) * 4;
                const int gk = k0 + krow, gr = r0 + rq;
                if (gk < kend) {
                    const float *src = P + (size_t)gk * ld + gr;
                    if (gr + 3 < rmax) {
                        val = load4_any_align(src);
                    } else {
                        if (gr + 0 < rmax) val.x = src[0];
                        if (gr + 1 < rmax) val.y = src[1];
                        if (gr + 2 < rmax) val.z = src[2];
                    }
                }
            }
        }
        reg[v] = val;
    }
}

template <bool KC, int R, int BK, int THREADS, int NV, bool PERM>
__device__ __forceinline__ void panel_store(float *lds, const floatx4 (&reg)[NV], int tid)
{
    constexpr int TOTAL = R * BK / 4;
    constexpr int LD = Panel<KC, R, BK, PERM>::LD;
#pragma unroll
    for (int v = 0; v < NV; ++v) {
        const int f = tid + v * THREADS;
        if (TOTAL % THREADS == 0 || f < TOTAL) {
            int off;
            if (KC) off = (f / (BK / 4)) * LD + ((f % (BK / 4)) ^ (PERM ? kc_chunk_key(f / (BK / 4)) : 0)) * 4;
            else off = (f / (R / 4)) * LD + (f % (R / 4)) * 4;
            *reinterpret_cast<floatx4 *>(lds + off) = reg[v];
        }
    }
}

// Operand values of one group of four 32x32x2 steps (k = 8*s + 4*h + t, t = 0..3) for 32 rows starting at `row`.
template <bool KC, int R, int BK, bool PERM>
__device__ __forceinline__ floatx4 panel_read(const float *lds, int row, int s, int l32, int h)
{
    constexpr int LD = Panel<KC, R, BK, PERM>::LD;
    if (KC) {
        return *reinterpret_cast<const floatx4 *>(lds + (row + l32) * LD +
                                                  ((s * 2 + h) ^ (PERM ? kc_chunk_key(row + l32) : 0)) * 4);
    } else {
        const float *p = lds + (s * 8 + h * 4) * LD + row + l32;
        floatx4 v;
        v.x = p[0];
        v.y = p[LD];
        v.z = p[2 * LD];
        v.w = p[3 * LD];
        return v;
    }
}

// Consecutive hardware workgroup ids are spread round-robin over the 8 XCDs (each with its own L2).  This maps
// id -> position so that each XCD receives a CONTIGUOUS range of positions 0..n-1 (a bijection for any n).
__device__ __forceinline__ int xcd_contiguous(int pid, int n)
{
    constexpr int XCDS = 8;
    const int q = n / XCDS, rem = n % XCDS;
    const int xcd = pid % XCDS, loc = pid / XCDS;
    return xcd * q + (xcd < rem ? xcd : rem) + loc;
}

// Tiles are walked in groups of GROUP_M tile rows, so that the A and B panels a group touches stay in L2.
__device__ __forceinline__ void grouped_tile(int lid, int tiles_m, int tiles_n, int &tm, int &tn)
{
    constexpr int GROUP_M = 8;
    const int group = GROUP_M * tiles_n;
    const int gid = lid / group;
    const int first_m = gid * GROUP_M;
    const int gsz = (tiles_m - first_m) < GROUP_M ? (tiles_m - first_m) : GROUP_M;
    tm = first_m + (lid % group) % gsz;
    tn = (lid % group) / gsz;
}

// Map the hardware workgroup id `hw` of a launch of tiles x splits workgroups (x fastest) to (tile, k split).
// The XCD-contiguous positions run over the WHOLE tiles x splits range, split-major: one XCD then works on a
// block of neighbouring tiles of ONE k slice at a time, so the operand panels those tiles share are fetched into
// that XCD's L2 once.  (Giving every XCD a share of every split made each panel a guest in several L2s: the
// hidden-delta product at 4096 patterns read 132 MB for 59 MB of operands.)  Within a split, tiles are grouped.
__device__ __forceinline__ void work_of_workgroup(int hw, int tiles_m, int tiles_n, int splits, int &tm, int &tn,
                                                  int &z)
{
    const int tiles = tiles_m * tiles_n;
    const int pos = xcd_contiguous(hw, tiles * splits);
    z = pos / tiles;
    grouped_tile(pos - z * tiles, tiles_m, tiles_n, tm, tn);
}

__device__ __forceinline__ float tanh_f32(float x)
{
    // tanh(x) = sign(x) * (1 - 2/(exp(2|x|)+1)); for small |x| the odd series avoids the cancellation
    const float ax = fabsf(x);
    float r;
    if (ax < 0.25f) {
        const float x2 = x * x;
        // x - x^3/3 + 2x^5/15 - 17x^7/315 + 62x^9/2835
        r = ax * (1.0f + x2 * (-0.33333333f + x2 * (0.13333333f + x2 * (-0.053968254f + x2 * 0.021869488f))));
    } else {
        const float e = __expf(2.0f * ax);
        r = 1.0f - 2.0f / (e + 1.0f);
    }
    return copysignf(r, x);
}

// Per-thread state of the unchecked fetch used for full k blocks.  The tile's base pointer (uniform) already
// points at (first row of the tile, first k of the workgroup); `off` is this thread's element offset from it
// and never changes, the base advances by BK (KC) or BK*ld (MC) per step.  A 16-byte load that lies wholly
// beyond the matrix edge is redirected to a valid address (row clamped for KC; for MC the first column of the
// tile, or the load that ends at the edge): its values only reach accumulators that are never stored.  An MC
// load that STRADDLES the edge (valid width not a multiple of 4; bit set in `edge`) is replaced by the 16-byte
// load that ENDS at the edge, and finish() moves its valid elements into place before the panel is stored.
// When the tile has fewer than 4 valid columns that load starts before the tile, so the caller moves the
// tile's base pointer back by `back` elements and every offset is `back` larger.  Only a matrix narrower than
// 4 falls back to guarded 4-byte loads.  No load ever touches an address outside the rows of the matrix.
template <bool KC, int R, int BK, int THREADS, int NV>
struct FastFetch {
    unsigned off[NV];
    unsigned edge;
    int valid;      // rows/columns of this tile inside the matrix
    int back;       // elements the caller must move the base pointer back (0 or 4)
    bool shifted;   // straddling loads are whole loads ending at the edge

    __device__ __forceinline__ void init(int ld, int r0, int rmax, int tid)
    {
        constexpr int TOTAL = R * BK / 4;
        edge = 0;
        valid = rmax - r0;
        back = 0;
        shifted = false;
        if (!KC && valid < R && (valid & 3) != 0) {
            if (valid >= 4) {
                shifted = true;
            } else if (r0 >= 4) {
                shifted = true;
                back = 4;
            }
        }
#pragma unroll
        for (int v = 0; v < NV; ++v) {
            int f = tid + v * THREADS;
            if (TOTAL % THREADS != 0 && f >= TOTAL) f = 0;   // nothing to fetch: repeat a valid load (not stored)
            if (KC) {
                int row = f / (BK / 4);
                const int kq = (f % (BK / 4)) * 4;
                row = row < valid ? row : valid - 1;
                off[v] = (unsigned)row * (unsigned)ld + (unsigned)kq;
            } else {
                const int krow = f / (R / 4);
                int rq = (f % (R / 4)) * 4;
                if (rq + 3 >= valid) {               // not wholly inside the matrix
                    if (shifted) {
                        if (rq < valid) edge |= 1u << v;
                        rq = valid - 4;              // >= -3, and rq + back >= 0
                    } else if ((valid & 3) == 0) {
                        rq = 0;                      // wholly outside, and the tile has >= 4 valid columns
                    } else {
                        edge |= 1u << v;             // guarded loads (they load nothing when wholly outside)
                        if (rq >= valid) rq = 0;
                    }
                }
                off[v] = (unsigned)krow * (unsigned)ld + (unsigned)(rq + back);
            }
        }
    }

    __device__ __forceinline__ void fetch(floatx4 (&reg)[NV], const float *__restrict__ base, int tid) const
    {
#pragma unroll
        for (int v = 0; v < NV; ++v) {
            const float *src = base + off[v];
            if (KC || shifted || !(edge >> v & 1)) {
                reg[v] = load4_any_align(src);
            } else {
                const int rq = ((tid + v * THREADS) % (R / 4)) * 4;
                floatx4 val = {0.f, 0.f, 0.f, 0.f};
                if (rq + 0 < valid) val.x = src[0];
                if (rq + 1 < valid) val.y = src[1];
                if (rq + 2 < valid) val.z = src[2];
                reg[v] = val;
            }
        }
    }

    // After fetch(), before the registers are stored to LDS: a straddling vector was loaded from the address
    // 4 - valid%4 elements lower, so its valid elements sit at the top of the register; move them down.
    // Written with selects only (no branches on valid%4).
    __device__ __forceinline__ void finish(floatx4 (&reg)[NV]) const
    {
        if (KC || !shifted || edge == 0) return;
        const bool r1 = (valid & 3) == 1, r2 = (valid & 3) == 2;
#pragma unroll
        for (int v = 0; v < NV; ++v) {
            const bool e = (edge >> v & 1) != 0;
            const floatx4 l = reg[v];
            floatx4 o;
            o.x = r1 ? l.w : (r2 ? l.z : l.y);
            o.y = r1 ? 0.f : (r2 ? l.w : l.z);
            o.z = (r1 || r2) ? 0.f : l.w;
            o.w = 0.f;
            reg[v].x = e ? o.x : l.x;
            reg[v].y = e ? o.y : l.y;
            reg[v].z = e ? o.z : l.z;
            reg[v].w = e ? o.w : l.w;
        }
    }
};

// Operand fragments of one group of four 32x32x2 products for a wavefront's whole sub-tile.
template <class Cfg>
struct Fragments {
    floatx4 a[Cfg::TM], b[Cfg::TN];
};

template <class Cfg, bool A_KC, bool B_KC>
__device__ __forceinline__ void read_fragments(Fragments<Cfg> &f, const float *la, const float *lb, int s, int wrow,
                                               int wcol, int l32, int h)
{
#pragma unroll
    for (int x = 0; x < Cfg::TM; ++x) f.a[x] = panel_read<A_KC, Cfg::BM, Cfg::BK, Cfg::PERMUTE_KC>(la, wrow + x * 32, s, l32, h);
#pragma unroll
    for (int y = 0; y < Cfg::TN; ++y) f.b[y] = panel_read<B_KC, Cfg::BN, Cfg::BK, Cfg::PERMUTE_KC>(lb, wcol + y * 32, s, l32, h);
}

// Products t0 <= t < t1 of a group, for every accumulator block of the wavefront.
template <class Cfg, int T0, int T1>
__device__ __forceinline__ void multiply(floatx16 (&acc)[Cfg::TM][Cfg::TN], const Fragments<Cfg> &f)
{
#pragma unroll
    for (int t = T0; t < T1; ++t)
#pragma unroll
        for (int x = 0; x < Cfg::TM; ++x)
#pragma unroll
            for (int y = 0; y < Cfg::TN; ++y)
                acc[x][y] = __builtin_amdgcn_mfma_f32_32x32x2f32(f.a[x][t], f.b[y][t], acc[x][y], 0, 0, 0);
}

// LDS floats one workgroup needs: two stages of an A panel and a B panel.
template <class Cfg, bool A_KC, bool B_KC>
constexpr int gemm_lds_floats()
{
    return 2 * (Panel<A_KC, Cfg::BM, Cfg::BK, Cfg::PERMUTE_KC>::SIZE + Panel<B_KC, Cfg::BN, Cfg::BK, Cfg::PERMUTE_KC>::SIZE);
}

// The product of one tile over the k range [kbeg, kend), followed by epilogue EPI written through `Cout`
// (row stride ldc).  `lds` points at gemm_lds_floats() floats of 16-byte
// aligned LDS; every thread of the workgroup must call this, and LDS is free again on return.
template <class Cfg, bool A_KC, bool B_KC, int EPI>
__device__ __forceinline__ void gemm_segment(const GemmArgs &g, const int tile_m, const int tile_n, const int kbeg,
                                             const int kend, float *Cout, const int ldc, float *lds)
{
    constexpr int BM = Cfg::BM, BN = Cfg::BN, BK = Cfg::BK, THREADS = Cfg::THREADS;
    constexpr int TM = Cfg::TM, TN = Cfg::TN;
    using PA = Panel<A_KC, BM, BK, Cfg::PERMUTE_KC>;
    using PB = Panel<B_KC, BN, BK, Cfg::PERMUTE_KC>;
    constexpr int NVA = (BM * BK / 4 + THREADS - 1) / THREADS;
    constexpr int NVB = (BN * BK / 4 + THREADS - 1) / THREADS;

    auto stage_a = [&](int st) { return lds + st * PA::SIZE; };
    auto stage_b = [&](int st) { return lds + 2 * PA::SIZE + st * PB::SIZE; };

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, h = lane >> 5;
    const int kw = wave / (Cfg::WM * Cfg::WN);               // which share of every k step (0 when KW == 1)
    const int wave_mn = wave % (Cfg::WM * Cfg::WN);
    const int wm = wave_mn / Cfg::WN, wn = wave_mn % Cfg::WN;
    const int wrow = wm * Cfg::WTM, wcol = wn * Cfg::WTN;

    const int i0 = tile_m * BM, j0 = tile_n * BN;
    const int nfull = (kend - kbeg) / BK;             // steps fetched without any check
    const bool tail = (kend - kbeg) % BK != 0;        // one last, partial step: checked fetch, zero filled
    const int nkb = nfull + (tail ? 1 : 0);

    floatx16 acc[TM][TN];
#pragma unroll
    for (int a = 0; a < TM; ++a)
#pragma unroll
        for (int b = 0; b < TN; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.f;

    FastFetch<A_KC, BM, BK, THREADS, NVA> fa;
    FastFetch<B_KC, BN, BK, THREADS, NVB> fb;
    fa.init(g.lda, i0, g.M, tid);
    fb.init(g.ldb, j0, g.N, tid);
    // uniform base pointers of the tile at k = kbeg, and their advance per step
    const float *pa = A_KC ? g.A + (size_t)i0 * g.lda + kbeg : g.A + (size_t)kbeg * g.lda + i0;
    const float *pb = B_KC ? g.B + (size_t)j0 * g.ldb + kbeg : g.B + (size_t)kbeg * g.ldb + j0;
    pa -= fa.back;
    pb -= fb.back;
    const size_t step_a = A_KC ? (size_t)BK : (size_t)BK * g.lda;
    const size_t step_b = B_KC ? (size_t)BK : (size_t)BK * g.ldb;

    floatx4 ra[NVA], rb[NVB];
#pragma unroll
    for (int v = 0; v < NVA; ++v) ra[v] = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int v = 0; v < NVB; ++v) rb[v] = floatx4{0.f, 0.f, 0.f, 0.f};

    constexpr int S = BK / 8;   // groups of four products per step

    if (nkb > 0) {
        if (nfull > 0) {
            fa.fetch(ra, pa, tid);
            fb.fetch(rb, pb, tid);
            fa.finish(ra);
            fb.finish(rb);
        } else {
            panel_fetch<A_KC, BM, BK, THREADS, NVA>(ra, g.A, g.lda, i0, g.M, kbeg, kend, tid);
            panel_fetch<B_KC, BN, BK, THREADS, NVB>(rb, g.B, g.ldb, j0, g.N, kbeg, kend, tid);
        }
        panel_store<A_KC, BM, BK, THREADS, NVA, Cfg::PERMUTE_KC>(stage_a(0), ra, tid);
        panel_store<B_KC, BN, BK, THREADS, NVB, Cfg::PERMUTE_KC>(stage_b(0), rb, tid);
    }
    __syncthreads();

    // All matrix-core work of one step on LDS stage `cur`.  Several workgroups share a compute unit, so the
    // latency of these LDS reads is covered by the products of the other workgroups' wavefronts.
    auto compute = [&](int cur) {
        const float *la = stage_a(cur), *lb = stage_b(cur);
        constexpr int SW = S / Cfg::KW;   // groups of four products per step for this wavefront
        Fragments<Cfg> f[SW];
#pragma unroll
        for (int sg = 0; sg < SW; ++sg)
            read_fragments<Cfg, A_KC, B_KC>(f[sg], la, lb, kw * SW + sg, wrow, wcol, l32, h);
#pragma unroll
        for (int sg = 0; sg < SW; ++sg) multiply<Cfg, 0, 4>(acc, f[sg]);
    };

    // full steps whose successor is also a full step: unchecked fetch
    int kb = 0;
    for (; kb + 1 < nfull; ++kb) {
        const int cur = kb & 1;
        pa += step_a;
        pb += step_b;
        fa.fetch(ra, pa, tid);
        fb.fetch(rb, pb, tid);
        compute(cur);
        fa.finish(ra);
        fb.finish(rb);
        panel_store<A_KC, BM, BK, THREADS, NVA, Cfg::PERMUTE_KC>(stage_a(cur ^ 1), ra, tid);
        panel_store<B_KC, BN, BK, THREADS, NVB, Cfg::PERMUTE_KC>(stage_b(cur ^ 1), rb, tid);
        __syncthreads();
    }
    // the last full step (its successor, if any, is the partial step: checked fetch), then the partial step
    for (; kb < nkb; ++kb) {
        const int cur = kb & 1;
        const bool more = kb + 1 < nkb;
        if (more) {
            const int k0 = kbeg + (kb + 1) * BK;
            panel_fetch<A_KC, BM, BK, THREADS, NVA>(ra, g.A, g.lda, i0, g.M, k0, kend, tid);
            panel_fetch<B_KC, BN, BK, THREADS, NVB>(rb, g.B, g.ldb, j0, g.N, k0, kend, tid);
        }
        compute(cur);
        if (more) {
            panel_store<A_KC, BM, BK, THREADS, NVA, Cfg::PERMUTE_KC>(stage_a(cur ^ 1), ra, tid);
            panel_store<B_KC, BN, BK, THREADS, NVB, Cfg::PERMUTE_KC>(stage_b(cur ^ 1), rb, tid);
        }
        __syncthreads();
    }

    if (Cfg::KW > 1) {
        // The k loop ended with a barrier, so the panels are dead: groups 1.. park their accumulators in LDS
        // (one 64-lane row per register: conflict free), group 0 adds them in group order and goes on alone.
        constexpr int PER_WAVE = TM * TN * 16 * 64;
        static_assert((Cfg::KW - 1) * Cfg::WM * Cfg::WN * PER_WAVE <= gemm_lds_floats<Cfg, A_KC, B_KC>(),
                      "LDS too small for the accumulator exchange");
        if (kw > 0) {
            float *dst = lds + ((kw - 1) * Cfg::WM * Cfg::WN + wave_mn) * PER_WAVE + lane;
#pragma unroll
            for (int x = 0; x < TM; ++x)
#pragma unroll
                for (int y = 0; y < TN; ++y)
#pragma unroll
                    for (int r = 0; r < 16; ++r) dst[((x * TN + y) * 16 + r) * 64] = acc[x][y][r];
        }
        __syncthreads();
        if (kw > 0) return;
#pragma unroll
        for (int g2 = 1; g2 < Cfg::KW; ++g2) {
            const float *src = lds + ((g2 - 1) * Cfg::WM * Cfg::WN + wave_mn) * PER_WAVE + lane;
#pragma unroll
            for (int x = 0; x < TM; ++x)
#pragma unroll
                for (int y = 0; y < TN; ++y)
#pragma unroll
                    for (int r = 0; r < 16; ++r) acc[x][y][r] += src[((x * TN + y) * 16 + r) * 64];
        }
    }
    // Epilogue.  Accumulator register r of a 32x32 block holds row 8*(r/4) + 4*h + r%4, column lane%32.
#pragma unroll
    for (int y = 0; y < TN; ++y) {
        const int j = j0 + wn * Cfg::WTN + y * 32 + l32;
        if (j >= g.N) continue;
        float bias = 0.f;
        if ((EPI == EPI_BIAS_TANH || EPI == EPI_BIAS) && g.bias) bias = g.bias[j];
#pragma unroll
        for (int x = 0; x < TM; ++x) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int i = i0 + wm * Cfg::WTM + x * 32 + 8 * (r / 4) + 4 * h + (r % 4);
                if (i >= g.M) continue;
                const float v = acc[x][y][r];
                float *dst = Cout + (size_t)i * ldc + j;
                if (EPI == EPI_AXPBY) {
                    float out = g.alpha * v;
                    if (g.beta != 0.f) out += g.beta * *dst;
                    *dst = out;
                } else if (EPI == EPI_PARTIAL) {
                    *dst = v;
                } else if (EPI == EPI_BIAS_TANH) {
                    *dst = tanh_f32(v + bias);
                } else if (EPI == EPI_BIAS) {
                    *dst = v + bias;
                } else {
                    const float hv = g.aux[(size_t)i * g.ldaux + j];
                    *dst = v * (1.0f - hv * hv);
                }
            }
        }
    }
}

// The work of one workgroup: `hw` is its position in the launch order of this problem's tiles x splits workgroups.
template <class Cfg, bool A_KC, bool B_KC, int EPI>
__device__ __forceinline__ void gemm_tile(const GemmArgs &g, const int hw, const int splits, float *lds)
{
    int tile_m, tile_n, z;
    work_of_workgroup(hw, g.tiles_m, g.tiles_n, splits, tile_m, tile_n, z);
    const int kbeg = z * g.kchunk;
    const int kend = (kbeg + g.kchunk < g.K) ? kbeg + g.kchunk : g.K;
    float *Cout = g.C;
    int ldc = g.ldc;
    if (EPI == EPI_PARTIAL) {
        Cout = g.C + (size_t)z * g.partial_stride;
        ldc = g.N;
    }
    gemm_segment<Cfg, A_KC, B_KC, EPI>(g, tile_m, tile_n, kbeg, kend, Cout, ldc, lds);
}

// One GEMM per launch: grid = (tiles, k splits).
template <class Cfg, bool A_KC, bool B_KC, int EPI>
__global__ __launch_bounds__(Cfg::THREADS, Cfg::WAVES_PER_SIMD) void gemm_kernel(const GemmArgs g)
{
    __shared__ __attribute__((aligned(16))) float lds[gemm_lds_floats<Cfg, A_KC, B_KC>()];
    const int hw = blockIdx.y * gridDim.x + blockIdx.x;
    gemm_tile<Cfg, A_KC, B_KC, EPI>(g, hw, gridDim.y, lds);
}

// Two independent GEMMs in one launch (1-D grid): workgroups [0, n1) work on g1, the rest on g2.  The second
// problem's workgroups start as the first one's finish, so the compute units stay full across the seam and
// one problem's stores overlap the other's products.  Both tile shapes must use the same number of threads.
template <class Cfg1, bool A_KC1, bool B_KC1, int EPI1, class Cfg2, bool A_KC2, bool B_KC2, int EPI2>
__global__ __launch_bounds__(Cfg1::THREADS, (Cfg1::WAVES_PER_SIMD < Cfg2::WAVES_PER_SIMD ? Cfg1::WAVES_PER_SIMD
                                                                                         : Cfg2::WAVES_PER_SIMD))
void gemm_pair_kernel(const GemmArgs g1, const GemmArgs g2, const int n1)
{
    static_assert(Cfg1::THREADS == Cfg2::THREADS, "paired tile shapes need equal workgroup sizes");
    constexpr int L1 = gemm_lds_floats<Cfg1, A_KC1, B_KC1>(), L2 = gemm_lds_floats<Cfg2, A_KC2, B_KC2>();
    __shared__ __attribute__((aligned(16))) float lds[L1 > L2 ? L1 : L2];
    const int id = blockIdx.x;
    if (id < n1) {
        gemm_tile<Cfg1, A_KC1, B_KC1, EPI1>(g1, id, n1 / (g1.tiles_m * g1.tiles_n), lds);
    } else {
        const int n2 = gridDim.x - n1;
        gemm_tile<Cfg2, A_KC2, B_KC2, EPI2>(g2, id - n1, n2 / (g2.tiles_m * g2.tiles_n), lds);
    }
}

}  // namespace ulsnn
