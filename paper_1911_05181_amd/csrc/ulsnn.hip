// Host side of the C ABI declared in include/ulsnn.h: argument checks, choice of tile shape and k split,
// workspace layout, and the stream-ordered launches.  No device memory is allocated here.
#include "../../include/ulsnn.h"

#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdint>

#include "gemm.hpp"
#include "mlp_kernels.hpp"

using namespace ulsnn;

namespace {

constexpr int NUM_CU = 256;          // MI355X: 8 XCDs x 32 compute units
constexpr int SLAB_ROWS = 16384;     // patterns processed per internal pass of the MLP gradient

inline bool is_n(char t) { return t == 'N' || t == 'n'; }
inline bool is_t(char t) { return t == 'T' || t == 't' || t == 'C' || t == 'c'; }
inline size_t round_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// ---------------------------------------------------------------------------------------------------------
// GEMM dispatch
// ---------------------------------------------------------------------------------------------------------

using Cfg128 = TileCfg<128, 128, 16, 2, 2>;   // 256 threads, wavefront tile 64 x 64
using Cfg64 = TileCfg<64, 64, 16, 2, 2>;      // 256 threads, wavefront tile 32 x 32 (small problems)

enum CfgId { CFG_128 = 0, CFG_64 = 1 };

struct GemmPlan {
    CfgId cfg;
    int bm, bn, bk;
    int tiles_m, tiles_n;
    int splits, kchunk;
};

inline void cfg_dims(CfgId c, int &bm, int &bn, int &bk)
{
    switch (c) {
        case CFG_128: bm = Cfg128::BM; bn = Cfg128::BN; bk = Cfg128::BK; break;
        default: bm = Cfg64::BM; bn = Cfg64::BN; bk = Cfg64::BK; break;
    }
}

// Choose a tile shape and, if allowed, a k split so that the launch has enough workgroups for 256 CUs.
GemmPlan plan_gemm(int m, int n, int k, bool allow_split)
{
    GemmPlan p;
    const long t128 = (long)((m + 127) / 128) * ((n + 127) / 128);
    p.cfg = (t128 >= NUM_CU || allow_split) ? CFG_128 : CFG_64;
    cfg_dims(p.cfg, p.bm, p.bn, p.bk);
    p.tiles_m = (m + p.bm - 1) / p.bm;
    p.tiles_n = (n + p.bn - 1) / p.bn;
    p.splits = 1;
    p.kchunk = std::max(k, 1);
    const long tiles = (long)p.tiles_m * p.tiles_n;
    if (allow_split && tiles < 2 * NUM_CU) {
        int want = (int)((2 * NUM_CU + tiles - 1) / tiles);
        const int max_by_k = std::max(1, k / (8 * p.bk));         // keep at least 8 k steps per split
        want = std::min(want, max_by_k);
        if (want > 1) {
            const int chunk = (int)round_up((size_t)(k + want - 1) / want, p.bk);
            p.kchunk = chunk;
            p.splits = (k + chunk - 1) / chunk;
        }
    }
    return p;
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

template <class Cfg>
hipError_t launch_cfg(bool a_kc, bool b_kc, int epi, const GemmArgs &a, int splits, hipStream_t s)
{
    switch (epi) {
        case EPI_AXPBY: return launch_layout<Cfg, EPI_AXPBY>(a_kc, b_kc, a, splits, s);
        case EPI_PARTIAL: return launch_layout<Cfg, EPI_PARTIAL>(a_kc, b_kc, a, splits, s);
        case EPI_BIAS_TANH: return launch_one<Cfg, true, false, EPI_BIAS_TANH>(a, splits, s);   // NN only
        case EPI_BIAS: return launch_one<Cfg, true, false, EPI_BIAS>(a, splits, s);             // NN only
        default: return launch_one<Cfg, true, true, EPI_TANHGRAD>(a, splits, s);                // NT only
    }
}

hipError_t launch_gemm(const GemmPlan &p, bool a_kc, bool b_kc, int epi, GemmArgs a, hipStream_t s)
{
    a.tiles_m = p.tiles_m;
    a.tiles_n = p.tiles_n;
    a.kchunk = p.kchunk;
    switch (p.cfg) {
        case CFG_128: return launch_cfg<Cfg128>(a_kc, b_kc, epi, a, p.splits, s);
        default: return launch_cfg<Cfg64>(a_kc, b_kc, epi, a, p.splits, s);
    }
}

inline unsigned grid_for(size_t elems)
{
    return (unsigned)std::min<size_t>((elems + 255) / 256, (size_t)NUM_CU * 8);
}

// One product of the MLP gradient: out = epilogue(op(A) op(B)), through a k split when the plan has one.
// epi is the single-launch epilogue; with a split the same effect is applied by the reduction.
hipError_t mlp_product(const GemmPlan &p, bool a_kc, bool b_kc, int epi, GemmArgs a, float *partial,
                       hipStream_t s)
{
    if (p.splits == 1) return launch_gemm(p, a_kc, b_kc, epi, a, s);
    GemmArgs pa = a;
    pa.C = partial;
    pa.partial_stride = (size_t)a.M * a.N;
    hipError_t e = launch_gemm(p, a_kc, b_kc, EPI_PARTIAL, pa, s);
    if (e != hipSuccess) return e;
    const size_t total = (size_t)a.M * a.N;
    if (epi == EPI_TANHGRAD) {
        hipLaunchKernelGGL(splitk_reduce_kernel<true>, dim3(grid_for(total)), dim3(256), 0, s, partial,
                           pa.partial_stride, p.splits, a.C, a.M, a.N, a.ldc, 1.0f, 0.0f, a.aux, a.ldaux);
    } else {
        hipLaunchKernelGGL(splitk_reduce_kernel<false>, dim3(grid_for(total)), dim3(256), 0, s, partial,
                           pa.partial_stride, p.splits, a.C, a.M, a.N, a.ldc, a.alpha, a.beta,
                           (const float *)nullptr, 0);
    }
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------------------
// MLP gradient: plans and workspace layout for one slab of patterns
// ---------------------------------------------------------------------------------------------------------

struct MlpLayout {
    int slab;                       // rows per pass
    int ldh, ldz;                   // row strides of H / dA1 and of Z / dO
    size_t off_h, off_z, off_da1, off_rowloss, off_partial, bytes;
};

struct SlabPlans {
    GemmPlan g1, g2, g3, g4, g5;
    size_t partial_floats;
};

SlabPlans plan_slab(int n_in, int n_hid, int n_out, int rows)
{
    SlabPlans s;
    s.g1 = plan_gemm(rows, n_hid, n_in, false);
    s.g2 = plan_gemm(rows, n_out, n_hid, false);
    s.g3 = plan_gemm(n_hid, n_out, rows, true);
    s.g4 = plan_gemm(rows, n_hid, n_out, true);
    s.g5 = plan_gemm(n_in, n_hid, rows, true);
    size_t p = 0;
    if (s.g3.splits > 1) p = std::max(p, (size_t)s.g3.splits * n_hid * n_out);
    if (s.g4.splits > 1) p = std::max(p, (size_t)s.g4.splits * rows * n_hid);
    if (s.g5.splits > 1) p = std::max(p, (size_t)s.g5.splits * n_in * n_hid);
    s.partial_floats = p;
    return s;
}

bool desc_ok(const ulsnn_mlp_desc *d)
{
    return d && d->n_in >= 1 && d->n_hid >= 1 && d->n_out >= 1;
}

// Upper bound on the split-k partial floats any pass of at most `slab` rows can need (non-decreasing in slab,
// so a workspace sized for a batch also serves every smaller one).
size_t partial_bound(int n_in, int n_hid, int n_out, int slab)
{
    int bm, bn, bk;
    cfg_dims(CFG_128, bm, bn, bk);
    const long by_k = std::max(1, slab / (8 * bk));
    auto want = [&](long tiles) { return std::min<long>((2 * NUM_CU + tiles - 1) / tiles, by_k); };
    const long t3 = (long)((n_hid + bm - 1) / bm) * ((n_out + bn - 1) / bn);
    const long t5 = (long)((n_in + bm - 1) / bm) * ((n_hid + bn - 1) / bn);
    size_t p = 0;
    if (want(t3) > 1) p = std::max(p, (size_t)want(t3) * n_hid * n_out);
    if (want(t5) > 1) p = std::max(p, (size_t)want(t5) * n_in * n_hid);
    // hidden delta: splits * rows <= 2*NUM_CU*bm / tiles_n + rows
    const long tn4 = (n_hid + bn - 1) / bn;
    p = std::max(p, (size_t)(2 * NUM_CU * bm / tn4 + slab + bm) * n_hid);
    return p;
}

MlpLayout mlp_layout(const ulsnn_mlp_desc *d, int batch)
{
    MlpLayout L;
    L.slab = std::max(1, std::min(batch, SLAB_ROWS));
    L.ldh = (int)round_up((size_t)d->n_hid, 32);
    L.ldz = (int)round_up((size_t)d->n_out, 32);
    const size_t partial = partial_bound(d->n_in, d->n_hid, d->n_out, L.slab);
    size_t off = 0;
    L.off_h = off;        off += round_up((size_t)L.slab * L.ldh * 4, 256);
    L.off_z = off;        off += round_up((size_t)L.slab * L.ldz * 4, 256);
    L.off_da1 = off;      off += round_up((size_t)L.slab * L.ldh * 4, 256);
    L.off_rowloss = off;  off += round_up((size_t)L.slab * 4, 256);
    L.off_partial = off;  off += round_up(partial * 4, 256);
    L.bytes = off;
    return L;
}

int check_mlp_args(const ulsnn_mlp_desc *d, const void *W1, const void *W2, const void *X, const int32_t *labels,
                   long long batch, float *dW1, float *dW2, float *loss)
{
    if (!d) return ULSNN_ERR_NULL;
    if (d->n_in < 1 || d->n_hid < 1 || d->n_out < 1 || batch < 0) return ULSNN_ERR_DIM;
    if (!W1 || !W2 || !dW1 || !dW2 || !loss) return ULSNN_ERR_NULL;
    if (batch > 0 && (!X || !labels)) return ULSNN_ERR_NULL;
    const int nb = (d->b1 != nullptr) + (d->b2 != nullptr) + (d->db1 != nullptr) + (d->db2 != nullptr);
    if (nb != 0 && nb != 4) return ULSNN_ERR_NULL;
    if (d->accumulate != 0 && d->accumulate != 1) return ULSNN_ERR_UNSUPPORTED;
    if (d->operand_dtype != 0) return ULSNN_ERR_UNSUPPORTED;
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
int mlp_grad_impl(const ulsnn_mlp_desc *d, const float *W1, const float *W2, const float *X,
                  const int32_t *labels, int batch, float *dW1, float *dW2, float *loss, bool accumulate,
                  hipEvent_t *ev = nullptr)
{
    hipStream_t s = (hipStream_t)d->hip_stream;
    const int n_in = d->n_in, n_hid = d->n_hid, n_out = d->n_out;
    const bool biases = d->b1 != nullptr;

    if (batch == 0) {
        if (!accumulate) {
            hipLaunchKernelGGL(zero_kernel, dim3(grid_for((size_t)n_in * n_hid)), dim3(256), 0, s, dW1,
                               (size_t)n_in * n_hid);
            hipLaunchKernelGGL(zero_kernel, dim3(grid_for((size_t)n_hid * n_out)), dim3(256), 0, s, dW2,
                               (size_t)n_hid * n_out);
            hipLaunchKernelGGL(zero_kernel, dim3(1), dim3(256), 0, s, loss, (size_t)1);
            if (biases) {
                hipLaunchKernelGGL(zero_kernel, dim3(grid_for(n_hid)), dim3(256), 0, s, d->db1, (size_t)n_hid);
                hipLaunchKernelGGL(zero_kernel, dim3(grid_for(n_out)), dim3(256), 0, s, d->db2, (size_t)n_out);
            }
            HIP_TRY(hipGetLastError());
        }
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
    float *partial = (float *)(ws + L.off_partial);

    for (int r0 = 0; r0 < batch; r0 += L.slab) {
        const int rows = std::min(L.slab, batch - r0);
        const SlabPlans P = plan_slab(n_in, n_hid, n_out, rows);
        if (L.off_partial + P.partial_floats * 4 > L.bytes) return ULSNN_ERR_WORKSPACE;   // cannot happen
        const float beta = (r0 > 0 || accumulate) ? 1.0f : 0.0f;
        const float *Xs = X + (size_t)r0 * n_in;
        const int32_t *ys = labels + r0;
        GemmArgs a{};
        MARK(0);

        // H = tanh(Xs W1 + b1)
        a = GemmArgs{};
        a.A = Xs; a.lda = n_in; a.B = W1; a.ldb = n_hid; a.C = H; a.ldc = L.ldh;
        a.M = rows; a.N = n_hid; a.K = n_in; a.alpha = 1.f; a.beta = 0.f; a.bias = d->b1;
        HIP_TRY(launch_gemm(P.g1, true, false, EPI_BIAS_TANH, a, s));
        MARK(1);

        // Z = H W2 + b2
        a = GemmArgs{};
        a.A = H; a.lda = L.ldh; a.B = W2; a.ldb = n_out; a.C = Z; a.ldc = L.ldz;
        a.M = rows; a.N = n_out; a.K = n_hid; a.alpha = 1.f; a.beta = 0.f; a.bias = d->b2;
        HIP_TRY(launch_gemm(P.g2, true, false, EPI_BIAS, a, s));
        MARK(2);

        // Z <- dO = softmax(Z) - onehot, row losses; loss (+)= their sum
        if (n_out <= 256 * 16) {
            hipLaunchKernelGGL((softmax_ce_kernel<256, 16>), dim3(rows), dim3(256), 0, s, Z, L.ldz, n_out, ys,
                               row_loss);
        } else {
            hipLaunchKernelGGL((softmax_ce_long_kernel<256>), dim3(rows), dim3(256), 0, s, Z, L.ldz, n_out, ys,
                               row_loss);
        }
        hipLaunchKernelGGL(loss_reduce_kernel, dim3(1), dim3(1024), 0, s, row_loss, (long long)rows, loss, beta);
        HIP_TRY(hipGetLastError());
        MARK(3);

        // dW2 (+)= H^T dO
        a = GemmArgs{};
        a.A = H; a.lda = L.ldh; a.B = Z; a.ldb = L.ldz; a.C = dW2; a.ldc = n_out;
        a.M = n_hid; a.N = n_out; a.K = rows; a.alpha = 1.f; a.beta = beta;
        HIP_TRY(mlp_product(P.g3, false, false, EPI_AXPBY, a, partial, s));
        MARK(4);
        if (biases) {
            hipLaunchKernelGGL(column_sum_kernel, dim3((n_out + 63) / 64), dim3(256), 0, s, Z, L.ldz, rows, n_out,
                               d->db2, beta);
            HIP_TRY(hipGetLastError());
        }

        MARK(5);

        // dA1 = (dO W2^T) * (1 - H*H)
        a = GemmArgs{};
        a.A = Z; a.lda = L.ldz; a.B = W2; a.ldb = n_out; a.C = dA1; a.ldc = L.ldh;
        a.M = rows; a.N = n_hid; a.K = n_out; a.alpha = 1.f; a.beta = 0.f; a.aux = H; a.ldaux = L.ldh;
        HIP_TRY(mlp_product(P.g4, true, true, EPI_TANHGRAD, a, partial, s));
        MARK(6);

        // dW1 (+)= Xs^T dA1
        a = GemmArgs{};
        a.A = Xs; a.lda = n_in; a.B = dA1; a.ldb = L.ldh; a.C = dW1; a.ldc = n_hid;
        a.M = n_in; a.N = n_hid; a.K = rows; a.alpha = 1.f; a.beta = beta;
        HIP_TRY(mlp_product(P.g5, false, false, EPI_AXPBY, a, partial, s));
        MARK(7);
        if (biases) {
            hipLaunchKernelGGL(column_sum_kernel, dim3((n_hid + 63) / 64), dim3(256), 0, s, dA1, L.ldh, rows,
                               n_hid, d->db1, beta);
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
    if (m == 0 || n == 0) return ULSNN_OK;
    if (!C) return ULSNN_ERR_NULL;
    hipStream_t s = (hipStream_t)hip_stream;
    if (k == 0 || alpha == 0.0f) {
        if (beta == 1.0f) return ULSNN_OK;
        hipLaunchKernelGGL(scale_kernel, dim3(grid_for((size_t)m * n)), dim3(256), 0, s, C, m, n, ldc, beta);
        return hipGetLastError() == hipSuccess ? ULSNN_OK : ULSNN_ERR_HIP;
    }
    if (!A || !B) return ULSNN_ERR_NULL;
    const GemmPlan p = plan_gemm(m, n, k, false);
    GemmArgs a{};
    a.A = A; a.B = B; a.C = C; a.M = m; a.N = n; a.K = k; a.lda = lda; a.ldb = ldb; a.ldc = ldc;
    a.alpha = alpha; a.beta = beta;
    return launch_gemm(p, is_n(transa), is_t(transb), EPI_AXPBY, a, s) == hipSuccess ? ULSNN_OK : ULSNN_ERR_HIP;
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
    const int rc = check_mlp_args(desc, W1, W2, X, labels, batch, dW1, dW2, loss);
    if (rc != ULSNN_OK) return rc;
    return mlp_grad_impl(desc, (const float *)W1, (const float *)W2, (const float *)X, labels, batch, dW1, dW2,
                         loss, desc->accumulate != 0);
}

int ulsnn_mlp_grad_epoch(const ulsnn_mlp_desc *desc, const void *W1, const void *W2, const void *X,
                         const int32_t *labels, int64_t n_patterns, int chunk, float *dW1, float *dW2,
                         float *loss)
{
    const int rc = check_mlp_args(desc, W1, W2, X, labels, (long long)n_patterns, dW1, dW2, loss);
    if (rc != ULSNN_OK) return rc;
    if (chunk < 1) return ULSNN_ERR_DIM;
    if (n_patterns == 0)
        return mlp_grad_impl(desc, (const float *)W1, (const float *)W2, nullptr, nullptr, 0, dW1, dW2, loss,
                             desc->accumulate != 0);
    const int first = (int)std::min<int64_t>(chunk, n_patterns);
    if (!desc->workspace || ((uintptr_t)desc->workspace & 255) ||
        desc->workspace_bytes < ulsnn_mlp_grad_workspace_bytes(desc, first))
        return ULSNN_ERR_WORKSPACE;
    const float *Xf = (const float *)X;
    for (int64_t p0 = 0; p0 < n_patterns; p0 += chunk) {
        const int rows = (int)std::min<int64_t>(chunk, n_patterns - p0);
        const int r = mlp_grad_impl(desc, (const float *)W1, (const float *)W2, Xf + (size_t)p0 * desc->n_in,
                                    labels + p0, rows, dW1, dW2, loss, p0 > 0 || desc->accumulate != 0);
        if (r != ULSNN_OK) return r;
    }
    return ULSNN_OK;
}

int ulsnn_mlp_grad_timed(const ulsnn_mlp_desc *desc, const void *W1, const void *W2, const void *X,
                         const int32_t *labels, int batch, float *dW1, float *dW2, float *loss, float *stage_ms)
{
    const int rc = check_mlp_args(desc, W1, W2, X, labels, batch, dW1, dW2, loss);
    if (rc != ULSNN_OK) return rc;
    if (!stage_ms) return ULSNN_ERR_NULL;
    if (batch < 1 || batch > SLAB_ROWS) return ULSNN_ERR_UNSUPPORTED;   // one internal pass only
    hipEvent_t ev[ULSNN_MLP_STAGES + 1];
    int made = 0, out = ULSNN_OK;
    for (; made <= ULSNN_MLP_STAGES; ++made)
        if (hipEventCreate(&ev[made]) != hipSuccess) { out = ULSNN_ERR_HIP; break; }
    if (out == ULSNN_OK)
        out = mlp_grad_impl(desc, (const float *)W1, (const float *)W2, (const float *)X, labels, batch, dW1, dW2,
                            loss, desc->accumulate != 0, ev);
    if (out == ULSNN_OK && hipEventSynchronize(ev[ULSNN_MLP_STAGES]) != hipSuccess) out = ULSNN_ERR_HIP;
    if (out == ULSNN_OK)
        for (int i = 0; i < ULSNN_MLP_STAGES; ++i)
            if (hipEventElapsedTime(&stage_ms[i], ev[i], ev[i + 1]) != hipSuccess) out = ULSNN_ERR_HIP;
    for (int i = 0; i < made; ++i) (void)hipEventDestroy(ev[i]);
    return out;
}

double ulsnn_sgemm_flops(int m, int n, int k) { return 2.0 * (double)m * (double)n * (double)k; }

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
