// Selective Mask training step (Sec. 3.2, Eq. (1); App. B.4 "Selective Mask"): value and gradient of
//   L(S) = mean_t corr_i( A[t][i], B[t][i] ) - lambda * sum_j sigma_j,     sigma = sigmoid(S / T),
//   A[t][i] = <gt_t, g_i>  (handed in),      B[t][i] = sum_j sigma_j^2 gt_t[j] g_i[j].
// Chain rule: with da, db the centred rows of A and B, c_t = da/(|da||db|) - corr_t db/|db|^2,
//   dL/dS_j = 2 sigma_j sigma_j' * (1/m) sum_t gt_t[j] (c_t G)[j]  -  lambda sigma_j',   sigma_j' = sigma_j (1 - sigma_j) / T.
// Both contractions over the data are GEMMs on the fp32 matrix cores:
//   B = (Gt * sigma^2) G^T      (m x n, contraction over p)
//   R = C G                     (m x p, contraction over n; G is transposed chunk by chunk so that both operands of
//                                the NT kernel are contiguous along the contraction)
// Everything else is a row statistic (fp64, fixed order) or elementwise.
#include <hip/hip_runtime.h>

#include "grass.h"
#include "grass_device.h"

namespace grass {

bool launch_gemm_dma_kmajor(bool a_kn, const float* A, const float* B, float* C, uint64_t M, uint64_t N, uint64_t K,
                            uint64_t lda, uint64_t ldb, uint64_t ldc, int accumulate, hipStream_t st, hipError_t* err,
                            uint32_t splits, float* partials, int lower_only, uint64_t k_rows, uint64_t b_cols_avail);
hipError_t gemm_nt_f32(const float* A, const float* B, float* C, uint64_t M, uint64_t N, uint64_t K, uint64_t lda,
                       uint64_t ldb, uint64_t ldc, int accumulate, int lower_only, hipStream_t st, uint32_t splits,
                       float* partials);
uint32_t gemm_nt_f32_splits(const float* A, const float* B, uint64_t M, uint64_t N, uint64_t K, uint64_t lda, uint64_t ldb,
                            uint32_t max_splits);
constexpr uint32_t kSmMaxSplits = 64;

__device__ __forceinline__ float sigmoidf(float x) { return 1.0f / (1.0f + expf(-x)); }

// Workgroup-wide sum of one double per thread (256 threads), result in every thread; fixed order.
__device__ __forceinline__ double block_sum(double v, double* red) {
    const int t = threadIdx.x;
    red[t] = v;
    __syncthreads();
    for (int off = 128; off > 0; off >>= 1) {
        if (t < off) red[t] += red[t + off];
        __syncthreads();
    }
    const double r = red[0];
    __syncthreads();
    return r;
}

// Gtw[t][j] = Gt[t][j] * sigma_j^2 (S null: Gt[t][j]) for a block of 256 columns and the rows blockIdx.y,
// blockIdx.y + gridDim.y, ...; columns p..ld_w are zero-filled.
// sig_part[blockIdx.x] = sum of sigma_j over the block's columns (written by the first row group).
__global__ void __launch_bounds__(256) sm_weight_kernel(const float* __restrict__ Gt, uint64_t ldgt, uint64_t m, uint64_t p,
                                                       const float* __restrict__ S, float inv_temp,
                                                       float* __restrict__ Gtw, uint64_t ld_w, double* sig_part) {
    __shared__ double red[256];
    const uint64_t j = (uint64_t)blockIdx.x * 256 + threadIdx.x;
    float w = 0.0f, sig = 0.0f;
    if (j < p) {
        if (S) { sig = sigmoidf(S[j] * inv_temp); w = sig * sig; }
        else w = 1.0f;                                     // no mask: plain inner products
    }
    if (j < ld_w) {
        if (j < p) {
#pragma unroll 4
            for (uint64_t t = blockIdx.y; t < m; t += gridDim.y) Gtw[t * ld_w + j] = Gt[t * ldgt + j] * w;
        } else {
            for (uint64_t t = blockIdx.y; t < m; t += gridDim.y) Gtw[t * ld_w + j] = 0.0f;
        }
    }
    if (blockIdx.y != 0) return;                           // uniform
    const double total = block_sum((double)sig, red);
    if (threadIdx.x == 0) sig_part[blockIdx.x] = total;
}

// One workgroup per test row t: Pearson correlation of A[t][:] and B[t][:] over the n train rows and the row
// C[t][i] = (da_i / (|da||db|) - corr * db_i / |db|^2) / m; columns n..ld_c of C are zero.
__global__ void __launch_bounds__(256) sm_corr_kernel(const float* A, uint64_t lda, const float* B, uint64_t ldb,
                                                     uint64_t n, uint64_t m, float* C, uint64_t ld_c, double* corr) {
    __shared__ double red[256];
    const uint64_t t = blockIdx.x;
    const float* a = A + t * lda;
    const float* b = B + t * ldb;
    double sa = 0.0, sb = 0.0;
    for (uint64_t i = threadIdx.x; i < n; i += 256) { sa += a[i]; sb += b[i]; }
    const double ma = block_sum(sa, red) / (double)n;
    const double mb = block_sum(sb, red) / (double)n;
    double saa = 0.0, sbb = 0.0, sab = 0.0;
    for (uint64_t i = threadIdx.x; i < n; i += 256) {
        const double da = a[i] - ma, db = b[i] - mb;
        saa += da * da; sbb += db * db; sab += da * db;
    }
    saa = block_sum(saa, red);
    sbb = block_sum(sbb, red);
    sab = block_sum(sab, red);
    const bool ok = saa > 0.0 && sbb > 0.0;
    const double nab = ok ? sqrt(saa) * sqrt(sbb) : 1.0;
    const double r = ok ? sab / nab : 0.0;
    if (threadIdx.x == 0) corr[t] = r;
    const double ka = ok ? 1.0 / (nab * (double)m) : 0.0, kb = ok ? r / (sbb * (double)m) : 0.0;
    if (!C) return;                                        // correlation only
    for (uint64_t i = threadIdx.x; i < ld_c; i += 256)
        C[t * ld_c + i] = i < n ? (float)(ka * (a[i] - ma) - kb * (b[i] - mb)) : 0.0f;
}

// One ascent step on the logits: S_j += lr * grad_j (sum in fp64, rounded to fp32 once).
__global__ void __launch_bounds__(256) sm_update_kernel(float* S, const float* grad, uint64_t p, double lr) {
    const uint64_t j = (uint64_t)blockIdx.x * 256 + threadIdx.x;
    if (j < p) S[j] = (float)((double)S[j] + lr * (double)grad[j]);
}

// grad[j] = 2 sigma_j sigma_j' * sum_t Gt[t][j] R[t][j - j0] - lambda sigma_j' for the columns [j0, j0 + pc).
// A workgroup takes 64 columns; its four wavefronts sum the rows t = w, w + 4, ... in fp64 and the four partial sums
// are added in a fixed order.
__global__ void __launch_bounds__(256) sm_grad_kernel(const float* __restrict__ Gt, uint64_t ldgt, uint64_t m,
                                                     const float* __restrict__ R, uint64_t ld_r, uint64_t j0, uint64_t pc,
                                                     const float* __restrict__ S, float inv_temp, float lambda,
                                                     float* __restrict__ grad) {
    __shared__ double part[4][64];
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const uint64_t c = (uint64_t)blockIdx.x * 64 + lane;
    const uint64_t j = j0 + c;
    double acc = 0.0;
    if (c < pc) {
#pragma unroll 4
        for (uint64_t t = w; t < m; t += 4) acc += (double)Gt[t * ldgt + j] * (double)R[t * ld_r + c];
    }
    part[w][lane] = acc;
    __syncthreads();
    if (w != 0 || c >= pc) return;
    acc = ((part[0][lane] + part[1][lane]) + part[2][lane]) + part[3][lane];
    const float sig = sigmoidf(S[j] * inv_temp);
    const float dsig = sig * (1.0f - sig) * inv_temp;
    grad[j] = (float)(2.0 * (double)sig * (double)dsig * acc - (double)lambda * (double)dsig);
}

// Samples that are sequences of tokens: X and Y are (m * Tt) x (n * T) matrices of token-pair products (row distance
// ldk), B[te][i] = sum over the Tt x T block of (te, i) of X * Y (fp64 sum, fixed order), i < n; columns n..n_write of B
// are zero (row distance ldb).  With one token per sample this is the elementwise product.
__global__ void __launch_bounds__(256) sm_block_dot_kernel(const float* X, const float* Y, uint64_t ldk, uint64_t m, uint64_t n,
                                                          uint64_t Tt, uint64_t T, float* B, uint64_t ldb, uint64_t n_write) {
    const uint64_t id = (uint64_t)blockIdx.x * 256 + threadIdx.x;
    if (id >= m * n_write) return;
    const uint64_t te = id / n_write, i = id - te * n_write;
    double acc = 0.0;
    if (i < n)
        for (uint64_t a = 0; a < Tt; ++a) {
            const uint64_t row = (te * Tt + a) * ldk + i * T;
            for (uint64_t b = 0; b < T; ++b) acc += (double)X[row + b] * (double)Y[row + b];
        }
    B[te * ldb + i] = (float)acc;
}

// D[v][u] = C[v / Tt][u / T] * K[v][u] for u < n_tok, 0 for n_tok <= u < ldd: the derivative of the objective with
// respect to one factor's token-pair products (C is the m x n row matrix of sm_corr_kernel, K the other factor's
// token-pair products).  The padding columns of the workspace matrices may hold anything, D must not.
__global__ void __launch_bounds__(256) sm_expand_kernel(const float* C, uint64_t ldc, const float* K, uint64_t ldk,
                                                       uint64_t m_tok, uint64_t n_tok, uint64_t Tt, uint64_t T, float* D,
                                                       uint64_t ldd) {
    const uint64_t id = (uint64_t)blockIdx.x * 256 + threadIdx.x;
    if (id >= m_tok * ldd) return;
    const uint64_t v = id / ldd, u = id - v * ldd;
    D[v * ldd + u] = u < n_tok ? C[(v / Tt) * ldc + u / T] * K[v * ldk + u] : 0.0f;
}

// objective = mean of corr - lambda * sum of the sigma partial sums; one workgroup, fixed order.
__global__ void __launch_bounds__(256) sm_objective_kernel(const double* corr, uint64_t m, const double* sig_part,
                                                          uint64_t parts, const double* sig_part2, uint64_t parts2,
                                                          double lambda, double* objective) {
    __shared__ double red[256];
    double c = 0.0, s = 0.0;
    for (uint64_t i = threadIdx.x; i < m; i += 256) c += corr[i];
    for (uint64_t i = threadIdx.x; i < parts; i += 256) s += sig_part[i];
    for (uint64_t i = threadIdx.x; i < parts2; i += 256) s += sig_part2[i];
    c = block_sum(c, red);
    s = block_sum(s, red);
    if (threadIdx.x == 0) *objective = c / (double)m - lambda * s;
}

struct SmLayout {
    uint64_t ld_w, n_pad, pc, parts;
    size_t off_gtw, off_b, off_c, off_corr, off_sig, off_gt, off_r, off_part, total;
};
static size_t up256(size_t x) { return (x + 255) / 256 * 256; }
// p: the widest factor the workspace has to serve.
static SmLayout sm_layout(uint64_t n, uint64_t m, uint64_t p) {
    SmLayout L;
    L.ld_w = (p + 3) / 4 * 4;
    L.n_pad = (n + 15) / 16 * 16;
    // columns per transposed chunk of G: about 1 GiB of workspace, at least 4,096 columns
    uint64_t pc = (1ull << 28) / L.n_pad;
    if (pc < 4096) pc = 4096;
    pc = pc / 64 * 64;
    if (pc > (p + 63) / 64 * 64) pc = (p + 63) / 64 * 64;
    L.pc = pc;
    L.parts = ceil_div(L.ld_w, 256);
    size_t o = 0;
    L.off_gtw = o; o += up256((size_t)m * L.ld_w * 4);
    L.off_b = o; o += up256((size_t)m * L.n_pad * 4);
    L.off_c = o; o += up256((size_t)m * L.n_pad * 4);
    L.off_corr = o; o += up256((size_t)m * 8);
    L.off_sig = o; o += up256((size_t)L.parts * 8);
    L.off_gt = o; o += up256((size_t)pc * L.n_pad * 4);
    L.off_r = o; o += up256((size_t)m * pc * 4);
    // K-range partial sums of B when its m x n output has too few tiles to fill the chip
    L.off_part = o;
    if (ceil_div(m, 128) * ceil_div(n, 128) < 1024) o += up256((size_t)kSmMaxSplits * m * n * 4);
    L.total = o;
    return L;
}

// B (m x n, row distance n_pad) = (Gt * sigma^2) G^T; sig_part receives the per-block sums of sigma.
static grass_status sm_masked_scores(const SmLayout& L, unsigned char* base, const float* G, uint64_t n, uint64_t ldg,
                                     const float* Gt, uint64_t m, uint64_t ldgt, uint64_t p, const float* S, float inv_temp,
                                     float* B, double* sig_part, hipStream_t hs) {
    float* Gtw = reinterpret_cast<float*>(base + L.off_gtw);
    const uint64_t ld_w = (p + 3) / 4 * 4;
    hipLaunchKernelGGL(sm_weight_kernel, dim3((uint32_t)ceil_div(ld_w, 256), (uint32_t)(m < 16 ? m : 16)), dim3(256), 0, hs, Gt,
                       ldgt, m, p, S, inv_temp, Gtw, ld_w, sig_part);
    // The direct-to-LDS GEMM contracts over whole 64-byte slices.  With 16-byte aligned rows of G the bulk of the
    // contraction (p rounded down to a multiple of 16) goes through it and the last p % 16 columns are added by a
    // second, tiny product; otherwise one product over all p columns runs on the register-staged kernel.
    uint64_t p_main = p;
    if (p % 16 != 0 && p >= 4096 && ldg % 4 == 0 && aligned(G, 16) && m >= 128 && n >= 128) p_main = p / 16 * 16;
    uint32_t splits = 1;
    if (ceil_div(m, 128) * ceil_div(n, 128) < 1024) splits = gemm_nt_f32_splits(Gtw, G, m, n, p_main, ld_w, ldg, kSmMaxSplits);
    if (splits > 1) {
        float* partials = reinterpret_cast<float*>(base + L.off_part);
        if (gemm_nt_f32(Gtw, G, nullptr, m, n, p_main, ld_w, ldg, n, 0, 0, hs, splits, partials) != hipSuccess) return GRASS_EHIP;
        hipLaunchKernelGGL(reduce_partials_kernel, dim3((uint32_t)ceil_div(m * n, 256)), dim3(256), 0, hs, partials, m,
                           (uint32_t)n, splits, 1.0f, B, L.n_pad);
    } else if (gemm_nt_f32(Gtw, G, B, m, n, p_main, ld_w, ldg, L.n_pad, 0, 0, hs, 1, nullptr) != hipSuccess) {
        return GRASS_EHIP;
    }
    if (p_main < p &&
        gemm_nt_f32(Gtw + p_main, G + p_main, B, m, n, p - p_main, ld_w, ldg, L.n_pad, 1, 0, hs, 1, nullptr) != hipSuccess)
        return GRASS_EHIP;
    return GRASS_OK;
}

// grad[j] = 2 sigma_j sigma_j' sum_t Gt[t][j] (C G)[t][j] - lambda sigma_j' for all p columns, G transposed in chunks.
static grass_status sm_backward(const SmLayout& L, unsigned char* base, const float* G, uint64_t n, uint64_t ldg,
                                const float* Gt, uint64_t m, uint64_t ldgt, uint64_t p, const float* S, float inv_temp,
                                float lambda, const float* C, float* grad, hipStream_t hs) {
    float* GTc = reinterpret_cast<float*>(base + L.off_gt);
    float* Rc = reinterpret_cast<float*>(base + L.off_r);
    const bool kmajor = m >= 128 && ldg % 4 == 0 && aligned(G, 16);      // chunk starts j0 are multiples of 64
    for (uint64_t j0 = 0; j0 < p; j0 += L.pc) {
        const uint64_t pc = j0 + L.pc <= p ? L.pc : p - j0;
        // Rc (m x pc) = C G[:, j0 : j0+pc], a contraction over the n rows of G.  With 16-byte aligned rows the GEMM
        // reads the column block of G in place as a K-major operand (C is zero beyond column n, G's rows end at n);
        // otherwise the block is transposed into the workspace first.
        bool taken = false;
        if (kmajor) {
            hipError_t derr = hipSuccess;
            taken = launch_gemm_dma_kmajor(false, C, G + j0, Rc, m, pc, L.n_pad, L.n_pad, ldg, L.pc, 0, hs, &derr, 1, nullptr,
                                           0, n, ldg - j0);
            if (taken && derr != hipSuccess) return GRASS_EHIP;
        }
        if (!taken) {
            // GTc (pc x n_pad) = transpose of the column block [j0, j0 + pc) of G
            hipLaunchKernelGGL(transpose_rows_kernel, dim3((uint32_t)ceil_div(pc, 64), (uint32_t)ceil_div(L.n_pad, 64)),
                               dim3(256), 0, hs, G + j0, ldg, (uint64_t)0, (uint32_t)n, (uint32_t)L.n_pad, (uint32_t)pc, GTc,
                               L.n_pad);
            if (gemm_nt_f32(C, GTc, Rc, m, pc, L.n_pad, L.n_pad, L.n_pad, L.pc, 0, 0, hs, 1, nullptr) != hipSuccess)
                return GRASS_EHIP;
        }
        hipLaunchKernelGGL(sm_grad_kernel, dim3((uint32_t)ceil_div(pc, 64)), dim3(256), 0, hs, Gt, ldgt, m, Rc, L.pc, j0, pc,
                           S, inv_temp, lambda, grad);
    }
    return GRASS_OK;
}

}  // namespace grass

using namespace grass;

static grass_status check_sm(uint64_t n, uint64_t m, uint64_t p) {
    if (n < 2 || m == 0 || p == 0) return GRASS_EINVAL;
    if (p >= (1ull << 31) || n >= (1ull << 31) || m >= (1ull << 31)) return GRASS_EUNSUPPORTED;
    return GRASS_OK;
}

extern "C" grass_status grass_selective_mask_grad_workspace_bytes(uint64_t n, uint64_t m, uint64_t p,
                                                                  size_t* host_bytes) {
    if (!host_bytes) return GRASS_EINVAL;
    grass_status st = check_sm(n, m, p);
    if (st != GRASS_OK) return st;
    *host_bytes = sm_layout(n, m, p).total;
    return GRASS_OK;
}

// Objective and gradient at S for one temperature: the body of grass_selective_mask_grad and of every training step.
static grass_status sm_value_and_grad(const SmLayout& L, unsigned char* base, const float* G, uint64_t n, uint64_t ldg,
                                      const float* Gt, uint64_t m, uint64_t ldgt, uint64_t p, const float* A, uint64_t lda,
                                      const float* S, double lambda, double temperature, float* grad, double* objective,
                                      hipStream_t hs) {
    grass_status st;
    float* B = reinterpret_cast<float*>(base + L.off_b);
    float* C = reinterpret_cast<float*>(base + L.off_c);
    double* corr = reinterpret_cast<double*>(base + L.off_corr);
    double* sig_part = reinterpret_cast<double*>(base + L.off_sig);
    const float inv_temp = (float)(1.0 / temperature);

    st = sm_masked_scores(L, base, G, n, ldg, Gt, m, ldgt, p, S, inv_temp, B, sig_part, hs);
    if (st != GRASS_OK) return st;
    hipLaunchKernelGGL(sm_corr_kernel, dim3((uint32_t)m), dim3(256), 0, hs, A, lda, B, L.n_pad, n, m, C, L.n_pad, corr);
    st = sm_backward(L, base, G, n, ldg, Gt, m, ldgt, p, S, inv_temp, (float)lambda, C, grad, hs);
    if (st != GRASS_OK) return st;
    if (objective)
        hipLaunchKernelGGL(sm_objective_kernel, dim3(1), dim3(256), 0, hs, corr, m, sig_part, ceil_div((p + 3) / 4 * 4, 256),
                           (const double*)nullptr, (uint64_t)0, lambda, objective);
    return launch_status();
}

extern "C" grass_status grass_selective_mask_grad(const float* G, uint64_t n, uint64_t ldg, const float* Gt, uint64_t m,
                                                  uint64_t ldgt, uint64_t p, const float* A, uint64_t lda,
                                                  const float* S, double lambda, double temperature, float* grad,
                                                  double* objective, void* ws, size_t ws_bytes, grass_stream stream) {
    grass_status st = check_sm(n, m, p);
    if (st != GRASS_OK) return st;
    if (!G || !Gt || !A || !S || !grad || ldg < p || ldgt < p || lda < n) return GRASS_EINVAL;
    if (!(temperature > 0.0) || !(lambda >= 0.0)) return GRASS_EINVAL;
    const SmLayout L = sm_layout(n, m, p);
    if (!ws || ws_bytes < L.total || !aligned(ws, 256)) return GRASS_EWORKSPACE;
    return sm_value_and_grad(L, static_cast<unsigned char*>(ws), G, n, ldg, Gt, m, ldgt, p, A, lda, S, lambda, temperature,
                             grad, objective, as_stream(stream));
}

// Training: `steps` plain gradient-ascent steps on the logits, step i at temperature host_temperatures[i], all
// enqueued back to back (the host only reads its own schedule array; nothing waits for the device).
extern "C" grass_status grass_selective_mask_train_workspace_bytes(uint64_t n, uint64_t m, uint64_t p,
                                                                   size_t* host_bytes) {
    if (!host_bytes) return GRASS_EINVAL;
    grass_status st = check_sm(n, m, p);
    if (st != GRASS_OK) return st;
    *host_bytes = sm_layout(n, m, p).total + up256((size_t)p * 4);
    return GRASS_OK;
}

extern "C" grass_status grass_selective_mask_train(const float* G, uint64_t n, uint64_t ldg, const float* Gt, uint64_t m,
                                                   uint64_t ldgt, uint64_t p, const float* A, uint64_t lda, float* S,
                                                   double lambda, double lr, const double* host_temperatures,
                                                   uint32_t steps, double* objectives, void* ws, size_t ws_bytes,
                                                   grass_stream stream) {
    grass_status st = check_sm(n, m, p);
    if (st != GRASS_OK) return st;
    if (!G || !Gt || !A || !S || ldg < p || ldgt < p || lda < n) return GRASS_EINVAL;
    if (!(lambda >= 0.0) || !(lr == lr) || (steps > 0 && !host_temperatures)) return GRASS_EINVAL;
    for (uint32_t i = 0; i < steps; ++i)
        if (!(host_temperatures[i] > 0.0)) return GRASS_EINVAL;
    const SmLayout L = sm_layout(n, m, p);
    if (!ws || ws_bytes < L.total + up256((size_t)p * 4) || !aligned(ws, 256)) return GRASS_EWORKSPACE;
    unsigned char* base = static_cast<unsigned char*>(ws);
    float* grad = reinterpret_cast<float*>(base + L.total);
    hipStream_t hs = as_stream(stream);
    for (uint32_t i = 0; i < steps; ++i) {
        st = sm_value_and_grad(L, base, G, n, ldg, Gt, m, ldgt, p, A, lda, S, lambda, host_temperatures[i], grad,
                               objectives ? objectives + i : nullptr, hs);
        if (st != GRASS_OK) return st;
        hipLaunchKernelGGL(sm_update_kernel, dim3((uint32_t)ceil_div(p, 256)), dim3(256), 0, hs, S, grad, p, lr);
    }
    return launch_status();
}

// Mean over the m rows of the Pearson correlation between row t of X and row t of Y (two m x n score matrices): the
// first term of Eq. (1) when Y holds the scores of masked gradients, and the agreement measure between exact and
// compressed attribution scores in general.
extern "C" grass_status grass_score_correlation_workspace_bytes(uint64_t m, size_t* host_bytes) {
    if (!host_bytes || m == 0) return GRASS_EINVAL;
    *host_bytes = up256((size_t)m * 8);
    return GRASS_OK;
}

extern "C" grass_status grass_score_correlation(const float* X, uint64_t ldx, const float* Y, uint64_t ldy, uint64_t m,
                                                uint64_t n, double* mean_corr, void* ws, size_t ws_bytes,
                                                grass_stream stream) {
    if (m == 0 || n < 2 || !X || !Y || !mean_corr || ldx < n || ldy < n) return GRASS_EINVAL;
    if (m >= (1ull << 31)) return GRASS_EUNSUPPORTED;
    if (!ws || ws_bytes < up256((size_t)m * 8) || !aligned(ws, 256)) return GRASS_EWORKSPACE;
    double* corr = static_cast<double*>(ws);
    hipStream_t hs = as_stream(stream);
    hipLaunchKernelGGL(sm_corr_kernel, dim3((uint32_t)m), dim3(256), 0, hs, X, ldx, Y, ldy, n, m, (float*)nullptr, (uint64_t)0,
                       corr);
    hipLaunchKernelGGL(sm_objective_kernel, dim3(1), dim3(256), 0, hs, corr, m, (const double*)nullptr, (uint64_t)0,
                       (const double*)nullptr, (uint64_t)0, 0.0, mean_corr);
    return launch_status();
}

// Factorised form for a linear layer (App. B.4 "Linear Layer"): gradients z_in (x) z_out, mask sigma(S_in) (x) sigma(S_out),
// <a (x) b, c (x) d> = <a, c><b, d>, so the masked scores are the elementwise product of the two factors' masked scores
// and each factor's gradient is the plain backward pass with C multiplied by the other factor's masked scores.  Samples
// that are sequences of tokens have gradients sum_t z_in_t (x) z_out_t (Eq. (2)): the factors' products are then taken
// between all tokens of a test and a train sample and summed over the token pairs; one token per sample is the case
// the paper writes out.
extern "C" grass_status grass_selective_mask_grad_factorized_workspace_bytes(uint64_t n, uint64_t m, uint64_t d_in,
                                                                             uint64_t d_out, size_t* host_bytes) {
    return grass_selective_mask_grad_factorized_seq_workspace_bytes(n, 1, m, 1, d_in, d_out, host_bytes);
}

// Sizes of the factorised problem on sequences: n samples of T tokens against m samples of Tt tokens.
struct SmSeq {
    uint64_t n, T, m, Tt, n_tok, m_tok, nb_pad;
};
static grass_status check_sm_factorized(uint64_t n, uint64_t T, uint64_t m, uint64_t Tt, uint64_t d_in, uint64_t d_out,
                                        SmSeq* q) {
    if (T == 0 || Tt == 0 || d_in == 0 || d_out == 0) return GRASS_EINVAL;
    if (n >= (1ull << 31) / T || m >= (1ull << 31) / Tt) return GRASS_EUNSUPPORTED;
    q->n = n; q->T = T; q->m = m; q->Tt = Tt; q->n_tok = n * T; q->m_tok = m * Tt; q->nb_pad = (n + 15) / 16 * 16;
    return check_sm(n, m, d_in > d_out ? d_in : d_out);
}
static grass_status check_sm_factorized_args(const SmSeq& q, uint64_t d_in, uint64_t d_out, const float* Z_in,
                                             const float* Z_out, uint64_t ld_zin, uint64_t ld_zout, const float* Zt_in,
                                             const float* Zt_out, uint64_t ld_ztin, uint64_t ld_ztout) {
    if (!Z_in || !Z_out || !Zt_in || !Zt_out) return GRASS_EINVAL;
    if (ld_zin < d_in || ld_ztin < d_in || ld_zout < d_out || ld_ztout < d_out) return GRASS_EINVAL;
    return GRASS_OK;
}
// workspace: sm_layout over the token matrices, then the second factor's token-pair products, its sigma partial sums,
// and the m x n matrices B and C
static size_t sm_factorized_bytes(const SmLayout& L, const SmSeq& q) {
    return L.total + up256((size_t)q.m_tok * L.n_pad * 4) + up256((size_t)L.parts * 8) + 2 * up256((size_t)q.m * q.nb_pad * 4);
}

// Value and both gradients.  Rows of Z_* are tokens (sample i owns rows i*T .. i*T + T - 1).
static grass_status sm_value_and_grad_factorized(
    const SmLayout& L, const SmSeq& q, unsigned char* base, const float* Z_in, const float* Z_out, uint64_t ld_zin,
    uint64_t ld_zout, const float* Zt_in, const float* Zt_out, uint64_t ld_ztin, uint64_t ld_ztout, uint64_t d_in,
    uint64_t d_out, const float* A, uint64_t lda, const float* S_in, const float* S_out, double lambda, double temperature,
    float* grad_in, float* grad_out, double* objective, hipStream_t hs) {
    const size_t tok_bytes = up256((size_t)q.m_tok * L.n_pad * 4), small = up256((size_t)q.m * q.nb_pad * 4);
    float* K_in = reinterpret_cast<float*>(base + L.off_b);            // token-pair products, m_tok x n_pad
    float* D = reinterpret_cast<float*>(base + L.off_c);               // derivative with respect to a factor's products
    double* corr = reinterpret_cast<double*>(base + L.off_corr);
    double* sig_in = reinterpret_cast<double*>(base + L.off_sig);
    float* K_out = reinterpret_cast<float*>(base + L.total);
    double* sig_out = reinterpret_cast<double*>(base + L.total + tok_bytes);
    float* B = reinterpret_cast<float*>(base + L.total + tok_bytes + up256((size_t)L.parts * 8));
    float* C = reinterpret_cast<float*>(reinterpret_cast<unsigned char*>(B) + small);
    const float inv_temp = (float)(1.0 / temperature);
    const uint32_t small_blocks = (uint32_t)ceil_div(q.m * q.nb_pad, 256);
    const uint32_t tok_blocks = (uint32_t)ceil_div(q.m_tok * L.n_pad, 256);

    grass_status st = sm_masked_scores(L, base, Z_in, q.n_tok, ld_zin, Zt_in, q.m_tok, ld_ztin, d_in, S_in, inv_temp, K_in, sig_in, hs);
    if (st != GRASS_OK) return st;
    st = sm_masked_scores(L, base, Z_out, q.n_tok, ld_zout, Zt_out, q.m_tok, ld_ztout, d_out, S_out, inv_temp, K_out, sig_out, hs);
    if (st != GRASS_OK) return st;
    // masked scores of the layer gradients (Kronecker products summed over tokens), their correlation with A, the row c
    hipLaunchKernelGGL(sm_block_dot_kernel, dim3(small_blocks), dim3(256), 0, hs, K_in, K_out, L.n_pad, q.m, q.n, q.Tt, q.T, B,
                       q.nb_pad, q.nb_pad);
    hipLaunchKernelGGL(sm_corr_kernel, dim3((uint32_t)q.m), dim3(256), 0, hs, A, lda, B, q.nb_pad, q.n, q.m, C, q.nb_pad, corr);
    // each factor's gradient is the plain backward pass over its token matrices with c spread over the token pairs and
    // multiplied by the other factor's products
    hipLaunchKernelGGL(sm_expand_kernel, dim3(tok_blocks), dim3(256), 0, hs, C, q.nb_pad, K_out, L.n_pad, q.m_tok, q.n_tok, q.Tt,
                       q.T, D, L.n_pad);
    st = sm_backward(L, base, Z_in, q.n_tok, ld_zin, Zt_in, q.m_tok, ld_ztin, d_in, S_in, inv_temp, (float)lambda, D, grad_in, hs);
    if (st != GRASS_OK) return st;
    hipLaunchKernelGGL(sm_expand_kernel, dim3(tok_blocks), dim3(256), 0, hs, C, q.nb_pad, K_in, L.n_pad, q.m_tok, q.n_tok, q.Tt,
                       q.T, D, L.n_pad);
    st = sm_backward(L, base, Z_out, q.n_tok, ld_zout, Zt_out, q.m_tok, ld_ztout, d_out, S_out, inv_temp, (float)lambda, D, grad_out, hs);
    if (st != GRASS_OK) return st;
    if (objective)
        hipLaunchKernelGGL(sm_objective_kernel, dim3(1), dim3(256), 0, hs, corr, q.m, sig_in, ceil_div((d_in + 3) / 4 * 4, 256),
                           (const double*)sig_out, ceil_div((d_out + 3) / 4 * 4, 256), lambda, objective);
    return launch_status();
}

extern "C" grass_status grass_selective_mask_grad_factorized_seq_workspace_bytes(uint64_t n, uint64_t T, uint64_t m, uint64_t Tt,
                                                                                 uint64_t d_in, uint64_t d_out,
                                                                                 size_t* host_bytes) {
    if (!host_bytes) return GRASS_EINVAL;
    SmSeq q;
    grass_status st = check_sm_factorized(n, T, m, Tt, d_in, d_out, &q);
    if (st != GRASS_OK) return st;
    *host_bytes = sm_factorized_bytes(sm_layout(q.n_tok, q.m_tok, d_in > d_out ? d_in : d_out), q);
    return GRASS_OK;
}

extern "C" grass_status grass_selective_mask_grad_factorized_seq(
    const float* Z_in, const float* Z_out, uint64_t n, uint64_t T, uint64_t ld_zin, uint64_t ld_zout, const float* Zt_in,
    const float* Zt_out, uint64_t m, uint64_t Tt, uint64_t ld_ztin, uint64_t ld_ztout, uint64_t d_in, uint64_t d_out,
    const float* A, uint64_t lda, const float* S_in, const float* S_out, double lambda, double temperature, float* grad_in,
    float* grad_out, double* objective, void* ws, size_t ws_bytes, grass_stream stream) {
    SmSeq q;
    grass_status st = check_sm_factorized(n, T, m, Tt, d_in, d_out, &q);
    if (st != GRASS_OK) return st;
    st = check_sm_factorized_args(q, d_in, d_out, Z_in, Z_out, ld_zin, ld_zout, Zt_in, Zt_out, ld_ztin, ld_ztout);
    if (st != GRASS_OK) return st;
    if (!A || lda < n || !S_in || !S_out || !grad_in || !grad_out) return GRASS_EINVAL;
    if (!(temperature > 0.0) || !(lambda >= 0.0)) return GRASS_EINVAL;
    const SmLayout L = sm_layout(q.n_tok, q.m_tok, d_in > d_out ? d_in : d_out);
    if (!ws || ws_bytes < sm_factorized_bytes(L, q) || !aligned(ws, 256)) return GRASS_EWORKSPACE;
    return sm_value_and_grad_factorized(L, q, static_cast<unsigned char*>(ws), Z_in, Z_out, ld_zin, ld_zout, Zt_in, Zt_out,
                                        ld_ztin, ld_ztout, d_in, d_out, A, lda, S_in, S_out, lambda, temperature, grad_in,
                                        grad_out, objective, as_stream(stream));
}

// Exact GradDot scores of the layer on sequences, A[te][i] = sum over token pairs of <z_in, zt_in> <z_out, zt_out>:
// the same token-pair products without weights, then the block sums.
extern "C" grass_status grass_graddot_factorized_workspace_bytes(uint64_t n, uint64_t T, uint64_t m, uint64_t Tt,
                                                                 uint64_t d_in, uint64_t d_out, size_t* host_bytes) {
    return grass_selective_mask_grad_factorized_seq_workspace_bytes(n, T, m, Tt, d_in, d_out, host_bytes);
}

extern "C" grass_status grass_graddot_factorized(const float* Z_in, const float* Z_out, uint64_t n, uint64_t T, uint64_t ld_zin,
                                                 uint64_t ld_zout, const float* Zt_in, const float* Zt_out, uint64_t m,
                                                 uint64_t Tt, uint64_t ld_ztin, uint64_t ld_ztout, uint64_t d_in, uint64_t d_out,
                                                 float* A, uint64_t lda, void* ws, size_t ws_bytes, grass_stream stream) {
    SmSeq q;
    grass_status st = check_sm_factorized(n, T, m, Tt, d_in, d_out, &q);
    if (st != GRASS_OK) return st;
    st = check_sm_factorized_args(q, d_in, d_out, Z_in, Z_out, ld_zin, ld_zout, Zt_in, Zt_out, ld_ztin, ld_ztout);
    if (st != GRASS_OK) return st;
    if (!A || lda < n) return GRASS_EINVAL;
    const SmLayout L = sm_layout(q.n_tok, q.m_tok, d_in > d_out ? d_in : d_out);
    if (!ws || ws_bytes < sm_factorized_bytes(L, q) || !aligned(ws, 256)) return GRASS_EWORKSPACE;
    unsigned char* base = static_cast<unsigned char*>(ws);
    float* K_in = reinterpret_cast<float*>(base + L.off_b);
    float* K_out = reinterpret_cast<float*>(base + L.total);
    double* sig = reinterpret_cast<double*>(base + L.off_sig);
    hipStream_t hs = as_stream(stream);
    st = sm_masked_scores(L, base, Z_in, q.n_tok, ld_zin, Zt_in, q.m_tok, ld_ztin, d_in, nullptr, 1.0f, K_in, sig, hs);
    if (st != GRASS_OK) return st;
    st = sm_masked_scores(L, base, Z_out, q.n_tok, ld_zout, Zt_out, q.m_tok, ld_ztout, d_out, nullptr, 1.0f, K_out, sig, hs);
    if (st != GRASS_OK) return st;
    hipLaunchKernelGGL(sm_block_dot_kernel, dim3((uint32_t)ceil_div(q.m * q.n, 256)), dim3(256), 0, hs, K_in, K_out, L.n_pad, q.m,
                       q.n, q.Tt, q.T, A, lda, q.n);                       // exactly the n columns of the caller's rows
    return launch_status();
}

extern "C" grass_status grass_selective_mask_grad_factorized(
    const float* Z_in, const float* Z_out, uint64_t n, uint64_t ld_zin, uint64_t ld_zout, const float* Zt_in,
    const float* Zt_out, uint64_t m, uint64_t ld_ztin, uint64_t ld_ztout, uint64_t d_in, uint64_t d_out, const float* A,
    uint64_t lda, const float* S_in, const float* S_out, double lambda, double temperature, float* grad_in, float* grad_out,
    double* objective, void* ws, size_t ws_bytes, grass_stream stream) {
    return grass_selective_mask_grad_factorized_seq(Z_in, Z_out, n, 1, ld_zin, ld_zout, Zt_in, Zt_out, m, 1, ld_ztin, ld_ztout,
                                                    d_in, d_out, A, lda, S_in, S_out, lambda, temperature, grad_in, grad_out,
                                                    objective, ws, ws_bytes, stream);
}

// Training of the factorised mask: both logit vectors take a plain gradient-ascent step per temperature of the host
// schedule, both derivatives taken at the logits before the step (the two updates run after both backward passes).
// Samples are sequences of T (train) and Tt (test) tokens; one token each is the case the paper writes out.
extern "C" grass_status grass_selective_mask_train_factorized_seq_workspace_bytes(uint64_t n, uint64_t T, uint64_t m,
                                                                                  uint64_t Tt, uint64_t d_in, uint64_t d_out,
                                                                                  size_t* host_bytes) {
    if (!host_bytes) return GRASS_EINVAL;
    SmSeq q;
    grass_status st = check_sm_factorized(n, T, m, Tt, d_in, d_out, &q);
    if (st != GRASS_OK) return st;
    *host_bytes = sm_factorized_bytes(sm_layout(q.n_tok, q.m_tok, d_in > d_out ? d_in : d_out), q) +
                  up256((size_t)d_in * 4) + up256((size_t)d_out * 4);
    return GRASS_OK;
}

extern "C" grass_status grass_selective_mask_train_factorized_seq(
    const float* Z_in, const float* Z_out, uint64_t n, uint64_t T, uint64_t ld_zin, uint64_t ld_zout, const float* Zt_in,
    const float* Zt_out, uint64_t m, uint64_t Tt, uint64_t ld_ztin, uint64_t ld_ztout, uint64_t d_in, uint64_t d_out,
    const float* A, uint64_t lda, float* S_in, float* S_out, double lambda, double lr, const double* host_temperatures,
    uint32_t steps, double* objectives, void* ws, size_t ws_bytes, grass_stream stream) {
    SmSeq q;
    grass_status st = check_sm_factorized(n, T, m, Tt, d_in, d_out, &q);
    if (st != GRASS_OK) return st;
    st = check_sm_factorized_args(q, d_in, d_out, Z_in, Z_out, ld_zin, ld_zout, Zt_in, Zt_out, ld_ztin, ld_ztout);
    if (st != GRASS_OK) return st;
    if (!A || lda < n || !S_in || !S_out) return GRASS_EINVAL;
    if (!(lambda >= 0.0) || !(lr == lr) || (steps > 0 && !host_temperatures)) return GRASS_EINVAL;
    for (uint32_t i = 0; i < steps; ++i)
        if (!(host_temperatures[i] > 0.0)) return GRASS_EINVAL;
    const SmLayout L = sm_layout(q.n_tok, q.m_tok, d_in > d_out ? d_in : d_out);
    const size_t fb = sm_factorized_bytes(L, q);
    if (!ws || ws_bytes < fb + up256((size_t)d_in * 4) + up256((size_t)d_out * 4) || !aligned(ws, 256))
        return GRASS_EWORKSPACE;
    unsigned char* base = static_cast<unsigned char*>(ws);
    float* grad_in = reinterpret_cast<float*>(base + fb);
    float* grad_out = reinterpret_cast<float*>(base + fb + up256((size_t)d_in * 4));
    hipStream_t hs = as_stream(stream);
    for (uint32_t i = 0; i < steps; ++i) {
        st = sm_value_and_grad_factorized(L, q, base, Z_in, Z_out, ld_zin, ld_zout, Zt_in, Zt_out, ld_ztin, ld_ztout, d_in, d_out,
                                          A, lda, S_in, S_out, lambda, host_temperatures[i], grad_in, grad_out,
                                          objectives ? objectives + i : nullptr, hs);
        if (st != GRASS_OK) return st;
        hipLaunchKernelGGL(sm_update_kernel, dim3((uint32_t)ceil_div(d_in, 256)), dim3(256), 0, hs, S_in, grad_in, d_in, lr);
        hipLaunchKernelGGL(sm_update_kernel, dim3((uint32_t)ceil_div(d_out, 256)), dim3(256), 0, hs, S_out, grad_out, d_out, lr);
    }
    return launch_status();
}

extern "C" grass_status grass_selective_mask_train_factorized_workspace_bytes(uint64_t n, uint64_t m, uint64_t d_in,
                                                                              uint64_t d_out, size_t* host_bytes) {
    return grass_selective_mask_train_factorized_seq_workspace_bytes(n, 1, m, 1, d_in, d_out, host_bytes);
}

extern "C" grass_status grass_selective_mask_train_factorized(
    const float* Z_in, const float* Z_out, uint64_t n, uint64_t ld_zin, uint64_t ld_zout, const float* Zt_in,
    const float* Zt_out, uint64_t m, uint64_t ld_ztin, uint64_t ld_ztout, uint64_t d_in, uint64_t d_out, const float* A,
    uint64_t lda, float* S_in, float* S_out, double lambda, double lr, const double* host_temperatures, uint32_t steps,
    double* objectives, void* ws, size_t ws_bytes, grass_stream stream) {
    return grass_selective_mask_train_factorized_seq(Z_in, Z_out, n, 1, ld_zin, ld_zout, Zt_in, Zt_out, m, 1, ld_ztin, ld_ztout,
                                                     d_in, d_out, A, lda, S_in, S_out, lambda, lr, host_temperatures, steps,
                                                     objectives, ws, ws_bytes, stream);
}
