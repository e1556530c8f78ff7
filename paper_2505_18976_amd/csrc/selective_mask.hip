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

hipError_t gemm_nt_f32(const float* A, const float* B, float* C, uint64_t M, uint64_t N, uint64_t K, uint64_t lda,
                       uint64_t ldb, uint64_t ldc, int accumulate, int lower_only, hipStream_t st, uint32_t splits,
                       float* partials);
uint32_t gemm_nt_f32_splits(const float* A, const float* B, uint64_t M, uint64_t N, uint64_t K, uint64_t lda, uint64_t ldb,
                            uint32_t max_splits);
constexpr uint32_t kSmMaxSplits = 8;

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

// Gtw[t][j] = Gt[t][j] * sigma_j^2 for a block of 256 columns and all m rows; columns p..ld_w are zero-filled.
// sig_part[blockIdx.x] = sum of sigma_j over the block's columns.
__global__ void __launch_bounds__(256) sm_weight_kernel(const float* Gt, uint64_t ldgt, uint64_t m, uint64_t p,
                                                       const float* S, float inv_temp, float* Gtw, uint64_t ld_w,
                                                       double* sig_part) {
    __shared__ double red[256];
    const uint64_t j = (uint64_t)blockIdx.x * 256 + threadIdx.x;
    float w = 0.0f, sig = 0.0f;
    if (j < p) { sig = sigmoidf(S[j] * inv_temp); w = sig * sig; }
    if (j < ld_w)
        for (uint64_t t = 0; t < m; ++t) Gtw[t * ld_w + j] = j < p ? Gt[t * ldgt + j] * w : 0.0f;
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
    for (uint64_t i = threadIdx.x; i < ld_c; i += 256)
        C[t * ld_c + i] = i < n ? (float)(ka * (a[i] - ma) - kb * (b[i] - mb)) : 0.0f;
}

// grad[j] = 2 sigma_j sigma_j' * sum_t Gt[t][j] R[t][j - j0] - lambda sigma_j' for the columns [j0, j0 + pc).
__global__ void __launch_bounds__(256) sm_grad_kernel(const float* Gt, uint64_t ldgt, uint64_t m, const float* R,
                                                     uint64_t ld_r, uint64_t j0, uint64_t pc, const float* S,
                                                     float inv_temp, float lambda, float* grad) {
    const uint64_t c = (uint64_t)blockIdx.x * 256 + threadIdx.x;
    if (c >= pc) return;
    const uint64_t j = j0 + c;
    double acc = 0.0;
    for (uint64_t t = 0; t < m; ++t) acc += (double)Gt[t * ldgt + j] * (double)R[t * ld_r + c];
    const float sig = sigmoidf(S[j] * inv_temp);
    const float dsig = sig * (1.0f - sig) * inv_temp;
    grad[j] = (float)(2.0 * (double)sig * (double)dsig * acc - (double)lambda * (double)dsig);
}

// objective = mean of corr - lambda * sum of the sigma partial sums; one workgroup, fixed order.
__global__ void __launch_bounds__(256) sm_objective_kernel(const double* corr, uint64_t m, const double* sig_part,
                                                          uint64_t parts, double lambda, double* objective) {
    __shared__ double red[256];
    double c = 0.0, s = 0.0;
    for (uint64_t i = threadIdx.x; i < m; i += 256) c += corr[i];
    for (uint64_t i = threadIdx.x; i < parts; i += 256) s += sig_part[i];
    c = block_sum(c, red);
    s = block_sum(s, red);
    if (threadIdx.x == 0) *objective = c / (double)m - lambda * s;
}

struct SmLayout {
    uint64_t ld_w, n_pad, pc, parts;
    size_t off_gtw, off_b, off_c, off_corr, off_sig, off_gt, off_r, off_part, total;
};
static size_t up256(size_t x) { return (x + 255) / 256 * 256; }
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
    unsigned char* base = static_cast<unsigned char*>(ws);
    float* Gtw = reinterpret_cast<float*>(base + L.off_gtw);
    float* B = reinterpret_cast<float*>(base + L.off_b);
    float* C = reinterpret_cast<float*>(base + L.off_c);
    double* corr = reinterpret_cast<double*>(base + L.off_corr);
    double* sig_part = reinterpret_cast<double*>(base + L.off_sig);
    float* GTc = reinterpret_cast<float*>(base + L.off_gt);
    float* Rc = reinterpret_cast<float*>(base + L.off_r);
    hipStream_t hs = as_stream(stream);
    const float inv_temp = (float)(1.0 / temperature);

    hipLaunchKernelGGL(sm_weight_kernel, dim3((uint32_t)L.parts), dim3(256), 0, hs, Gt, ldgt, m, p, S, inv_temp, Gtw, L.ld_w,
                       sig_part);
    uint32_t splits = 1;
    if (ceil_div(m, 128) * ceil_div(n, 128) < 1024) splits = gemm_nt_f32_splits(Gtw, G, m, n, p, L.ld_w, ldg, kSmMaxSplits);
    if (splits > 1) {
        float* partials = reinterpret_cast<float*>(base + L.off_part);
        if (gemm_nt_f32(Gtw, G, nullptr, m, n, p, L.ld_w, ldg, n, 0, 0, hs, splits, partials) != hipSuccess) return GRASS_EHIP;
        hipLaunchKernelGGL(reduce_partials_kernel, dim3((uint32_t)ceil_div(m * n, 256)), dim3(256), 0, hs, partials, m,
                           (uint32_t)n, splits, 1.0f, B, L.n_pad);
    } else if (gemm_nt_f32(Gtw, G, B, m, n, p, L.ld_w, ldg, L.n_pad, 0, 0, hs, 1, nullptr) != hipSuccess) {
        return GRASS_EHIP;
    }
    hipLaunchKernelGGL(sm_corr_kernel, dim3((uint32_t)m), dim3(256), 0, hs, A, lda, B, L.n_pad, n, m, C, L.n_pad, corr);
    for (uint64_t j0 = 0; j0 < p; j0 += L.pc) {
        const uint64_t pc = j0 + L.pc <= p ? L.pc : p - j0;
        // GTc (pc x n_pad) = transpose of the column block [j0, j0 + pc) of G
        hipLaunchKernelGGL(transpose_rows_kernel, dim3((uint32_t)ceil_div(pc, 64), (uint32_t)(L.n_pad / 64 + (L.n_pad % 64 != 0))),
                           dim3(256), 0, hs, G + j0, ldg, (uint64_t)0, (uint32_t)n, (uint32_t)L.n_pad, (uint32_t)pc, GTc,
                           L.n_pad);
        if (gemm_nt_f32(C, GTc, Rc, m, pc, L.n_pad, L.n_pad, L.n_pad, L.pc, 0, 0, hs, 1, nullptr) != hipSuccess)
            return GRASS_EHIP;
        hipLaunchKernelGGL(sm_grad_kernel, dim3((uint32_t)ceil_div(pc, 256)), dim3(256), 0, hs, Gt, ldgt, m, Rc, L.pc, j0, pc,
                           S, inv_temp, (float)lambda, grad);
    }
    if (objective)
        hipLaunchKernelGGL(sm_objective_kernel, dim3(1), dim3(256), 0, hs, corr, m, sig_part, L.parts, lambda, objective);
    return launch_status();
}
