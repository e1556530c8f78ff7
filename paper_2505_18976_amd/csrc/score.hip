// Dense contractions on the matrix cores: the attribute-stage score GEMM
// (Sec. 2.1: all-pair inner products of compressed gradients) and the dense
// Gaussian projection baseline (Sec. 2.2: g_hat = P g, P_ij ~ N(0, 1/k)).
//
// Both are C[M x N] (+)= A[M x K] * B[N x K]^T with A and B row-major and K
// contiguous ("NT" GEMM).  A workgroup of 4 wavefronts (2 x 2) computes a
// 128 x 128 tile of C; each wavefront owns 64 x 64 = 2 x 2 MFMA tiles of 32 x 32.
// K is consumed in slices of 32 staged through LDS, with the next slice
// prefetched into registers while the current one feeds the MFMAs.
//   mode 0: v_mfma_f32_32x32x2_f32, LDS holds fp32 laid out [k][m].
//   mode 1: operands rounded to bf16 (nearest even) when staged,
//           v_mfma_f32_32x32x16_bf16 with fp32 accumulation, LDS laid out [m][k].
// Workgroup ids are remapped so that each XCD (ids are dealt round-robin to the
// 8 XCDs) walks a contiguous range of tiles and re-uses its operands in its L2.
#include "grass_device.h"

namespace grass {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int BM = 128, BN = 128, BK = 32;
constexpr int kGemmThreads = 256;
constexpr int kLdF32 = BM + 2;     // floats per k-row in mode 0 (see bank note below)
constexpr int kLdBf16 = BK + 8;    // bf16 per m-row in mode 1 (80 bytes)

struct GemmArgs {
    const float* A;   // M x K
    const float* B;   // N x K
    float* C;         // M x N
    uint64_t M, N, K, lda, ldb, ldc;
    uint32_t tiles_m, tiles_n;
    int accumulate;   // C += instead of C =
    uint64_t kt_per_split;     // split-K: workgroup (split, tile) contracts K slices [split*kps, (split+1)*kps)
    uint64_t split_stride_c;   //          into C + split*split_stride_c
};

__device__ __forceinline__ uint16_t f32_to_bf16_rne(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (uint16_t)((u >> 16) | 0x40u);   // NaN stays NaN
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

// Loads 4 consecutive k of one row with the widest access the alignment allows;
// out-of-range rows and k read as zero.
template <int V>
__device__ __forceinline__ float4 load4(const float* base, uint64_t ld, uint64_t row, uint64_t rows, uint64_t k0,
                                        uint64_t K) {
    float4 r = make_float4(0.f, 0.f, 0.f, 0.f);
    if (row >= rows) return r;
    const float* p = base + row * ld + k0;
    if (k0 + 4 <= K) {
        if constexpr (V == 4) {
            r = *reinterpret_cast<const float4*>(p);
        } else if constexpr (V == 2) {
            const float2 a = *reinterpret_cast<const float2*>(p);
            const float2 b = *reinterpret_cast<const float2*>(p + 2);
            r = make_float4(a.x, a.y, b.x, b.y);
        } else {
            r = make_float4(p[0], p[1], p[2], p[3]);
        }
    } else {
        if (k0 + 0 < K) r.x = p[0];
        if (k0 + 1 < K) r.y = p[1];
        if (k0 + 2 < K) r.z = p[2];
        if (k0 + 3 < K) r.w = p[3];
    }
    return r;
}

template <int MODE, int V>
__global__ void __launch_bounds__(kGemmThreads) __attribute__((amdgpu_waves_per_eu(3, 3))) gemm_nt_kernel(GemmArgs a) {
    extern __shared__ __align__(16) unsigned char smem[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;

    // XCD-aware tile order: consecutive logical tiles share the same B (train) tile.
    const uint32_t total = a.tiles_m * a.tiles_n;
    const uint32_t split = blockIdx.x / total;
    const uint32_t bid = blockIdx.x - split * total;
    a.C += split * a.split_stride_c;
    const uint32_t per_xcd = (total + 7) / 8;
    uint32_t logical = (bid % 8) * per_xcd + bid / 8;
    if (total % 8 != 0) logical = bid;              // ragged grids keep the plain order
    if (logical >= total) return;
    const uint32_t tn = logical / a.tiles_m, tm = logical % a.tiles_m;
    const uint64_t m0 = (uint64_t)tm * BM, n0 = (uint64_t)tn * BN;

    // staging map: 8 lanes cover the 32 k of one row (coalesced 128-byte rows)
    const int kq = tid & 7;            // which group of 4 k
    const int r0 = tid >> 3;           // row 0..31, +32 per step

    f32x16 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;

    float4 ra[4], rb[4];
    auto fetch = [&](uint64_t k0) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            ra[i] = load4<V>(a.A, a.lda, m0 + r0 + 32 * i, a.M, k0 + kq * 4, a.K);
            rb[i] = load4<V>(a.B, a.ldb, n0 + r0 + 32 * i, a.N, k0 + kq * 4, a.K);
        }
    };

    const uint64_t nkt_all = (a.K + BK - 1) / BK;
    const uint64_t kt_begin = (uint64_t)split * a.kt_per_split;
    const uint64_t nkt = kt_begin + a.kt_per_split < nkt_all ? kt_begin + a.kt_per_split : nkt_all;
    fetch(kt_begin * BK);
    for (uint64_t kt = kt_begin; kt < nkt; ++kt) {
        __syncthreads();    // everyone is done reading the previous slice
        if constexpr (MODE == 0) {
            float* As = reinterpret_cast<float*>(smem);            // [BK][kLdF32]
            float* Bs = As + BK * kLdF32;
            // bank of (k, m) = (k*kLdF32 + m) % 32; kLdF32 = 130 puts the 8 k-groups of a
            // wavefront 8 banks apart, so a store sees at most 2 lanes per bank.
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int row = r0 + 32 * i;
                As[(kq * 4 + 0) * kLdF32 + row] = ra[i].x; As[(kq * 4 + 1) * kLdF32 + row] = ra[i].y;
                As[(kq * 4 + 2) * kLdF32 + row] = ra[i].z; As[(kq * 4 + 3) * kLdF32 + row] = ra[i].w;
                Bs[(kq * 4 + 0) * kLdF32 + row] = rb[i].x; Bs[(kq * 4 + 1) * kLdF32 + row] = rb[i].y;
                Bs[(kq * 4 + 2) * kLdF32 + row] = rb[i].z; Bs[(kq * 4 + 3) * kLdF32 + row] = rb[i].w;
            }
        } else {
            uint16_t* As = reinterpret_cast<uint16_t*>(smem);      // [BM][kLdBf16]
            uint16_t* Bs = As + BM * kLdBf16;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int row = r0 + 32 * i;
                ushort4 pa, pb;
                pa.x = f32_to_bf16_rne(ra[i].x); pa.y = f32_to_bf16_rne(ra[i].y);
                pa.z = f32_to_bf16_rne(ra[i].z); pa.w = f32_to_bf16_rne(ra[i].w);
                pb.x = f32_to_bf16_rne(rb[i].x); pb.y = f32_to_bf16_rne(rb[i].y);
                pb.z = f32_to_bf16_rne(rb[i].z); pb.w = f32_to_bf16_rne(rb[i].w);
                *reinterpret_cast<ushort4*>(As + row * kLdBf16 + kq * 4) = pa;
                *reinterpret_cast<ushort4*>(Bs + row * kLdBf16 + kq * 4) = pb;
            }
        }
        __syncthreads();
        if (kt + 1 < nkt) fetch((kt + 1) * BK);

        if constexpr (MODE == 0) {
            const float* As = reinterpret_cast<const float*>(smem);
            const float* Bs = As + BK * kLdF32;
#pragma unroll
            for (int kk = 0; kk < BK; kk += 2) {
                const int krow = kk + (lane >> 5);
                float fa[2], fb[2];
#pragma unroll
                for (int i = 0; i < 2; ++i) fa[i] = As[krow * kLdF32 + wm * 64 + i * 32 + (lane & 31)];
#pragma unroll
                for (int j = 0; j < 2; ++j) fb[j] = Bs[krow * kLdF32 + wn * 64 + j * 32 + (lane & 31)];
#pragma unroll
                for (int i = 0; i < 2; ++i)
#pragma unroll
                    for (int j = 0; j < 2; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[i], fb[j], acc[i][j], 0, 0, 0);
            }
        } else {
            const uint16_t* As = reinterpret_cast<const uint16_t*>(smem);
            const uint16_t* Bs = As + BM * kLdBf16;
#pragma unroll
            for (int kk = 0; kk < BK; kk += 16) {
                bf16x8 fa[2], fb[2];
#pragma unroll
                for (int i = 0; i < 2; ++i)
                    fa[i] = *reinterpret_cast<const bf16x8*>(As + (wm * 64 + i * 32 + (lane & 31)) * kLdBf16 + kk +
                                                             (lane >> 5) * 8);
#pragma unroll
                for (int j = 0; j < 2; ++j)
                    fb[j] = *reinterpret_cast<const bf16x8*>(Bs + (wn * 64 + j * 32 + (lane & 31)) * kLdBf16 + kk +
                                                             (lane >> 5) * 8);
#pragma unroll
                for (int i = 0; i < 2; ++i)
#pragma unroll
                    for (int j = 0; j < 2; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
            }
        }
    }

    // accumulator element e of a lane: row 8*(e/4) + 4*(lane/32) + e%4, column lane%32
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const uint64_t col = n0 + wn * 64 + j * 32 + (lane & 31);
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const uint64_t row = m0 + wm * 64 + i * 32 + 8 * (e >> 2) + 4 * (lane >> 5) + (e & 3);
                if (row < a.M && col < a.N) {
                    float* c = a.C + row * a.ldc + col;
                    *c = a.accumulate ? *c + acc[i][j][e] : acc[i][j][e];
                }
            }
        }
}

static int vec_width(const float* p, uint64_t ld) {
    if (aligned(p, 16) && ld % 4 == 0) return 4;
    if (aligned(p, 8) && ld % 2 == 0) return 2;
    return 1;
}

// defined in gemm_bf16.hip: 256 x 256 tiles fed by direct-to-LDS loads
bool launch_gemm_dma(bool f32, const void* A, const void* B, float* C, uint64_t M, uint64_t N, uint64_t K, uint64_t lda,
                     uint64_t ldb, uint64_t ldc, int accumulate, hipStream_t st, hipError_t* err, uint32_t splits,
                     float* partials, int lower_only);
uint32_t gemm_dma_splits(uint64_t M, uint64_t N, uint64_t K, bool f32, uint32_t max_splits);
bool gemm_dma_eligible(bool f32, const void* A, const void* B, uint64_t K, uint64_t lda, uint64_t ldb);
hipError_t convert_to_bf16(const float* src, uint64_t rows, uint64_t cols, uint64_t cols_pad, uint64_t ld_src, uint16_t* dst,
                           uint64_t ld_dst, hipStream_t st);

// splits > 1 (fp32 mode only): K-range partial products go to `partials`, see launch_gemm_dma.
static hipError_t launch_gemm(const GemmArgs& a, int mode, hipStream_t st, uint32_t splits = 1,
                              float* partials = nullptr, int lower_only = 0) {
    if (mode == 0 && a.M >= 128 && a.N >= 128) {       // large fp32 problems: the direct-to-LDS pipeline
        hipError_t derr = hipSuccess;
        if (launch_gemm_dma(true, a.A, a.B, a.C, a.M, a.N, a.K, a.lda, a.ldb, a.ldc, a.accumulate, st, &derr, splits,
                            partials, lower_only))
            return derr;
    }
    GemmArgs g = a;
    g.tiles_m = (uint32_t)ceil_div(a.M, BM);
    g.tiles_n = (uint32_t)ceil_div(a.N, BN);
    const uint64_t nkt = ceil_div(a.K, BK);
    if (splits < 1 || !partials) splits = 1;
    if (splits > nkt) return hipErrorInvalidValue;
    g.kt_per_split = ceil_div(nkt, splits);
    if (ceil_div(nkt, g.kt_per_split) != splits) return hipErrorInvalidValue;      // every K range non-empty
    g.split_stride_c = 0;
    if (splits > 1) { g.C = partials; g.ldc = a.N; g.split_stride_c = a.M * a.N; }
    const uint64_t total = (uint64_t)g.tiles_m * g.tiles_n * splits;
    if (total == 0 || total > 0x7FFFFFFFull) return hipErrorInvalidValue;
    int v = vec_width(a.A, a.lda);
    const int vb = vec_width(a.B, a.ldb);
    if (vb < v) v = vb;
    const size_t lds = mode == 0 ? (size_t)2 * BK * kLdF32 * sizeof(float) : (size_t)2 * BM * kLdBf16 * sizeof(uint16_t);
    dim3 grid((uint32_t)total), block(kGemmThreads);
#define GRASS_GEMM(MODE, V) hipLaunchKernelGGL((gemm_nt_kernel<MODE, V>), grid, block, lds, st, g)
    if (mode == 0) {
        if (v == 4) GRASS_GEMM(0, 4); else if (v == 2) GRASS_GEMM(0, 2); else GRASS_GEMM(0, 1);
    } else {
        if (v == 4) GRASS_GEMM(1, 4); else if (v == 2) GRASS_GEMM(1, 2); else GRASS_GEMM(1, 1);
    }
#undef GRASS_GEMM
    return hipGetLastError();
}

// C (M x N) = or += A (M x K) B^T (N x K), fp32 MFMA; used by the FIM and the inverse-FIM-vector product.
// lower_only: A == B and the caller reads only the tiles on or below the diagonal (the others may be left unwritten).
// splits > 1: the partial product of K range s goes to partials + s*M*N (dense) instead of C; needs M, N >= 128,
// K a multiple of 16 with at least `splits` slices of 16, 16-byte aligned operands.
hipError_t gemm_nt_f32(const float* A, const float* B, float* C, uint64_t M, uint64_t N, uint64_t K, uint64_t lda,
                       uint64_t ldb, uint64_t ldc, int accumulate, int lower_only, hipStream_t st, uint32_t splits,
                       float* partials) {
    GemmArgs a;
    a.A = A; a.B = B; a.C = C;
    a.M = M; a.N = N; a.K = K; a.lda = lda; a.ldb = ldb; a.ldc = ldc;
    a.accumulate = accumulate;
    return launch_gemm(a, 0, st, splits, partials, lower_only);
}

// Number of K ranges gemm_nt_f32 should be given (with a partials buffer of that many M x N matrices) so that a product
// with few output tiles still fills the chip; 1 = no split.
uint32_t gemm_nt_f32_splits(const float* A, const float* B, uint64_t M, uint64_t N, uint64_t K, uint64_t lda, uint64_t ldb,
                            uint32_t max_splits) {
    if (M >= 128 && N >= 128 && gemm_dma_eligible(true, A, B, K, lda, ldb)) return gemm_dma_splits(M, N, K, true, max_splits);
    const uint64_t tiles = ceil_div(M, BM) * ceil_div(N, BN), slices = ceil_div(K, BK);
    if (tiles == 0 || tiles >= 2 * kNumCU || slices < 128) return 1;
    uint64_t s = ceil_div(2 * kNumCU, tiles);
    if (s > max_splits) s = max_splits;
    if (s > slices / 64) s = slices / 64;
    if (s < 2) return 1;
    return (uint32_t)ceil_div(slices, ceil_div(slices, s));
}

// P[a, b] for b in [p0, p0+pc): one Box-Muller normal per hash, scaled to variance 1/k.
// blockIdx.x: a run of 256 columns, blockIdx.y (+ stride): rows.
// BF16: the value is rounded to bf16 (nearest even) and columns pc..pc_pad are zero-filled (whole K slices for the
// bf16 GEMM); otherwise pc_pad == pc.
template <bool BF16>
__global__ void __launch_bounds__(256) gauss_matrix_kernel(uint64_t sub, uint64_t p, uint32_t k, uint64_t p0,
                                                           uint64_t pc, uint64_t pc_pad, void* Pv, uint64_t ldP,
                                                           float inv_sqrt_k) {
    const uint64_t col = (uint64_t)blockIdx.x * 256 + threadIdx.x;
    if (col >= pc_pad) return;
    for (uint32_t row = blockIdx.y; row < k; row += gridDim.y) {
        float v = 0.0f;
        if (col < pc) {
            const uint64_t h = sm(sub, (uint64_t)row * p + p0 + col);
            const float u1 = ((float)(uint32_t)(h >> 41) + 0.5f) * (1.0f / 8388608.0f);           // (0, 1), exact
            const float u2 = (float)(uint32_t)((h >> 16) & 0xFFFFFFu) * (1.0f / 16777216.0f);      // [0, 1)
            // hardware transcendentals: v_log_f32 is log2, v_cos_f32 takes its argument in revolutions (cos(2 pi u2))
            v = __builtin_amdgcn_sqrtf(-1.3862943611198906f * __builtin_amdgcn_logf(u1)) * __builtin_amdgcn_cosf(u2) * inv_sqrt_k;
        }
        if constexpr (BF16) static_cast<uint16_t*>(Pv)[(uint64_t)row * ldP + col] = f32_to_bf16_rne(v);
        else static_cast<float*>(Pv)[(uint64_t)row * ldP + col] = v;
    }
}

static void launch_gauss_matrix(uint64_t sub, uint64_t p, uint32_t k, uint64_t p0, uint64_t pc, uint64_t pc_pad, bool bf16,
                                void* P, uint64_t ldP, hipStream_t hs) {
    const uint32_t gx = (uint32_t)ceil_div(pc_pad, 256);
    uint32_t gy = k;                                   // about 16K workgroups keep every CU busy
    if ((uint64_t)gx * gy > 16384) gy = (uint32_t)(16384 / gx > 0 ? 16384 / gx : 1);
    if (gy > 65535) gy = 65535;
    const float scale = 1.0f / sqrtf((float)k);
    if (bf16)
        hipLaunchKernelGGL(gauss_matrix_kernel<true>, dim3(gx, gy), dim3(256), 0, hs, sub, p, k, p0, pc, pc_pad, P, ldP, scale);
    else
        hipLaunchKernelGGL(gauss_matrix_kernel<false>, dim3(gx, gy), dim3(256), 0, hs, sub, p, k, p0, pc, pc_pad, P, ldP, scale);
}

}  // namespace grass

using namespace grass;

// Workspace plan of grass_score: bf16 copies of both operands (mode 1) and K-range partial sums when the M x N
// output has too few tiles to fill the chip.
constexpr uint32_t kScoreMaxSplits = 32;      // K ranges of a score product with few output tiles (8 tiles still fill 256 CUs)
struct ScorePlan {
    uint64_t kp;               // K rounded up to whole 64-byte bf16 slices
    size_t off_test, off_train, off_part, total;
    bool may_split;
};
static size_t up256s(size_t x) { return (x + 255) / 256 * 256; }
static ScorePlan score_plan(uint64_t N, uint64_t M, uint64_t K, int mode) {
    ScorePlan P;
    P.kp = (K + 31) / 32 * 32;
    size_t o = 0;
    P.off_test = o;  if (mode == 1) o += up256s((size_t)M * P.kp * 2);
    P.off_train = o; if (mode == 1) o += up256s((size_t)N * P.kp * 2);
    P.may_split = ceil_div(M, 128) * ceil_div(N, 128) < 1024 && K >= 4096;
    P.off_part = o;  if (P.may_split) o += up256s((size_t)kScoreMaxSplits * M * N * 4);
    P.total = o;
    return P;
}

extern "C" grass_status grass_score_workspace_bytes(uint64_t N, uint64_t M, uint64_t K, int compute_mode,
                                                    size_t* host_bytes) {
    if (!host_bytes || K == 0 || (compute_mode != 0 && compute_mode != 1)) return GRASS_EINVAL;
    *host_bytes = (N == 0 || M == 0) ? 0 : score_plan(N, M, K, compute_mode).total;
    return GRASS_OK;
}

extern "C" grass_status grass_score(const float* train, const float* test, int compute_mode, uint64_t N, uint64_t M,
                                    uint64_t K, uint64_t ld_train, uint64_t ld_test, float* scores,
                                    uint64_t ld_scores, void* ws, size_t ws_bytes, grass_stream stream) {
    if (K == 0 || (compute_mode != 0 && compute_mode != 1)) return GRASS_EINVAL;
    if (N == 0 || M == 0) return GRASS_OK;
    if (!train || !test || !scores || ld_train < K || ld_test < K || ld_scores < N) return GRASS_EINVAL;
    hipStream_t hs = as_stream(stream);
    const ScorePlan P = score_plan(N, M, K, compute_mode);
    const bool have_ws = ws != nullptr && ws_bytes >= P.total && P.total > 0;
    if (ws != nullptr && P.total > 0 && (ws_bytes < P.total || !aligned(ws, 256))) return GRASS_EWORKSPACE;
    unsigned char* base = static_cast<unsigned char*>(ws);
    GemmArgs a;
    a.A = test; a.B = train; a.C = scores;
    a.M = M; a.N = N; a.K = K; a.lda = ld_test; a.ldb = ld_train; a.ldc = ld_scores;
    a.accumulate = 0;
    if (compute_mode == 1 && have_ws) {
        // round both operands once, then the bf16 direct-to-LDS kernel (zero-padded to whole K slices)
        uint16_t* te = reinterpret_cast<uint16_t*>(base + P.off_test);
        uint16_t* tr = reinterpret_cast<uint16_t*>(base + P.off_train);
        if (convert_to_bf16(test, M, K, P.kp, ld_test, te, P.kp, hs) != hipSuccess) return GRASS_EHIP;
        if (convert_to_bf16(train, N, K, P.kp, ld_train, tr, P.kp, hs) != hipSuccess) return GRASS_EHIP;
        uint32_t splits = P.may_split ? gemm_dma_splits(M, N, P.kp, false, kScoreMaxSplits) : 1;
        float* partials = reinterpret_cast<float*>(base + P.off_part);
        hipError_t derr = hipSuccess;
        if (launch_gemm_dma(false, te, tr, scores, M, N, P.kp, P.kp, P.kp, ld_scores, 0, hs, &derr, splits,
                            splits > 1 ? partials : nullptr, 0)) {
            if (derr != hipSuccess) return GRASS_EHIP;
            if (splits > 1)
                hipLaunchKernelGGL(reduce_partials_kernel, dim3((uint32_t)ceil_div(M * N, 256)), dim3(256), 0, hs, partials, M,
                                   (uint32_t)N, splits, 1.0f, scores, ld_scores);
            return launch_status();
        }
        // not reachable with the padded copies; fall through to the on-the-fly kernel
    }
    if (compute_mode == 0 && have_ws && P.may_split) {
        const uint32_t splits = gemm_nt_f32_splits(test, train, M, N, K, ld_test, ld_train, kScoreMaxSplits);
        if (splits > 1) {
            float* partials = reinterpret_cast<float*>(base + P.off_part);
            if (launch_gemm(a, 0, hs, splits, partials) != hipSuccess) return GRASS_EHIP;
            hipLaunchKernelGGL(reduce_partials_kernel, dim3((uint32_t)ceil_div(M * N, 256)), dim3(256), 0, hs, partials, M,
                               (uint32_t)N, splits, 1.0f, scores, ld_scores);
            return launch_status();
        }
    }
    return launch_gemm(a, compute_mode, hs) == hipSuccess ? GRASS_OK : GRASS_EHIP;
}

extern "C" grass_status grass_gauss_matrix(uint64_t seed, uint64_t stream_id, uint64_t p, uint32_t k, uint64_t p0,
                                           uint64_t pc, float* P, uint64_t ldP, grass_stream stream) {
    if (p == 0 || k == 0 || pc == 0 || p0 + pc > p || !P || ldP < pc) return GRASS_EINVAL;
    if (ceil_div(pc, 256) > 0x7FFFFFFFull) return GRASS_EUNSUPPORTED;
    launch_gauss_matrix(substream(seed, stream_id), p, k, p0, pc, pc, false, P, ldP, as_stream(stream));
    return launch_status();
}

// dst (rows x cols_pad, row distance ld_dst) = src (rows x cols), columns cols..cols_pad zero; rows dealt to blockIdx.y.
__global__ void __launch_bounds__(256) copy_pad_f32_kernel(const float* src, uint64_t ld_src, uint64_t rows, uint64_t cols,
                                                           uint64_t cols_pad, float* dst, uint64_t ld_dst) {
    const uint64_t c = (uint64_t)blockIdx.x * 256 + threadIdx.x;
    if (c >= cols_pad) return;
    for (uint64_t r = blockIdx.y; r < rows; r += gridDim.y)
        dst[r * ld_dst + c] = c < cols ? __builtin_nontemporal_load(src + r * ld_src + c) : 0.0f;
}

static uint64_t gauss_chunk(uint64_t p, uint64_t p_chunk) {
    uint64_t pc = p_chunk == 0 ? 8192 : p_chunk;
    pc = (pc + 31) / 32 * 32;              // whole 64-byte K slices of fp32 and of bf16
    return pc > p ? (p + 31) / 32 * 32 : pc;
}

// Workspace plan of grass_gauss_project.  mode 0: the fp32 chunk of P.  mode 1 (n, k >= 128): bf16 chunks of P and
// of g.  Both: K-range partial sums when the n x k output has too few tiles to fill the chip.
struct GaussPlan {
    uint64_t pc;
    uint32_t splits;           // K ranges of the first (largest) chunk's product; later chunks never use more
    bool bf16_path;
    size_t off_p, off_g, off_part, total;
};
static GaussPlan gauss_plan(uint64_t n, uint64_t p, uint32_t k, uint64_t p_chunk, int mode) {
    GaussPlan G;
    G.pc = gauss_chunk(p, p_chunk);
    const bool big = n >= 128 && k >= 128;
    G.bf16_path = mode == 1 && big;
    const uint64_t first = G.pc < p ? G.pc : p;
    G.splits = 1;
    if (big && (mode == 0 || G.bf16_path) && first % 32 == 0) G.splits = gemm_dma_splits(n, k, first, mode == 0, 8);
    size_t o = 0;
    G.off_p = o; o += up256s((size_t)k * G.pc * (G.bf16_path ? 2 : 4));
    // a chunk of g: rounded to bf16 (mode 1), or copied to 16-byte aligned rows when g's own rows are not (mode 0;
    // the query does not know the alignment, so the room is always there)
    G.off_g = o; if (G.bf16_path) o += up256s((size_t)n * G.pc * 2); else if (big && mode == 0) o += up256s((size_t)n * G.pc * 4);
    G.off_part = o; if (G.splits > 1) o += up256s((size_t)G.splits * n * k * 4);
    G.total = o;
    return G;
}

extern "C" grass_status grass_gauss_project_workspace_bytes(uint64_t n, uint64_t p, uint32_t k, uint64_t p_chunk,
                                                            size_t* host_bytes) {
    if (!host_bytes || p == 0 || k == 0) return GRASS_EINVAL;
    const size_t a = gauss_plan(n, p, k, p_chunk, 0).total, b = gauss_plan(n, p, k, p_chunk, 1).total;
    *host_bytes = a > b ? a : b;           // the mode is not an argument of the query: enough for either
    return GRASS_OK;
}

extern "C" grass_status grass_gauss_project(const float* g, uint64_t n, uint64_t p, uint64_t ldg, uint32_t k,
                                            uint64_t seed, uint64_t stream_id, uint64_t p_chunk, int compute_mode,
                                            float* out, uint64_t ldo, void* ws, size_t ws_bytes,
                                            grass_stream stream) {
    if (p == 0 || k == 0 || (compute_mode != 0 && compute_mode != 1)) return GRASS_EINVAL;
    if (n == 0) return GRASS_OK;
    if (!g || !out || ldg < p || ldo < k) return GRASS_EINVAL;
    GaussPlan G = gauss_plan(n, p, k, p_chunk, compute_mode);
    const uint64_t pc = G.pc;
    if (ceil_div(pc, 256) > 0x7FFFFFFFull) return GRASS_EUNSUPPORTED;
    if (!ws || ws_bytes < G.total || !aligned(ws, 256)) return GRASS_EWORKSPACE;
    // the fp32 direct-to-LDS kernel needs 16-byte aligned rows: chunks of a g that has none are copied to the workspace
    // first (2 x 4 bytes of traffic per element against 2k flops: nothing next to the product)
    const bool stage_g = compute_mode == 0 && n >= 128 && k >= 128 && (!aligned(g, 16) || ldg % 4 != 0);
    unsigned char* base = static_cast<unsigned char*>(ws);
    float* partials = G.splits > 1 ? reinterpret_cast<float*>(base + G.off_part) : nullptr;
    hipStream_t hs = as_stream(stream);
    const uint64_t sub = substream(seed, stream_id);
    for (uint64_t p0 = 0; p0 < p; p0 += pc) {
        const uint64_t cur = p0 + pc <= p ? pc : p - p0;
        const int accumulate = p0 != 0;
        if (G.bf16_path) {
            // P and g chunks rounded to bf16 once (zero-padded to whole K slices), bf16 matrix cores, fp32 accumulation
            const uint64_t cur_pad = (cur + 31) / 32 * 32;
            uint16_t* Pb = reinterpret_cast<uint16_t*>(base + G.off_p);
            uint16_t* gb = reinterpret_cast<uint16_t*>(base + G.off_g);
            launch_gauss_matrix(sub, p, k, p0, cur, cur_pad, true, Pb, pc, hs);
            if (convert_to_bf16(g + p0, n, cur, cur_pad, ldg, gb, pc, hs) != hipSuccess) return GRASS_EHIP;
            uint32_t s_cur = G.splits > 1 ? gemm_dma_splits(n, k, cur_pad, false, G.splits) : 1;
            if (s_cur > G.splits) s_cur = G.splits;
            float* C = G.splits > 1 ? partials : out;
            const uint64_t ldc = G.splits > 1 ? k : ldo;
            hipError_t derr = hipSuccess;
            if (!launch_gemm_dma(false, gb, Pb, C, n, k, cur_pad, pc, pc, ldc, accumulate, hs, &derr, s_cur,
                                 s_cur > 1 ? partials : nullptr, 0) || derr != hipSuccess)
                return GRASS_EHIP;
            continue;
        }
        float* P = reinterpret_cast<float*>(base + G.off_p);
        GemmArgs a;
        a.A = g + p0; a.B = P; a.C = out;
        a.M = n; a.N = k; a.K = cur; a.lda = ldg; a.ldb = pc; a.ldc = ldo;
        a.accumulate = accumulate;
        if (stage_g) {
            const uint64_t cur_pad = (cur + 15) / 16 * 16;         // zero-padded to whole K slices, like P
            float* gs = reinterpret_cast<float*>(base + G.off_g);
            hipLaunchKernelGGL(copy_pad_f32_kernel, dim3((uint32_t)ceil_div(cur_pad, 256), (uint32_t)(n < 65535 ? n : 65535)),
                               dim3(256), 0, hs, g + p0, ldg, n, cur, cur_pad, gs, pc);
            launch_gauss_matrix(sub, p, k, p0, cur, cur_pad, false, P, pc, hs);
            a.A = gs; a.lda = pc; a.K = cur_pad;
        } else {
            launch_gauss_matrix(sub, p, k, p0, cur, cur, false, P, pc, hs);
        }
        if (G.splits > 1) {
            uint32_t s_cur = a.K % 16 == 0 ? gemm_dma_splits(n, k, a.K, true, G.splits) : 1;
            if (s_cur > G.splits) s_cur = G.splits;
            if (s_cur == 1) {                              // short or ragged tail: a one-range product into partial 0
                a.C = partials; a.ldc = k;
                if (launch_gemm(a, 0, hs) != hipSuccess) return GRASS_EHIP;
            } else if (launch_gemm(a, 0, hs, s_cur, partials) != hipSuccess) {
                return GRASS_EHIP;
            }
        } else if (launch_gemm(a, compute_mode, hs) != hipSuccess) {
            return GRASS_EHIP;
        }
    }
    if (G.splits > 1) {
        const uint64_t total = n * (uint64_t)k;
        if (ceil_div(total, 256) > 0x7FFFFFFFull) return GRASS_EUNSUPPORTED;
        hipLaunchKernelGGL(reduce_partials_kernel, dim3((uint32_t)ceil_div(total, 256)), dim3(256), 0, hs, partials, n, k,
                           G.splits, 1.0f, out, ldo);
    }
    return launch_status();
}
