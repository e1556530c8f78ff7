// Cache stage after compression (Sec. 2.1 steps 2 and 3 on compressed gradients, Sec. 2.2 "projected FIM",
// damping of App. B):
//   grass_fim          F = (1/N) G^T G                      fp32 MFMA (transpose + NT GEMM, lower tiles only)
//   grass_fim_inverse  W = (F + lambda I)^{-1}              fp64: blocked Cholesky, recursive triangular inverse,
//                                                           W = L^{-T} L^{-1}; fp64 MFMA for every product
//   grass_ifvp         out = G W  (row i = W g_i)           fp32 MFMA NT GEMM (W is symmetric)
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

// ------------------------------------------------------------------------------------------------ FIM (fp32)
// F[a][b] = F[b][a] = scale * S[a][b] for a >= b: applies 1/N and mirrors the computed lower triangle.  S is F itself
// (splits == 0) or the sum, in ascending order, of `splits` dense k x k partial products.
__global__ void __launch_bounds__(256) fim_finish_kernel(float* F, uint64_t ldf, uint32_t k, float scale,
                                                        const float* partials, uint32_t splits) {
    // one 64 x 64 tile on or below the diagonal per workgroup; the mirrored tile is written from an LDS copy so that
    // both stores run along rows
    __shared__ float tile[64][65];
    if (blockIdx.x > blockIdx.y) return;
    const uint32_t a0 = blockIdx.y * 64, b0 = blockIdx.x * 64;
    const uint32_t c = threadIdx.x & 63, r0 = threadIdx.x >> 6;
    // phase 1: a thread owns 4 adjacent columns of 4 rows (16-byte loads when the columns exist and are aligned)
    {
        const uint32_t c4 = (threadIdx.x & 15) * 4, rr = threadIdx.x >> 4;
        const bool vec = b0 + c4 + 4 <= k && k % 4 == 0 && ldf % 4 == 0 && ((uintptr_t)F & 15) == 0 &&
                         ((uintptr_t)partials & 15) == 0;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const uint32_t r = rr + 16 * i, a = a0 + r;
            if (a >= k) continue;
            float v[4] = {0.0f, 0.0f, 0.0f, 0.0f};
            if (vec) {
                if (splits == 0) {
                    const float4 q = *reinterpret_cast<const float4*>(F + (uint64_t)a * ldf + b0 + c4);
                    v[0] = q.x; v[1] = q.y; v[2] = q.z; v[3] = q.w;
                }
                for (uint32_t s = 0; s < splits; ++s) {
                    const float4 q = *reinterpret_cast<const float4*>(partials + ((uint64_t)s * k + a) * k + b0 + c4);
                    v[0] += q.x; v[1] += q.y; v[2] += q.z; v[3] += q.w;
                }
            } else {
                for (int e = 0; e < 4; ++e) {
                    const uint32_t bb = b0 + c4 + e;
                    if (bb >= k) continue;
                    if (splits == 0) v[e] = F[(uint64_t)a * ldf + bb];
                    for (uint32_t s = 0; s < splits; ++s) v[e] += partials[((uint64_t)s * k + a) * k + bb];
                }
            }
            const bool whole = vec && a >= b0 + c4 + 3;          // all four on or below the diagonal
            if (whole) {
                float4 q;
                q.x = v[0] * scale; q.y = v[1] * scale; q.z = v[2] * scale; q.w = v[3] * scale;
                *reinterpret_cast<float4*>(F + (uint64_t)a * ldf + b0 + c4) = q;
            }
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const uint32_t bb = b0 + c4 + e;
                if (bb >= k || a < bb) continue;                 // above the diagonal: not computed, not stored
                const float w = v[e] * scale;
                if (!whole) F[(uint64_t)a * ldf + bb] = w;
                tile[r][c4 + e] = w;
            }
        }
    }
    __syncthreads();
    // element (b0 + r, a0 + c) of the upper triangle = element (a0 + c, b0 + r) of the lower one
    for (uint32_t r = r0; r < 64; r += 4) {
        const uint32_t row = b0 + r, col = a0 + c;
        if (row < k && col < k && col > row) F[(uint64_t)row * ldf + col] = tile[c][r];
    }
}

// ------------------------------------------------------------------------------------- fp64 building blocks
constexpr int NB = 64;                        // block size of the factorisation
typedef double f64x4 __attribute__((ext_vector_type(4)));

// A64 (kp x kp, row distance ld): lower triangle of F + lambda I, identity on the padding rows; X64 = 0.
__global__ void __launch_bounds__(256) fim_load_kernel(const float* F, uint64_t ldf, uint32_t k, double lambda,
                                                      double* A64, double* X64, uint32_t kp, uint32_t ld) {
    const uint64_t t = (uint64_t)blockIdx.x * 256 + threadIdx.x;
    if (t >= (uint64_t)kp * kp) return;
    const uint32_t a = (uint32_t)(t / kp), b = (uint32_t)(t - (uint64_t)a * kp);
    double v = 0.0;
    if (a < k && b <= a) v = (double)F[(uint64_t)a * ldf + b] + (a == b ? lambda : 0.0);
    else if (a >= k && a == b) v = 1.0;
    A64[(uint64_t)a * ld + b] = v;
    X64[(uint64_t)a * ld + b] = 0.0;
}

// Value of lane `src` (a compile-time constant) of a double, as a wavefront-uniform scalar.
__device__ __forceinline__ double lane_bcast(double v, int src) {
    const int lo = __builtin_amdgcn_readlane(__double2loint(v), src);
    const int hi = __builtin_amdgcn_readlane(__double2hiint(v), src);
    return __hiloint2double(hi, lo);
}

// Cholesky factor of the NB x NB diagonal block j (lower, in place) and its inverse D = L_jj^{-1} into the
// same block of X64 (zeros above the diagonal).  A non-positive pivot records its 1-based index in *info
// (first one wins) and is replaced by 1 so that the run stays finite.
// Two wavefronts and one barrier (at the start): the column recurrence is a chain of dependent fp64 operations (32
// cycles each on this chip), so what matters is the length of that chain and the number of instructions a wavefront
// has to issue, not parallel width.
//   Wavefront 0 factorises.  Lane r keeps row r of the block in registers.  In step c every lane scales its entry of
//   column c and writes it to LDS; the entries l[q][c] that the trailing update a[r][q] -= l[r][c] l[q][c] needs come
//   back as broadcast reads of two doubles each (all lanes read the same address).  (Fetching them with two v_readlane
//   per value instead took 16,700 instructions, 8,500 of them v_readlane and 3,300 hazard nops, against 12,600.)
//   Wavefront 1 inverts, one column behind: lane t keeps column t of X = L^{-1}, x[q] = delta_qt - sum_{m<c} l[q][m]
//   X[m][t] after c steps; in step c it finishes X[c][t] = x[c] / l[c][c] and subtracts l[q][c] X[c][t] from the x[q]
//   below, with the same broadcast reads of column c.  It waits for column c on a counter in LDS that wavefront 0
//   advances after its writes of the column (LDS operations of one wavefront complete in order); wavefront 0 never
//   waits for anybody, so every wait ends.  Doing the inverse afterwards in the factorising wavefront (forward
//   substitution with the rows of L read back from LDS) took 39 us per block against 24 us for the two in step.
// The loop bodies must stay free of branches (every lane stores the same 1/pivot): with a conditional store per
// column the compiler sank the trailing updates of far columns across 30 to 40 basic blocks towards their use and
// spilled 2,200 registers to scratch.  The empty asm statements bound how far it may move LDS reads.
struct f64x2 { double x, y; };
// The two wavefronts' work, for threads 0..127 of a workgroup.  `tile` is the block to factorise (row distance
// tile_ld, global memory or LDS); its factor goes to Lout (row distance ld, global; may be null: nobody needs the
// diagonal blocks of L once their inverses exist) and the inverse to Xb (row distance ld, global).  *columns_done
// must be 0 and visible to both wavefronts (a barrier after it is set) on entry; no barrier inside.
__device__ __forceinline__ void potrf_two_wavefronts(double (*Lc)[NB], double* Ys, int* columns_done, const double* tile,
                                                     uint32_t tile_ld, double* Lout, double* Xb, uint32_t ld,
                                                     uint32_t j, int* info) {
    const int r = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    if (wave == 0) {
        double a[NB];
#pragma unroll
        for (int q = 0; q < NB; ++q) a[q] = tile[(uint64_t)r * tile_ld + q];
        int bad = 0;
#pragma unroll
        for (int c = 0; c < NB; ++c) {
            const double piv = lane_bcast(a[c], c);
            const bool ok = piv > 0.0;                                   // false for NaN too
            if (!ok && bad == 0) bad = c + 1;
            const double pv = ok ? piv : 1.0;
            double y = __builtin_amdgcn_rsq(pv);                         // pivot^(-1/2): estimate + two Newton steps
            y = fma(0.5 * y, fma(-pv * y, y, 1.0), y);
            y = fma(0.5 * y, fma(-pv * y, y, 1.0), y);
            Ys[c] = y;                                                   // every lane stores the same value: no branch
            const double lc = r == c ? pv * y : (r > c ? a[c] * y : 0.0);
            a[c] = lc;
            Lc[c][r] = lc;                                               // LDS operations of one wavefront stay in order
            __hip_atomic_store(columns_done, c + 1, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_WORKGROUP);
            if (c + 1 < NB) {
#pragma unroll
                for (int q0 = (c + 1) & ~1; q0 < NB; q0 += 2) {          // pairs (q0, q0 + 1), q0 even
                    const f64x2 l = *reinterpret_cast<const f64x2*>(&Lc[c][q0]);
                    if (q0 > c) a[q0] = fma(-lc, l.x, a[q0]);            // only rows r >= q are used later
                    a[q0 + 1] = fma(-lc, l.y, a[q0 + 1]);
                    if ((q0 & 14) == 14) asm volatile("" ::: "memory");   // at most 8 reads in flight (measured best)
                }
            }
            asm volatile("" ::: "memory");
        }
        if (r == 0 && bad != 0 && info) atomicCAS(info, 0, (int)(j * NB) + bad);
        if (Lout) {
#pragma unroll
            for (int q = 0; q < NB; ++q) Lout[(uint64_t)r * ld + q] = q <= r ? a[q] : 0.0;
        }
    } else if (wave == 1) {
        const uint32_t done_addr = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) int*)columns_done;   // LDS offset
        double x[NB];
#pragma unroll
        for (int q = 0; q < NB; ++q) x[q] = q == r ? 1.0 : 0.0;
#pragma unroll
        for (int c = 0; c < NB; ++c) {
            // wait until *columns_done > c.  The polling loop lives inside one asm statement: as a loop of the C++
            // source it would split every unrolled step into basic blocks (see above).  The value read stays inside
            // the statement and has arrived (lgkmcnt(0)) before the statement ends.
            {
                uint32_t seen;
                asm volatile("1:\n\t"
                             "ds_read_b32 %0, %1\n\t"
                             "s_waitcnt lgkmcnt(0)\n\t"
                             "v_cmp_gt_i32_e32 vcc, %2, %0\n\t"
                             "s_sleep 1\n\t"
                             "s_cbranch_vccnz 1b"
                             : "=&v"(seen)
                             : "v"(done_addr), "v"(c + 1)
                             : "vcc", "memory");
            }
            const double xc = x[c] * Ys[c];                              // X[c][t], final; zero for t > c
            Xb[(uint64_t)c * ld + r] = xc;
            if (c + 1 < NB) {
#pragma unroll
                for (int q0 = (c + 1) & ~1; q0 < NB; q0 += 2) {
                    const f64x2 l = *reinterpret_cast<const f64x2*>(&Lc[c][q0]);      // l[q0][c], l[q0 + 1][c]
                    if (q0 > c) x[q0] = fma(-l.x, xc, x[q0]);
                    x[q0 + 1] = fma(-l.y, xc, x[q0 + 1]);
                    if ((q0 & 14) == 14) asm volatile("" ::: "memory");
                }
            }
            asm volatile("" ::: "memory");
        }
    }
}

__global__ void __launch_bounds__(128) potrf_block_kernel(double* A64, double* X64, uint32_t ld, uint32_t j, int* info) {
    __shared__ __align__(16) double Lc[NB][NB];          // Lc[c][q] = L[q][c]: column c contiguous
    __shared__ __align__(16) double Ys[NB];              // 1 / L[c][c]
    __shared__ int columns_done;
    double* Ab = A64 + ((uint64_t)j * NB) * ld + (uint64_t)j * NB;
    double* Xb = X64 + ((uint64_t)j * NB) * ld + (uint64_t)j * NB;
    if (threadIdx.x == 0) columns_done = 0;
    __syncthreads();
    potrf_two_wavefronts(Lc, Ys, &columns_done, Ab, ld, nullptr, Xb, ld, j, info);
}

// C = alpha * A B + beta * C in fp64 with v_mfma_f64_16x16x4_f64.  A is M x K, B is K x N, C is M x N, each given
// by element strides (rs = row stride, cs = column stride), so transposed operands need no copy.  M, N, K are
// multiples of 64.  64 x 64 tile per workgroup, 4 wavefronts of 32 x 32 (2 x 2 MFMA blocks), K steps of 16 through
// LDS stored k-major with a row stride of 80 doubles (operand reads of one half-wavefront cover all 64 banks).
// Structure flags restrict the contraction range of a tile at (m0, n0) when an operand is triangular:
//   K_FROM_ROW: k >= m0      K_FROM_COL: k >= n0      K_TO_ROW: k < m0 + 64
// LOWER_TILES computes only tiles with m0 >= n0; MIRROR (fp32 output only) also writes the transposed element of
// off-diagonal tiles.  blockIdx.z is a batch index with strides bsA/bsB/bsC.
enum : int { K_FROM_ROW = 1, K_FROM_COL = 2, K_TO_ROW = 4, LOWER_TILES = 8, MIRROR = 16 };
struct DgemmArgs {
    const double* A; const double* B; double* C; float* Cf;
    int64_t rsA, csA, rsB, csB, rsC, csC;
    int64_t bsA, bsB, bsC;
    uint32_t M, N, K;
    double alpha, beta;
    int flags;
};
constexpr int kDLd = 80;

// Pipeline: the operands of the next four K steps travel in four rotating register sets (every tile's K range is a
// multiple of 64, so the loop runs in rounds of four steps with static set numbers and unconditional loads, and the
// compiler's wait counts leave the three newer sets in flight), two LDS stages, one barrier per step.  With one set
// and two barriers per step the kernel needed eight workgroups per CU to cover the load latency, and the tiles with
// the longest K range, each at an eighth of a CU's speed, set the time of the triangular products.
// Workgroups are numbered so that the tiles with the longest K range start first (the hardware hands out workgroups
// in launch order): by columns for K_FROM_COL, by rows from the bottom for K_TO_ROW, by rows from the top otherwise.
__global__ void __launch_bounds__(256) dgemm_kernel(DgemmArgs g) {
    __shared__ double As[2][16][kDLd];
    __shared__ double Bs[2][16][kDLd];
    uint32_t tm = blockIdx.y, tn = blockIdx.x;
    {
        const uint32_t t = blockIdx.y * gridDim.x + blockIdx.x;
        if (g.flags & K_FROM_COL) { tn = t / gridDim.y; tm = t % gridDim.y; }
        else if (g.flags & K_TO_ROW) { tm = gridDim.y - 1 - blockIdx.y; }
    }
    const uint32_t m0 = tm * 64, n0 = tn * 64;
    if ((g.flags & LOWER_TILES) && n0 > m0) return;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const double* A = g.A + (int64_t)blockIdx.z * g.bsA;
    const double* B = g.B + (int64_t)blockIdx.z * g.bsB;

    uint32_t kb = 0, ke = g.K;
    if ((g.flags & K_FROM_ROW) && m0 > kb) kb = m0;
    if ((g.flags & K_FROM_COL) && n0 > kb) kb = n0;
    if ((g.flags & K_TO_ROW) && m0 + 64 < ke) ke = m0 + 64;

    // staging map: the contiguous direction of each operand goes to adjacent lanes, 4 doubles per thread
    const bool a_k_contig = g.csA == 1, b_k_contig = g.rsB == 1;
    int ai, ak, bi, bk;                       // first (i, k) element of this thread, 4 elements along the contiguous dimension
    if (a_k_contig) { ai = tid >> 2; ak = (tid & 3) * 4; } else { ak = tid >> 4; ai = (tid & 15) * 4; }
    if (b_k_contig) { bi = tid >> 2; bk = (tid & 3) * 4; } else { bk = tid >> 4; bi = (tid & 15) * 4; }
    // a thread's 4 elements are adjacent in memory (the host checks that each operand has a unit stride and 32-byte
    // aligned rows): one 32-byte load instead of four 8-byte ones, whole 128-byte lines per wavefront instruction
    const double* ap = A + (int64_t)(m0 + ai) * g.rsA + (int64_t)ak * g.csA;
    const double* bp = B + (int64_t)bk * g.rsB + (int64_t)(n0 + bi) * g.csB;

    f64x4 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) acc[i][j] = f64x4{0.0, 0.0, 0.0, 0.0};

    if (kb < ke) {                                              // uniform
        const uint32_t klast = ke - 16;
        f64x4 ra[4], rb[4];
        auto fetch = [&](int set, uint32_t k0) {               // steps past the end re-read the last one (never used)
            const uint32_t kq = k0 < klast ? k0 : klast;
            ra[set] = *reinterpret_cast<const f64x4*>(ap + (int64_t)kq * g.csA);
            rb[set] = *reinterpret_cast<const f64x4*>(bp + (int64_t)kq * g.rsB);
        };
        auto stash = [&](int set, int stage) {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                if (a_k_contig) As[stage][ak + q][ai] = ra[set][q]; else As[stage][ak][ai + q] = ra[set][q];
                if (b_k_contig) Bs[stage][bk + q][bi] = rb[set][q]; else Bs[stage][bk][bi + q] = rb[set][q];
            }
        };
#pragma unroll
        for (int u = 0; u < 4; ++u) fetch(u, kb + 16 * u);
        stash(0, 0);
        __syncthreads();
        for (uint32_t k0 = kb; k0 < ke; k0 += 64) {            // four steps per round; step u computes out of stage u & 1
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                fetch(u, k0 + 16 * (u + 4));                   // set u went to LDS one step ago
#pragma unroll
                for (int kk = 0; kk < 16; kk += 4) {
                    const int kr = kk + (lane >> 4);
                    double fa[2], fb[2];
#pragma unroll
                    for (int i = 0; i < 2; ++i) fa[i] = As[u & 1][kr][wm * 32 + i * 16 + (lane & 15)];
#pragma unroll
                    for (int j = 0; j < 2; ++j) fb[j] = Bs[u & 1][kr][wn * 32 + j * 16 + (lane & 15)];
#pragma unroll
                    for (int i = 0; i < 2; ++i)
#pragma unroll
                        for (int j = 0; j < 2; ++j)
                            acc[i][j] = __builtin_amdgcn_mfma_f64_16x16x4f64(fa[i], fb[j], acc[i][j], 0, 0, 0);
                }
                stash((u + 1) & 3, (u + 1) & 1);               // the next step's operands (past the end: unused)
                __syncthreads();                               // that stage is complete; everybody is done with this one
            }
        }
    }

    // accumulator element e of a lane: row 4*e + lane/16, column lane%16 of the 16 x 16 block
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const uint32_t row = m0 + wm * 32 + i * 16 + 4 * e + (lane >> 4);
                const uint32_t col = n0 + wn * 32 + j * 16 + (lane & 15);
                double v = g.alpha * acc[i][j][e];
                if (g.Cf) {
                    float* c = g.Cf + (int64_t)blockIdx.z * g.bsC;
                    c[(int64_t)row * g.rsC + (int64_t)col * g.csC] = (float)v;
                    if ((g.flags & MIRROR) && m0 != n0) c[(int64_t)col * g.rsC + (int64_t)row * g.csC] = (float)v;
                } else {
                    double* c = g.C + (int64_t)blockIdx.z * g.bsC + (int64_t)row * g.rsC + (int64_t)col * g.csC;
                    if (g.beta != 0.0) v += g.beta * *c;
                    *c = v;
                }
            }
}

// The product for K = 64 exactly (the panel scaling and the rank-64 updates inside an outer block of the
// factorisation): such a launch is a few tiles deep and its time is memory latency, so a tile asks for everything it
// needs at once - all four K steps of both operands and, for beta != 0, its tile of C - and then runs the steps out of
// registers.  beta != 0 requires alpha = -1 or 1 (the accumulators start from C * beta / alpha, exact for those).
__global__ void __launch_bounds__(256) dgemm_k64_kernel(DgemmArgs g) {
    __shared__ double As[16][kDLd];
    __shared__ double Bs[16][kDLd];
    const uint32_t m0 = blockIdx.y * 64, n0 = blockIdx.x * 64;
    if ((g.flags & LOWER_TILES) && n0 > m0) return;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const double* A = g.A + (int64_t)blockIdx.z * g.bsA;
    const double* B = g.B + (int64_t)blockIdx.z * g.bsB;
    double* C = g.C + (int64_t)blockIdx.z * g.bsC;
    const bool a_k_contig = g.csA == 1, b_k_contig = g.rsB == 1;
    int ai, ak, bi, bk;
    if (a_k_contig) { ai = tid >> 2; ak = (tid & 3) * 4; } else { ak = tid >> 4; ai = (tid & 15) * 4; }
    if (b_k_contig) { bi = tid >> 2; bk = (tid & 3) * 4; } else { bk = tid >> 4; bi = (tid & 15) * 4; }
    const double* ap = A + (int64_t)(m0 + ai) * g.rsA + (int64_t)ak * g.csA;
    const double* bp = B + (int64_t)bk * g.rsB + (int64_t)(n0 + bi) * g.csB;
    f64x4 ra[4], rb[4];
#pragma unroll
    for (int s = 0; s < 4; ++s) {
        ra[s] = *reinterpret_cast<const f64x4*>(ap + (int64_t)(16 * s) * g.csA);
        rb[s] = *reinterpret_cast<const f64x4*>(bp + (int64_t)(16 * s) * g.rsB);
    }
    f64x4 acc[2][2];
    const double c_scale = g.beta / g.alpha;
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const uint32_t row = m0 + wm * 32 + i * 16 + 4 * e + (lane >> 4);
                const uint32_t col = n0 + wn * 32 + j * 16 + (lane & 15);
                acc[i][j][e] = g.beta != 0.0 ? c_scale * C[(int64_t)row * g.rsC + (int64_t)col * g.csC] : 0.0;
            }
#pragma unroll
    for (int s = 0; s < 4; ++s) {
        if (s) __syncthreads();                            // previous step's reads are done
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            if (a_k_contig) As[ak + q][ai] = ra[s][q]; else As[ak][ai + q] = ra[s][q];
            if (b_k_contig) Bs[bk + q][bi] = rb[s][q]; else Bs[bk][bi + q] = rb[s][q];
        }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < 16; kk += 4) {
            const int kr = kk + (lane >> 4);
            double fa[2], fb[2];
#pragma unroll
            for (int i = 0; i < 2; ++i) fa[i] = As[kr][wm * 32 + i * 16 + (lane & 15)];
#pragma unroll
            for (int j = 0; j < 2; ++j) fb[j] = Bs[kr][wn * 32 + j * 16 + (lane & 15)];
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f64_16x16x4f64(fa[i], fb[j], acc[i][j], 0, 0, 0);
        }
    }
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const uint32_t row = m0 + wm * 32 + i * 16 + 4 * e + (lane >> 4);
                const uint32_t col = n0 + wn * 32 + j * 16 + (lane & 15);
                C[(int64_t)row * g.rsC + (int64_t)col * g.csC] = g.alpha * acc[i][j][e];
            }
}

// One step of the factorisation inside an outer block, fused into one launch because every dependent launch costs
// about 6 us here whatever it computes: for the factorised diagonal block j (inverse D_j in X64) workgroup (m, n), n <= m,
// of the grid (inner column blocks, row blocks below j)
//   1. scales its two row blocks of the panel itself, P_m = A[m][j] D_j^T and P_n = A[n][j] D_j^T (the unscaled panel in
//      A64 is only read in this launch; the workgroups of column 0 write P_m to the same block position of X64, where
//      the lower blocks of L live from here on),
//   2. updates its tile, A[m][n] -= P_m P_n^T,
//   3. and workgroup (0, 0), whose tile is the next diagonal block, goes on to factorise and invert it
//      (potrf_two_wavefronts out of LDS), so the next step can start right away.
// Everything a tile needs (two panel blocks, D_j, its tile of A) is requested at the start.  All blocks are 64 x 64.
constexpr int kStepBuf = 64 * kDLd;                    // doubles per LDS operand buffer ([k][row], 64 k)
constexpr size_t kStepLdsBytes = (size_t)(3 * kStepBuf + NB) * sizeof(double) + 16;

__global__ void __launch_bounds__(256) chol_step_kernel(double* A64, double* X64, uint32_t ld, uint32_t j, int* info) {
    extern __shared__ __align__(16) double step_lds[];
    const uint32_t m = blockIdx.y, n = blockIdx.x;
    if (n > m) return;
    double* buf0 = step_lds;
    double* buf1 = step_lds + kStepBuf;
    double* buf2 = step_lds + 2 * kStepBuf;
    double* Ys = step_lds + 3 * kStepBuf;
    int* columns_done = reinterpret_cast<int*>(Ys + NB);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const uint64_t j0 = (uint64_t)j * NB, j1 = j0 + NB;
    const double* Am = A64 + (j1 + (uint64_t)m * NB) * ld + j0;
    const double* An = A64 + (j1 + (uint64_t)n * NB) * ld + j0;
    const double* Dj = X64 + j0 * ld + j0;
    double* Ct = A64 + (j1 + (uint64_t)m * NB) * ld + j1 + (uint64_t)n * NB;
    const bool square = m == n;                        // uniform: P_n is P_m

    // row-major 64 x 64 blocks: thread -> row tid/4, columns (tid%4)*4 + 16 s .. + 3
    const int srow = tid >> 2, scol = (tid & 3) * 4;
    f64x4 ra[4], rn[4], rd[4];
#pragma unroll
    for (int s4 = 0; s4 < 4; ++s4) {
        ra[s4] = *reinterpret_cast<const f64x4*>(Am + (uint64_t)srow * ld + scol + 16 * s4);
        rd[s4] = *reinterpret_cast<const f64x4*>(Dj + (uint64_t)srow * ld + scol + 16 * s4);
        rn[s4] = *reinterpret_cast<const f64x4*>(An + (uint64_t)srow * ld + scol + 16 * s4);
    }
    // accumulator element e of block (bi, bj): row wm*32 + bi*16 + 4e + lane/16, column wn*32 + bj*16 + lane%16
    f64x4 accC[2][2];
#pragma unroll
    for (int bi = 0; bi < 2; ++bi)
#pragma unroll
        for (int bj = 0; bj < 2; ++bj)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int row = wm * 32 + bi * 16 + 4 * e + (lane >> 4), col = wn * 32 + bj * 16 + (lane & 15);
                accC[bi][bj][e] = -Ct[(uint64_t)row * ld + col];       // result = -(-C + P_m P_n^T)
            }
#pragma unroll
    for (int s4 = 0; s4 < 4; ++s4)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int k = scol + 16 * s4 + q;
            buf0[k * kDLd + srow] = ra[s4][q];                          // [k][i]  = A[m][i][k]
            buf1[k * kDLd + srow] = rn[s4][q];
            buf2[k * kDLd + srow] = rd[s4][q];                          // [k][n'] = D[n'][k]
        }
    __syncthreads();
    auto product = [&](const double* Aop, const double* Bop, f64x4 (&acc)[2][2]) {      // acc += Aop^T-layout x Bop, K = 64
#pragma unroll
        for (int kk = 0; kk < NB; kk += 4) {
            const int kr = kk + (lane >> 4);
            double fa[2], fb[2];
#pragma unroll
            for (int bi = 0; bi < 2; ++bi) fa[bi] = Aop[kr * kDLd + wm * 32 + bi * 16 + (lane & 15)];
#pragma unroll
            for (int bj = 0; bj < 2; ++bj) fb[bj] = Bop[kr * kDLd + wn * 32 + bj * 16 + (lane & 15)];
#pragma unroll
            for (int bi = 0; bi < 2; ++bi)
#pragma unroll
                for (int bj = 0; bj < 2; ++bj)
                    acc[bi][bj] = __builtin_amdgcn_mfma_f64_16x16x4f64(fa[bi], fb[bj], acc[bi][bj], 0, 0, 0);
        }
    };
    f64x4 accP[2][2], accQ[2][2];
#pragma unroll
    for (int bi = 0; bi < 2; ++bi)
#pragma unroll
        for (int bj = 0; bj < 2; ++bj) { accP[bi][bj] = f64x4{0.0, 0.0, 0.0, 0.0}; accQ[bi][bj] = f64x4{0.0, 0.0, 0.0, 0.0}; }
    product(buf0, buf2, accP);                                           // P_m = A_m D^T
    if (!square) product(buf1, buf2, accQ);                              // P_n = A_n D^T
    __syncthreads();                                                     // everybody is done reading the operands
    double* Pout = X64 + (j1 + (uint64_t)m * NB) * ld + j0;
#pragma unroll
    for (int bi = 0; bi < 2; ++bi)
#pragma unroll
        for (int bj = 0; bj < 2; ++bj)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int row = wm * 32 + bi * 16 + 4 * e + (lane >> 4), col = wn * 32 + bj * 16 + (lane & 15);
                buf0[col * kDLd + row] = accP[bi][bj][e];                // [k][i] = P_m[i][k]
                if (!square) buf1[col * kDLd + row] = accQ[bi][bj][e];   // [k][n] = P_n[n][k]
                if (n == 0) Pout[(uint64_t)row * ld + col] = accP[bi][bj][e];
            }
    __syncthreads();
    product(buf0, square ? buf0 : buf1, accC);
    const bool next_diagonal = m == 0;                                   // (0, 0): uniform
#pragma unroll
    for (int bi = 0; bi < 2; ++bi)
#pragma unroll
        for (int bj = 0; bj < 2; ++bj)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int row = wm * 32 + bi * 16 + 4 * e + (lane >> 4), col = wn * 32 + bj * 16 + (lane & 15);
                const double v = -accC[bi][bj][e];
                Ct[(uint64_t)row * ld + col] = v;
                if (next_diagonal) buf2[row * kDLd + col] = v;           // row-major copy for the factorisation
            }
    if (!next_diagonal) return;
    if (tid == 0) *columns_done = 0;
    __syncthreads();                                                     // the tile copy and the counter are visible; buf0 is free
    if (tid < 128)
        potrf_two_wavefronts(reinterpret_cast<double (*)[NB]>(buf0), Ys, columns_done, buf2, kDLd, nullptr,
                             X64 + j1 * ld + j1, ld, j + 1, info);
}

// W[a][b] = (float) S[max(a,b)][min(a,b)] for the leading k x k part of a matrix (row distance ld) whose lower triangle is valid.
__global__ void __launch_bounds__(256) fim_store_kernel(const double* S, uint32_t ld, uint32_t k, float* W, uint64_t ldw) {
    const uint64_t t = (uint64_t)blockIdx.x * 256 + threadIdx.x;
    if (t >= (uint64_t)k * k) return;
    const uint32_t a = (uint32_t)(t / k), b = (uint32_t)(t - (uint64_t)a * k);
    const uint32_t hi = a > b ? a : b, lo = a > b ? b : a;
    W[(uint64_t)a * ldw + b] = (float)S[(uint64_t)hi * ld + lo];
}

__global__ void fill_i32_kernel(int* p, int count, int value) {
    if ((int)threadIdx.x < count) p[threadIdx.x] = value;
}

static hipError_t dgemm(const DgemmArgs& g, uint32_t batch, hipStream_t st) {
    if (g.M == 0 || g.N == 0 || batch == 0) return hipSuccess;
    if (g.M % 64 || g.N % 64 || g.K % 64) return hipErrorInvalidValue;
    // the kernels load 4 adjacent doubles at once: one unit stride per operand, the other stride and the base keep
    // 32-byte alignment
    const bool a_ok = (g.csA == 1 && g.rsA % 4 == 0) || (g.rsA == 1 && g.csA % 4 == 0);
    const bool b_ok = (g.rsB == 1 && g.csB % 4 == 0) || (g.csB == 1 && g.rsB % 4 == 0);
    if (!a_ok || !b_ok || !aligned(g.A, 32) || !aligned(g.B, 32) || g.bsA % 4 || g.bsB % 4) return hipErrorInvalidValue;
    if (g.K == 64 && !g.Cf && (g.flags & ~LOWER_TILES) == 0 && (g.beta == 0.0 || g.alpha == 1.0 || g.alpha == -1.0)) {
        hipLaunchKernelGGL(dgemm_k64_kernel, dim3(g.N / 64, g.M / 64, batch), dim3(256), 0, st, g);
        return hipGetLastError();
    }
    hipLaunchKernelGGL(dgemm_kernel, dim3(g.N / 64, g.M / 64, batch), dim3(256), 0, st, g);
    return hipGetLastError();
}

static uint32_t padded(uint32_t k) { return (k + NB - 1) / NB * NB; }
// Row distance of the fp64 work matrices: 16 doubles (one 128-byte line) more than the padded size.  With a power-of-two
// row distance (k = 4,096: 32 KB) the rows of an operand tile all fall on the same memory channels.
static uint32_t row_distance(uint32_t kp) { return kp + 16; }

}  // namespace grass

using namespace grass;

// --------------------------------------------------------------------------------------------------- C ABI
// rows of G per transposed chunk: long enough that each K range of a chunk product amortises its pipeline fill
static uint64_t fim_chunk_rows(uint64_t N) { return N < 16384 ? (N + 15) / 16 * 16 : 16384; }

// K ranges of the product.  The lower-triangle tiles of a 256 x 256 tiling are few (136 for k = 4,096 on 256 CUs)
// and all workgroups of a launch take equally long, so the launch runs in rounds of 256 workgroups: the number of
// ranges (at most 16, each at least 16 groups of 32 rows long) is the one that leaves the last round fullest, with a
// small penalty per range for its k x k partial sum (k = 4,096: 15 ranges = 2,040 workgroups = 7.97 rounds, where 8
// ranges = 4.25 rounds idle a quarter of the chip for a fifth of the time).
static uint32_t fim_splits(uint64_t N, uint32_t k) {
    if (k < 128) return 1;
    const uint64_t t = ((uint64_t)k + 255) / 256, lower = t * (t + 1) / 2;
    const uint64_t groups = ceil_div(N, 32);
    uint32_t best = 1;
    double best_score = -1.0;
    for (uint32_t s = 1; s <= 16; ++s) {
        if (s > 1 && groups < (uint64_t)s * 16) break;
        const uint64_t wg = lower * s;
        const double fill = (double)wg / (double)(ceil_div(wg, kNumCU) * kNumCU);
        const double score = fill - 0.003 * s;
        if (score > best_score) { best_score = score; best = s; }
    }
    return best;
}

static size_t fim_gt_bytes(uint64_t N, uint32_t k) { return ((size_t)k * fim_chunk_rows(N) * sizeof(float) + 255) / 256 * 256; }

extern "C" grass_status grass_fim_workspace_bytes(uint64_t N, uint32_t k, size_t* host_bytes) {
    if (!host_bytes || k == 0) return GRASS_EINVAL;
    if (N == 0) N = 1;
    const uint32_t splits = fim_splits(N, k);
    *host_bytes = fim_gt_bytes(N, k) + (splits > 1 ? (size_t)splits * k * k * sizeof(float) : 0);
    return GRASS_OK;
}

extern "C" grass_status grass_fim(const float* G, uint64_t N, uint32_t k, uint64_t ldg, float* F, uint64_t ldf, void* ws,
                                  size_t ws_bytes, grass_stream stream) {
    if (k == 0 || N == 0) return GRASS_EINVAL;
    if (!G || !F || ldg < k || ldf < k) return GRASS_EINVAL;
    const uint64_t rows = fim_chunk_rows(N);
    const uint32_t splits = fim_splits(N, k);
    const size_t need = fim_gt_bytes(N, k) + (splits > 1 ? (size_t)splits * k * k * sizeof(float) : 0);
    if (!ws || ws_bytes < need || !aligned(ws, 256)) return GRASS_EWORKSPACE;
    float* Gt = static_cast<float*>(ws);
    float* partials = splits > 1 ? reinterpret_cast<float*>(static_cast<unsigned char*>(ws) + fim_gt_bytes(N, k)) : nullptr;
    hipStream_t hs = as_stream(stream);
    // G^T G contracts over the rows of G: with 16-byte aligned rows the GEMM takes G itself as both (K-major)
    // operands in one launch, the N rows interleaved between the K ranges; otherwise chunks of G are transposed
    // into the workspace first.
    if (k >= 128 && k % 4 == 0 && ldg % 4 == 0 && aligned(G, 16)) {
        uint32_t s_cur = splits;
        const uint64_t groups = ceil_div(N, 32);
        if (s_cur > 1 && groups < (uint64_t)s_cur * 16) s_cur = (uint32_t)(groups / 16);       // short inputs: fewer ranges
        if (s_cur < 2) s_cur = 1;
        hipError_t derr = hipSuccess;
        const bool taken = s_cur > 1
            ? launch_gemm_dma_kmajor(true, G, G, nullptr, k, k, N, ldg, ldg, k, 0, hs, &derr, s_cur, partials, 1, 0, 0)
            : launch_gemm_dma_kmajor(true, G, G, F, k, k, N, ldg, ldg, ldf, 0, hs, &derr, 1, nullptr, 1, 0, 0);
        if (taken) {
            if (derr != hipSuccess) return GRASS_EHIP;
            hipLaunchKernelGGL(fim_finish_kernel, dim3((k + 63) / 64, (k + 63) / 64), dim3(256), 0, hs, F, ldf, k,
                               (float)(1.0 / (double)N), partials, s_cur > 1 ? s_cur : 0);
            return launch_status();
        }
    }
    uint32_t ranges_used = 0;                 // partial products the first chunk initialises; later chunks use no more
    for (uint64_t r0 = 0; r0 < N; r0 += rows) {
        const uint32_t rc = (uint32_t)(r0 + rows <= N ? rows : N - r0);
        const uint32_t rc_pad = (rc + 15) / 16 * 16;                 // the GEMM contracts over whole 64-byte slices
        hipLaunchKernelGGL(transpose_rows_kernel, dim3((k + 63) / 64, (rc_pad + 63) / 64), dim3(256), 0, hs, G, ldg, r0, rc,
                           rc_pad, k, Gt, rows);
        hipError_t e;
        if (splits > 1) {
            // a short chunk uses fewer ranges: the first chunk (accumulate = 0) initialises the ones it uses, a
            // shorter last chunk adds to a subset of them, and only those are summed at the end (a first chunk that
            // is itself short - few rows in all - must not leave the sum reading partial products nobody wrote)
            uint32_t s_cur = splits;
            if ((uint64_t)rc_pad / 16 < (uint64_t)s_cur * 32) s_cur = rc_pad / 16 / 32;
            if (r0 == 0) ranges_used = s_cur >= 2 ? s_cur : 1;
            if (s_cur >= 2)
                e = gemm_nt_f32(Gt, Gt, nullptr, k, k, rc_pad, rows, rows, k, r0 != 0, 1, hs, s_cur, partials);
            else
                e = gemm_nt_f32(Gt, Gt, partials, k, k, rc_pad, rows, rows, k, r0 != 0, 1, hs, 1, nullptr);
        } else {
            e = gemm_nt_f32(Gt, Gt, F, k, k, rc_pad, rows, rows, ldf, r0 != 0, 1, hs, 1, nullptr);
        }
        if (e != hipSuccess) return GRASS_EHIP;
    }
    hipLaunchKernelGGL(fim_finish_kernel, dim3((k + 63) / 64, (k + 63) / 64), dim3(256), 0, hs, F, ldf, k,
                       (float)(1.0 / (double)N), partials, splits > 1 ? ranges_used : 0);
    return launch_status();
}

extern "C" grass_status grass_fim_inverse_workspace_bytes(uint32_t k, size_t* host_bytes) {
    if (!host_bytes || k == 0) return GRASS_EINVAL;
    const size_t kp = padded(k);
    *host_bytes = 2 * kp * row_distance((uint32_t)kp) * sizeof(double);
    return GRASS_OK;
}

extern "C" grass_status grass_fim_inverse(const float* F, uint32_t k, uint64_t ldf, double lambda, float* W, uint64_t ldw,
                                          int32_t* info, void* ws, size_t ws_bytes, grass_stream stream) {
    if (k == 0 || !(lambda >= 0.0)) return GRASS_EINVAL;
    if (!F || !W || ldf < k || ldw < k) return GRASS_EINVAL;
    if (k > 32768) return GRASS_EUNSUPPORTED;
    const uint32_t kp = padded(k), nblk = kp / NB;
    const int64_t ld = row_distance(kp);
    const size_t mat = (size_t)kp * ld * sizeof(double);
    if (!ws || ws_bytes < 2 * mat || !aligned(ws, 256)) return GRASS_EWORKSPACE;
    double* A64 = static_cast<double*>(ws);
    double* X64 = A64 + (size_t)kp * ld;
    hipStream_t hs = as_stream(stream);

    if (info) hipLaunchKernelGGL(fill_i32_kernel, dim3(1), dim3(64), 0, hs, info, 1, 0);
    hipLaunchKernelGGL(fim_load_kernel, dim3((uint32_t)ceil_div((uint64_t)kp * kp, 256)), dim3(256), 0, hs, F, ldf, k, lambda,
                       A64, X64, kp, (uint32_t)ld);

    // Blocked Cholesky, A = L L^T.  Two levels: inside an outer block of kOuter diagonal blocks (512 columns) every
    // factorised 64-column panel updates the remaining columns of the outer block only (right-looking, K = 64, one
    // fused launch per step, see chol_step_kernel); the rest of the matrix receives the whole outer block at once
    // (K = 512).  A rank-64 update of the full trailing matrix moves 16 bytes of C per 128 flops and was bound by that
    // traffic (58 us for the first one, 1.8 ms over the factorisation).  The inverses of the diagonal blocks and the
    // scaled panels (the lower blocks of L) go to X64; A64 keeps the matrix being updated.  Wider outer blocks make the
    // steps longer than the factorisation of the next diagonal block that hides behind them (16: no faster).
    constexpr uint32_t kOuter = 8;
    static LdsOptIn step_opt_in;
    if (allow_large_lds(step_opt_in, reinterpret_cast<const void*>(chol_step_kernel)) != hipSuccess) return GRASS_EHIP;
    bool factorised = false;                               // block j already factorised by the step before it
    for (uint32_t j = 0; j < nblk; ++j) {
        if (!factorised)
            hipLaunchKernelGGL(potrf_block_kernel, dim3(1), dim3(128), 0, hs, A64, X64, (uint32_t)ld, j, info);
        factorised = false;
        const uint32_t below = kp - (j + 1) * NB;
        if (below == 0) break;
        const uint32_t outer_end = (j / kOuter + 1) * kOuter < nblk ? (j / kOuter + 1) * kOuter : nblk;   // first block after this outer block
        const uint32_t inner_blocks = outer_end - (j + 1);
        if (inner_blocks > 0) {
            // panel scaling, update of the remaining columns of the outer block, factorisation of block j + 1
            hipLaunchKernelGGL(chol_step_kernel, dim3(inner_blocks, below / NB), dim3(256), kStepLdsBytes, hs, A64, X64,
                               (uint32_t)ld, j, info);
            if (hipGetLastError() != hipSuccess) return GRASS_EHIP;
            factorised = true;
            continue;
        }
        // last block of the outer block: scaled panel (into X64), then the rest of the matrix -= P P^T with P the
        // rows of the whole outer block below it
        DgemmArgs p{};
        p.A = A64 + (size_t)(j + 1) * NB * ld + (size_t)j * NB; p.rsA = ld; p.csA = 1;
        p.B = X64 + (size_t)j * NB * ld + (size_t)j * NB; p.rsB = 1; p.csB = ld;          // B[kk][n] = D[n][kk]
        p.C = X64 + (size_t)(j + 1) * NB * ld + (size_t)j * NB; p.rsC = ld; p.csC = 1;
        p.M = below; p.N = NB; p.K = NB; p.alpha = 1.0; p.beta = 0.0; p.flags = 0;
        if (dgemm(p, 1, hs) != hipSuccess) return GRASS_EHIP;
        if (outer_end < nblk) {
            const uint32_t c0 = (outer_end - kOuter) * NB, r0 = outer_end * NB;
            const double* P = X64 + (size_t)r0 * ld + c0;
            DgemmArgs u{};
            u.A = P; u.rsA = ld; u.csA = 1;
            u.B = P; u.rsB = 1; u.csB = ld;
            u.C = A64 + (size_t)r0 * ld + r0; u.rsC = ld; u.csC = 1;
            u.M = kp - r0; u.N = kp - r0; u.K = kOuter * NB; u.alpha = -1.0; u.beta = 1.0; u.flags = LOWER_TILES;
            if (dgemm(u, 1, hs) != hipSuccess) return GRASS_EHIP;
        }
    }

    // X = L^{-1} by doubling: with the inverses X11, X22 of two adjacent diagonal blocks of size b in place,
    // X21 = -X22 (L21 X11).  T = L21 X11 is parked transposed in the unused upper triangle of A64.
    for (uint32_t b = NB; b < kp; b *= 2) {
        const uint32_t full = kp / (2 * b);                // pairs with a complete second block
        const uint32_t rest = kp - full * 2 * b;           // a last pair with a shorter second block if rest > b
        for (int pass = 0; pass < 2; ++pass) {
            const uint32_t batch = pass == 0 ? full : (rest > b ? 1 : 0);
            if (batch == 0) continue;
            const uint32_t M2 = pass == 0 ? b : rest - b;
            const size_t o = pass == 0 ? 0 : (size_t)full * 2 * b;
            const int64_t bs = (int64_t)2 * b * (ld + 1);  // next pair: 2b down the diagonal
            DgemmArgs t{};                                 // T (M2 x b) = L21 * X11, X11 lower: k >= n0
            t.A = X64 + (o + b) * ld + o; t.rsA = ld; t.csA = 1; t.bsA = bs;      // L21 (scaled panels live in X64)
            t.B = X64 + o * ld + o; t.rsB = ld; t.csB = 1; t.bsB = bs;
            t.C = A64 + o * ld + (o + b); t.rsC = 1; t.csC = ld; t.bsC = bs;      // T[r][c] at A64[o+c][o+b+r]
            t.M = M2; t.N = b; t.K = b; t.alpha = 1.0; t.beta = 0.0; t.flags = K_FROM_COL;
            if (dgemm(t, batch, hs) != hipSuccess) return GRASS_EHIP;
            DgemmArgs x{};                                 // X21 (M2 x b) = -X22 * T, X22 lower: k < m0 + 64
            x.A = X64 + (o + b) * ld + (o + b); x.rsA = ld; x.csA = 1; x.bsA = bs;
            x.B = A64 + o * ld + (o + b); x.rsB = 1; x.csB = ld; x.bsB = bs;      // B[kk][n] = T[kk][n]
            x.C = X64 + (o + b) * ld + o; x.rsC = ld; x.csC = 1; x.bsC = bs;
            x.M = M2; x.N = b; x.K = M2; x.alpha = -1.0; x.beta = 0.0; x.flags = K_TO_ROW;
            if (dgemm(x, batch, hs) != hipSuccess) return GRASS_EHIP;
        }
    }

    // W = X^T X (lower tiles, mirrored), written as fp32; only the leading k x k part leaves the workspace
    if (kp == k) {
        DgemmArgs w{};
        w.A = X64; w.rsA = 1; w.csA = ld;                   // A[i][kk] = X[kk][i]
        w.B = X64; w.rsB = ld; w.csB = 1;
        w.Cf = W; w.rsC = (int64_t)ldw; w.csC = 1;
        w.M = kp; w.N = kp; w.K = kp; w.alpha = 1.0; w.beta = 0.0; w.flags = K_FROM_ROW | LOWER_TILES | MIRROR;
        if (dgemm(w, 1, hs) != hipSuccess) return GRASS_EHIP;
    } else {                                                // padded: go through A64 (free now), then copy k x k
        DgemmArgs w{};
        w.A = X64; w.rsA = 1; w.csA = ld;
        w.B = X64; w.rsB = ld; w.csB = 1;
        w.C = A64; w.rsC = ld; w.csC = 1;
        w.M = kp; w.N = kp; w.K = kp; w.alpha = 1.0; w.beta = 0.0; w.flags = K_FROM_ROW | LOWER_TILES;
        if (dgemm(w, 1, hs) != hipSuccess) return GRASS_EHIP;
        hipLaunchKernelGGL(fim_store_kernel, dim3((uint32_t)ceil_div((uint64_t)k * k, 256)), dim3(256), 0, hs, A64, (uint32_t)ld, k, W,
                           ldw);
    }
    return launch_status();
}

extern "C" grass_status grass_ifvp(const float* G, uint64_t N, uint32_t k, uint64_t ldg, const float* W, uint64_t ldw,
                                   float* out, uint64_t ldo, grass_stream stream) {
    if (k == 0) return GRASS_EINVAL;
    if (N == 0) return GRASS_OK;
    if (!G || !W || !out || ldg < k || ldw < k || ldo < k) return GRASS_EINVAL;
    // out[i][a] = sum_c G[i][c] W[a][c]  (W symmetric)
    return gemm_nt_f32(G, W, out, N, k, k, ldg, ldw, ldo, 0, 0, as_stream(stream), 1, nullptr) == hipSuccess ? GRASS_OK
                                                                                                             : GRASS_EHIP;
}
