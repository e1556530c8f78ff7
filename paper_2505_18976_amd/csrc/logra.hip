// LoGra baseline: factorised dense projection Gauss_{k_in (x) k_out} for one
// linear layer (Sec. 3.3.2 "Recap on LoGra", Eq. (3)):
//     out_i = sum_t (P_in x_t) (x) (P_out g_t),   flat index a*k_out + b,
// with P_in (k_in x d_in) and P_out (k_out x d_out) dense (Gaussian) matrices
// supplied by the caller in bf16.  This is the method FactGraSS is compared with;
// it has to read every column of x and g, where FactGraSS reads k' of them.
//
// One workgroup (4 wavefronts) owns one sample and one chunk of its tokens.
//   Stage 1: a = X_chunk P_in^T and b = G_chunk P_out^T, 64 tokens at a time, bf16
//            MFMA with fp32 accumulation; K (= d_in, d_out) is streamed in slices
//            of 128 through two LDS stages with the next two slices prefetched in
//            registers (128 KB per workgroup in flight: one workgroup per CU has to
//            cover the HBM latency by itself).
//            Wavefronts 0,1 compute a (token halves), wavefronts 2,3 compute b.
//   Stage 2: acc[a][b] += sum_t a_t[a] * b_t[b] on the fp32 matrix cores from LDS.
// Per-chunk partial k_in x k_out blocks are added in a fixed order by
// reduce_partials_kernel.
#include "grass_device.h"

namespace grass {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int LT = 64;                 // tokens per stage-1 tile
constexpr int LK = 128;                // K slice
constexpr int LRS = LK + 8;            // bf16 per LDS row (272 bytes: conflict-free 16-byte fragment reads)
constexpr int LP = 64;                 // projected width handled (k_in, k_out <= 64, zero padded)
constexpr int kTileElems = 64 * LRS;   // one 64-row tile
constexpr int kLograStage = 4 * kTileElems;   // X, G, P_in, P_out
constexpr int kLograThreads = 256;

struct LograArgs {
    const uint16_t* x;      // (n, T, d_in) bf16
    const uint16_t* g;      // (n, T, d_out) bf16
    const uint16_t* pin;    // k_in x d_in bf16
    const uint16_t* pout;   // k_out x d_out bf16
    float* dst;
    uint64_t T, ld_dst, chunk_stride;
    uint32_t d_in, d_out, k_in, k_out;
    uint32_t tokens_per_block;
};

__global__ void __launch_bounds__(kLograThreads) logra_kernel(LograArgs a) {
    extern __shared__ __align__(16) uint16_t lds[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wg = wave >> 1, wh = wave & 1;          // stage 1: which product, which token half
    const uint64_t sample = blockIdx.y;
    const uint64_t t_begin = (uint64_t)blockIdx.x * a.tokens_per_block;
    const uint64_t t_end = t_begin + a.tokens_per_block < a.T ? t_begin + a.tokens_per_block : a.T;
    const uint16_t* xs = a.x + sample * a.T * a.d_in;
    const uint16_t* gs = a.g + sample * a.T * a.d_out;
    const uint32_t dmax = a.d_in > a.d_out ? a.d_in : a.d_out;
    const uint32_t nslices = (dmax + LK - 1) / LK;
    // Workgroups walk through the K slices in rotated order (workgroup w starts at slice 5w mod nslices): all of them
    // run in lockstep otherwise and would ask the same few L2 channels for the same slice of P_in / P_out at the same
    // time.  The contraction is a sum over all slices either way.
    const uint32_t rot = (uint32_t)((blockIdx.x + (uint64_t)blockIdx.y * gridDim.x) * 5 % nslices);
    auto K0 = [&](uint32_t i) {                         // i < nslices
        const uint32_t q = i + rot;
        return (q >= nslices ? q - nslices : q) * (uint32_t)LK;
    };

    // staging map: chunk c = tid + 256*i (i = 0..3) of a 64 x 128 tile: row c/16, 16-byte chunk c%16
    constexpr int CPR = LK / 8;                         // 16-byte chunks per row
    constexpr int NI = 64 * CPR / kLograThreads;        // chunks per thread and tile
    constexpr int RSTEP = kLograThreads / CPR;          // rows between a thread's chunks
    const int srow = tid / CPR, skc = tid % CPR;

    f32x16 acc2;                                        // stage 2: one 32 x 32 tile of the k_in x k_out block
#pragma unroll
    for (int v = 0; v < 16; ++v) acc2[v] = 0.0f;
    const int ta = wave >> 1, tb = wave & 1;

    struct RegSet { u32x4 rx[NI], rg[NI], rpi[NI], rpo[NI]; };
    for (uint64_t t0 = t_begin; t0 < t_end; t0 += LT) {
        // Loads are issued unconditionally from addresses clamped into the tensors (rows past the end re-read the last
        // valid row, columns past d re-read the last 16-byte chunk) and the out-of-range parts are zeroed when the
        // registers are stored to LDS: a load under a branch makes the compiler wait for every outstanding load.
        const uint32_t din8 = a.d_in - 8, dout8 = a.d_out - 8;          // d_in, d_out are multiples of 8, >= 8
        const uint64_t trow_last = t_end - 1;
        auto fetch = [&](RegSet& r, uint32_t k0) {
            const uint32_t kk = k0 + skc * 8;           // a 16-byte chunk is all in or all out
            const uint32_t kx = kk < a.d_in ? kk : din8, kg = kk < a.d_out ? kk : dout8;
#pragma unroll
            for (int i = 0; i < NI; ++i) {
                const uint32_t row = srow + RSTEP * i;
                const uint64_t t = t0 + row < trow_last ? t0 + row : trow_last;
                // x and g are read exactly once (non-temporal: they must not push the projection matrices, which
                // every workgroup re-reads, out of L2)
                r.rx[i] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(xs + t * a.d_in + kx));
                r.rg[i] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(gs + t * a.d_out + kg));
                r.rpi[i] = *reinterpret_cast<const u32x4*>(a.pin + (uint64_t)(row < a.k_in ? row : a.k_in - 1) * a.d_in + kx);
                r.rpo[i] = *reinterpret_cast<const u32x4*>(a.pout + (uint64_t)(row < a.k_out ? row : a.k_out - 1) * a.d_out + kg);
            }
        };
        auto stash = [&](const RegSet& r, int stage, uint32_t k0) {
            uint16_t* base = lds + stage * kLograStage;
            const uint32_t kk = k0 + skc * 8;
            const uint32_t mx = kk < a.d_in ? ~0u : 0u, mg = kk < a.d_out ? ~0u : 0u;
#pragma unroll
            for (int i = 0; i < NI; ++i) {
                const uint32_t row = srow + RSTEP * i;
                const int off = row * LRS + skc * 8;
                const uint32_t mt = t0 + row < t_end ? ~0u : 0u;
                const uint32_t mxi = mx & mt, mgi = mg & mt;
                const uint32_t mpi = mx & (row < a.k_in ? ~0u : 0u), mpo = mg & (row < a.k_out ? ~0u : 0u);
                *reinterpret_cast<u32x4*>(base + off) = r.rx[i] & u32x4(mxi);
                *reinterpret_cast<u32x4*>(base + kTileElems + off) = r.rg[i] & u32x4(mgi);
                *reinterpret_cast<u32x4*>(base + 2 * kTileElems + off) = r.rpi[i] & u32x4(mpi);
                *reinterpret_cast<u32x4*>(base + 3 * kTileElems + off) = r.rpo[i] & u32x4(mpo);
            }
        };

        f32x16 acc1[2];                                 // 32 tokens x 64 projected columns
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc1[j][v] = 0.0f;
        auto multiply = [&](int cur, uint32_t sl) {
            // operand tiles of this wavefront: tokens (X or G) and projection rows (P_in or P_out)
            const uint16_t* tok = lds + cur * kLograStage + wg * kTileElems + (wh * 32 + (lane & 31)) * LRS + (lane >> 5) * 8;
            const uint16_t* prj = lds + cur * kLograStage + (2 + wg) * kTileElems + (lane & 31) * LRS + (lane >> 5) * 8;
            const bool live = K0(sl) < (wg == 0 ? a.d_in : a.d_out);       // uniform per wavefront
            if (live) {
#pragma unroll
                for (int ks = 0; ks < LK / 16; ++ks) {
                    const bf16x8 tf = *reinterpret_cast<const bf16x8*>(tok + ks * 16);
#pragma unroll
                    for (int j = 0; j < 2; ++j) {
                        const bf16x8 pf = *reinterpret_cast<const bf16x8*>(prj + j * 32 * LRS + ks * 16);
                        acc1[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(tf, pf, acc1[j], 0, 0, 0);
                    }
                }
            }
        };

        // Two K slices are in flight in registers behind the one being multiplied (set B holds the odd slices, set A
        // the even ones); loads complete in order, so storing slice s+1 to LDS waits for that slice only.
        RegSet A, B;
        __syncthreads();                                // stage-2 reads of the previous token tile are done
        fetch(A, K0(0));
        stash(A, 0, K0(0));
        uint32_t sl = 0;
        if (nslices > 4) {
            // Steady state (both prefetches exist on every path into and around the loop): the same straight-line
            // code every iteration, so the compiler can count how many newer loads may stay in flight when a register
            // set is stored to LDS (a prefetch under a condition anywhere on the way in would make it wait for all).
            fetch(B, K0(1));
            fetch(A, K0(2));
            __syncthreads();
            for (; sl + 4 < nslices; sl += 2) {
                multiply(0, sl);                            // stage 0: slice sl
                stash(B, 1, K0(sl + 1));
                fetch(B, K0(sl + 3));
                __syncthreads();
                multiply(1, sl + 1);                        // stage 1: slice sl + 1
                stash(A, 0, K0(sl + 2));
                fetch(A, K0(sl + 4));
                __syncthreads();
            }
        } else {
            if (nslices > 1) fetch(B, K0(1));                  // branches around whole slices are uniform
            if (nslices > 2) fetch(A, K0(2));
            __syncthreads();
        }
        // the last slices, with the bounds checks
        for (; sl < nslices; sl += 2) {
            multiply(0, sl);
            if (sl + 1 < nslices) stash(B, 1, K0(sl + 1));
            if (sl + 3 < nslices) fetch(B, K0(sl + 3));
            __syncthreads();
            if (sl + 1 >= nslices) break;
            multiply(1, sl + 1);
            if (sl + 2 < nslices) stash(A, 0, K0(sl + 2));
            if (sl + 4 < nslices) fetch(A, K0(sl + 4));
            __syncthreads();
        }

        // a (wavefronts 0,1) and b (wavefronts 2,3) as fp32 [token][64] over the staging area
        float* ab = reinterpret_cast<float*>(lds) + wg * (LT * LP);
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int row = wh * 32 + 8 * (e >> 2) + 4 * (lane >> 5) + (e & 3);     // token
                ab[row * LP + j * 32 + (lane & 31)] = acc1[j][e];
            }
        __syncthreads();
        const float* as = reinterpret_cast<const float*>(lds);
        const float* bs = as + LT * LP;
#pragma unroll 8
        for (int t = 0; t < LT; t += 2) {
            const float fa = as[(t + (lane >> 5)) * LP + ta * 32 + (lane & 31)];
            const float fb = bs[(t + (lane >> 5)) * LP + tb * 32 + (lane & 31)];
            acc2 = __builtin_amdgcn_mfma_f32_32x32x2f32(fa, fb, acc2, 0, 0, 0);
        }
    }

    float* o = a.dst + (uint64_t)blockIdx.x * a.chunk_stride + sample * a.ld_dst;
#pragma unroll
    for (int e = 0; e < 16; ++e) {
        const uint32_t ai = ta * 32 + 8 * (e >> 2) + 4 * (lane >> 5) + (e & 3);
        const uint32_t bi = tb * 32 + (lane & 31);
        if (ai < a.k_in && bi < a.k_out) o[(uint64_t)ai * a.k_out + bi] = acc2[e];
    }
}

struct LograPlan {
    uint32_t tokens_per_block, chunks;
    size_t ws_bytes;
};

static void plan_logra(uint64_t n, uint64_t T, uint32_t k_in, uint32_t k_out, LograPlan* pl) {
    // larger chunks re-read P_in / P_out less often; keep at least one workgroup per CU when possible
    uint64_t tpb = 64;
    for (uint64_t cand : {256ull, 128ull}) {
        if (n * ceil_div(T, cand) >= (uint64_t)kNumCU) { tpb = cand; break; }
    }
    uint64_t chunks = ceil_div(T, tpb);
    if (chunks > 65535) { tpb = ceil_div(ceil_div(T, 65535), LT) * LT; chunks = ceil_div(T, tpb); }
    pl->tokens_per_block = (uint32_t)tpb;
    pl->chunks = (uint32_t)chunks;
    pl->ws_bytes = chunks > 1 ? (size_t)chunks * n * k_in * k_out * sizeof(float) : 0;
}

}  // namespace grass

using namespace grass;

static grass_status check_logra(uint64_t n, uint64_t T, uint32_t k_in, uint32_t k_out) {
    if (T == 0 || k_in == 0 || k_out == 0) return GRASS_EINVAL;
    if (n > 65535 || k_in > LP || k_out > LP) return GRASS_EUNSUPPORTED;
    return GRASS_OK;
}

extern "C" grass_status logra_linear_workspace_bytes(uint64_t n, uint64_t T, uint32_t k_in, uint32_t k_out,
                                                     size_t* host_bytes) {
    if (!host_bytes) return GRASS_EINVAL;
    grass_status st = check_logra(n, T, k_in, k_out);
    if (st != GRASS_OK) return st;
    if (n == 0) { *host_bytes = 0; return GRASS_OK; }
    LograPlan pl;
    plan_logra(n, T, k_in, k_out, &pl);
    *host_bytes = pl.ws_bytes;
    return GRASS_OK;
}

extern "C" grass_status logra_linear(const void* x, const void* gout, uint64_t n, uint64_t T, uint32_t d_in,
                                     uint32_t d_out, const void* P_in, uint32_t k_in, const void* P_out,
                                     uint32_t k_out, float* out, uint64_t ldo, void* ws, size_t ws_bytes,
                                     grass_stream stream) {
    grass_status st = check_logra(n, T, k_in, k_out);
    if (st != GRASS_OK) return st;
    if (d_in == 0 || d_out == 0) return GRASS_EINVAL;
    if (n == 0) return GRASS_OK;
    const uint64_t kk = (uint64_t)k_in * k_out;
    if (!x || !gout || !P_in || !P_out || !out || ldo < kk) return GRASS_EINVAL;
    // 16-byte chunks along the feature dimension
    if (d_in % 8 != 0 || d_out % 8 != 0 || !aligned(x, 16) || !aligned(gout, 16) || !aligned(P_in, 16) ||
        !aligned(P_out, 16))
        return GRASS_EUNSUPPORTED;
    LograPlan pl;
    plan_logra(n, T, k_in, k_out, &pl);
    if (pl.ws_bytes > 0 && (!ws || ws_bytes < pl.ws_bytes || !aligned(ws, 256))) return GRASS_EWORKSPACE;

    LograArgs a;
    a.x = static_cast<const uint16_t*>(x);
    a.g = static_cast<const uint16_t*>(gout);
    a.pin = static_cast<const uint16_t*>(P_in);
    a.pout = static_cast<const uint16_t*>(P_out);
    a.T = T; a.d_in = d_in; a.d_out = d_out; a.k_in = k_in; a.k_out = k_out;
    a.tokens_per_block = pl.tokens_per_block;
    if (pl.chunks == 1) {
        a.dst = out; a.ld_dst = ldo; a.chunk_stride = 0;
    } else {
        a.dst = static_cast<float*>(ws); a.ld_dst = kk; a.chunk_stride = n * kk;
    }
    hipStream_t hs = as_stream(stream);
    static LdsOptIn opt_in;
    const size_t lds_bytes = (size_t)2 * kLograStage * sizeof(uint16_t);
    if (allow_large_lds(opt_in, reinterpret_cast<const void*>(logra_kernel)) != hipSuccess) return GRASS_EHIP;
    hipLaunchKernelGGL(logra_kernel, dim3(pl.chunks, (uint32_t)n), dim3(kLograThreads), lds_bytes, hs, a);
    if (hipGetLastError() != hipSuccess) return GRASS_EHIP;
    if (pl.chunks > 1) {
        const uint64_t total = n * kk;
        hipLaunchKernelGGL(reduce_partials_kernel, dim3((uint32_t)ceil_div(total, 256)), dim3(256), 0, hs,
                           static_cast<const float*>(ws), n, (uint32_t)kk, pl.chunks, 1.0f, out, ldo);
        if (hipGetLastError() != hipSuccess) return GRASS_EHIP;
    }
    return GRASS_OK;
}
