// LoGra baseline: factorised dense projection Gauss_{k_in (x) k_out} for one
// linear layer (Sec. 3.3.2 "Recap on LoGra", Eq. (3)):
//     out_i = sum_t (P_in x_t) (x) (P_out g_t),   flat index a*k_out + b,
// with P_in (k_in x d_in) and P_out (k_out x d_out) dense (Gaussian) matrices
// supplied by the caller in bf16.  This is the method FactGraSS is compared with;
// it has to read every column of x and g, where FactGraSS reads k' of them.
//
// One workgroup (8 wavefronts) owns one sample and one chunk of its tokens.
//   Stage 1: a = X_chunk P_in^T and b = G_chunk P_out^T, 64 tokens at a time, bf16
//            MFMA with fp32 accumulation; K (= d_in, d_out) is streamed in slices
//            of 128 through two LDS stages.  Four producer wavefronts stream x and g,
//            64 columns at a time, through eight rotating register sets (seven loads
//            of 16 KB in flight behind the one being stored to LDS: one workgroup per
//            CU has to cover the HBM latency by itself); four consumer wavefronts
//            fetch the slices of P_in and P_out, which come out of L2, two slices
//            ahead, stage them, and multiply the staged slice (consumers 0,1 compute a
//            for the two token halves, 2,3 compute b), so the matrix and LDS-read work
//            runs under the producers' wait for memory.
//   Stage 2: acc[a][b] += sum_t a_t[a] * b_t[b] on the fp32 matrix cores from LDS
//            (consumers).
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
constexpr int kLograThreads = 512;       // 4 producer + 4 consumer wavefronts

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

constexpr int kHalf = 64;               // columns per register set of the producers (half an LDS slice)
constexpr int kSets = 8;                // rotating register sets of x and g: seven halves stay in flight behind the one being stored

__global__ void __launch_bounds__(kLograThreads) logra_kernel(LograArgs a) {
    extern __shared__ __align__(16) uint16_t lds[];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);     // uniform: the role branches below are scalar
    const bool producer = wave < 4;                   // wavefronts 0..3 stream x and g, 4..7 fetch P and multiply
    const int ptid = tid & 255;                       // thread index inside its role
    const int cw = wave & 3;                          // consumer wavefront
    const int wg = cw >> 1, wh = cw & 1;              // stage 1: which product (a or b), which token half
    const uint64_t sample = blockIdx.y;
    const uint64_t t_begin = (uint64_t)blockIdx.x * a.tokens_per_block;
    const uint64_t t_end = t_begin + a.tokens_per_block < a.T ? t_begin + a.tokens_per_block : a.T;
    const uint16_t* xs = a.x + sample * a.T * a.d_in;
    const uint16_t* gs = a.g + sample * a.T * a.d_out;
    const uint32_t dmax = a.d_in > a.d_out ? a.d_in : a.d_out;
    const uint32_t ngroups = (dmax + LK - 1) / LK;    // LDS slices of 128 columns
    const uint32_t nhalves = 2 * ngroups;             // producer loads of 64 columns
    // Workgroups walk through the K slices in rotated order (workgroup w starts at slice 5w mod ngroups): all of them
    // run in lockstep otherwise and would ask the same few L2 channels for the same slice of P_in / P_out at the same
    // time.  The contraction is a sum over all slices either way.
    const uint32_t rot = (uint32_t)((blockIdx.x + (uint64_t)blockIdx.y * gridDim.x) * 5 % ngroups);
    auto KG = [&](uint32_t g) {                         // first column of group g of this workgroup's order; g >= ngroups
        if (g >= ngroups) return dmax + (uint32_t)LK;   // gives a column past every operand (loads clamp, stores zero)
        const uint32_t q = g + rot;
        return (q >= ngroups ? q - ngroups : q) * (uint32_t)LK;
    };
    auto KH = [&](uint32_t j) { return KG(j >> 1) + (j & 1) * (uint32_t)kHalf; };   // first column of half j
    const uint32_t din8 = a.d_in - 8, dout8 = a.d_out - 8;              // d_in, d_out are multiples of 8, >= 8

    f32x16 acc2;                                        // stage 2: one 32 x 32 tile of the k_in x k_out block
#pragma unroll
    for (int v = 0; v < 16; ++v) acc2[v] = 0.0f;
    const int ta = cw >> 1, tb = cw & 1;

    for (uint64_t t0 = t_begin; t0 < t_end; t0 += LT) {
        // Loads are issued unconditionally from addresses clamped into the tensors (rows past the end re-read the last
        // valid row, columns past d re-read the last 16-byte chunk) and the out-of-range parts are zeroed when the
        // registers are stored to LDS: a load under a branch makes the compiler wait for every outstanding load.
        // Addresses are a uniform 64-bit base (tile of tokens, or the projection matrix) plus a 32-bit byte offset
        // per lane (the host refuses d > 2^24, so 64 rows of 2-byte elements stay below 2^32): the per-lane part of
        // an address then costs one register instead of two per outstanding load.
        //
        // Half j of x and g (64 columns of both token tiles) travels in register set j mod 8 of the producers and lands
        // in LDS stage (j / 2) mod 2: seven halves (112 KB per workgroup) stay in flight behind the one being stored,
        // which is what it takes to cover the HBM latency with one workgroup per CU.  The projection matrices come
        // out of L2 with a shorter latency; the consumers fetch them themselves, a whole slice of 128 columns two slices
        // ahead, so they do not take the producers' registers and - loads return in order within a wavefront - do
        // not wait behind the long queue of x and g.  While the consumers multiply group g out of stage g mod 2, both
        // roles store group g + 1 into the other stage.  Every wavefront passes the same barriers: one at the start
        // of the tile, one after each group is staged (which is also: after the group before it has been multiplied),
        // one after the last group has been multiplied.
        __syncthreads();                                // stage-2 reads of the previous token tile are done
        if (producer) {
            // staging map of the 256 producer threads for one half (64 rows x 64 columns per tile): chunk c = ptid +
            // 256*i (i = 0, 1): row c/8, 16-byte chunk c%8
            constexpr int CPR = kHalf / 8, NI = 64 * CPR / 256, RSTEP = 256 / CPR;
            const int srow = ptid / CPR, skc = ptid % CPR;
            const uint32_t rows_left = (uint32_t)(t_end - t0 < LT ? t_end - t0 : LT);
            const char* xb = reinterpret_cast<const char*>(xs + t0 * a.d_in);
            const char* gb = reinterpret_cast<const char*>(gs + t0 * a.d_out);
            uint32_t ox[NI], og[NI];
#pragma unroll
            for (int i = 0; i < NI; ++i) {
                const uint32_t row = srow + RSTEP * i;
                const uint32_t trow = row < rows_left ? row : rows_left - 1;
                ox[i] = trow * a.d_in * 2; og[i] = trow * a.d_out * 2;
            }
            struct RegSet { u32x4 rx[NI], rg[NI]; };
            auto fetch = [&](RegSet& r, uint32_t k0) {
                const uint32_t kk = k0 + skc * 8;           // a 16-byte chunk is all in or all out
                const uint32_t kx = (kk < a.d_in ? kk : din8) * 2, kg = (kk < a.d_out ? kk : dout8) * 2;
#pragma unroll
                for (int i = 0; i < NI; ++i) {
                    // x and g are read exactly once (non-temporal: they must not push the projection matrices, which
                    // every workgroup re-reads, out of L2)
                    r.rx[i] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(xb + (ox[i] + kx)));
                    r.rg[i] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(gb + (og[i] + kg)));
                }
            };
            // half j goes to LDS stage (j >> 1) & 1, columns (j & 1) * 64 .. + 63 of the 128-column rows
            auto stash = [&](const RegSet& r, uint32_t j, uint32_t k0) {
                uint16_t* base = lds + ((j >> 1) & 1) * kLograStage + (j & 1) * kHalf;
                const uint32_t kk = k0 + skc * 8;
                const uint32_t mx = kk < a.d_in ? ~0u : 0u, mg = kk < a.d_out ? ~0u : 0u;
#pragma unroll
                for (int i = 0; i < NI; ++i) {
                    const uint32_t row = srow + RSTEP * i;
                    const int off = row * LRS + skc * 8;
                    const uint32_t mt = t0 + row < t_end ? ~0u : 0u;
                    *reinterpret_cast<u32x4*>(base + off) = r.rx[i] & u32x4(mx & mt);
                    *reinterpret_cast<u32x4*>(base + kTileElems + off) = r.rg[i] & u32x4(mg & mt);
                }
            };
            RegSet S[kSets];
#pragma unroll
            for (int q = 0; q < kSets; ++q) fetch(S[q], KH(q));            // unconditional (clamped past the end)
            uint32_t j = 0;                                                // next half to store; a multiple of 8
            // steady state: every fetch is unconditional on every path into and around the loop, so the wait counts
            // the compiler derives keep the seven newer register sets in flight
            for (; j + 2 * kSets - 1 < nhalves; j += kSets) {
#pragma unroll
                for (int u = 0; u < kSets; ++u) {
                    stash(S[u], j + u, KH(j + u));
                    fetch(S[u], KH(j + u + kSets));
                    if (u & 1) __syncthreads();        // group (j+u)/2 is staged, group (j+u)/2 - 1 has been multiplied
                }
            }
            // the last halves, with the bounds checks (uniform branches)
            for (; j < nhalves; j += kSets) {
#pragma unroll
                for (int u = 0; u < kSets; ++u) {
                    if (j + u < nhalves) {
                        stash(S[u], j + u, KH(j + u));
                        if (j + u + kSets < nhalves) fetch(S[u], KH(j + u + kSets));
                        if (u & 1) __syncthreads();
                    }
                }
            }
            __syncthreads();                                               // the last group has been multiplied
        } else {
            // staging map of the 256 consumer threads for one group of P_in and of P_out (64 rows x 128 columns each):
            // chunk c = ptid + 256*i (i = 0..3): row c/16, 16-byte chunk c%16
            constexpr int PCPR = LK / 8, PNI = 64 * PCPR / 256, PRSTEP = 256 / PCPR;
            const int prow = ptid / PCPR, pkc = ptid % PCPR;
            const char* pib = reinterpret_cast<const char*>(a.pin);
            const char* pob = reinterpret_cast<const char*>(a.pout);
            uint32_t opi[PNI], opo[PNI];
#pragma unroll
            for (int i = 0; i < PNI; ++i) {
                const uint32_t row = prow + PRSTEP * i;
                opi[i] = (row < a.k_in ? row : a.k_in - 1) * a.d_in * 2;
                opo[i] = (row < a.k_out ? row : a.k_out - 1) * a.d_out * 2;
                // The projection offsets do not depend on the token tile; hidden from the optimiser here, or it computes
                // the complete 64-bit addresses of the first loads of a tile once, outside the tile loop, and keeps
                // (spills) them all.
                asm volatile("" : "+v"(opi[i]), "+v"(opo[i]));
            }
            struct PSet { u32x4 rpi[PNI], rpo[PNI]; };
            auto fetch_p = [&](PSet& r, uint32_t k0) {
                const uint32_t kk = k0 + pkc * 8;
                const uint32_t kx = (kk < a.d_in ? kk : din8) * 2, kg = (kk < a.d_out ? kk : dout8) * 2;
#pragma unroll
                for (int i = 0; i < PNI; ++i) {
                    r.rpi[i] = *reinterpret_cast<const u32x4*>(pib + (opi[i] + kx));
                    r.rpo[i] = *reinterpret_cast<const u32x4*>(pob + (opo[i] + kg));
                }
            };
            auto stash_p = [&](const PSet& r, uint32_t g, uint32_t k0) {
                uint16_t* base = lds + (g & 1) * kLograStage + 2 * kTileElems;
                const uint32_t kk = k0 + pkc * 8;
                const uint32_t mx = kk < a.d_in ? ~0u : 0u, mg = kk < a.d_out ? ~0u : 0u;
#pragma unroll
                for (int i = 0; i < PNI; ++i) {
                    const uint32_t row = prow + PRSTEP * i;
                    const int off = row * LRS + pkc * 8;
                    *reinterpret_cast<u32x4*>(base + off) = r.rpi[i] & u32x4(mx & (row < a.k_in ? ~0u : 0u));
                    *reinterpret_cast<u32x4*>(base + kTileElems + off) = r.rpo[i] & u32x4(mg & (row < a.k_out ? ~0u : 0u));
                }
            };
            f32x16 acc1[2];                                 // 32 tokens x 64 projected columns
#pragma unroll
            for (int jj = 0; jj < 2; ++jj)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc1[jj][v] = 0.0f;
            auto multiply = [&](int cur, uint32_t g) {
                // operand tiles of this wavefront: tokens (X or G) and projection rows (P_in or P_out)
                const uint16_t* tok = lds + cur * kLograStage + wg * kTileElems + (wh * 32 + (lane & 31)) * LRS + (lane >> 5) * 8;
                const uint16_t* prj = lds + cur * kLograStage + (2 + wg) * kTileElems + (lane & 31) * LRS + (lane >> 5) * 8;
                const bool live = KG(g) < (wg == 0 ? a.d_in : a.d_out);        // uniform per wavefront
                if (live) {
#pragma unroll
                    for (int ks = 0; ks < LK / 16; ++ks) {
                        const bf16x8 tf = *reinterpret_cast<const bf16x8*>(tok + ks * 16);
#pragma unroll
                        for (int jj = 0; jj < 2; ++jj) {
                            const bf16x8 pf = *reinterpret_cast<const bf16x8*>(prj + jj * 32 * LRS + ks * 16);
                            acc1[jj] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(tf, pf, acc1[jj], 0, 0, 0);
                        }
                    }
                }
            };
            PSet P0, P1;                                    // groups 0, 2, 4, ... travel in P0, the odd ones in P1
            fetch_p(P0, KG(0));
            fetch_p(P1, KG(1));
            stash_p(P0, 0, KG(0));
            fetch_p(P0, KG(2));
            __syncthreads();                                               // group 0 is staged
            uint32_t g = 0;
            for (; g + 1 < ngroups; g += 2) {                              // two groups per round: static register sets
                multiply(0, g);
                stash_p(P1, g + 1, KG(g + 1));
                fetch_p(P1, KG(g + 3));
                __syncthreads();
                multiply(1, g + 1);
                stash_p(P0, g + 2, KG(g + 2));                             // past the end: zeros into a stage nobody reads
                fetch_p(P0, KG(g + 4));
                __syncthreads();
            }
            if (g < ngroups) {                                             // an odd number of groups: the last one
                multiply(0, g);
                __syncthreads();
            }
            // a (consumers 0,1) and b (consumers 2,3) as fp32 [token][64] over the staging area, which nobody reads
            // or writes any more after the last barrier
            float* ab = reinterpret_cast<float*>(lds) + wg * (LT * LP);
#pragma unroll
            for (int jj = 0; jj < 2; ++jj)
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const int row = wh * 32 + 8 * (e >> 2) + 4 * (lane >> 5) + (e & 3);     // token
                    ab[row * LP + jj * 32 + (lane & 31)] = acc1[jj][e];
                }
        }
        __syncthreads();
        if (!producer) {
            const float* as = reinterpret_cast<const float*>(lds);
            const float* bs = as + LT * LP;
#pragma unroll 8
            for (int t = 0; t < LT; t += 2) {
                const float fa = as[(t + (lane >> 5)) * LP + ta * 32 + (lane & 31)];
                const float fb = bs[(t + (lane >> 5)) * LP + tb * 32 + (lane & 31)];
                acc2 = __builtin_amdgcn_mfma_f32_32x32x2f32(fa, fb, acc2, 0, 0, 0);
            }
        }
    }

    if (!producer) {
        float* o = a.dst + (uint64_t)blockIdx.x * a.chunk_stride + sample * a.ld_dst;
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            const uint32_t ai = ta * 32 + 8 * (e >> 2) + 4 * (lane >> 5) + (e & 3);
            const uint32_t bi = tb * 32 + (lane & 31);
            if (ai < a.k_in && bi < a.k_out) o[(uint64_t)ai * a.k_out + bi] = acc2[e];
        }
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
    if (d_in > (1u << 24) || d_out > (1u << 24)) return GRASS_EUNSUPPORTED;   // 32-bit byte offsets inside a tile
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
