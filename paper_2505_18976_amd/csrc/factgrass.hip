// FactGraSS for one linear layer (Sec. 3.3.2, Eq. (2) and Eq. (3)).
//
// Stage 1 (sparsification): gather k_in' columns of every token's layer input
// and k_out' columns of its pre-activation gradient.  Stage 2 (reconstruction):
// v[a*k_out' + b] = sum_t x'_t[a] * g'_t[b], a (k_in' x T)(T x k_out') contraction
// done on the matrix cores in bf16 with fp32 accumulation.  Stage 3 (sparse
// projection): SJLT of the k_in'*k_out' accumulator straight from registers into
// k LDS buckets (fp64 buckets with the fp64 LDS atomic add when they fit, which
// is an order of magnitude faster on gfx950 than the native fp32 LDS atomic add;
// fp32 buckets with a compare-and-swap loop otherwise).  The d_out x d_in layer
// gradient is never formed.
//
// A workgroup (4 wavefronts) owns one sample and one chunk of its tokens.
// Because the SJLT is linear, each chunk is projected on its own and the
// per-chunk k-vectors are added in a fixed order by a second kernel.
//
// factgrass_layers runs many layers of one model pass (same n, T, mask widths
// and k; per-layer shapes, indices, SJLT stream and output block) in a single
// launch: blockIdx.z selects the layer descriptor, so the gather latency of one
// workgroup overlaps with the matrix and SJLT phases of the others and the
// launch cost is paid once.
#include <type_traits>

#include <algorithm>
#include <cmath>
#include <vector>

#include "grass_device.h"

namespace grass {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kTokTile = 32;              // tokens staged per step (two MFMA k-steps of 16)
constexpr int kTokStride = kTokTile + 8;  // bf16 elements per LDS row: 80 bytes keeps 16-byte reads conflict-free
constexpr int kFgThreads = 256;

// Per-layer part of the arguments (device-resident array in the many-layer call).
struct FgLayer {
    const uint16_t* x;      // (n, T, d_in) bf16 bits
    const uint16_t* g;      // (n, T, d_out) bf16 bits
    const int32_t* idx_in;
    const int32_t* idx_out;
    float* out;             // n x k block of this layer (row distance ldo), used when there is one chunk
    uint64_t sub;           // sub-seed of the layer's SJLT stream
    uint32_t d_in, d_out;
};

struct FgArgs {
    FgLayer one;            // the layer, when `many` is null
    const FgLayer* many;    // device array indexed by blockIdx.z
    float* partial;         // [layer][chunk][n][k] when chunks > 1
    uint64_t T, n;
    uint64_t ldo;
    uint32_t ka, kb;
    uint32_t k, s, m;
    uint32_t tokens_per_block, chunks;
    float scale;
    uint32_t identity;      // 1: no SJLT, out[a*kb + b] = v[a*kb + b] (the factorised mask Mask_{k_in x k_out})
};

// Up to 64 layer descriptors handed over as kernel arguments (56 bytes each, under the 4 KB argument limit).
constexpr int kLayersPerPack = 64;
struct FgLayerPack {
    FgLayer l[kLayersPerPack];
    uint32_t first, count;
};
static_assert(sizeof(FgLayerPack) <= 4096, "kernel arguments are limited to 4 KB");
__global__ void __launch_bounds__(kLayersPerPack) fg_store_layers_kernel(FgLayerPack pack, FgLayer* table) {
    if (threadIdx.x < pack.count) table[pack.first + threadIdx.x] = pack.l[threadIdx.x];
}

// TA, TB: number of 32-wide tiles covering k_in' and k_out'.
template <int TA, int TB, bool F64>
__global__ void __launch_bounds__(kFgThreads) factgrass_kernel(FgArgs a) {
    using bucket_t = typename std::conditional<F64, double, float>::type;
    extern __shared__ __align__(16) unsigned char smem[];
    uint16_t* xs = reinterpret_cast<uint16_t*>(smem);                 // two stages of [TA*32][kTokStride] ...
    uint16_t* gs = xs + TA * 32 * kTokStride;                          // ... followed by [TB*32][kTokStride]
    bucket_t* sk = reinterpret_cast<bucket_t*>(smem);                  // [k], reuses the staging area afterwards

    constexpr int KA = TA * 32, KB = TB * 32;
    constexpr int NT = TA * TB;                    // output tiles
    constexpr int TPW = (NT + 3) / 4;              // tiles per wavefront
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const FgLayer L = a.many ? a.many[blockIdx.z] : a.one;       // uniform
    const uint64_t sample = blockIdx.y;
    const uint64_t t_begin = (uint64_t)blockIdx.x * a.tokens_per_block;
    const uint64_t t_end = t_begin + a.tokens_per_block < a.T ? t_begin + a.tokens_per_block : a.T;

    // each thread gathers a fixed column of x and a fixed column of g
    const int xa = tid % KA, xt0 = tid / KA;       // kFgThreads % KA == 0
    const int gb = tid % KB, gt0 = tid / KB;
    constexpr int XSTEP = kFgThreads / KA, GSTEP = kFgThreads / KB;
    const int32_t xcol = (uint32_t)xa < a.ka ? L.idx_in[xa] : -1;
    const int32_t gcol = (uint32_t)gb < a.kb ? L.idx_out[gb] : -1;
    const uint16_t* xrow = L.x + sample * a.T * L.d_in;
    const uint16_t* grow = L.g + sample * a.T * L.d_out;

    f32x16 acc[TPW];
#pragma unroll
    for (int i = 0; i < TPW; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[i][v] = 0.0f;

    // The gather of a token tile is pure latency (every 2-byte pick is its own 128-byte line, read once: non-temporal
    // loads), so two tiles are kept in flight in two register sets behind the tile being multiplied, and the LDS
    // staging area is double-buffered: one barrier per tile (the barrier of tile t+1 also tells that every wavefront
    // has finished reading the stage that tile t+2 will overwrite).
    constexpr int NX = kTokTile / XSTEP, NG = kTokTile / GSTEP;
    constexpr int kStageElems = (KA + KB) * kTokStride;
    // Every load is issued unconditionally from an address clamped into the chunk (padding columns read column 0,
    // tokens past the end read the last token) and the value is zeroed when it is stored to LDS: a load under a
    // branch would make the compiler wait for it on the spot, one round trip to HBM per load.
    // The layer descriptor comes out of memory, so the compiler cannot see that its pointers are global: say so
    // (generic-address loads count against both the memory and the LDS counters and force a full wait each time).
    typedef const __attribute__((address_space(1))) uint16_t* gptr_t;
    const gptr_t xbase = (gptr_t)(xrow + t_begin * L.d_in + (xcol >= 0 ? xcol : 0));
    const gptr_t gbase = (gptr_t)(grow + t_begin * L.d_out + (gcol >= 0 ? gcol : 0));
    const uint32_t nt = (uint32_t)(t_end - t_begin);      // tokens of this chunk (at most tokens_per_block), > 0
    const uint32_t xkeep = xcol >= 0 ? 0xFFFFu : 0u, gkeep = gcol >= 0 ? 0xFFFFu : 0u;
    uint32_t xv0[NX], gv0[NG], xv1[NX], gv1[NG];
    // r0: first token of the tile, relative to the chunk
    auto gather = [&](uint32_t (&xv)[NX], uint32_t (&gv)[NG], uint32_t r0) {
#pragma unroll
        for (int i = 0; i < NX; ++i) {
            const uint32_t r = r0 + xt0 + i * XSTEP;
            xv[i] = __builtin_nontemporal_load(xbase + (uint64_t)(r < nt ? r : nt - 1) * L.d_in);
        }
#pragma unroll
        for (int i = 0; i < NG; ++i) {
            const uint32_t r = r0 + gt0 + i * GSTEP;
            gv[i] = __builtin_nontemporal_load(gbase + (uint64_t)(r < nt ? r : nt - 1) * L.d_out);
        }
    };
    auto stash = [&](const uint32_t (&xv)[NX], const uint32_t (&gv)[NG], int stage, uint32_t r0) {
        uint16_t* xs_ = xs + stage * kStageElems;
        uint16_t* gs_ = gs + stage * kStageElems;
#pragma unroll
        for (int i = 0; i < NX; ++i)
            xs_[xa * kTokStride + xt0 + i * XSTEP] = (uint16_t)(xv[i] & xkeep & (r0 + xt0 + i * XSTEP < nt ? 0xFFFFu : 0u));
#pragma unroll
        for (int i = 0; i < NG; ++i)
            gs_[gb * kTokStride + gt0 + i * GSTEP] = (uint16_t)(gv[i] & gkeep & (r0 + gt0 + i * GSTEP < nt ? 0xFFFFu : 0u));
    };
    auto multiply = [&](int stage) {
        const uint16_t* xs_ = xs + stage * kStageElems;
        const uint16_t* gs_ = gs + stage * kStageElems;
#pragma unroll
        for (int i = 0; i < TPW; ++i) {
            const int tile = wave + 4 * i;
            if (tile < NT) {
                const int ta = tile / TB, tb = tile % TB;
#pragma unroll
                for (int ks = 0; ks < kTokTile / 16; ++ks) {
                    const bf16x8 af = *reinterpret_cast<const bf16x8*>(
                        xs_ + (ta * 32 + (lane & 31)) * kTokStride + ks * 16 + (lane >> 5) * 8);
                    const bf16x8 bf = *reinterpret_cast<const bf16x8*>(
                        gs_ + (tb * 32 + (lane & 31)) * kTokStride + ks * 16 + (lane >> 5) * 8);
                    acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af, bf, acc[i], 0, 0, 0);
                }
            }
        }
    };
    gather(xv0, gv0, 0);
    uint32_t r0 = 0;
    if (nt > 3 * kTokTile) {
        // Steady state: both lookahead gathers exist on every path into and around this loop, so the compiler can
        // count how many newer loads may stay in flight when a register set is stored (a gather under a condition on
        // the way in would make it wait for all of them).
        gather(xv1, gv1, kTokTile);
        for (; r0 + 3 * kTokTile < nt; r0 += 2 * kTokTile) {
            stash(xv0, gv0, 0, r0);                       // waits for the older set only: loads return in order
            __syncthreads();
            gather(xv0, gv0, r0 + 2 * kTokTile);
            multiply(0);
            stash(xv1, gv1, 1, r0 + kTokTile);
            __syncthreads();
            gather(xv1, gv1, r0 + 3 * kTokTile);
            multiply(1);
        }
    } else if (kTokTile < nt) {
        gather(xv1, gv1, kTokTile);                       // the branches around whole tiles are uniform
    }
    for (; r0 < nt; r0 += 2 * kTokTile) {                 // the last tiles, with the bounds checks
        stash(xv0, gv0, 0, r0);
        __syncthreads();
        if (r0 + 2 * kTokTile < nt) gather(xv0, gv0, r0 + 2 * kTokTile);
        multiply(0);
        if (r0 + kTokTile >= nt) break;
        stash(xv1, gv1, 1, r0 + kTokTile);
        __syncthreads();
        if (r0 + 3 * kTokTile < nt) gather(xv1, gv1, r0 + 3 * kTokTile);
        multiply(1);
    }
    __syncthreads();
    for (uint32_t b = tid; b < a.k; b += kFgThreads) sk[b] = (bucket_t)0;
    __syncthreads();

    // SJLT of this chunk's partial v.  Accumulator element e of a lane sits at
    // row (a') = 8*(e/4) + 4*(lane/32) + e%4 and column (b') = lane%32 of its tile.
#pragma unroll
    for (int i = 0; i < TPW; ++i) {
        const int tile = wave + 4 * i;
        if (tile < NT) {
            const int ta = tile / TB, tb = tile % TB;
            const uint32_t bq = tb * 32 + (lane & 31);
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const uint32_t aq = ta * 32 + 8 * (e >> 2) + 4 * (lane >> 5) + (e & 3);
                const float val = acc[i][e];
                if (a.identity) {                                  // every (a', b') belongs to exactly one lane
                    if (aq < a.ka && bq < a.kb) sk[aq * a.kb + bq] = (bucket_t)val;
                } else if (aq < a.ka && bq < a.kb && val != 0.0f) {
                    uint64_t c = ((uint64_t)aq * a.kb + bq) * a.s;
                    for (uint32_t rr = 0; rr < a.s; ++rr, ++c) {
                        const uint64_t h = sm(L.sub, c);
                        const uint32_t bucket = rr * a.m + bucket_of(h, a.m);
                        const float sv = __uint_as_float(__float_as_uint(val) ^ signbit_of(h));
                        if constexpr (F64) {
                            __hip_atomic_fetch_add(sk + bucket, (double)sv, __ATOMIC_RELAXED,
                                                   __HIP_MEMORY_SCOPE_WORKGROUP);
                        } else {
                            uint32_t* pb = reinterpret_cast<uint32_t*>(sk + bucket);
                            uint32_t old = *reinterpret_cast<volatile uint32_t*>(pb), assumed;
                            do {
                                assumed = old;
                                old = atomicCAS(pb, assumed, __float_as_uint(__uint_as_float(assumed) + sv));
                            } while (old != assumed);
                        }
                    }
                }
            }
        }
    }
    __syncthreads();
    float* o;
    float scale = a.scale;
    if (a.chunks == 1) {
        o = L.out + sample * a.ldo;
    } else {
        o = a.partial + (((uint64_t)blockIdx.z * a.chunks + blockIdx.x) * a.n + sample) * a.k;
        scale = 1.0f;
    }
    for (uint32_t b = tid; b < a.k; b += kFgThreads) o[b] = (float)sk[b] * scale;
}

// out_l[i, b] = scale * sum_c partial[l][c][i][b], c ascending (fixed order).
__global__ void __launch_bounds__(256) fg_reduce_kernel(FgArgs a) {
    const FgLayer L = a.many ? a.many[blockIdx.y] : a.one;
    const uint64_t total = a.n * a.k;
    const uint64_t t = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= total) return;
    const uint64_t i = t / a.k;
    const uint32_t b = (uint32_t)(t - i * a.k);
    const float* p = a.partial + (uint64_t)blockIdx.y * a.chunks * total + t;
    float sum = 0.0f;
    uint32_t c = 0;
    for (; c + 8 <= a.chunks; c += 8) {                   // eight loads in flight, added in chunk order
        float v[8];
#pragma unroll
        for (int q = 0; q < 8; ++q) v[q] = __builtin_nontemporal_load(p + (uint64_t)(c + q) * total);
#pragma unroll
        for (int q = 0; q < 8; ++q) sum += v[q];
    }
    for (; c < a.chunks; ++c) sum += p[(uint64_t)c * total];
    L.out[i * a.ldo + b] = sum * a.scale;
}

struct FgPlan {
    int TA, TB;
    bool f64;
    uint32_t tokens_per_block, chunks;
    size_t lds_bytes, ws_bytes;
};

static int tiles_for(uint32_t kq) { return kq <= 32 ? 1 : (kq <= 64 ? 2 : 4); }

static bool plan_fg(uint64_t n_layers, uint64_t n, uint64_t T, uint32_t ka, uint32_t kb, uint32_t k, FgPlan* pl,
                    const grass_tuning* tune = nullptr) {
    const int tune_tokens = tune ? tune->factgrass_tokens_per_block : 0;   // override of this call; 0 = heuristic
    if (ka == 0 || kb == 0 || ka > GRASS_MAX_FACTOR || kb > GRASS_MAX_FACTOR) return false;
    pl->TA = tiles_for(ka);
    pl->TB = tiles_for(kb);
    // tokens per workgroup: every workgroup pays a fixed price (SJLT of its partial accumulator, one k-vector
    // written and re-read), so take the largest chunk that still yields enough workgroups: about one per CU for
    // chunks of 256 tokens and more (many layers in one launch: up to whole sequences, no partial sums at all),
    // half a workgroup per CU for the short chunks of a single small layer (measured on 7 ... 112 layers of
    // 8 x 1,024 tokens and on one layer of 32 x 512 tokens).
    uint64_t tpb = 32;
    for (uint64_t cand : {1024ull, 512ull, 256ull, 128ull, 64ull}) {
        const uint64_t need = cand >= 256 ? (uint64_t)kNumCU * 7 / 8 : (uint64_t)kNumCU / 2;
        if (n_layers * n * ceil_div(T, cand) >= need) { tpb = cand; break; }
    }
    if (tpb > ceil_div(T, kTokTile) * kTokTile) tpb = ceil_div(T, kTokTile) * kTokTile;
    if (tune_tokens > 0) tpb = ceil_div((uint64_t)tune_tokens, kTokTile) * kTokTile;
    uint64_t chunks = ceil_div(T, tpb);
    if (chunks > 65535) { chunks = 65535; tpb = ceil_div(ceil_div(T, chunks), kTokTile) * kTokTile; chunks = ceil_div(T, tpb); }
    pl->tokens_per_block = (uint32_t)tpb;
    pl->chunks = (uint32_t)chunks;
    const size_t stage = (size_t)2 * (pl->TA + pl->TB) * 32 * kTokStride * sizeof(uint16_t);   // double-buffered
    pl->f64 = (size_t)k * sizeof(double) <= 64 * 1024;      // keeps at least two workgroups per CU
    const size_t buckets = (size_t)k * (pl->f64 ? sizeof(double) : sizeof(float));
    pl->lds_bytes = stage > buckets ? stage : buckets;
    pl->ws_bytes = chunks > 1 ? (size_t)n_layers * chunks * n * k * sizeof(float) : 0;
    return pl->lds_bytes <= kLdsBytes - 1024;
}

template <int TA, int TB, bool F64>
static hipError_t launch_fg2(const FgArgs& a, const FgPlan& pl, uint64_t n, uint32_t n_layers, hipStream_t st) {
    auto kern = factgrass_kernel<TA, TB, F64>;
    static LdsOptIn opt_in;
    const hipError_t e = allow_large_lds(opt_in, reinterpret_cast<const void*>(kern));
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, dim3(pl.chunks, (uint32_t)n, n_layers), dim3(kFgThreads), pl.lds_bytes, st, a);
    return hipGetLastError();
}

template <int TA, int TB>
static hipError_t launch_fg(const FgArgs& a, const FgPlan& pl, uint64_t n, uint32_t n_layers, hipStream_t st) {
    return pl.f64 ? launch_fg2<TA, TB, true>(a, pl, n, n_layers, st) : launch_fg2<TA, TB, false>(a, pl, n, n_layers, st);
}

// Launches the compression kernel and, when tokens were chunked, the fixed-order reduction.
static grass_status run_fg(FgArgs& a, const FgPlan& pl, uint32_t n_layers, hipStream_t hs) {
    hipError_t e = hipErrorInvalidValue;
    switch (pl.TA * 10 + pl.TB) {
        case 11: e = launch_fg<1, 1>(a, pl, a.n, n_layers, hs); break;
        case 12: e = launch_fg<1, 2>(a, pl, a.n, n_layers, hs); break;
        case 14: e = launch_fg<1, 4>(a, pl, a.n, n_layers, hs); break;
        case 21: e = launch_fg<2, 1>(a, pl, a.n, n_layers, hs); break;
        case 22: e = launch_fg<2, 2>(a, pl, a.n, n_layers, hs); break;
        case 24: e = launch_fg<2, 4>(a, pl, a.n, n_layers, hs); break;
        case 41: e = launch_fg<4, 1>(a, pl, a.n, n_layers, hs); break;
        case 42: e = launch_fg<4, 2>(a, pl, a.n, n_layers, hs); break;
        case 44: e = launch_fg<4, 4>(a, pl, a.n, n_layers, hs); break;
        default: return GRASS_EUNSUPPORTED;
    }
    if (e != hipSuccess) return GRASS_EHIP;
    if (pl.chunks > 1) {
        const uint64_t total = a.n * a.k;
        hipLaunchKernelGGL(fg_reduce_kernel, dim3((uint32_t)ceil_div(total, 256), n_layers), dim3(256), 0, hs, a);
        if (hipGetLastError() != hipSuccess) return GRASS_EHIP;
    }
    return GRASS_OK;
}

}  // namespace grass

using namespace grass;

static grass_status check_fg(uint64_t n, uint64_t T, uint32_t ka, uint32_t kb, uint32_t k, uint32_t s) {
    if (T == 0 || ka == 0 || kb == 0 || k == 0 || s == 0 || k % s != 0) return GRASS_EINVAL;
    if (n > 65535 || ka > GRASS_MAX_FACTOR || kb > GRASS_MAX_FACTOR || k > GRASS_MAX_K) return GRASS_EUNSUPPORTED;
    return GRASS_OK;
}

extern "C" grass_status factgrass_linear_workspace_bytes(uint64_t n, uint64_t T, uint32_t kin_p, uint32_t kout_p,
                                                         uint32_t k, uint32_t s, const grass_tuning* host_tuning,
                                                         size_t* host_bytes) {
    if (!host_bytes) return GRASS_EINVAL;
    grass_status st = check_fg(n, T, kin_p, kout_p, k, s);
    if (st != GRASS_OK) return st;
    if (n == 0) { *host_bytes = 0; return GRASS_OK; }
    FgPlan pl;
    if (!plan_fg(1, n, T, kin_p, kout_p, k, &pl, host_tuning)) return GRASS_EUNSUPPORTED;
    *host_bytes = pl.ws_bytes;
    return GRASS_OK;
}

static void fill_common(FgArgs& a, const FgPlan& pl, uint64_t n, uint64_t T, uint32_t ka, uint32_t kb, uint32_t k,
                        uint32_t s, uint64_t ldo) {
    a.many = nullptr; a.partial = nullptr;
    a.T = T; a.n = n; a.ldo = ldo; a.ka = ka; a.kb = kb;
    a.k = k; a.s = s; a.m = k / s;
    a.tokens_per_block = pl.tokens_per_block; a.chunks = pl.chunks;
    a.scale = 1.0f / sqrtf((float)s);
    a.identity = 0;
}

extern "C" grass_status factgrass_linear(const void* x, const void* gout, uint64_t n, uint64_t T, uint32_t d_in,
                                         uint32_t d_out, const int32_t* idx_in, uint32_t kin_p,
                                         const int32_t* idx_out, uint32_t kout_p, uint32_t k, uint32_t s,
                                         uint64_t seed, uint64_t stream_id, float* out, uint64_t ldo, void* ws,
                                         size_t ws_bytes, const grass_tuning* host_tuning, grass_stream stream) {
    grass_status st = check_fg(n, T, kin_p, kout_p, k, s);
    if (st != GRASS_OK) return st;
    if (kin_p > d_in || kout_p > d_out) return GRASS_EINVAL;
    if (n == 0) return GRASS_OK;
    if (!x || !gout || !idx_in || !idx_out || !out || ldo < k) return GRASS_EINVAL;
    FgPlan pl;
    if (!plan_fg(1, n, T, kin_p, kout_p, k, &pl, host_tuning)) return GRASS_EUNSUPPORTED;
    if (pl.ws_bytes > 0 && (!ws || ws_bytes < pl.ws_bytes || !aligned(ws, 256))) return GRASS_EWORKSPACE;

    FgArgs a;
    fill_common(a, pl, n, T, kin_p, kout_p, k, s, ldo);
    a.one.x = static_cast<const uint16_t*>(x);
    a.one.g = static_cast<const uint16_t*>(gout);
    a.one.idx_in = idx_in; a.one.idx_out = idx_out; a.one.out = out;
    a.one.sub = substream(seed, stream_id);
    a.one.d_in = d_in; a.one.d_out = d_out;
    a.partial = static_cast<float*>(ws);
    return run_fg(a, pl, 1, as_stream(stream));
}

static size_t layers_table_bytes(uint32_t n_layers) { return ((size_t)n_layers * sizeof(FgLayer) + 255) / 256 * 256; }

extern "C" grass_status factgrass_layers_workspace_bytes(uint32_t n_layers, uint64_t n, uint64_t T, uint32_t kin_p,
                                                         uint32_t kout_p, uint32_t k, uint32_t s,
                                                         const grass_tuning* host_tuning, size_t* host_bytes) {
    if (!host_bytes || n_layers == 0) return GRASS_EINVAL;
    if (n_layers > 65535) return GRASS_EUNSUPPORTED;
    grass_status st = check_fg(n, T, kin_p, kout_p, k, s);
    if (st != GRASS_OK) return st;
    if (n == 0) { *host_bytes = 0; return GRASS_OK; }
    FgPlan pl;
    if (!plan_fg(n_layers, n, T, kin_p, kout_p, k, &pl, host_tuning)) return GRASS_EUNSUPPORTED;
    *host_bytes = layers_table_bytes(n_layers) + pl.ws_bytes;
    return GRASS_OK;
}

extern "C" grass_status factgrass_layers(const factgrass_layer* host_layers, uint32_t n_layers, uint64_t n, uint64_t T,
                                         uint32_t kin_p, uint32_t kout_p, uint32_t k, uint32_t s, uint64_t seed,
                                         uint64_t ldo, void* ws, size_t ws_bytes, const grass_tuning* host_tuning,
                                         grass_stream stream) {
    if (!host_layers || n_layers == 0) return GRASS_EINVAL;
    if (n_layers > 65535) return GRASS_EUNSUPPORTED;
    grass_status st = check_fg(n, T, kin_p, kout_p, k, s);
    if (st != GRASS_OK) return st;
    if (n == 0) return GRASS_OK;
    if (ldo < k) return GRASS_EINVAL;
    for (uint32_t l = 0; l < n_layers; ++l) {
        const factgrass_layer& h = host_layers[l];
        if (!h.x || !h.gout || !h.idx_in || !h.idx_out || !h.out) return GRASS_EINVAL;
        if (kin_p > h.d_in || kout_p > h.d_out) return GRASS_EINVAL;
    }
    FgPlan pl;
    if (!plan_fg(n_layers, n, T, kin_p, kout_p, k, &pl, host_tuning)) return GRASS_EUNSUPPORTED;
    const size_t table = layers_table_bytes(n_layers);
    if (!ws || ws_bytes < table + pl.ws_bytes || !aligned(ws, 256)) return GRASS_EWORKSPACE;

    // The descriptor table travels to the head of the workspace as kernel arguments, 64 layers per launch: the
    // arguments are copied when the launch is enqueued, so nothing depends on host memory staying alive or on how
    // the runtime treats pageable copies, and the call stays asynchronous.
    hipStream_t hs = as_stream(stream);
    // Workgroups are handed out in launch order, layer after layer, and a workgroup's time follows the number of
    // 128-byte lines its picks touch per token, which depends on the layer's widths: the layers go into the table
    // most expensive first, so that the last round of workgroups is made of the cheap ones (every layer writes to
    // its own `out`, so the order is free).
    std::vector<uint32_t> order(n_layers);
    std::vector<double> cost(n_layers);
    for (uint32_t l = 0; l < n_layers; ++l) {
        auto lines = [](double d, double picks) {               // expected distinct lines of `picks` random 2-byte columns
            const double L = d * 2.0 / 128.0 < 1.0 ? 1.0 : d * 2.0 / 128.0;
            return L * (1.0 - std::pow(1.0 - 1.0 / L, picks));
        };
        order[l] = l;
        cost[l] = lines((double)host_layers[l].d_in, (double)kin_p) + lines((double)host_layers[l].d_out, (double)kout_p);
    }
    std::stable_sort(order.begin(), order.end(), [&](uint32_t a, uint32_t b) { return cost[a] > cost[b]; });
    FgLayer first_layer{};
    for (uint32_t l0 = 0; l0 < n_layers; l0 += kLayersPerPack) {
        FgLayerPack pack;
        pack.first = l0;
        pack.count = n_layers - l0 < (uint32_t)kLayersPerPack ? n_layers - l0 : (uint32_t)kLayersPerPack;
        for (uint32_t q = 0; q < pack.count; ++q) {
            const factgrass_layer& h = host_layers[order[l0 + q]];
            FgLayer& d = pack.l[q];
            d.x = static_cast<const uint16_t*>(h.x);
            d.g = static_cast<const uint16_t*>(h.gout);
            d.idx_in = h.idx_in; d.idx_out = h.idx_out; d.out = h.out;
            d.sub = substream(seed, h.stream_id);
            d.d_in = h.d_in; d.d_out = h.d_out;
        }
        for (uint32_t q = pack.count; q < (uint32_t)kLayersPerPack; ++q) pack.l[q] = FgLayer{};
        if (l0 == 0) first_layer = pack.l[0];
        hipLaunchKernelGGL(fg_store_layers_kernel, dim3(1), dim3(kLayersPerPack), 0, hs, pack, static_cast<FgLayer*>(ws));
        if (hipGetLastError() != hipSuccess) return GRASS_EHIP;
    }
    FgArgs a;
    fill_common(a, pl, n, T, kin_p, kout_p, k, s, ldo);
    a.one = first_layer;
    a.many = static_cast<const FgLayer*>(ws);
    a.partial = reinterpret_cast<float*>(static_cast<char*>(ws) + table);
    return run_fg(a, pl, n_layers, hs);
}

// Mask_{k_in x k_out} (Sec. 3.3.2, the factorised mask used as a baseline in Table 2 and as stage 1-2 of FactGraSS):
// out_i[a*k_out' + b] = sum_t x_t[idx_in[a]] * g_t[idx_out[b]], no sparse projection afterwards.
extern "C" grass_status factmask_linear_workspace_bytes(uint64_t n, uint64_t T, uint32_t kin_p, uint32_t kout_p,
                                                        size_t* host_bytes) {
    if (!host_bytes) return GRASS_EINVAL;
    if (kin_p == 0 || kout_p == 0 || kin_p > GRASS_MAX_FACTOR || kout_p > GRASS_MAX_FACTOR) return GRASS_EINVAL;
    return factgrass_linear_workspace_bytes(n, T, kin_p, kout_p, kin_p * kout_p, 1, nullptr, host_bytes);
}

extern "C" grass_status factmask_linear(const void* x, const void* gout, uint64_t n, uint64_t T, uint32_t d_in,
                                        uint32_t d_out, const int32_t* idx_in, uint32_t kin_p, const int32_t* idx_out,
                                        uint32_t kout_p, float* out, uint64_t ldo, void* ws, size_t ws_bytes,
                                        grass_stream stream) {
    if (kin_p == 0 || kout_p == 0 || kin_p > GRASS_MAX_FACTOR || kout_p > GRASS_MAX_FACTOR) return GRASS_EINVAL;
    const uint32_t k = kin_p * kout_p;
    grass_status st = check_fg(n, T, kin_p, kout_p, k, 1);
    if (st != GRASS_OK) return st;
    if (kin_p > d_in || kout_p > d_out) return GRASS_EINVAL;
    if (n == 0) return GRASS_OK;
    if (!x || !gout || !idx_in || !idx_out || !out || ldo < k) return GRASS_EINVAL;
    FgPlan pl;
    if (!plan_fg(1, n, T, kin_p, kout_p, k, &pl)) return GRASS_EUNSUPPORTED;
    if (pl.ws_bytes > 0 && (!ws || ws_bytes < pl.ws_bytes || !aligned(ws, 256))) return GRASS_EWORKSPACE;
    FgArgs a;
    fill_common(a, pl, n, T, kin_p, kout_p, k, 1, ldo);
    a.identity = 1;
    a.one.x = static_cast<const uint16_t*>(x);
    a.one.g = static_cast<const uint16_t*>(gout);
    a.one.idx_in = idx_in; a.one.idx_out = idx_out; a.one.out = out;
    a.one.sub = 0;
    a.one.d_in = d_in; a.one.d_out = d_out;
    a.partial = static_cast<float*>(ws);
    return run_fg(a, pl, 1, as_stream(stream));
}
