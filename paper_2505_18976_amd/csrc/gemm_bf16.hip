// Score GEMM (Sec. 2.1, attribute stage: all-pair inner products of compressed
// gradients) on the direct-to-LDS pipeline: bf16 operands for callers that keep
// the compressed gradients in bf16 (plus the fp32 -> bf16 conversion they need),
// and fp32 operands (also used by the dense Gaussian baseline of Sec. 2.2).
//
// C[M x N] = A[M x K] * B[N x K]^T, A and B row-major bf16 with K contiguous,
// fp32 accumulation.  One workgroup of 8 wavefronts (2 x 4) owns a 256 x 256 tile
// of C; each wavefront owns 128 x 64 = 4 x 2 MFMA tiles (v_mfma_f32_32x32x16_bf16,
// 128 accumulator registers per lane).  Two wavefronts per SIMD are needed: one
// wavefront alone sustains only about one 16-byte-per-lane LDS read every 64
// cycles (measured), exactly what a 128 x 128 tile would ask of it.
// K is consumed in slices of 32 through three LDS stages and four register
// sets: in iteration t the MFMAs read stage t, slice t+2 moves from its register
// set to stage t+2, the global loads of slice t+6 are issued into the freed set
// (four iterations of MFMA work cover the HBM/L2 latency), and the first
// fragments of slice t+1 (complete since the previous barrier) are prefetched, so
// the matrix pipe waits neither for the barrier nor for memory.  LDS rows are
// padded to 80 bytes so that the 16-byte fragment reads (one row per lane) are
// bank-conflict free.  Workgroup ids are dealt round-robin to the 8 XCDs; the
// tile order gives every XCD a contiguous range of tiles in which the M-tiles
// sharing a B tile are adjacent.
#include "grass_device.h"

namespace grass {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int TM = 256, TN = 256, TK = 32;
constexpr int RS = TK + 8;                       // bf16 elements per LDS row (80 bytes)
constexpr int kStageElems = (TM + TN) * RS;      // one stage: A tile then B tile
constexpr int kStages = 3;
constexpr int kBf16Threads = 512;

struct GemmBf16Args {
    const uint16_t* A;    // M x K
    const uint16_t* B;    // N x K
    float* C;             // M x N
    uint64_t M, N, K, lda, ldb, ldc;
    uint32_t tiles_m, tiles_n;
};

struct Frags {
    bf16x8 a[4], b[2];
};

__global__ void __launch_bounds__(kBf16Threads) gemm_bf16_nt_kernel(GemmBf16Args a) {
    extern __shared__ __align__(16) uint16_t lds[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 2, wn = wave & 3;

    const uint32_t total = a.tiles_m * a.tiles_n;
    const uint32_t bid = blockIdx.x;
    uint32_t logical = bid;
    if (total % 8 == 0) logical = (bid % 8) * (total / 8) + bid / 8;
    const uint32_t tn = logical / a.tiles_m, tm = logical % a.tiles_m;
    const uint64_t m0 = (uint64_t)tm * TM, n0 = (uint64_t)tn * TN;

    // staging map: 4 lanes cover the 64 bytes of one row slice, a wavefront covers 16 rows
    constexpr int NS = 2;             // row steps per thread and operand
    const int srow = tid >> 2;        // 0..127, +128 per step
    const int skc = tid & 3;          // 16-byte chunk inside the 32-element slice
    const uint16_t* arow[NS];
    const uint16_t* brow[NS];
#pragma unroll
    for (int i = 0; i < NS; ++i) {
        uint64_t r = m0 + srow + 128 * i;
        arow[i] = a.A + (r < a.M ? r : a.M - 1) * a.lda + skc * 8;     // rows past the edge re-read the last row;
        r = n0 + srow + 128 * i;                                        // their products are never stored
        brow[i] = a.B + (r < a.N ? r : a.N - 1) * a.ldb + skc * 8;
    }

    constexpr int kSets = 4;          // register sets of global loads in flight
    u32x4 ra[kSets][NS], rb[kSets][NS];
    const uint64_t nkt = (a.K + TK - 1) / TK;
    auto fetch = [&](u32x4 (&xa)[NS], u32x4 (&xb)[NS], uint64_t slice) {
        const uint64_t k0 = slice * TK;
        const bool in_k = slice < nkt && k0 + skc * 8 < a.K;      // K is a multiple of 8: a chunk is all in or all out
#pragma unroll
        for (int i = 0; i < NS; ++i) {
            xa[i] = in_k ? *reinterpret_cast<const u32x4*>(arow[i] + k0) : u32x4(0u);
            xb[i] = in_k ? *reinterpret_cast<const u32x4*>(brow[i] + k0) : u32x4(0u);
        }
    };
    auto stash = [&](const u32x4 (&xa)[NS], const u32x4 (&xb)[NS], int stage) {
        uint16_t* sa = lds + stage * kStageElems;
        uint16_t* sb = sa + TM * RS;
#pragma unroll
        for (int i = 0; i < NS; ++i) {
            *reinterpret_cast<u32x4*>(sa + (srow + 128 * i) * RS + skc * 8) = xa[i];
            *reinterpret_cast<u32x4*>(sb + (srow + 128 * i) * RS + skc * 8) = xb[i];
        }
    };
    const int a_off = (wm * 128 + (lane & 31)) * RS + (lane >> 5) * 8;
    const int b_off = TM * RS + (wn * 64 + (lane & 31)) * RS + (lane >> 5) * 8;
    auto load_frags = [&](Frags& f, int stage, int ks) {
        const uint16_t* base = lds + stage * kStageElems + ks * 16;
#pragma unroll
        for (int i = 0; i < 4; ++i) f.a[i] = *reinterpret_cast<const bf16x8*>(base + a_off + i * 32 * RS);
#pragma unroll
        for (int j = 0; j < 2; ++j) f.b[j] = *reinterpret_cast<const bf16x8*>(base + b_off + j * 32 * RS);
    };

    f32x16 acc[4][2];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;
    auto mma = [&](const Frags& f) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.a[i], f.b[j], acc[i][j], 0, 0, 0);
    };

    // prologue: slices 0 and 1 go straight to stages 0 and 1; slices 2..5 start travelling.
    // Slice j always uses register set j % 4.
    fetch(ra[0], rb[0], 0);
    fetch(ra[1], rb[1], 1);
    stash(ra[0], rb[0], 0);
    stash(ra[1], rb[1], 1);
    fetch(ra[2], rb[2], 2);
    fetch(ra[3], rb[3], 3);
    fetch(ra[0], rb[0], 4);
    fetch(ra[1], rb[1], 5);
    __syncthreads();
    Frags f0, f1;
    load_frags(f0, 0, 0);
    int s_cur = 0, s_next = 1, s_fill = 2;
    for (uint64_t kt = 0; kt < nkt; kt += kSets) {
#pragma unroll
        for (int u = 0; u < kSets; ++u) {
            const uint64_t it = kt + u;
            if (it < nkt) {                                     // uniform
                constexpr int kDummy = 0; (void)kDummy;
                const int q = (u + 2) % kSets;                  // register set of slice it+2 (kt is a multiple of 4)
                if (it + 2 < nkt) stash(ra[q], rb[q], s_fill);  // stage last read in iteration it-1
                fetch(ra[q], rb[q], it + 2 + kSets);
                load_frags(f1, s_cur, 1);
                mma(f0);
                if (it + 1 < nkt) load_frags(f0, s_next, 0);    // complete since the previous barrier
                mma(f1);
                __syncthreads();
                const int t = s_cur; s_cur = s_next; s_next = s_fill; s_fill = t;
            }
        }
    }

    // accumulator element e of a lane: row 8*(e/4) + 4*(lane/32) + e%4, column lane%32
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const uint64_t col = n0 + wn * 64 + j * 32 + (lane & 31);
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const uint64_t row = m0 + wm * 128 + i * 32 + 8 * (e >> 2) + 4 * (lane >> 5) + (e & 3);
                if (row < a.M && col < a.N) a.C[row * a.ldc + col] = acc[i][j][e];
            }
        }
}

// ---------------------------------------------------------------------------
// Fast path (K a multiple of 64 bytes): the operands travel HBM/L2 -> LDS directly
// (global_load_lds_dwordx4: lane i of a wavefront deposits its 16 bytes at
// LDS base + 16*i), so no registers are spent on staging.  A stage holds 128
// bytes (two 64-byte slices: 64 bf16 or 32 fp32) of each of the 512 tile rows,
// and two stages of 64 KB alternate.  A wavefront load covers whole 128-byte
// lines (with 64-byte rows every line was requested twice, one iteration apart)
// and there is one barrier per 64 (32) k instead of per 32 (16): measured 4 to
// 19 % faster than four stages of 64-byte rows, depending on shape and data.
// Rows are stored unpadded; the
// 16-byte chunk kc of row r sits at position kc ^ ((r >> 1) & 7), which makes the
// fragment reads of 16 consecutive rows hit the 16 distinct 16-byte bank groups.
constexpr int kDmaStages = 2;
constexpr int kDmaStageBytes = (TM + TN) * 128;        // 64 KB

__device__ __forceinline__ void wait_vmcnt_0() { __builtin_amdgcn_s_waitcnt(0x0F70); }     // vmcnt==0, others free
__device__ __forceinline__ void wait_lgkmcnt_0() { __builtin_amdgcn_s_waitcnt(0xC07F); }   // lgkmcnt==0, others free
// Workgroup barrier without the memory fence of __syncthreads(): the fence would
// wait for every outstanding direct-to-LDS load, including the slices that are
// meant to stay in flight.  Each wavefront waits for its own loads of the slice
// that must be visible (vmcnt) before it arrives here, which is all the ordering
// the pipeline needs; the empty asm statements keep the compiler from moving LDS
// accesses across the barrier.
__device__ __forceinline__ void bare_barrier() {
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
}

// F32 = false: bf16 operands, v_mfma_f32_32x32x16_bf16, a slice is 32 elements.
// F32 = true:  fp32 operands, v_mfma_f32_32x32x2_f32, a slice is 16 elements.  The
//   LDS image is the same (64-byte rows of four 16-byte chunks); a lane's chunk
//   holds 4 consecutive k, and MFMA step e of a chunk pair uses element e of the
//   lower lanes' chunk (k = 4c + e) and of the upper lanes' chunk (k = 4c + 4 + e),
//   the same pairing for both operands.
struct GemmDmaArgs {
    const void* A;        // M x K
    const void* B;        // N x K
    float* C;             // M x N
    uint64_t M, N, K, lda, ldb, ldc;
    uint32_t tiles_m, tiles_n;
    int accumulate;       // C += instead of C =
    uint32_t splits;             // split-K: workgroup (split, tile) contracts the 128-byte groups split, split + splits,
    uint64_t split_stride_c;     //          split + 2*splits, ... of K into C + split*split_stride_c
    int lower_only;              // symmetric product: tiles strictly above the diagonal are skipped
    uint64_t m_read, n_read;     // K-major operands: columns that may be read (a multiple of 4, >= M resp. N)
    uint64_t k_rows;             // K-major operands: rows that exist (<= K); k-rows from there on count as zero
};

// AKN / BKN (fp32 only): the operand is stored K-major, A as K x M (row distance lda) and B as K x N, i.e. the
// contraction runs over the rows of a row-major matrix (G^T G, C G) and no transposed copy is needed.  Its part of a
// stage is then 32 k-rows of 256 columns (1 KB each, one load instruction per k-row); a lane takes 4 (A) or 2 (B)
// adjacent columns of one k-row per read and feeds one MFMA tile with each, so tile i of a wavefront owns the rows
// 4q + i (q = 0..31) of its 128 and tile j the columns 2q + j of its 64.  k-rows at or past K are loaded from a zero
// word, so K needs no padding for such an operand.
__device__ __align__(16) const uint32_t g_dma_zeros[4] = {0u, 0u, 0u, 0u};

// SKINNY (row-major A): for products with at most 128 (or 257 to 384) rows of A - a handful of test gradients against
// many train gradients - the square tile would spend half of its matrix work on rows that do not exist.  With a
// row-major B the same 512 stage rows split 128 : 384, i.e. a 128 x 384 tile of C with the wavefronts 2 x 4 over it,
// 64 x 96 = 2 x 3 MFMA tiles each.  With a K-major B the stage keeps the square tile's image (B's 32 k-rows of 256
// columns behind 256 row slots, of which A fills 128): a 128 x 256 tile of C, 64 x 64 per wavefront.
template <bool F32, bool AKN, bool BKN, bool SKINNY = false>
__global__ void __launch_bounds__(kBf16Threads) gemm_dma_kernel(GemmDmaArgs a) {
    static_assert(F32 || (!AKN && !BKN), "K-major operands are built for fp32 only");
    static_assert(!SKINNY || !AKN, "the tiles of 128 rows are built for a row-major A only");
    extern __shared__ __align__(16) unsigned char smem[];
    constexpr int ESZ = F32 ? 4 : 2;                 // bytes per element
    constexpr int SK = 64 / ESZ;                     // elements per slice (64-byte rows)
    constexpr int TMk = SKINNY ? 128 : TM, TNk = SKINNY ? (BKN ? 256 : 384) : TN;      // tile of C
    constexpr int WM = TMk / 2, WN = TNk / 4;        // wavefront tile
    constexpr int MI = WM / 32, NJ = WN / 32;        // MFMA tiles per wavefront
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 2, wn = wave & 3;

    // lower_only: only the tiles_m*(tiles_m+1)/2 tiles on or below the diagonal are launched, numbered row by row
    const uint32_t total = a.lower_only ? a.tiles_m * (a.tiles_m + 1) / 2 : a.tiles_m * a.tiles_n;
    const uint32_t split = blockIdx.x / total;
    const uint32_t bid = blockIdx.x - split * total;
    uint32_t logical = bid;
    if (total % 8 == 0) logical = (bid % 8) * (total / 8) + bid / 8;      // consecutive tiles stay on one XCD
    uint32_t tn, tm;
    if (a.lower_only) {
        tm = (uint32_t)((sqrtf(8.0f * (float)logical + 1.0f) - 1.0f) * 0.5f);
        while (tm * (tm + 1) / 2 > logical) --tm;
        while ((tm + 1) * (tm + 2) / 2 <= logical) ++tm;
        tn = logical - tm * (tm + 1) / 2;
    } else if (total % 256 == 0 && a.tiles_m % 8 == 0 && a.tiles_n % 4 == 0 && a.tiles_m >= 16) {
        // Tall products: the 32 tiles that run on an XCD at a time form a block of 8 x 4 tiles (12 operand tiles
        // for its L2 to hold per K group) instead of a run of 32 along M (33 operand tiles).
        const uint32_t block = logical >> 5, within = logical & 31, blocks_m = a.tiles_m / 8;
        tm = (block % blocks_m) * 8 + (within & 7);
        tn = (block / blocks_m) * 4 + (within >> 3);
    } else {
        tn = logical / a.tiles_m;
        tm = logical % a.tiles_m;
    }
    const uint64_t m0 = (uint64_t)tm * TMk, n0 = (uint64_t)tn * TNk;
    a.C += split * a.split_stride_c;

    // DMA map: a stage is 512 rows (A then B) of 128 bytes; wavefront w moves rows 64w..64w+63 with 8
    // instructions of 8 rows; lane i moves row 8j + i/8, LDS chunk position i%8 = global chunk (i%8) ^ swizzle(row).
    // In the half group that ends an odd number of slices the lanes of chunks 4..7 re-read chunks 0..3 (in
    // bounds; their LDS data is never used).
    const uint64_t nk_all = (a.K + SK - 1) / SK;   // 64-byte slices; a K that is not a multiple needs K-major operands
    // Groups of two slices = 128 bytes per row.  The K ranges of a split-K launch are interleaved group by group
    // (split s takes groups s, s + splits, ...): all workgroups walk along the rows together and touch one
    // narrow window of every row at a time, and no range boundary has to be rounded to a group.
    const uint64_t ng_all = (nk_all + 1) / 2, gstride = a.splits;
    const uint64_t ng = (ng_all - split + gstride - 1) / gstride;          // >= 1: the host keeps splits <= ng_all
    const bool half_tail = (nk_all & 1) != 0 && (ng_all - 1) % gstride == split;   // this split owns the half group
    const bool is_a = wave * 64 < TMk;           // wavefront w moves stage rows 64w .. 64w+63: the A part comes first
    const bool dma_idle = SKINNY && BKN && !is_a && wave < 4;      // 128 x 256 tile: stage rows 128..255 stay unused
    const bool kmajor = is_a ? AKN : BKN;        // uniform per wavefront
    const int wq = wave & 3;                     // K-major operands (square tile): wavefront within its operand
    const int op_row0 = is_a ? wave * 64 : wave * 64 - TMk;        // first row of this wavefront inside its operand's tile
    const unsigned char* gsrc[8];
    uint64_t gadv;                               // bytes from one group of this split to its next
    if (kmajor) {
        // instruction j moves k-row 8*wq + j of the group: 256 columns, lane i the columns 4i..4i+3
        const uint64_t lim = is_a ? a.m_read : a.n_read, ld = is_a ? a.lda : a.ldb;
        uint64_t col = (is_a ? m0 : n0) + 4 * (uint64_t)lane;
        if (col + 4 > lim) col = lim - 4;                               // columns past the edge: never stored
        const unsigned char* mat = static_cast<const unsigned char*>(is_a ? a.A : a.B) + col * 4;
#pragma unroll
        for (int j = 0; j < 8; ++j) gsrc[j] = mat + ((uint64_t)split * 32 + 8 * wq + j) * ld * 4;
        gadv = gstride * 32 * ld * 4;
    } else {
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int r = op_row0 + j * 8 + (lane >> 3);               // row of the operand's tile
            const int kc = (lane & 7) ^ ((r >> 1) & 7);
            const uint64_t row = (is_a ? m0 : n0) + r, lim = is_a ? a.M : a.N;   // rows past the edge re-read the
            gsrc[j] = static_cast<const unsigned char*>(is_a ? a.A : a.B) +       // last row; never stored
                      ((row < lim ? row : lim - 1) * (is_a ? a.lda : a.ldb)) * ESZ + kc * 16 + (uint64_t)split * 128;
        }
        gadv = gstride * 128;
    }
    const int upper = (lane >> 2) & 1;        // row-major operand: chunk >= 4 for even j, chunk < 4 for odd j
    auto dma = [&](uint64_t group, int stage) {
        if (dma_idle) return;                                                        // uniform per wavefront
        unsigned char* base = smem + stage * kDmaStageBytes + wave * 8192;
        const bool tail = half_tail && group == ng - 1;
        const uint64_t krow0 = ((uint64_t)split + group * gstride) * 32 + 8 * wq;   // K-major: first k-row of this wavefront
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const unsigned char* src;
            if (kmajor) {
                src = krow0 + j < a.k_rows ? gsrc[j] + group * gadv : reinterpret_cast<const unsigned char*>(g_dma_zeros);
            } else {
                const int back = (tail && (upper ^ (j & 1))) ? 64 : 0;
                src = gsrc[j] + group * gadv - back;
            }
            __builtin_amdgcn_global_load_lds(reinterpret_cast<const uint32_t*>(src),
                                             reinterpret_cast<uint32_t*>(base + j * 1024), 16, 0, 0);
        }
    };

    // fragment addresses.  Row-major operand: row*128 + ((2*ks + lane/32) ^ swizzle) * 16, the swizzle depends on
    // lane only; MFMA step e of k-step ks uses element e of the chunk (k = 8ks + 4*(lane/32) + e).  K-major operand:
    // k-row (8ks + 4*(lane/32) + e) * 1024 + column * 4, one read per step e.
    const int fl = (lane >> 1) & 7;
    const int a_row = (wm * WM + (lane & 31)) * 128;
    const int b_row = (TMk + wn * WN + (lane & 31)) * 128;
    const int a_kn = (4 * (lane >> 5)) * 1024 + (wm * 128 + 4 * (lane & 31)) * 4;
    const int b_kn = TM * 128 + (4 * (lane >> 5)) * 1024 + (wn * 64 + 2 * (lane & 31)) * 4;
    struct RawFrags { u32x4 a[4]; uint32_t b[4 * (SKINNY ? 3 : 2)]; };
    auto load_frags = [&](RawFrags& f, int stage, int ks) {
        const unsigned char* st = smem + stage * kDmaStageBytes;
        const unsigned char* base = st + (((2 * ks + (lane >> 5)) ^ fl) * 16);
        if constexpr (AKN) {
#pragma unroll
            for (int e = 0; e < 4; ++e) f.a[e] = *reinterpret_cast<const u32x4*>(st + a_kn + (8 * ks + e) * 1024);
        } else {
#pragma unroll
            for (int i = 0; i < MI; ++i) f.a[i] = *reinterpret_cast<const u32x4*>(base + a_row + i * 32 * 128);
        }
        if constexpr (BKN) {
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const u32x2 v = *reinterpret_cast<const u32x2*>(st + b_kn + (8 * ks + e) * 1024);
                f.b[2 * e] = v[0]; f.b[2 * e + 1] = v[1];
            }
        } else {
#pragma unroll
            for (int j = 0; j < NJ; ++j) {
                const u32x4 v = *reinterpret_cast<const u32x4*>(base + b_row + j * 32 * 128);
#pragma unroll
                for (int e = 0; e < 4; ++e) f.b[4 * j + e] = v[e];
            }
        }
    };

    f32x16 acc[MI][NJ];
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NJ; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;
    auto mma = [&](const RawFrags& f) {
#pragma unroll
        for (int i = 0; i < MI; ++i)
#pragma unroll
            for (int j = 0; j < NJ; ++j) {
                if constexpr (F32) {
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const uint32_t av = AKN ? f.a[e][i] : f.a[i][e];
                        const uint32_t bv = BKN ? f.b[2 * e + j] : f.b[4 * j + e];
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(av), __uint_as_float(bv),
                                                                         acc[i][j], 0, 0, 0);
                    }
                } else {
                    u32x4 bv;
#pragma unroll
                    for (int e = 0; e < 4; ++e) bv[e] = f.b[4 * j + e];
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, f.a[i]),
                                                                        __builtin_bit_cast(bf16x8, bv), acc[i][j],
                                                                        0, 0, 0);
                }
            }
    };

    // Two stages.  The barrier of group g sits before its last multiply step: by then every wavefront has all
    // fragments of stage g in registers (the stage may be overwritten) and its own part of group g+1 has landed
    // (the other stage may be read).  Behind it the loads of group g+2 are issued, the first fragments of group
    // g+1 are requested, and the last step of group g covers their latency.
    dma(0, 0);
    wait_vmcnt_0();
    bare_barrier();
    if (ng > 1) dma(1, 1);
    RawFrags f0, f1;
    load_frags(f0, 0, 0);
    for (uint64_t g = 0; g < ng; ++g) {
        const int cur = (int)(g & 1);
        load_frags(f1, cur, 1);
        mma(f0);
        if (!(half_tail && g == ng - 1)) {                       // uniform
            load_frags(f0, cur, 2);
            mma(f1);
            load_frags(f1, cur, 3);
            mma(f0);
        }
        wait_lgkmcnt_0();
        wait_vmcnt_0();
        bare_barrier();
        if (g + 2 < ng) dma(g + 2, cur);
        if (g + 1 < ng) load_frags(f0, cur ^ 1, 0);
        mma(f1);
    }

    // accumulator element e of a lane belongs to row 8*(e/4) + 4*(lane/32) + e%4 and column lane%32 of its MFMA tile;
    // which rows and columns of C a tile owns depends on the operand layouts (see above)
    const bool interior = m0 + TMk <= a.M && n0 + TNk <= a.N;     // uniform
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NJ; ++j) {
            const uint64_t col = BKN ? n0 + wn * WN + 2 * (lane & 31) + j : n0 + wn * WN + j * 32 + (lane & 31);
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int rit = 8 * (e >> 2) + 4 * (lane >> 5) + (e & 3);
                const uint64_t row = AKN ? m0 + wm * WM + 4 * rit + i : m0 + wm * WM + i * 32 + rit;
                if (interior && !a.accumulate) {
                    a.C[row * a.ldc + col] = acc[i][j][e];
                } else if (row < a.M && col < a.N) {
                    float* c = a.C + row * a.ldc + col;
                    *c = a.accumulate ? *c + acc[i][j][e] : acc[i][j][e];
                }
            }
        }
}

// Operands the direct-to-LDS kernel can take: whole 64-byte K slices, 16-byte aligned rows.  (A variant with
// 4-byte loads for rows of any alignment was measured at 92 TFLOP/s against 120-130 of this one, no better than the
// register-staged kernel that takes such operands, and was dropped.)
bool gemm_dma_eligible(bool f32, const void* A, const void* B, uint64_t K, uint64_t lda, uint64_t ldb) {
    const uint64_t esz = f32 ? 4 : 2, sk = 64 / esz;
    return K > 0 && K % sk == 0 && (lda * esz) % 16 == 0 && (ldb * esz) % 16 == 0 && aligned(A, 16) && aligned(B, 16);
}

// Split-K factor when there are few output tiles.  All workgroups of a launch take equally long, so it runs in rounds
// of one workgroup per CU: among the admissible numbers of K ranges (at most max_splits, at least 32 slices each)
// take the one that leaves the last round fullest, with a small penalty per range for its partial sum.
// Row-major products with few rows of A (up to 128, or 257 to 384: three tile rows of 128 instead of two of 256) take
// the 128 x 384 tile when that is less work for the chip.  One workgroup runs per CU at a time, so a launch with
// enough tiles to do without K ranges costs (rounds of 256 tiles) x (tile area): 65,536 rows of B against 300 rows of
// A are 512 square tiles = 2 rounds, but 513 tiles of 128 x 384 = 3 rounds, and the square tile wins although 41 % of
// its rows are padding.  With few tiles the K ranges fill the chip either way and the smaller padding decides.
static bool gemm_dma_skinny(uint64_t M, uint64_t N, uint64_t tile_n = 384) {
    if (!(M <= 128 || (M > 256 && M <= 384))) return false;
    const uint64_t sq = ceil_div(M, TM) * ceil_div(N, TN), sk = ceil_div(M, 128) * ceil_div(N, tile_n);
    if (sq < 128) return true;
    return ceil_div(sk, kNumCU) * (128 * tile_n) < ceil_div(sq, kNumCU) * (uint64_t)(TM * TN);
}

uint32_t gemm_dma_splits(uint64_t M, uint64_t N, uint64_t K, bool f32, uint32_t max_splits) {
    const uint64_t tiles = gemm_dma_skinny(M, N) ? ceil_div(M, 128) * ceil_div(N, 384) : ceil_div(M, TM) * ceil_div(N, TN);
    const uint64_t slices = K / (f32 ? 16 : 32);
    if (tiles == 0 || tiles >= (uint64_t)kNumCU || slices < 64) return 1;
    uint32_t best = 1;
    double best_score = -1.0;
    for (uint32_t s = 1; s <= max_splits; ++s) {
        if (s > 1 && slices / 32 < s) break;
        const uint64_t wg = tiles * s;
        const double fill = (double)wg / (double)(ceil_div(wg, kNumCU) * kNumCU);
        const double score = fill - 0.003 * s;
        if (score > best_score) { best_score = score; best = s; }
    }
    return best;
}

// Host-side launch shared by the score GEMMs and the Gaussian baseline.  Returns
// false when the operands do not qualify (K not a multiple of the slice width,
// leading dimensions or bases not 16-byte aligned); the caller then falls back.
// splits > 1 (a value from gemm_dma_splits) writes the partial product of K range
// s to partials + s*M*N (dense M x N, accumulate applies to it) instead of C.
// lower_only (A == B, M == N): only tiles on or below the diagonal are computed.
// a_kn / b_kn (fp32 only): that operand is K-major (K x M resp. K x N, row distance lda / ldb).  A K-major operand
// needs 16-byte aligned rows and base, a column count that is a multiple of 4, and takes any K; a row-major
// operand needs K in whole 64-byte slices.
static bool launch_gemm_dma_any(bool f32, bool a_kn, bool b_kn, const void* A, const void* B, float* C, uint64_t M,
                                uint64_t N, uint64_t K, uint64_t lda, uint64_t ldb, uint64_t ldc, int accumulate,
                                hipStream_t st, hipError_t* err, uint32_t splits, float* partials, int lower_only,
                                uint64_t k_rows = 0, uint64_t b_cols_avail = 0) {
    const uint64_t esz = f32 ? 4 : 2, sk = 64 / esz;
    if ((a_kn || b_kn) && !f32) return false;
    if (K == 0 || M == 0 || N == 0) return false;
    if ((lda * esz) % 16 != 0 || (ldb * esz) % 16 != 0 || !aligned(A, 16) || !aligned(B, 16)) return false;
    if ((!a_kn || !b_kn) && K % sk != 0) return false;
    // a K-major operand is read in 16-byte pieces: its column count rounded up to 4 must exist in every row
    if (k_rows == 0 || k_rows > K) k_rows = K;
    if (b_cols_avail == 0) b_cols_avail = ldb;
    const uint64_t n_read = (N + 3) / 4 * 4;
    if (a_kn && (M % 4 != 0 || lda < M)) return false;
    if (b_kn && (n_read > b_cols_avail || b_cols_avail > ldb)) return false;
    GemmDmaArgs a;
    a.A = A; a.B = B; a.C = C; a.M = M; a.N = N; a.K = K; a.lda = lda; a.ldb = ldb; a.ldc = ldc;
    a.m_read = M; a.n_read = n_read; a.k_rows = k_rows;
    a.accumulate = accumulate;
    a.lower_only = lower_only;
    const uint64_t skinny_n = b_kn ? 256 : 384;                           // a K-major B keeps the square tile's stage image
    const bool skinny = !a_kn && !lower_only && gemm_dma_skinny(M, N, skinny_n);
    a.tiles_m = (uint32_t)ceil_div(M, skinny ? 128 : TM);
    a.tiles_n = (uint32_t)ceil_div(N, skinny ? skinny_n : TN);
    const uint64_t slices = ceil_div(K, sk);
    if (splits < 1 || !partials) splits = 1;
    if (splits > ceil_div(slices, 2)) return false;                        // every split gets at least one group
    a.splits = splits;
    a.split_stride_c = 0;
    if (splits > 1) { a.C = partials; a.ldc = N; a.split_stride_c = M * N; }
    if (lower_only && a.tiles_m != a.tiles_n) return false;
    const uint64_t total = (lower_only ? (uint64_t)a.tiles_m * (a.tiles_m + 1) / 2 : (uint64_t)a.tiles_m * a.tiles_n) * splits;
    if (total == 0 || total > 0x7FFFFFFFull) return false;
    int variant = !f32 ? 0 : (a_kn ? (b_kn ? 3 : -1) : (b_kn ? 2 : 1));
    if (variant < 0) return false;                                         // K-major A with row-major B: not built
    if (skinny) variant = !f32 ? 4 : (b_kn ? 6 : 5);
    static LdsOptIn opt_in[7];
    const void* fns[7] = {reinterpret_cast<const void*>(gemm_dma_kernel<false, false, false>),
                          reinterpret_cast<const void*>(gemm_dma_kernel<true, false, false>),
                          reinterpret_cast<const void*>(gemm_dma_kernel<true, false, true>),
                          reinterpret_cast<const void*>(gemm_dma_kernel<true, true, true>),
                          reinterpret_cast<const void*>(gemm_dma_kernel<false, false, false, true>),
                          reinterpret_cast<const void*>(gemm_dma_kernel<true, false, false, true>),
                          reinterpret_cast<const void*>(gemm_dma_kernel<true, false, true, true>)};
    *err = allow_large_lds(opt_in[variant], fns[variant]);
    if (*err != hipSuccess) return true;
    const size_t lds = (size_t)kDmaStages * kDmaStageBytes;
    const dim3 grid((uint32_t)total), block(kBf16Threads);
    switch (variant) {
        case 0: hipLaunchKernelGGL((gemm_dma_kernel<false, false, false>), grid, block, lds, st, a); break;
        case 1: hipLaunchKernelGGL((gemm_dma_kernel<true, false, false>), grid, block, lds, st, a); break;
        case 2: hipLaunchKernelGGL((gemm_dma_kernel<true, false, true>), grid, block, lds, st, a); break;
        case 3: hipLaunchKernelGGL((gemm_dma_kernel<true, true, true>), grid, block, lds, st, a); break;
        case 4: hipLaunchKernelGGL((gemm_dma_kernel<false, false, false, true>), grid, block, lds, st, a); break;
        case 5: hipLaunchKernelGGL((gemm_dma_kernel<true, false, false, true>), grid, block, lds, st, a); break;
        default: hipLaunchKernelGGL((gemm_dma_kernel<true, false, true, true>), grid, block, lds, st, a); break;
    }
    *err = hipGetLastError();
    return true;
}

bool launch_gemm_dma(bool f32, const void* A, const void* B, float* C, uint64_t M, uint64_t N, uint64_t K, uint64_t lda,
                     uint64_t ldb, uint64_t ldc, int accumulate, hipStream_t st, hipError_t* err, uint32_t splits,
                     float* partials, int lower_only) {
    return launch_gemm_dma_any(f32, false, false, A, B, C, M, N, K, lda, ldb, ldc, accumulate, st, err, splits, partials,
                               lower_only);
}

// fp32 products with K-major operands: C (M x N) = A^T B for A stored K x M and B stored K x N (a_kn and b_kn), or
// C = A B for A stored M x K and B stored K x N (b_kn only).  k_rows (0 = K): rows the K-major operands really have;
// K itself may be larger when a row-major A is zero-padded to whole slices.  b_cols_avail (0 = ldb): columns that
// exist from B's base to the end of a row (B may be a column block of a wider matrix).  Same return convention as
// launch_gemm_dma.
bool launch_gemm_dma_kmajor(bool a_kn, const float* A, const float* B, float* C, uint64_t M, uint64_t N, uint64_t K,
                            uint64_t lda, uint64_t ldb, uint64_t ldc, int accumulate, hipStream_t st, hipError_t* err,
                            uint32_t splits, float* partials, int lower_only, uint64_t k_rows, uint64_t b_cols_avail) {
    return launch_gemm_dma_any(true, a_kn, true, A, B, C, M, N, K, lda, ldb, ldc, accumulate, st, err, splits, partials,
                               lower_only, k_rows, b_cols_avail);
}

// fp32 -> bf16, round to nearest even; 4 elements per thread.  Columns cols..cols_pad of dst are zero-filled.
// VEC: rows and bases are 16-byte (src) and 8-byte (dst) aligned, so a thread moves one 16-byte load and one 8-byte
// store (non-temporal: the source is read once).
__device__ __forceinline__ uint16_t bf16_rne_bits(uint32_t u) {
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (uint16_t)((u >> 16) | 0x40u);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}
template <bool VEC>
__global__ void __launch_bounds__(256) to_bf16_kernel(const float* src, uint64_t rows, uint64_t cols, uint64_t cols_pad,
                                                      uint64_t ld_src, uint16_t* dst, uint64_t ld_dst) {
    const uint64_t quads = (cols_pad + 3) / 4;
    const uint64_t t = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= rows * quads) return;
    const uint64_t r = t / quads, c0 = (t - r * quads) * 4;
    if (VEC && c0 + 4 <= cols) {
        const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(src + r * ld_src + c0));
        u32x2 o;
        o[0] = (uint32_t)bf16_rne_bits(v[0]) | ((uint32_t)bf16_rne_bits(v[1]) << 16);
        o[1] = (uint32_t)bf16_rne_bits(v[2]) | ((uint32_t)bf16_rne_bits(v[3]) << 16);
        *reinterpret_cast<u32x2*>(dst + r * ld_dst + c0) = o;
        return;
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        if (c0 + j < cols) dst[r * ld_dst + c0 + j] = bf16_rne_bits(__float_as_uint(src[r * ld_src + c0 + j]));
        else if (c0 + j < cols_pad) dst[r * ld_dst + c0 + j] = 0;
    }
}

// dst (rows x ld_dst bf16) = src rounded to nearest even, zero-padded up to cols_pad columns.
hipError_t convert_to_bf16(const float* src, uint64_t rows, uint64_t cols, uint64_t cols_pad, uint64_t ld_src, uint16_t* dst,
                           uint64_t ld_dst, hipStream_t st) {
    const uint64_t total = rows * ((cols_pad + 3) / 4);
    if (total == 0) return hipSuccess;
    if (ceil_div(total, 256) > 0x7FFFFFFFull) return hipErrorInvalidValue;
    const bool vec = aligned(src, 16) && ld_src % 4 == 0 && aligned(dst, 8) && ld_dst % 4 == 0;
    if (vec)
        hipLaunchKernelGGL(to_bf16_kernel<true>, dim3((uint32_t)ceil_div(total, 256)), dim3(256), 0, st, src, rows, cols,
                           cols_pad, ld_src, dst, ld_dst);
    else
        hipLaunchKernelGGL(to_bf16_kernel<false>, dim3((uint32_t)ceil_div(total, 256)), dim3(256), 0, st, src, rows, cols,
                           cols_pad, ld_src, dst, ld_dst);
    return hipGetLastError();
}

}  // namespace grass

using namespace grass;

extern "C" grass_status grass_to_bf16(const float* src, uint64_t rows, uint64_t cols, uint64_t ld_src, void* dst,
                                      uint64_t ld_dst, grass_stream stream) {
    if (cols == 0) return GRASS_EINVAL;
    if (rows == 0) return GRASS_OK;
    if (!src || !dst || ld_src < cols || ld_dst < cols) return GRASS_EINVAL;
    if (ceil_div(rows * ((cols + 3) / 4), 256) > 0x7FFFFFFFull) return GRASS_EUNSUPPORTED;
    return convert_to_bf16(src, rows, cols, cols, ld_src, static_cast<uint16_t*>(dst), ld_dst, as_stream(stream)) == hipSuccess
               ? GRASS_OK : GRASS_EHIP;
}

extern "C" grass_status grass_score_bf16(const void* train, const void* test, uint64_t N, uint64_t M, uint64_t K,
                                         uint64_t ld_train, uint64_t ld_test, float* scores, uint64_t ld_scores,
                                         grass_stream stream) {
    if (K == 0) return GRASS_EINVAL;
    if (N == 0 || M == 0) return GRASS_OK;
    if (!train || !test || !scores || ld_train < K || ld_test < K || ld_scores < N) return GRASS_EINVAL;
    // 16-byte chunks: K and the leading dimensions in multiples of 8 elements, 16-byte aligned bases
    if (K % 8 != 0 || ld_train % 8 != 0 || ld_test % 8 != 0 || !aligned(train, 16) || !aligned(test, 16))
        return GRASS_EUNSUPPORTED;
    GemmBf16Args a;
    a.A = static_cast<const uint16_t*>(test);
    a.B = static_cast<const uint16_t*>(train);
    a.C = scores;
    a.M = M; a.N = N; a.K = K; a.lda = ld_test; a.ldb = ld_train; a.ldc = ld_scores;
    a.tiles_m = (uint32_t)ceil_div(M, TM);
    a.tiles_n = (uint32_t)ceil_div(N, TN);
    const uint64_t total = (uint64_t)a.tiles_m * a.tiles_n;
    if (total > 0x7FFFFFFFull) return GRASS_EUNSUPPORTED;
    static LdsOptIn opt_in;
    const size_t lds_bytes = (size_t)kStages * kStageElems * sizeof(uint16_t);
    if (allow_large_lds(opt_in, reinterpret_cast<const void*>(gemm_bf16_nt_kernel)) != hipSuccess) return GRASS_EHIP;
    hipError_t derr = hipSuccess;
    if (launch_gemm_dma(false, test, train, scores, M, N, K, ld_test, ld_train, ld_scores, 0, as_stream(stream), &derr, 1,
                        nullptr, 0))
        return derr == hipSuccess ? GRASS_OK : GRASS_EHIP;
    hipLaunchKernelGGL(gemm_bf16_nt_kernel, dim3((uint32_t)total), dim3(kBf16Threads), lds_bytes, as_stream(stream), a);
    return launch_status();
}
