// SJLT and fused GraSS (mask + SJLT) kernels.
//
// Sec. 3.1: SJLT scans the input and lets every coordinate add itself to, or
// subtract itself from, s output coordinates.  Sec. 3.3.1: GraSS applies the
// same scan to the masked sub-vector g[idx].
//
// Mapping to the GPU: a workgroup owns R rows (samples) and one contiguous
// chunk of the SJLT's input positions.  In the fused case the rows are
// consecutive.  In the unmasked case they are row0 + q*P with P the period after
// which row start addresses repeat modulo 128 bytes (P = 32 / gcd(ld mod 32, 32)
// rows of fp32): all R rows then share one alignment, the vector loop starts on
// a 128-byte line and every 16-byte load and every wavefront's 1 KB of loads
// covers whole lines.  With consecutive rows of an odd-sized matrix each
// wavefront load straddles a line that its neighbour fetches again (streaming
// loads are not retained in L2): measured +20 % HBM reads on 11,173,962 columns.  It keeps an R x k accumulator
// in LDS (row-major: for a fixed row, random buckets spread evenly over the LDS
// banks; a bucket-major layout would confine each row to 1/R of the banks).
// A thread reads the same V consecutive positions of all R
// rows (coalesced 4V-byte loads; a gather through idx in the fused case),
// evaluates the hash of each position once in registers and reuses bucket and
// sign for the R rows.  Exact zeros are skipped (the sparsity of per-sample
// gradients reduces LDS traffic, not HBM traffic).  If the input positions are
// split over several chunks the per-chunk partial rows go to the workspace and
// a second kernel adds them in a fixed order; no global atomics anywhere.
//
// How a value is added to its LDS bucket is a template policy, because on
// gfx950 the native fp32 LDS atomic add retires about one lane every three
// cycles per CU, an order of magnitude below the other LDS operations:
//   ACC_F64: fp64 accumulators updated with the fp64 LDS atomic add (fast,
//            order-insensitive to well below fp32 resolution, half as many rows
//            fit in LDS);
//   ACC_CAS: fp32 accumulators updated with a compare-and-swap loop.
#include <cstdio>
#include <mutex>

#include "grass_device.h"

namespace grass {

// Scratch memory of grass_sjlt_noalloc: partial sums of the column chunks and, when it fits behind them, the
// transient (bucket, sign) table.  One copy per GPU inside the loaded code object, held until the process ends.
// In host code the array's name is only a handle for hipGetSymbolAddress; kernels and copies get the address that
// call returns for the current device.
static __device__ __align__(256) unsigned char scratch[GRASS_NOALLOC_SCRATCH_BYTES];

enum { ACC_CAS = 2, ACC_F64 = 3 };
template <int ACC> struct AccT { using type = float; };
template <> struct AccT<ACC_F64> { using type = double; };

struct SjltArgs {
    const void* g;        // fp32 or bf16 words, see the kernel's element type
    const int32_t* idx;   // nullptr: positions are columns
    float* dst;           // out (direct) or partial workspace
    uint64_t ldg;
    uint64_t n;
    uint64_t d;           // number of SJLT input positions (p or k')
    uint64_t ld_dst;      // row distance in dst
    uint64_t chunk_stride;  // elements between consecutive chunks in dst (0 when direct)
    uint64_t pos_per_chunk;
    uint64_t sub;         // sub-seed of the SJLT stream
    uint32_t k, s, m;
    uint32_t shift;       // 32 - log2(m) when m is a power of two >= 2
    float scale;          // applied when writing directly
    const uint16_t* table;  // MODE_TABLE: bucket | sign << 15 of every position (s == 1)
    uint32_t row_period;  // P: the rows of a workgroup are first + q*P (1 = consecutive rows)
    uint32_t align_lines; // unmasked, V == 4: start the vector loop on a 128-byte line
};

template <int ACC>
__device__ __forceinline__ void lds_add(typename AccT<ACC>::type* addr, float v) {
    if constexpr (ACC == ACC_F64) {
        __hip_atomic_fetch_add(addr, (double)v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    } else {
        uint32_t* p = reinterpret_cast<uint32_t*>(addr);
        uint32_t old = *reinterpret_cast<volatile uint32_t*>(p), assumed;
        do {
            assumed = old;
            old = atomicCAS(p, assumed, __float_as_uint(__uint_as_float(assumed) + v));
        } while (old != assumed);
    }
}

// Adds the R values of one input position to their buckets.  z is the generator
// state of the position's first non-zero, i.e. sub + (pos*s + 1)*gamma.
// How bucket and sign of a position are obtained:
//   MODE_GENERAL  hash per non-zero, bucket by multiply-high (any s, any m);
//   MODE_FAST     s == 1 and m a power of two >= 2: bucket by shift, no loop over s;
//   MODE_TABLE    s == 1, unmasked, line-aligned rows: read from a table of 16-bit entries that the call builds first
//                 (11 million positions cost 22 MB and a few microseconds).  Every row group re-evaluates the same p
//                 hashes otherwise, and with 8 quarter-rate integer multiplies each they were 12 % of the launch
//                 on the ResNet-scale input; the table is shared through L2 by the workgroups of an XCD.
enum { MODE_GENERAL = 0, MODE_FAST = 1, MODE_TABLE = 2 };
template <int R, int ACC, int MODE>
__device__ __forceinline__ void scatter_position(typename AccT<ACC>::type* acc, const float (&v)[R], uint64_t z,
                                                 const SjltArgs& a) {
    bool any = false;
#pragma unroll
    for (int r = 0; r < R; ++r) any |= (v[r] != 0.0f);
    if (!any) return;
    if constexpr (MODE == MODE_FAST) {
        const uint64_t h = finalise(z);
        const uint32_t b = (uint32_t)(h >> 32) >> a.shift;
        const uint32_t sg = signbit_of(h);
        typename AccT<ACC>::type* slot = acc + b;
#pragma unroll
        for (int r = 0; r < R; ++r) {
            if (v[r] != 0.0f) lds_add<ACC>(slot + (uint32_t)r * a.k, __uint_as_float(__float_as_uint(v[r]) ^ sg));
        }
    } else {
        for (uint32_t rr = 0; rr < a.s; ++rr, z += kGamma) {
            const uint64_t h = finalise(z);
            const uint32_t b = rr * a.m + bucket_of(h, a.m);
            const uint32_t sg = signbit_of(h);
            typename AccT<ACC>::type* slot = acc + b;
#pragma unroll
            for (int r = 0; r < R; ++r) {
                if (v[r] != 0.0f) lds_add<ACC>(slot + (uint32_t)r * a.k, __uint_as_float(__float_as_uint(v[r]) ^ sg));
            }
        }
    }
}

// The same with bucket and sign taken from a table entry.
template <int R, int ACC>
__device__ __forceinline__ void scatter_entry(typename AccT<ACC>::type* acc, const float (&v)[R], uint32_t e,
                                              const SjltArgs& a) {
    typename AccT<ACC>::type* slot = acc + (e & 0x7FFFu);
    const uint32_t sg = (e >> 15) << 31;
#pragma unroll
    for (int r = 0; r < R; ++r) {
        if (v[r] != 0.0f) lds_add<ACC>(slot + (uint32_t)r * a.k, __uint_as_float(__float_as_uint(v[r]) ^ sg));
    }
}

// Input element types: fp32, or bf16 handed over as raw 16-bit words (exact in fp32: the word is the upper half).
template <typename T> struct Elem;
template <> struct Elem<float> {
    static constexpr uint32_t per_line = 32;                       // elements per 128-byte line
    static __device__ __forceinline__ float f(float v) { return v; }
};
template <> struct Elem<uint16_t> {
    static constexpr uint32_t per_line = 64;
    static __device__ __forceinline__ float f(uint16_t v) { return __uint_as_float((uint32_t)v << 16); }
};
template <typename T, int V> struct VecT { typedef T type __attribute__((ext_vector_type(V))); };
template <typename T> struct VecT<T, 1> { using type = T; };

// V consecutive table entries; only the alignment of one entry may be assumed of its address.
template <int V> struct alignas(2) TableVec { uint16_t e[V]; };

template <typename T, int V>
__device__ __forceinline__ void unpack(const typename VecT<T, V>::type& x, float* o) {
    if constexpr (V == 1) {
        o[0] = Elem<T>::f(x);
    } else {
#pragma unroll
        for (int i = 0; i < V; ++i) o[i] = Elem<T>::f(x[i]);
    }
}

// The gradient matrix is read exactly once: non-temporal loads keep it from
// displacing anything in the caches and sustain a higher HBM rate.
template <typename T>
__device__ __forceinline__ T stream_load(const T* p) { return __builtin_nontemporal_load(p); }

// R rows per workgroup, V positions per load (unmasked only), U loads in flight
// per row and thread.
template <typename T, int R, int V, int U, bool MASKED, int ACC, int MODE>
__global__ void __launch_bounds__(1024) sjlt_kernel(SjltArgs a) {
    constexpr int HMODE = MODE == MODE_TABLE ? MODE_GENERAL : MODE;   // hash path of the few scalar positions
    using acc_t = typename AccT<ACC>::type;
    extern __shared__ __align__(16) unsigned char smem[];
    acc_t* acc = reinterpret_cast<acc_t*>(smem);
    const uint32_t nt = blockDim.x;
    // rows of this workgroup: blocks of P*R rows, group (blockIdx.x % P) of a block takes every P-th row
    const uint64_t P = a.row_period;
    const uint64_t row0 = ((uint64_t)blockIdx.x / P) * (P * R) + (uint64_t)blockIdx.x % P;
    if (row0 >= a.n) return;                                  // uniform: a group past the last row
    int nrows = 0;
#pragma unroll
    for (int r = 0; r < R; ++r) nrows += (row0 + (uint64_t)r * P < a.n) ? 1 : 0;      // valid rows are the first nrows
    for (uint32_t t = threadIdx.x; t < (uint32_t)R * a.k; t += nt) acc[t] = (acc_t)0;
    __syncthreads();

    const uint64_t begin = (uint64_t)blockIdx.y * a.pos_per_chunk;
    const uint64_t end = (begin + a.pos_per_chunk < a.d) ? begin + a.pos_per_chunk : a.d;
    const T* rowp[R];
#pragma unroll
    for (int r = 0; r < R; ++r)
        rowp[r] = static_cast<const T*>(a.g) + (row0 + (r < nrows ? (uint64_t)r * P : 0)) * a.ldg;

    const uint64_t zpos = (uint64_t)a.s * kGamma;             // generator-state distance between positions

    if constexpr (MASKED) {
        // one position per thread and step; U steps in flight
        const uint64_t zstep = zpos * nt;
        uint64_t base = begin + threadIdx.x;
        uint64_t z = a.sub + (base * a.s + 1) * kGamma;
        for (; base < end; base += (uint64_t)nt * U, z += zstep * U) {
            int32_t col[U];
            float v[U][R];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const uint64_t pos = base + (uint64_t)u * nt;
                col[u] = pos < end ? a.idx[pos] : -1;
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
#pragma unroll
                for (int r = 0; r < R; ++r)
                    v[u][r] = (col[u] >= 0 && r < nrows) ? Elem<T>::f(stream_load(rowp[r] + col[u])) : 0.0f;
            }
#pragma unroll
            for (int u = 0; u < U; ++u) scatter_position<R, ACC, HMODE>(acc, v[u], z + zstep * u, a);
        }
    } else {
        using VT = typename VecT<T, V>::type;
        constexpr uint32_t E = Elem<T>::per_line;
        // vector range [vbeg, vend): the chunk shifted to the first 128-byte line of these rows
        uint64_t lead = 0;
        if (a.align_lines) lead = (E - (uint32_t)((reinterpret_cast<uintptr_t>(rowp[0]) / sizeof(T)) & (E - 1))) & (E - 1);
        const uint64_t vbeg = begin + lead < a.d ? begin + lead : a.d;
        const uint64_t vend = end + lead < a.d ? end + lead : a.d;          // the last chunk has end == d
        if (blockIdx.y == 0 && threadIdx.x < lead && threadIdx.x < a.d) {   // fewer than a line of leading positions
            float v[R];
#pragma unroll
            for (int r = 0; r < R; ++r) v[r] = r < nrows ? Elem<T>::f(rowp[r][threadIdx.x]) : 0.0f;
            scatter_position<R, ACC, HMODE>(acc, v, a.sub + ((uint64_t)threadIdx.x * a.s + 1) * kGamma, a);
        }
        const uint64_t nvec = (vend - vbeg) / V;
        const uint64_t zstep = zpos * V * nt;
        uint64_t vb = threadIdx.x;
        uint64_t z = a.sub + ((vbeg + vb * V) * a.s + 1) * kGamma;
        for (; vb < nvec; vb += (uint64_t)nt * U, z += zstep * U) {
            VT x[U][R];
            TableVec<V> te[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const uint64_t vi = vb + (uint64_t)u * nt;
#pragma unroll
                for (int r = 0; r < R; ++r) {
                    if (vi < nvec && r < nrows)
                        x[u][r] = stream_load(reinterpret_cast<const VT*>(rowp[r] + vbeg + vi * V));
                    else
                        x[u][r] = VT{};
                }
                if constexpr (MODE == MODE_TABLE) {
                    // the vector loop starts on a line of g, which is any position of the table: 2-byte aligned only
                    te[u] = vi < nvec ? *reinterpret_cast<const TableVec<V>*>(a.table + vbeg + vi * V) : TableVec<V>{};
                }
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                float e[R][V];
#pragma unroll
                for (int r = 0; r < R; ++r) unpack<T, V>(x[u][r], e[r]);
#pragma unroll
                for (int c = 0; c < V; ++c) {
                    float v[R];
#pragma unroll
                    for (int r = 0; r < R; ++r) v[r] = e[r][c];
                    if constexpr (MODE == MODE_TABLE) {
                        scatter_entry<R, ACC>(acc, v, te[u].e[c], a);
                    } else {
                        scatter_position<R, ACC, MODE>(acc, v, z + zstep * u + zpos * c, a);   // all-zero past nvec: skipped
                    }
                }
            }
        }
        // ragged tail of fewer than V positions
        const uint64_t tail = vbeg + nvec * V + threadIdx.x;
        if (tail < vend) {
            float v[R];
#pragma unroll
            for (int r = 0; r < R; ++r) v[r] = r < nrows ? Elem<T>::f(rowp[r][tail]) : 0.0f;
            scatter_position<R, ACC, HMODE>(acc, v, a.sub + (tail * a.s + 1) * kGamma, a);
        }
    }
    __syncthreads();

    float* dst = a.dst + (uint64_t)blockIdx.y * a.chunk_stride;
    for (int r = 0; r < nrows; ++r) {
        float* o = dst + (row0 + (uint64_t)r * P) * a.ld_dst;
        for (uint32_t b = threadIdx.x; b < a.k; b += nt) o[b] = (float)acc[(uint32_t)r * a.k + b] * a.scale;
    }
}

// table[j] = bucket | sign << 15 of position j (s == 1, m = k <= 32768).
__global__ void __launch_bounds__(256) sjlt_table_kernel(uint64_t sub, uint64_t d, uint32_t m, uint16_t* table) {
    const uint64_t j = (uint64_t)blockIdx.x * 256 + threadIdx.x;
    if (j >= d) return;
    const uint64_t h = sm(sub, j);
    table[j] = (uint16_t)(bucket_of(h, m) | (signbit_of(h) ? 0x8000u : 0u));
}

struct SjltPlan {
    int R, V, threads, acc;
    uint32_t row_period;      // P of the kernel's row mapping
    bool align_lines;
    bool table;               // bucket/sign table in the workspace behind the partial sums (optional)
    size_t table_offset, table_bytes;
    uint32_t chunks;
    uint64_t pos_per_chunk;
    size_t lds_bytes;
    size_t ws_bytes;
};

// force_v != 0 (workspace query, where the alignment of g is unknown): consecutive rows and that vector width;
// consecutive rows give the fewest row groups and so the most chunks, an upper bound for every layout.
// in_bytes: 4 (fp32 input) or 2 (bf16 input).
static bool plan_sjlt(uint64_t n, uint64_t d, bool masked, uint32_t k, const void* g, uint64_t ldg,
                      SjltPlan* pl, int force_v, uint32_t in_bytes, uint32_t s, const grass_tuning* tune) {
    // launch-shape overrides of this call (experiments); zero = heuristic
    const int tune_rows = tune ? tune->sjlt_rows_per_block : 0;
    const int tune_chunks = tune ? tune->sjlt_column_chunks : 0;
    const int tune_threads = tune ? tune->sjlt_threads : 0;
    const int tune_acc = tune ? tune->sjlt_accumulator : 0;
    if ((size_t)k * 4 > 128 * 1024) return false;
    int acc = ACC_F64;
    if ((size_t)k * 8 > 128 * 1024) acc = ACC_CAS;            // fp64 buckets of one row no longer fit
    if ((tune_acc == ACC_CAS || tune_acc == ACC_F64) && (size_t)k * (tune_acc == ACC_F64 ? 8 : 4) <= 128 * 1024)
        acc = tune_acc;
    const size_t esz = acc == ACC_F64 ? 8 : 4;
    int R = 8;
    while (R > 1 && (size_t)R * k * esz > 128 * 1024) R >>= 1;
    // no point holding more rows than there are samples
    while (R > 1 && (uint64_t)R > n) R >>= 1;
    // short rows (a few iterations of one workgroup): the launch is latency-bound, so one chunk (no second
    // kernel for the partial sums) and fewer rows per workgroup until there are 32 workgroups
    const bool short_rows = d <= 32768;
    if (short_rows) while (R > 1 && ceil_div(n, R) < 32) R >>= 1;
    // long masked rows are bound by the gather (one 128-byte line per kept coordinate): up to a few hundred rows,
    // one workgroup per CU matters more than sharing the hash of a position between the rows of a workgroup
    if (masked && !short_rows) while (R > 1 && ceil_div(n, R) < (uint64_t)kNumCU) R >>= 1;
    if (tune_rows == 1 || tune_rows == 2 || tune_rows == 4 || tune_rows == 8) {
        if ((size_t)tune_rows * k * esz <= kLdsBytes) R = tune_rows;
    }
    int threads = 1024;
    if ((size_t)R * k * esz <= 64 * 1024) threads = 512;      // two or more groups per CU anyway
    if (short_rows && ceil_div(n, R) <= (uint64_t)kNumCU) threads = 1024;   // one workgroup per CU at most: widest
    if (tune_threads == 256 || tune_threads == 512 || tune_threads == 1024) threads = tune_threads;
    int V = 1;
    uint32_t P = 1;
    bool align_lines = false;
    if (!masked && force_v != 0) {
        V = force_v;
    } else if (!masked) {
        // rows P apart start at the same offset inside a 128-byte line; group them if there are enough rows
        const uint32_t E = 128 / in_bytes, vmax = 16 / in_bytes;   // elements per line, per 16-byte load
        uint32_t rem = (uint32_t)(ldg % E), gcd = E;
        while (rem % gcd != 0) gcd >>= 1;                     // gcd(ld mod E, E); E when ld mod E == 0
        const uint32_t period = E / gcd;
        if (period == 1 || n >= 4ull * period * R) {
            P = period; V = (int)vmax; align_lines = true;
        } else if (aligned(g, 16) && ldg % vmax == 0) V = (int)vmax;
        else if (in_bytes == 4 && aligned(g, 8) && ldg % 2 == 0) V = 2;
    }
    const uint64_t row_groups = ceil_div(n, (uint64_t)P * R) * P;
    // chunks: enough workgroups to fill the chip, but keep the partial-sum
    // traffic (2 * chunks * n * k * 4 bytes) small against the input traffic.
    const uint64_t step = (uint64_t)threads * V * 2;
    uint64_t max_chunks_work = d / (step * 2);
    if (max_chunks_work < 1) max_chunks_work = 1;
    uint64_t max_chunks_traffic = (d * (masked ? 8 : 1)) / (8ull * k);
    if (max_chunks_traffic < 1) max_chunks_traffic = 1;
    // unmasked: four rounds of workgroups even out the tail, but no more than 16 chunks of partial sums per row
    // unless it takes more to give every CU one workgroup (measured for n = 1 ... 1,024 at p = 11 million)
    uint64_t chunks = ceil_div(4 * kNumCU, row_groups);
    if (chunks > 16) chunks = 16;
    if (chunks < ceil_div(kNumCU, row_groups)) chunks = ceil_div(kNumCU, row_groups);
    if (chunks > 128) chunks = 128;
    if (masked) {                                             // gather-bound: fill the chip once; every further chunk
        chunks = ceil_div(kNumCU, row_groups);                // only adds partial sums (measured for n = 4 ... 2,048)
        if (chunks > 16) chunks = 16;
    }
    if (chunks > max_chunks_work) chunks = max_chunks_work;
    if (chunks > max_chunks_traffic) chunks = max_chunks_traffic;
    if (short_rows) chunks = 1;
    if (tune_chunks > 0) chunks = tune_chunks;
    if (chunks > 65535) chunks = 65535;
    uint64_t ppc = ceil_div(d, chunks);
    ppc = ceil_div(ppc, step) * step;             // keeps chunk starts V-aligned
    chunks = ceil_div(d, ppc);
    if (chunks < 1) chunks = 1;
    pl->R = R; pl->V = V; pl->threads = threads; pl->acc = acc;
    pl->row_period = P; pl->align_lines = align_lines;
    pl->chunks = (uint32_t)chunks;
    pl->pos_per_chunk = ppc;
    pl->lds_bytes = (size_t)R * k * esz;
    pl->ws_bytes = chunks > 1 ? (size_t)chunks * n * k * 4 : 0;
    // the table pays when many row groups would repeat the same hashes over a long row.  Its conditions do not depend
    // on the alignment of g, so that the workspace query (which does not know it) reserves the room; a call whose
    // rows are not grouped by line offset, or whose workspace has no room for it, hashes as before.
    pl->table = !masked && s == 1 && acc == ACC_F64 && k <= 32768 && d >= 65536 && ceil_div(n, R) >= 16;
    pl->table_offset = (pl->ws_bytes + 255) / 256 * 256;
    pl->table_bytes = pl->table ? d * sizeof(uint16_t) : 0;
    if (!align_lines && force_v == 0) pl->table = false;
    return true;
}

template <typename T, int R, int V, int U, bool MASKED, int ACC, int MODE>
static hipError_t launch_one(const SjltArgs& a, const SjltPlan& pl, hipStream_t st) {
    auto kern = sjlt_kernel<T, R, V, U, MASKED, ACC, MODE>;
    static LdsOptIn opt_in;
    const hipError_t e = allow_large_lds(opt_in, reinterpret_cast<const void*>(kern));
    if (e != hipSuccess) return e;
    dim3 grid((uint32_t)(ceil_div(a.n, (uint64_t)pl.row_period * R) * pl.row_period), pl.chunks);
    hipLaunchKernelGGL(kern, grid, dim3(pl.threads), pl.lds_bytes, st, a);
    return hipGetLastError();
}

template <typename T, int R, int ACC, int MODE>
static hipError_t launch_raf(const SjltArgs& a, const SjltPlan& pl, bool masked, hipStream_t st) {
    constexpr int VMAX = 16 / sizeof(T);
    if constexpr (MODE == MODE_TABLE) {
        return launch_one<T, R, VMAX, (R >= 8 ? 1 : 2), false, ACC, MODE>(a, pl, st);   // the plan guarantees V == VMAX
    } else {
        if (masked) return launch_one<T, R, 1, (R >= 8 ? 2 : 4), true, ACC, MODE>(a, pl, st);
        if (pl.V == VMAX) return launch_one<T, R, VMAX, (R >= 8 ? 1 : 2), false, ACC, MODE>(a, pl, st);
        if constexpr (sizeof(T) == 4) {
            if (pl.V == 2) return launch_one<T, R, 2, (R >= 8 ? 2 : 4), false, ACC, MODE>(a, pl, st);
        }
        return launch_one<T, R, 1, (R >= 8 ? 2 : 4), false, ACC, MODE>(a, pl, st);
    }
}

template <typename T, int R>
static hipError_t launch_r(const SjltArgs& a, const SjltPlan& pl, bool masked, int mode, hipStream_t st) {
    if (mode == MODE_TABLE) return launch_raf<T, R, ACC_F64, MODE_TABLE>(a, pl, masked, st);
    if (pl.acc == ACC_CAS)
        return mode == MODE_FAST ? launch_raf<T, R, ACC_CAS, MODE_FAST>(a, pl, masked, st)
                                 : launch_raf<T, R, ACC_CAS, MODE_GENERAL>(a, pl, masked, st);
    return mode == MODE_FAST ? launch_raf<T, R, ACC_F64, MODE_FAST>(a, pl, masked, st)
                             : launch_raf<T, R, ACC_F64, MODE_GENERAL>(a, pl, masked, st);
}

template <typename T>
static hipError_t launch_t(const SjltArgs& a, const SjltPlan& pl, bool masked, int mode, hipStream_t st) {
    switch (pl.R) {
        case 8: return launch_r<T, 8>(a, pl, masked, mode, st);
        case 4: return launch_r<T, 4>(a, pl, masked, mode, st);
        case 2: return launch_r<T, 2>(a, pl, masked, mode, st);
        default: return launch_r<T, 1>(a, pl, masked, mode, st);
    }
}

}  // namespace grass

using namespace grass;

static grass_status check_sjlt_dims(uint64_t n, uint64_t p, bool masked, uint32_t kprime, uint32_t k, uint32_t s) {
    (void)n;
    if (p == 0 || p >= (1ull << 31)) return GRASS_EINVAL;
    if (k == 0 || s == 0 || k % s != 0) return GRASS_EINVAL;
    if (masked && (kprime == 0 || kprime > p)) return GRASS_EINVAL;
    if (k > GRASS_MAX_K) return GRASS_EUNSUPPORTED;
    return GRASS_OK;
}

extern "C" grass_status grass_sjlt_workspace_bytes(uint64_t n, uint64_t p, uint32_t kprime_or_0, uint32_t k,
                                                   uint32_t s, const grass_tuning* host_tuning, size_t* host_bytes) {
    if (!host_bytes) return GRASS_EINVAL;
    const bool masked = kprime_or_0 != 0;
    grass_status st = check_sjlt_dims(n, p, masked, kprime_or_0, k, s);
    if (st != GRASS_OK) return st;
    if (n == 0) { *host_bytes = 0; return GRASS_OK; }
    // the vector width depends on the alignment of g, which is unknown here: chunking
    // uses the widest step, so take the largest chunk count any width can give.
    size_t worst = 0;
    for (int v = 1; v <= 4; v *= 2) {
        SjltPlan pl;
        if (!plan_sjlt(n, masked ? kprime_or_0 : p, masked, k, nullptr, 0, &pl, v, 4, s, host_tuning)) return GRASS_EUNSUPPORTED;
        const size_t need = pl.table ? pl.table_offset + pl.table_bytes : pl.ws_bytes;
        if (need > worst) worst = need;
    }
    *host_bytes = worst;
    return GRASS_OK;
}

static grass_status run_sjlt(const void* g, uint32_t in_bytes, uint64_t n, uint64_t p, uint64_t ldg, const int32_t* idx,
                             uint32_t kprime, uint32_t k, uint32_t s, uint64_t seed, uint64_t stream_id, float* out,
                             uint64_t ldo, void* ws, size_t ws_bytes, const grass_tuning* tune, grass_stream stream) {
    const bool masked = idx != nullptr;
    grass_status st = check_sjlt_dims(n, p, masked, kprime, k, s);
    if (st != GRASS_OK) return st;
    if (n == 0) return GRASS_OK;
    if (!g || !out || ldg < p || ldo < k || !aligned(g, in_bytes) || !aligned(out, 4)) return GRASS_EINVAL;
    if (n * ldg >= (1ull << 62)) return GRASS_EINVAL;
    const uint64_t d = masked ? kprime : p;
    SjltPlan pl;
    if (!plan_sjlt(n, d, masked, k, g, ldg, &pl, 0, in_bytes, s, tune)) return GRASS_EUNSUPPORTED;
    if (pl.ws_bytes > 0 && (!ws || ws_bytes < pl.ws_bytes || !aligned(ws, 256))) return GRASS_EWORKSPACE;

    SjltArgs a;
    a.g = g; a.idx = idx; a.ldg = ldg; a.n = n; a.d = d;
    a.k = k; a.s = s; a.m = k / s;
    a.shift = 0;
    int mode = MODE_GENERAL;
    if (s == 1 && a.m >= 2 && (a.m & (a.m - 1)) == 0) {
        uint32_t lg = 0;
        while ((1u << lg) < a.m) ++lg;
        a.shift = 32 - lg;
        mode = MODE_FAST;
    }
    a.sub = substream(seed, stream_id);
    a.table = nullptr;
    hipStream_t hs = as_stream(stream);
    if (pl.table && ws && aligned(ws, 256) && ws_bytes >= pl.table_offset + pl.table_bytes) {
        uint16_t* table = reinterpret_cast<uint16_t*>(static_cast<char*>(ws) + pl.table_offset);
        hipLaunchKernelGGL(sjlt_table_kernel, dim3((uint32_t)ceil_div(d, 256)), dim3(256), 0, hs, a.sub, d, a.m, table);
        if (hipGetLastError() != hipSuccess) return GRASS_EHIP;
        a.table = table;
        mode = MODE_TABLE;
    }
    a.pos_per_chunk = pl.pos_per_chunk;
    a.row_period = pl.row_period;
    a.align_lines = pl.align_lines ? 1u : 0u;
    const float scale = 1.0f / sqrtf((float)s);
    if (pl.chunks == 1) {
        a.dst = out; a.ld_dst = ldo; a.chunk_stride = 0; a.scale = scale;
    } else {
        a.dst = static_cast<float*>(ws); a.ld_dst = k; a.chunk_stride = n * k; a.scale = 1.0f;
    }
    const hipError_t e = in_bytes == 4 ? launch_t<float>(a, pl, masked, mode, hs) : launch_t<uint16_t>(a, pl, masked, mode, hs);
    if (e != hipSuccess) return GRASS_EHIP;
    if (pl.chunks > 1) {
        const uint64_t total = n * k;
        hipLaunchKernelGGL(reduce_partials_kernel, dim3((uint32_t)ceil_div(total, 256)), dim3(256), 0, hs,
                           static_cast<const float*>(ws), n, k, pl.chunks, scale, out, ldo);
        if (hipGetLastError() != hipSuccess) return GRASS_EHIP;
    }
    return GRASS_OK;
}

extern "C" grass_status grass_sjlt(const float* g, uint64_t n, uint64_t p, uint64_t ldg, const int32_t* idx,
                                   uint32_t kprime, uint32_t k, uint32_t s, uint64_t seed, uint64_t stream_id,
                                   float* out, uint64_t ldo, void* ws, size_t ws_bytes,
                                   const grass_tuning* host_tuning, grass_stream stream) {
    return run_sjlt(g, 4, n, p, ldg, idx, kprime, k, s, seed, stream_id, out, ldo, ws, ws_bytes, host_tuning, stream);
}

extern "C" grass_status grass_sjlt_bf16(const void* g, uint64_t n, uint64_t p, uint64_t ldg, const int32_t* idx,
                                        uint32_t kprime, uint32_t k, uint32_t s, uint64_t seed, uint64_t stream_id,
                                        float* out, uint64_t ldo, void* ws, size_t ws_bytes,
                                        const grass_tuning* host_tuning, grass_stream stream) {
    return run_sjlt(g, 2, n, p, ldg, idx, kprime, k, s, seed, stream_id, out, ldo, ws, ws_bytes, host_tuning, stream);
}

// Which instantiation a plan launches, spelled the way a profiler lists it (without spaces): the template arguments
// are <input type, rows per workgroup, positions per load, loads in flight, fused mask, accumulator, hash mode>.
extern "C" grass_status grass_sjlt_describe(const void* g, int input_is_bf16, uint64_t n, uint64_t p, uint64_t ldg,
                                            uint32_t kprime_or_0, uint32_t k, uint32_t s, int with_workspace,
                                            const grass_tuning* host_tuning, char* host_text, size_t host_text_bytes) {
    if (!host_text || host_text_bytes == 0) return GRASS_EINVAL;
    const bool masked = kprime_or_0 != 0;
    grass_status st = check_sjlt_dims(n, p, masked, kprime_or_0, k, s);
    if (st != GRASS_OK) return st;
    if (n == 0 || ldg < p) return GRASS_EINVAL;
    const uint32_t in_bytes = input_is_bf16 ? 2 : 4;
    SjltPlan pl;
    if (!plan_sjlt(n, masked ? kprime_or_0 : p, masked, k, g, ldg, &pl, 0, in_bytes, s, host_tuning)) return GRASS_EUNSUPPORTED;
    const uint32_t m = k / s;
    int mode = (s == 1 && m >= 2 && (m & (m - 1)) == 0) ? MODE_FAST : MODE_GENERAL;
    if (pl.table && with_workspace) mode = MODE_TABLE;
    const int vmax = 16 / (int)in_bytes;
    const int V = masked ? 1 : pl.V;
    const int U = (!masked && V == vmax) ? (pl.R >= 8 ? 1 : 2) : (pl.R >= 8 ? 2 : 4);
    const int acc = mode == MODE_TABLE ? ACC_F64 : pl.acc;
    const unsigned long long groups = ceil_div(n, (uint64_t)pl.row_period * pl.R) * pl.row_period;
    const int len = snprintf(host_text, host_text_bytes,
                             "sjlt_kernel<%s,%d,%d,%d,%s,%d,%d> grid=%llux%u block=%d lds=%zu chunks=%u reduce=%d table=%d",
                             input_is_bf16 ? "unsignedshort" : "float", pl.R, V, U, masked ? "true" : "false", acc, mode,
                             groups, pl.chunks, pl.threads, pl.lds_bytes, pl.chunks, pl.chunks > 1 ? 1 : 0,
                             mode == MODE_TABLE ? 1 : 0);
    return (len < 0 || (size_t)len >= host_text_bytes) ? GRASS_EINVAL : GRASS_OK;
}

// Device address of `scratch` on the current device, looked up once per device.
static hipError_t scratch_address(void** out) {
    static std::mutex lock;
    static void* ptr[64] = {};
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= 64) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> guard(lock);
    if (!ptr[dev]) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        ptr[dev] = p;
    }
    *out = ptr[dev];
    return hipSuccess;
}

extern "C" grass_status grass_sjlt_noalloc(const float* g, uint64_t n, uint64_t p, uint64_t ldg, const int32_t* idx,
                                           uint32_t kprime, uint32_t k, uint32_t s, uint64_t seed, uint64_t stream_id,
                                           float* out, uint64_t ldo, grass_stream stream) {
    // all argument and size checks first: nothing below them can fail on the host side except the HIP runtime
    const bool masked = idx != nullptr;
    grass_status st = check_sjlt_dims(n, p, masked, kprime, k, s);
    if (st != GRASS_OK) return st;
    if (n == 0) return GRASS_OK;
    if (!g || !out || ldg < p || ldo < k || !aligned(g, 4) || !aligned(out, 4)) return GRASS_EINVAL;
    SjltPlan pl;
    if (!plan_sjlt(n, masked ? kprime : p, masked, k, g, ldg, &pl, 0, 4, s, nullptr)) return GRASS_EUNSUPPORTED;
    if (pl.ws_bytes > (size_t)GRASS_NOALLOC_SCRATCH_BYTES) return GRASS_ETOOLARGE;
    void* ws = nullptr;
    if (pl.ws_bytes > 0 || pl.table) {
        if (scratch_address(&ws) != hipSuccess) return GRASS_EHIP;
    }
    // the partial sums of every (chunk, row) pair and every table entry are written before they are read, so the
    // contents the previous call left behind need no clearing
    return run_sjlt(g, 4, n, p, ldg, idx, kprime, k, s, seed, stream_id, out, ldo, ws,
                    ws ? (size_t)GRASS_NOALLOC_SCRATCH_BYTES : 0, nullptr, stream);
}
