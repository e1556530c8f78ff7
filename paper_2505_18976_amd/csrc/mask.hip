// Random Mask index generation, Selective Mask index extraction, mask gather, SJLT table dump, index check.
//
// Sec. 3.2: Random Mask keeps a random subset of k' of the p coordinates; as a
// matrix it is a binary selection matrix with one non-repeating non-zero per
// row, and applying it is an index gather.
//
// Index generation never stores the p keys: key_j = H(seed, stream, j) is
// recomputed wherever needed.  A 4-pass radix select (16 bits per pass, global
// histogram) finds the k'-th smallest key T exactly; a counting pass and an
// ordered compaction then emit, in ascending j, every j with key_j < T plus the
// first `need` coordinates with key_j == T.
#include <mutex>

#include "grass_device.h"

namespace grass {

constexpr int kHistBins = 1 << 16;
constexpr int kSelThreads = 256;
constexpr int kSelItems = 8;                       // consecutive coordinates per thread
constexpr int kSelTile = kSelThreads * kSelItems;  // coordinates per workgroup

struct SelectState {
    unsigned long long prefix;   // high bits of T fixed so far
    uint32_t need;               // how many keys are still wanted inside the current prefix class
    uint32_t pad;
};

// Key sources of the select kernels.  HashKeys: Random Mask, key_j = H(seed, stream, j), never stored.
// LogitKeys: Selective Mask with an exact count (App. B.4 "ensuring exact k"): the largest logits first, so the key
// is the bitwise complement of the order-preserving integer image of S_j (-0 is folded into +0), in the upper word.
struct HashKeys {
    static constexpr bool kClustered = false;                  // hashed keys: a wavefront's digits are all different
    uint64_t sub;
    __device__ __forceinline__ uint64_t operator()(uint64_t j) const { return sm(sub, j); }
};
__device__ __forceinline__ uint64_t logit_key(float v) {
    uint32_t u = __float_as_uint(v + 0.0f);
    u = (u & 0x80000000u) ? ~u : (u | 0x80000000u);          // ascending in v
    return (uint64_t)(~u) << 32;                                // ascending key = descending logit
}
struct LogitKeys {
    static constexpr bool kClustered = true;                   // logits: many keys share their leading digits
    const float* S;
    __device__ __forceinline__ uint64_t operator()(uint64_t j) const { return logit_key(S[j]); }
};

__global__ void fill_u32_kernel(uint32_t* p, uint64_t count, uint32_t v) {
    uint64_t t = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
    for (; t < count; t += stride) p[t] = v;
}

__global__ void select_init_kernel(SelectState* st, unsigned long long prefix, uint32_t need) {
    st->prefix = prefix;
    st->need = need;
    st->pad = 0;
}

// Counter of histogram bin b: neighbouring bins sit 32 words apart, in different 128-byte lines.  Keys that cluster in
// a run of neighbouring bins (logits of similar size share their leading bits) then spread their additions over as
// many lines as bins instead of queueing up on a few.
__device__ __forceinline__ uint32_t hist_slot(uint32_t bin) { return ((bin & 2047u) << 5) | (bin >> 11); }
__device__ __forceinline__ uint32_t hist_bin_of_slot(uint32_t slot) { return ((slot & 31u) << 11) | (slot >> 5); }
static_assert(kHistBins == 65536, "hist_slot permutes 16-bit bins");

// pass = 0..3: histogram of bits [48-16*pass, 64-16*pass) among keys whose
// higher bits equal the prefix.
template <class KeyFn>
__global__ void __launch_bounds__(256) select_hist_kernel(KeyFn kf, uint64_t p, int pass,
                                                          const SelectState* st, uint32_t* hist) {
    const unsigned long long prefix = st->prefix;
    const int shift = 48 - 16 * pass;
    uint64_t j = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
    for (; j < p; j += stride) {
        const uint64_t key = kf(j);
        const bool in_class = pass == 0 ? true : ((key >> (shift + 16)) == prefix);
        const uint32_t bin = (uint32_t)((key >> shift) & 0xFFFFull);
        if constexpr (KeyFn::kClustered) {
            // Keys that cluster in a few bins would serialise on those counters: the lanes of a wavefront that share
            // a bin send one addition of their number (a few rounds; whatever is left after eight adds singly).
            bool todo = in_class;
            for (int round = 0; round < 8; ++round) {
                const unsigned long long pending = __ballot(todo);
                if (pending == 0) break;                                        // uniform
                const int leader = __ffsll((long long)pending) - 1;
                const uint32_t lead_bin = (uint32_t)__shfl((int)bin, leader);
                const unsigned long long same = __ballot(todo && bin == lead_bin);
                if ((int)(threadIdx.x & 63) == leader) atomicAdd(&hist[hist_slot(lead_bin)], (uint32_t)__popcll(same));
                if (bin == lead_bin) todo = false;
            }
            if (todo) atomicAdd(&hist[hist_slot(bin)], 1u);
        } else {
            if (in_class) atomicAdd(&hist[hist_slot(bin)], 1u);
        }
    }
}

// One workgroup: find the bin in which the cumulative count reaches `need`.
__global__ void __launch_bounds__(1024) select_pick_kernel(SelectState* st, const uint32_t* hist) {
    __shared__ uint32_t part[1024];
    __shared__ uint32_t chosen_bin, chosen_before;
    const int t = threadIdx.x;
    constexpr int per = kHistBins / 1024;   // 64 bins per thread
    // part[t] = count of the bins t*per .. t*per + per - 1; the counters are read in storage order (coalesced)
    part[t] = 0;
    __syncthreads();
    uint32_t c[per];
#pragma unroll
    for (int q = 0; q < per; ++q) c[q] = hist[(uint32_t)t + 1024u * q];            // all loads in flight together
#pragma unroll
    for (int q = 0; q < per; ++q)
        if (c[q]) atomicAdd(&part[hist_bin_of_slot((uint32_t)t + 1024u * q) / per], c[q]);
    __syncthreads();
    // inclusive scan over the 1024 partial sums: within each wavefront by shuffles, then the totals of the earlier
    // wavefronts are added
    __shared__ uint32_t wave_total[16];
    {
        const int lane = t & 63, w = t >> 6;
        uint32_t v = part[t];
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const uint32_t u = (uint32_t)__shfl_up((int)v, off);
            if (lane >= off) v += u;
        }
        if (lane == 63) wave_total[w] = v;
        __syncthreads();
        uint32_t base = 0;
        for (int q = 0; q < w; ++q) base += wave_total[q];
        part[t] = v + base;
        __syncthreads();
    }
    const uint32_t need = st->need;
    const uint32_t before = (t == 0) ? 0u : part[t - 1];
    if (before < need && need <= part[t]) {
        uint32_t run = before;
        uint32_t mine[per];
#pragma unroll
        for (int b = 0; b < per; ++b) mine[b] = hist[hist_slot((uint32_t)(t * per + b))];     // loads in flight together
#pragma unroll
        for (int b = 0; b < per; ++b) {
            const uint32_t c = mine[b];
            if (run < need && need <= run + c) {
                chosen_bin = (uint32_t)(t * per + b);
                chosen_before = run;
            }
            run += c;
        }
    }
    __syncthreads();
    if (t == 0) {
        st->prefix = (st->prefix << 16) | (unsigned long long)chosen_bin;
        st->need = need - chosen_before;
    }
}

// Workgroup-wide exclusive scan of two counters per thread (256 threads).
__device__ __forceinline__ void block_scan2(uint32_t a, uint32_t b, uint32_t* ea, uint32_t* eb,
                                            uint32_t* ta, uint32_t* tb) {
    __shared__ uint32_t sa[kSelThreads], sb[kSelThreads];
    const int t = threadIdx.x;
    sa[t] = a; sb[t] = b;
    __syncthreads();
    for (int off = 1; off < kSelThreads; off <<= 1) {
        uint32_t va = (t >= off) ? sa[t - off] : 0u;
        uint32_t vb = (t >= off) ? sb[t - off] : 0u;
        __syncthreads();
        sa[t] += va; sb[t] += vb;
        __syncthreads();
    }
    *ea = sa[t] - a; *eb = sb[t] - b;
    *ta = sa[kSelThreads - 1]; *tb = sb[kSelThreads - 1];
    __syncthreads();
}

// Per tile of kSelTile coordinates: how many keys are below T, how many equal T.
template <class KeyFn>
__global__ void __launch_bounds__(kSelThreads) select_count_kernel(KeyFn kf, uint64_t p,
                                                                   const SelectState* st, uint32_t* tile_less,
                                                                   uint32_t* tile_eq) {
    const unsigned long long T = st->prefix;
    const uint64_t j0 = (uint64_t)blockIdx.x * kSelTile + (uint64_t)threadIdx.x * kSelItems;
    uint32_t less = 0, eq = 0;
#pragma unroll
    for (int i = 0; i < kSelItems; ++i) {
        const uint64_t j = j0 + i;
        if (j < p) {
            const uint64_t key = kf(j);
            less += key < T;
            eq += key == T;
        }
    }
    uint32_t el, ee, tl, te;
    block_scan2(less, eq, &el, &ee, &tl, &te);
    if (threadIdx.x == 0) { tile_less[blockIdx.x] = tl; tile_eq[blockIdx.x] = te; }
}

// One workgroup: exclusive scan of the per-tile counts, in place.
// total_less (may be null) receives the number of keys below T.
__global__ void __launch_bounds__(1024) select_scan_tiles_kernel(uint32_t* tile_less, uint32_t* tile_eq,
                                                                 uint64_t tiles, uint32_t* total_less) {
    __shared__ uint32_t sa[1024], sb[1024];
    const int t = threadIdx.x;
    const uint64_t per = (tiles + 1023) / 1024;
    const uint64_t lo = (uint64_t)t * per;
    const uint64_t hi = lo + per < tiles ? lo + per : tiles;
    uint32_t a = 0, b = 0;
    for (uint64_t i = lo; i < hi; ++i) { a += tile_less[i]; b += tile_eq[i]; }
    sa[t] = a; sb[t] = b;
    __syncthreads();
    for (int off = 1; off < 1024; off <<= 1) {
        uint32_t va = (t >= off) ? sa[t - off] : 0u;
        uint32_t vb = (t >= off) ? sb[t - off] : 0u;
        __syncthreads();
        sa[t] += va; sb[t] += vb;
        __syncthreads();
    }
    if (t == 1023 && total_less) *total_less = sa[1023];
    uint32_t ra = sa[t] - a, rb = sb[t] - b;
    for (uint64_t i = lo; i < hi; ++i) {
        const uint32_t ca = tile_less[i], cb = tile_eq[i];
        tile_less[i] = ra; tile_eq[i] = rb;
        ra += ca; rb += cb;
    }
}

// Ordered compaction: coordinate j is kept iff key_j < T, or key_j == T and
// fewer than `need` equal keys precede it; its output slot is the number of
// kept coordinates before it.
template <class KeyFn>
__global__ void __launch_bounds__(kSelThreads) select_compact_kernel(KeyFn kf, uint64_t p,
                                                                     const SelectState* st,
                                                                     const uint32_t* tile_less,
                                                                     const uint32_t* tile_eq, int32_t* idx,
                                                                     uint32_t kprime) {
    const unsigned long long T = st->prefix;
    const uint32_t need = st->need;
    const uint64_t j0 = (uint64_t)blockIdx.x * kSelTile + (uint64_t)threadIdx.x * kSelItems;
    uint32_t less = 0, eq = 0;
    uint32_t flag_less = 0, flag_eq = 0;
#pragma unroll
    for (int i = 0; i < kSelItems; ++i) {
        const uint64_t j = j0 + i;
        if (j < p) {
            const uint64_t key = kf(j);
            if (key < T) { ++less; flag_less |= 1u << i; }
            if (key == T) { ++eq; flag_eq |= 1u << i; }
        }
    }
    uint32_t el, ee, tl, te;
    block_scan2(less, eq, &el, &ee, &tl, &te);
    uint32_t nl = tile_less[blockIdx.x] + el;
    uint32_t ne = tile_eq[blockIdx.x] + ee;
#pragma unroll
    for (int i = 0; i < kSelItems; ++i) {
        const bool is_less = (flag_less >> i) & 1u;
        const bool is_eq = (flag_eq >> i) & 1u;
        if (is_less || (is_eq && ne < need)) {
            const uint32_t slot = nl + (ne < need ? ne : need);
            if (slot < kprime) idx[slot] = (int32_t)(j0 + i);
        }
        nl += is_less;
        ne += is_eq;
    }
}

__global__ void __launch_bounds__(1024) mask_gather_kernel(const float* g, uint64_t ldg, const int32_t* idx,
                                                          uint32_t kprime, float* out, uint64_t ldo,
                                                          uint64_t n, uint32_t rows_per_block) {
    const uint32_t jp = blockIdx.x * blockDim.x + threadIdx.x;
    if (jp >= kprime) return;
    const int32_t col = idx[jp];
    const uint64_t r0 = (uint64_t)blockIdx.y * rows_per_block;
    const uint64_t r1 = r0 + rows_per_block < n ? r0 + rows_per_block : n;
    uint64_t r = r0;
    for (; r + 8 <= r1; r += 8) {
        // read-once, write-once data: non-temporal accesses sustain a higher rate on scattered lines;
        // eight rows in flight per thread
        float v[8];
#pragma unroll
        for (int q = 0; q < 8; ++q) v[q] = __builtin_nontemporal_load(g + (r + q) * ldg + col);
#pragma unroll
        for (int q = 0; q < 8; ++q) __builtin_nontemporal_store(v[q], out + (r + q) * ldo + jp);
    }
    for (; r < r1; ++r) out[r * ldo + jp] = g[r * ldg + col];
}

__global__ void __launch_bounds__(256) sjlt_tables_kernel(uint64_t sub, uint64_t total, uint32_t s, uint32_t m,
                                                          uint32_t* bucket, int8_t* sign) {
    uint64_t c = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
    for (; c < total; c += stride) {
        const uint64_t h = sm(sub, c);
        const uint32_t r = (uint32_t)(c % s);
        bucket[c] = r * m + bucket_of(h, m);
        sign[c] = signbit_of(h) ? (int8_t)-1 : (int8_t)1;
    }
}

// P[row(j', r)][col(j')] = sign(j', r) / sqrt(s) for the SJLT positions j' in [0, d): col(j') = idx[j'] for the fused
// mask (P is then the product of the SJLT matrix and the selection matrix), j' itself otherwise.  P is zero-filled first.
__global__ void __launch_bounds__(256) projection_matrix_kernel(uint64_t sub, uint64_t d, const int32_t* idx, uint32_t s,
                                                               uint32_t m, float value, float* P, uint64_t ldP) {
    const uint64_t total = d * s;
    uint64_t c = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
    for (; c < total; c += stride) {
        const uint64_t jp = c / s;
        const uint32_t r = (uint32_t)(c - jp * s);
        const uint64_t h = sm(sub, c);
        const uint64_t col = idx ? (uint64_t)idx[jp] : jp;
        P[(uint64_t)(r * m + bucket_of(h, m)) * ldP + col] = signbit_of(h) ? -value : value;
    }
}

__global__ void __launch_bounds__(256) zero_rows_kernel(float* P, uint64_t rows, uint64_t cols, uint64_t ld) {
    const uint64_t t = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= rows * cols) return;
    const uint64_t r = t / cols;
    P[r * ld + (t - r * cols)] = 0.0f;
}

__global__ void __launch_bounds__(256) check_indices_kernel(const int32_t* idx, uint32_t kprime, uint64_t p,
                                                            uint32_t* bad) {
    const uint32_t t = blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= kprime) return;
    const int32_t v = idx[t];
    bool ok = v >= 0 && (uint64_t)v < p;
    if (t > 0) ok = ok && idx[t - 1] < v;
    if (!ok) atomicOr(bad, 1u);
}

// Result word of grass_check_indices (one per device, inside the code object).  The call synchronises anyway, so a
// host mutex held from the reset of the word to its read-back makes concurrent calls from several threads safe.
__device__ uint32_t bad_flag;
static std::mutex bad_flag_mutex;

struct SelectLayout {
    size_t off_state, off_hist, off_less, off_eq, total;
    uint64_t tiles;
};

static SelectLayout select_layout(uint64_t p) {
    SelectLayout L;
    L.tiles = ceil_div(p, kSelTile);
    L.off_state = 0;
    L.off_hist = 256;
    L.off_less = L.off_hist + (size_t)4 * kHistBins * sizeof(uint32_t);
    L.off_eq = L.off_less + ((L.tiles * 4 + 255) / 256) * 256;
    L.total = L.off_eq + ((L.tiles * 4 + 255) / 256) * 256;
    return L;
}

}  // namespace grass

using namespace grass;

extern "C" grass_status grass_mask_indices_workspace_bytes(uint64_t p, uint32_t kprime, size_t* host_bytes) {
    if (!host_bytes || p == 0 || p >= (1ull << 31) || kprime == 0 || kprime > p) return GRASS_EINVAL;
    *host_bytes = select_layout(p).total;
    return GRASS_OK;
}

// k smallest (key, j) pairs in ascending j.  radix = false skips the search for the threshold key: the state is
// preset to (T, 0) and every j with key_j < T is emitted (their number goes to *count).
template <class KeyFn>
static grass_status run_select(KeyFn kf, uint64_t p, uint32_t k, bool radix, unsigned long long preset_T, int32_t* idx,
                               uint32_t capacity, uint32_t* count, void* ws, hipStream_t hs) {
    const SelectLayout L = select_layout(p);
    char* base = static_cast<char*>(ws);
    SelectState* st = reinterpret_cast<SelectState*>(base + L.off_state);
    uint32_t* hist = reinterpret_cast<uint32_t*>(base + L.off_hist);
    uint32_t* tile_less = reinterpret_cast<uint32_t*>(base + L.off_less);
    uint32_t* tile_eq = reinterpret_cast<uint32_t*>(base + L.off_eq);
    if (radix) {
        hipLaunchKernelGGL(fill_u32_kernel, dim3(256), dim3(256), 0, hs, hist, (uint64_t)4 * kHistBins, 0u);
        hipLaunchKernelGGL(select_init_kernel, dim3(1), dim3(1), 0, hs, st, 0ull, k);
        uint32_t hist_blocks = (uint32_t)ceil_div(p, 256);
        if (hist_blocks > 4096) hist_blocks = 4096;
        for (int pass = 0; pass < 4; ++pass) {
            uint32_t* h = hist + (size_t)pass * kHistBins;
            hipLaunchKernelGGL(select_hist_kernel<KeyFn>, dim3(hist_blocks), dim3(256), 0, hs, kf, p, pass, st, h);
            hipLaunchKernelGGL(select_pick_kernel, dim3(1), dim3(1024), 0, hs, st, h);
        }
    } else {
        hipLaunchKernelGGL(select_init_kernel, dim3(1), dim3(1), 0, hs, st, preset_T, 0u);
    }
    hipLaunchKernelGGL(select_count_kernel<KeyFn>, dim3((uint32_t)L.tiles), dim3(kSelThreads), 0, hs, kf, p, st,
                       tile_less, tile_eq);
    hipLaunchKernelGGL(select_scan_tiles_kernel, dim3(1), dim3(1024), 0, hs, tile_less, tile_eq, L.tiles, count);
    hipLaunchKernelGGL(select_compact_kernel<KeyFn>, dim3((uint32_t)L.tiles), dim3(kSelThreads), 0, hs, kf, p, st,
                       tile_less, tile_eq, idx, capacity);
    return launch_status();
}

extern "C" grass_status grass_mask_indices(uint64_t seed, uint64_t stream_id, uint64_t p, uint32_t kprime,
                                           int32_t* idx, void* ws, size_t ws_bytes, grass_stream stream) {
    if (p == 0 || p >= (1ull << 31) || kprime == 0 || kprime > p || !idx) return GRASS_EINVAL;
    if (!ws || ws_bytes < select_layout(p).total || !aligned(ws, 256)) return GRASS_EWORKSPACE;
    return run_select(HashKeys{substream(seed, stream_id)}, p, kprime, true, 0ull, idx, kprime, nullptr, ws,
                      as_stream(stream));
}

extern "C" grass_status grass_selective_mask_indices_workspace_bytes(uint64_t p, size_t* host_bytes) {
    if (!host_bytes || p == 0 || p >= (1ull << 31)) return GRASS_EINVAL;
    *host_bytes = select_layout(p).total;
    return GRASS_OK;
}

extern "C" grass_status grass_selective_mask_indices(const float* S, uint64_t p, uint32_t k, int32_t* idx,
                                                     uint32_t* count, void* ws, size_t ws_bytes, grass_stream stream) {
    if (p == 0 || p >= (1ull << 31) || k > p || !S || !idx) return GRASS_EINVAL;
    if (k == 0 && !count) return GRASS_EINVAL;
    if (!ws || ws_bytes < select_layout(p).total || !aligned(ws, 256)) return GRASS_EWORKSPACE;
    hipStream_t hs = as_stream(stream);
    if (k == 0) {
        // sigma(S_j) >= 1/2  <=>  S_j >= 0  <=>  key_j <= key(+0)  <=>  key_j < key(+0) + 2^32 (low word is zero)
        const uint32_t zero_image = 0x80000000u;                                // order-preserving image of +0.0f
        const unsigned long long thr = ((unsigned long long)(~zero_image) << 32) + (1ull << 32);
        return run_select(LogitKeys{S}, p, 0, false, thr, idx, (uint32_t)p, count, ws, hs);
    }
    grass_status st = run_select(LogitKeys{S}, p, k, true, 0ull, idx, k, nullptr, ws, hs);
    if (st == GRASS_OK && count) {
        hipLaunchKernelGGL(fill_u32_kernel, dim3(1), dim3(1), 0, hs, count, (uint64_t)1, k);
        st = launch_status();
    }
    return st;
}

extern "C" grass_status grass_projection_matrix(uint64_t seed, uint64_t stream_id, uint64_t p, const int32_t* idx,
                                                uint32_t kprime, uint32_t k, uint32_t s, float* P, uint64_t ldP,
                                                grass_stream stream) {
    if (p == 0 || p >= (1ull << 31) || k == 0 || s == 0 || k % s != 0 || !P || ldP < p) return GRASS_EINVAL;
    if (idx && (kprime == 0 || kprime > p)) return GRASS_EINVAL;
    if (ceil_div((uint64_t)k * p, 256) > 0x7FFFFFFFull) return GRASS_EUNSUPPORTED;
    const uint64_t d = idx ? kprime : p;
    hipStream_t hs = as_stream(stream);
    hipLaunchKernelGGL(zero_rows_kernel, dim3((uint32_t)ceil_div((uint64_t)k * p, 256)), dim3(256), 0, hs, P, (uint64_t)k, p,
                       ldP);
    const uint64_t total = d * s;
    const uint32_t blocks = (uint32_t)(ceil_div(total, 256) > 8192 ? 8192 : ceil_div(total, 256));
    hipLaunchKernelGGL(projection_matrix_kernel, dim3(blocks), dim3(256), 0, hs, substream(seed, stream_id), d, idx, s, k / s,
                       1.0f / sqrtf((float)s), P, ldP);
    return launch_status();
}

extern "C" grass_status grass_check_indices(const int32_t* idx, uint32_t kprime, uint64_t p, int* host_ok,
                                            grass_stream stream) {
    if (!idx || !host_ok || kprime == 0 || p == 0) return GRASS_EINVAL;
    std::lock_guard<std::mutex> guard(bad_flag_mutex);
    uint32_t* dflag = nullptr;
    if (hipGetSymbolAddress(reinterpret_cast<void**>(&dflag), HIP_SYMBOL(bad_flag)) != hipSuccess) return GRASS_EHIP;
    hipStream_t hs = as_stream(stream);
    hipLaunchKernelGGL(fill_u32_kernel, dim3(1), dim3(1), 0, hs, dflag, (uint64_t)1, 0u);
    hipLaunchKernelGGL(check_indices_kernel, dim3((uint32_t)ceil_div(kprime, 256)), dim3(256), 0, hs, idx, kprime,
                       p, dflag);
    uint32_t h = 1;
    if (hipMemcpyAsync(&h, dflag, sizeof(h), hipMemcpyDeviceToHost, hs) != hipSuccess) return GRASS_EHIP;
    if (hipStreamSynchronize(hs) != hipSuccess) return GRASS_EHIP;
    *host_ok = h == 0;
    return GRASS_OK;
}

extern "C" grass_status grass_mask(const float* g, uint64_t n, uint64_t p, uint64_t ldg, const int32_t* idx,
                                   uint32_t kprime, float* out, uint64_t ldo, grass_stream stream) {
    if (p == 0 || p >= (1ull << 31) || kprime == 0 || kprime > p) return GRASS_EINVAL;
    if (n == 0) return GRASS_OK;
    if (!g || !idx || !out || ldg < p || ldo < kprime) return GRASS_EINVAL;
    // rows per workgroup: keep idx reuse high, still fill the chip
    // 1,024 consecutive kept columns of the same few rows per workgroup: neighbouring wavefronts walk through
    // neighbouring DRAM pages of one row at the same time
    const uint32_t gather_threads = kprime >= 4096 ? 1024 : 256;
    const uint32_t col_blocks = (uint32_t)ceil_div(kprime, gather_threads);
    uint32_t rows_per_block = 8;
    const uint64_t row_blocks = ceil_div(n, rows_per_block);
    if (row_blocks > 65535) rows_per_block = (uint32_t)ceil_div(n, 65535);
    hipLaunchKernelGGL(mask_gather_kernel, dim3(col_blocks, (uint32_t)ceil_div(n, rows_per_block)),
                       dim3(gather_threads), 0, as_stream(stream), g, ldg, idx, kprime, out, ldo, n, rows_per_block);
    return launch_status();
}

extern "C" grass_status grass_sjlt_tables(uint64_t seed, uint64_t stream_id, uint64_t d, uint32_t k, uint32_t s,
                                          uint32_t* bucket, int8_t* sign, grass_stream stream) {
    if (d == 0 || k == 0 || s == 0 || k % s != 0 || !bucket || !sign) return GRASS_EINVAL;
    const uint64_t total = d * s;
    uint32_t blocks = (uint32_t)(ceil_div(total, 256) > 8192 ? 8192 : ceil_div(total, 256));
    hipLaunchKernelGGL(sjlt_tables_kernel, dim3(blocks), dim3(256), 0, as_stream(stream),
                       substream(seed, stream_id), total, s, k / s, bucket, sign);
    return launch_status();
}
