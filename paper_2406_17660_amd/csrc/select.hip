// grass_select_rows: compute_P of Section 3.2 on the device.
//
// The work is O(m) integer operations on a few thousand row statistics, so it is latency
// bound, not bandwidth bound: one workgroup of 1024 threads (16 wavefronts) runs the whole
// rule, using LDS histograms, wavefront scans and ballots.  No host round trip: idx and
// rho stay on the device for the calls that follow.
//
//   Top-r           4-pass radix select (8 bits per pass, LDS histogram) on the bit
//                   patterns of sumsq, then an order-preserving compaction by block scan.
//   with repl.      fixed-point weights -> 64-bit inclusive prefix sums in the workspace;
//                   the r draws are independent: Philox word, 64x64 high multiply, binary
//                   search; a per-row hit counter plus a scan emits idx sorted.
//   without repl.   draws are sequential by definition.  A radix-64 sum tree over the
//                   weights (in LDS when it fits in 144 KiB, else in the workspace) lets
//                   one wavefront do a draw in log64(m) steps: 64 children per load, a
//                   wavefront scan and a ballot pick the child; the path is then
//                   decremented.  Chosen leaves have weight 0; a scan compacts them.
//
// Selection arithmetic is integer (or correctly rounded IEEE double sqrt / divide) so
// that the indices are reproducible bit for bit.
#include <atomic>

#include "common.hpp"

// Scratch memory of grass_select_rows_static, the entry point for callers that cannot
// allocate: one copy per GPU, held until the process ends.  In host code this name is only a
// handle for hipGetSymbolAddress; kernels are given the address that call returns.
constexpr size_t kStaticScratchBytes = size_t{1} << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace grass {
namespace {

constexpr int kThreads = 1024;
constexpr int kWaves = kThreads / kWave;
constexpr size_t kHeaderBytes = 256;       // status word + padding
constexpr size_t kLdsTreeBytes = 144 * 1024;
constexpr int kMaxLevels = 6;              // 64^6 > 2^31 rows

struct Shared {
    uint32_t hist[256];
    unsigned long long scan_tot[kWaves];
    double red[kWaves];
    unsigned long long bcast64;
    uint32_t prefix;
    uint32_t need;
    int bad;
};

__device__ __forceinline__ uint32_t key_of(float s) { return s == 0.0f ? 0u : __float_as_uint(s); }
__device__ __forceinline__ bool is_bad(float s) { return !(s >= 0.0f) || isinf(s); }

// Philox4x32-10 (Salmon et al., SC'11): counter = (j, refresh_id), key = seed.
__device__ __forceinline__ unsigned long long draw_word(unsigned long long seed,
                                                        unsigned long long refresh,
                                                        unsigned long long j) {
    uint32_t c0 = static_cast<uint32_t>(j), c1 = static_cast<uint32_t>(j >> 32);
    uint32_t c2 = static_cast<uint32_t>(refresh), c3 = static_cast<uint32_t>(refresh >> 32);
    uint32_t k0 = static_cast<uint32_t>(seed), k1 = static_cast<uint32_t>(seed >> 32);
#pragma unroll
    for (int i = 0; i < 10; ++i) {
        const uint32_t h0 = __umulhi(0xD2511F53u, c0), l0 = 0xD2511F53u * c0;
        const uint32_t h1 = __umulhi(0xCD9E8D57u, c2), l1 = 0xCD9E8D57u * c2;
        const uint32_t n0 = h1 ^ c1 ^ k0, n2 = h0 ^ c3 ^ k1;
        c0 = n0; c1 = l1; c2 = n2; c3 = l0;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    return static_cast<unsigned long long>(c0) | (static_cast<unsigned long long>(c1) << 32);
}

__device__ __forceinline__ double weight_of(float s, int method) {
    const double d = static_cast<double>(s);
    return method == GRASS_SEL_UNIFORM ? 1.0 : (method == GRASS_SEL_MULTI_NORM ? sqrt(d) : d);
}
__device__ __forceinline__ unsigned long long quantise(double w, double wmax) {
    if (wmax == 0.0) return 1ull;
    return static_cast<unsigned long long>(floor(w / wmax * 1099511627776.0)) + 1ull;
}

// Exclusive prefix sum of one value per thread across the workgroup; `total` is the sum.
// Two barriers; `sh->scan_tot` is reused by every call.
template <typename T>
__device__ __forceinline__ T block_exclusive_scan(T v, Shared* sh, T& total) {
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    const T incl = wave_inclusive_scan(v);
    __syncthreads();  // previous users of scan_tot are done
    if (lane == kWave - 1) sh->scan_tot[wave] = static_cast<unsigned long long>(incl);
    __syncthreads();
    T before = 0, all = 0;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
        const T t = static_cast<T>(sh->scan_tot[w]);
        if (w < wave) before += t;
        all += t;
    }
    total = all;
    return before + incl - v;
}

__device__ __forceinline__ double block_max(double v, Shared* sh) {
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    v = wave_max(v);
    __syncthreads();
    if (lane == 0) sh->red[wave] = v;
    __syncthreads();
    double r = sh->red[0];
#pragma unroll
    for (int w = 1; w < kWaves; ++w) r = sh->red[w] > r ? sh->red[w] : r;
    return r;
}

// Common prologue: reject NaN / Inf / negative statistics.  Returns true (for every
// thread) when the input is bad, after writing the placeholder selection.
__device__ bool reject_nonfinite(const float* sumsq, int64_t m, int64_t r, int32_t* idx,
                                 float* rho, int32_t* status, Shared* sh) {
    if (threadIdx.x == 0) sh->bad = 0;
    __syncthreads();
    bool bad = false;
    for (int64_t k = threadIdx.x; k < m; k += kThreads) bad |= is_bad(sumsq[k]);
    if (bad) sh->bad = 1;
    __syncthreads();
    if (!sh->bad) {
        if (threadIdx.x == 0) *status = GRASS_OK;
        return false;
    }
    if (threadIdx.x == 0) *status = GRASS_ERR_NONFINITE;
    for (int64_t j = threadIdx.x; j < r; j += kThreads) {
        idx[j] = static_cast<int32_t>((j * m) / r);  // ascending and inside [0, m)
        rho[j] = 1.0f;
    }
    return true;
}

// ------------------------------------------------------------------------------ Top-r
__global__ __launch_bounds__(kThreads) void select_topr_kernel(
    const float* __restrict__ sumsq, int64_t m, int64_t r, int32_t* __restrict__ idx,
    float* __restrict__ rho, int32_t* __restrict__ status) {
    __shared__ Shared sh;
    if (reject_nonfinite(sumsq, m, r, idx, rho, status, &sh)) return;
    if (r == 0) return;  // nothing to select: only the status word is written
    const int tid = threadIdx.x;

    // Radix select: after the four passes `prefix` is the r-th largest key and `need`
    // how many rows carrying exactly that key are still wanted.
    uint32_t prefix = 0, need = static_cast<uint32_t>(r);
    for (int pass = 3; pass >= 0; --pass) {
        const int shift = pass * 8;
        if (tid < 256) sh.hist[tid] = 0;
        __syncthreads();
        for (int64_t k = tid; k < m; k += kThreads) {
            const uint32_t key = key_of(sumsq[k]);
            const bool match = pass == 3 || (key >> (shift + 8)) == (prefix >> (shift + 8));
            if (match) atomicAdd(&sh.hist[(key >> shift) & 255u], 1u);
        }
        __syncthreads();
        if (tid < kWave) {
            // lane L owns digits 255-4L .. 252-4L (descending); find the digit at which the
            // count of rows with a larger digit first reaches `need`
            uint32_t h[4], s = 0;
#pragma unroll
            for (int e = 0; e < 4; ++e) { h[e] = sh.hist[255 - 4 * tid - e]; s += h[e]; }
            const uint32_t incl = wave_inclusive_scan(s);
            uint32_t above = incl - s;
            if (above < need && need <= incl) {
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    if (need <= above + h[e]) {
                        sh.prefix = prefix | (static_cast<uint32_t>(255 - 4 * tid - e) << shift);
                        sh.need = need - above;
                        break;
                    }
                    above += h[e];
                }
            }
        }
        __syncthreads();
        prefix = sh.prefix;
        need = sh.need;
    }

    // Compaction in row order: every key above the threshold, and the first `need` rows
    // that equal it (ties go to the lower index).
    unsigned long long carry = 0;  // low 32 bits: rows above so far; high: rows equal so far
    for (int64_t base = 0; base < m; base += kThreads) {
        const int64_t k = base + tid;
        bool gt = false, eq = false;
        if (k < m) {
            const uint32_t key = key_of(sumsq[k]);
            gt = key > prefix;
            eq = key == prefix;
        }
        const unsigned long long mine = (gt ? 1ull : 0ull) | (eq ? (1ull << 32) : 0ull);
        unsigned long long total;
        const unsigned long long before = carry + block_exclusive_scan(mine, &sh, total);
        const uint32_t gt_before = static_cast<uint32_t>(before);
        const uint32_t eq_before = static_cast<uint32_t>(before >> 32);
        if (gt || (eq && eq_before < need)) {
            const uint32_t pos = gt_before + (eq_before < need ? eq_before : need);
            idx[pos] = static_cast<int32_t>(k);
            rho[pos] = 1.0f;
        }
        carry += total;
    }
}

// ------------------------------------------------------------------------------ with replacement
__global__ __launch_bounds__(kThreads) void select_repl_kernel(
    const float* __restrict__ sumsq, int64_t m, int64_t r, int method, int rescale,
    unsigned long long seed, unsigned long long refresh, int32_t* __restrict__ idx,
    float* __restrict__ rho, int32_t* __restrict__ status, unsigned long long* __restrict__ csum,
    uint32_t* __restrict__ hits) {
    __shared__ Shared sh;
    if (reject_nonfinite(sumsq, m, r, idx, rho, status, &sh)) return;
    if (r == 0) return;  // nothing to select: only the status word is written
    const int tid = threadIdx.x;

    double wmax = 0.0;
    for (int64_t k = tid; k < m; k += kThreads) {
        const double w = weight_of(sumsq[k], method);
        wmax = w > wmax ? w : wmax;
    }
    wmax = block_max(wmax, &sh);

    // inclusive prefix sums of the integer weights
    unsigned long long carry = 0;
    for (int64_t base = 0; base < m; base += kThreads) {
        const int64_t k = base + tid;
        const unsigned long long wq = k < m ? quantise(weight_of(sumsq[k], method), wmax) : 0ull;
        unsigned long long total;
        const unsigned long long before = block_exclusive_scan(wq, &sh, total);
        if (k < m) {
            csum[k] = carry + before + wq;
            hits[k] = 0;
        }
        carry += total;
    }
    const unsigned long long total_w = carry;
    __threadfence_block();
    __syncthreads();

    // independent draws: first k with csum[k] > target
    for (int64_t j = tid; j < r; j += kThreads) {
        const unsigned long long target = __umul64hi(draw_word(seed, refresh, j), total_w);
        int64_t lo = 0, hi = m - 1;
        while (lo < hi) {
            const int64_t mid = (lo + hi) >> 1;
            if (csum[mid] > target) hi = mid; else lo = mid + 1;
        }
        atomicAdd(&hits[lo], 1u);
    }
    __threadfence_block();
    __syncthreads();

    // emit rows in ascending order, each as often as it was hit
    uint32_t out_carry = 0;
    for (int64_t base = 0; base < m; base += kThreads) {
        const int64_t k = base + tid;
        const uint32_t h = k < m ? hits[k] : 0u;
        uint32_t total;
        const uint32_t pos = out_carry + block_exclusive_scan(h, &sh, total);
        if (h) {
            float rk = 1.0f;
            if (rescale) {
                const unsigned long long wq = csum[k] - (k ? csum[k - 1] : 0ull);
                const double q = static_cast<double>(wq) / static_cast<double>(total_w);
                rk = static_cast<float>(1.0 / sqrt(static_cast<double>(r) * q));
            }
            for (uint32_t e = 0; e < h; ++e) {
                idx[pos + e] = static_cast<int32_t>(k);
                rho[pos + e] = rk;
            }
        }
        out_carry += total;
    }
}

// ------------------------------------------------------------------------------ without replacement
// Sampling without replacement is r sequential draws from the weights that are left (the
// weight of a drawn row is taken out before the next draw).  The weights sit in a radix-64
// tree whose nodes store, instead of their own sum, the INCLUSIVE PREFIX of the sums inside
// their group of 64 siblings.  One wavefront then walks a draw down the tree with one load,
// one compare and one ballot per level (the first lane whose prefix exceeds the target is
// the child to enter; the prefix of the lane before it is what the target loses), and takes
// the drawn weight w out by subtracting w from the prefixes at and after the path's lane in
// each of the path's groups.  Every value is an exact integer, so the draws are those of the
// sequential definition.  Every level is padded to whole groups; padding carries weight 0.
struct TreeShape {
    int levels;                  // level 0 = leaves
    int64_t groups[kMaxLevels];  // groups of 64 entries per level (the top level has one)
    int64_t offset[kMaxLevels];  // first entry of the level inside the node array
};

__device__ __forceinline__ unsigned long long read_lane64(unsigned long long v, int l) {
    const uint32_t lo = __builtin_amdgcn_readlane(static_cast<uint32_t>(v), l);
    const uint32_t hi = __builtin_amdgcn_readlane(static_cast<uint32_t>(v >> 32), l);
    return (static_cast<unsigned long long>(hi) << 32) | lo;
}

// The r draws, by one wavefront.  TreePtr is an LDS or a global pointer; kFence orders the
// updates of a global tree before the next draw's loads.
template <int LEVELS, bool kFence, typename TreePtr>
__device__ __forceinline__ void draw_without_replacement(TreePtr tree, const TreeShape& shape,
                                                         int64_t r, unsigned long long seed,
                                                         unsigned long long refresh,
                                                         unsigned long long total_w, int lane) {
    unsigned long long remaining = total_w;
    for (int64_t j0 = 0; j0 < r; j0 += kWave) {
        // the Philox words of the next 64 draws, one per lane
        const unsigned long long words = draw_word(seed, refresh, static_cast<unsigned long long>(j0 + lane));
        const int in_block = r - j0 < kWave ? static_cast<int>(r - j0) : kWave;
        for (int jj = 0; jj < in_block; ++jj) {
            unsigned long long target = __umul64hi(read_lane64(words, jj), remaining);
            unsigned long long prefix[LEVELS];
            int64_t entry[LEVELS];
            int first[LEVELS];
            unsigned long long w = 0;
            int64_t node = 0;
#pragma unroll
            for (int L = LEVELS - 1; L >= 0; --L) {
                entry[L] = shape.offset[L] + node * kWave + lane;
                prefix[L] = tree[entry[L]];
                const unsigned long long hit = __ballot(prefix[L] > target);
                const int f = __ffsll(static_cast<long long>(hit)) - 1;  // hit != 0: target < total
                const unsigned long long before = f > 0 ? read_lane64(prefix[L], f - 1) : 0ull;
                if (L == 0) w = read_lane64(prefix[0], f) - before;  // the leaf drawn
                target -= before;
                first[L] = f;
                node = node * kWave + f;
            }
#pragma unroll
            for (int L = 0; L < LEVELS; ++L)
                if (lane >= first[L]) tree[entry[L]] = prefix[L] - w;
            remaining -= w;
            if (kFence) __threadfence_block();
        }
    }
}

template <bool kFence, typename TreePtr>
__device__ __forceinline__ void draw_dispatch(TreePtr tree, const TreeShape& shape, int64_t r,
                                              unsigned long long seed, unsigned long long refresh,
                                              unsigned long long total_w, int lane) {
    switch (shape.levels) {
        case 1: draw_without_replacement<1, kFence>(tree, shape, r, seed, refresh, total_w, lane); break;
        case 2: draw_without_replacement<2, kFence>(tree, shape, r, seed, refresh, total_w, lane); break;
        case 3: draw_without_replacement<3, kFence>(tree, shape, r, seed, refresh, total_w, lane); break;
        case 4: draw_without_replacement<4, kFence>(tree, shape, r, seed, refresh, total_w, lane); break;
        case 5: draw_without_replacement<5, kFence>(tree, shape, r, seed, refresh, total_w, lane); break;
        default: draw_without_replacement<6, kFence>(tree, shape, r, seed, refresh, total_w, lane); break;
    }
}

template <bool kTreeInLds>
__global__ __launch_bounds__(kThreads) void select_norepl_kernel(
    const float* __restrict__ sumsq, int64_t m, int64_t r, int method, int rescale,
    unsigned long long seed, unsigned long long refresh, int32_t* __restrict__ idx,
    float* __restrict__ rho, int32_t* __restrict__ status, unsigned long long* ws_tree,
    TreeShape shape) {
    __shared__ Shared sh;
    extern __shared__ unsigned long long lds_tree[];
    if (reject_nonfinite(sumsq, m, r, idx, rho, status, &sh)) return;
    if (r == 0) return;  // nothing to select: only the status word is written
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
    unsigned long long* tree = kTreeInLds ? lds_tree : ws_tree;

    double wmax = 0.0;
    for (int64_t k = tid; k < m; k += kThreads) {
        const double w = weight_of(sumsq[k], method);
        wmax = w > wmax ? w : wmax;
    }
    wmax = block_max(wmax, &sh);

    // padding entries of the inner levels (children that do not exist) weigh 0
    for (int L = 1; L < shape.levels; ++L)
        for (int64_t e = shape.groups[L - 1] + tid; e < shape.groups[L] * kWave; e += kThreads)
            tree[shape.offset[L] + e] = 0ull;
    __threadfence_block();
    __syncthreads();
    // level by level: prefix sums inside each group; the group's sum goes up one level
    for (int L = 0; L < shape.levels; ++L) {
        for (int64_t g = wave; g < shape.groups[L]; g += kWaves) {
            const int64_t e = g * kWave + lane;
            unsigned long long v;
            if (L == 0) v = e < m ? quantise(weight_of(sumsq[e], method), wmax) : 0ull;
            else v = tree[shape.offset[L] + e];
            v = wave_inclusive_scan(v);
            tree[shape.offset[L] + e] = v;
            if (lane == kWave - 1 && L + 1 < shape.levels) tree[shape.offset[L + 1] + g] = v;
        }
        __threadfence_block();
        __syncthreads();
    }
    const unsigned long long total_w = tree[shape.offset[shape.levels - 1] + kWave - 1];

    if (wave == 0) draw_dispatch<!kTreeInLds>(tree, shape, r, seed, refresh, total_w, lane);
    __threadfence_block();
    __syncthreads();

    // chosen leaves now weigh 0 (every weight started >= 1): compact them in row order
    uint32_t carry = 0;
    for (int64_t base = 0; base < m; base += kThreads) {
        const int64_t k = base + tid;
        uint32_t chosen = 0;
        if (k < m) {
            const unsigned long long here = tree[k];  // level 0 starts at offset 0
            const unsigned long long before = (k & (kWave - 1)) ? tree[k - 1] : 0ull;
            chosen = here == before ? 1u : 0u;
        }
        uint32_t total;
        const uint32_t pos = carry + block_exclusive_scan(chosen, &sh, total);
        if (chosen) {
            float rk = 1.0f;
            if (rescale) {
                const unsigned long long wq = quantise(weight_of(sumsq[k], method), wmax);
                const double q = static_cast<double>(wq) / static_cast<double>(total_w);
                rk = static_cast<float>(1.0 / sqrt(static_cast<double>(r) * q));
            }
            idx[pos] = static_cast<int32_t>(k);
            rho[pos] = rk;
        }
        carry += total;
    }
}

TreeShape tree_shape(int64_t m) {
    TreeShape s;
    s.levels = 0;
    int64_t groups = m > 0 ? (m + kWave - 1) / kWave : 1, off = 0;
    while (true) {
        s.groups[s.levels] = groups;
        s.offset[s.levels] = off;
        ++s.levels;
        if (groups == 1 || s.levels == kMaxLevels) break;
        off += groups * kWave;
        groups = (groups + kWave - 1) / kWave;
    }
    return s;
}

size_t tree_bytes(const TreeShape& s) {
    return static_cast<size_t>(s.offset[s.levels - 1] + s.groups[s.levels - 1] * kWave) *
           sizeof(unsigned long long);
}

}  // namespace

size_t select_workspace_bytes(int64_t m, int64_t r, grass_method method, int replacement) {
    (void)r;
    if (m < 0) m = 0;
    if (method == GRASS_SEL_TOPR) return kHeaderBytes;
    if (replacement) return kHeaderBytes + static_cast<size_t>(m) * 8 + static_cast<size_t>(m) * 4;
    return kHeaderBytes + tree_bytes(tree_shape(m));
}

// `status`: the device status word; `body`: select_workspace_bytes(...) - kHeaderBytes bytes of
// device scratch (prefix sums and hit counters, or the tree), 256-byte aligned.
static grass_status launch_select_kernels(const float* sumsq, int64_t m, int64_t r,
                                          grass_method method, int replacement, grass_scale scale,
                                          uint64_t seed, uint64_t refresh_id, int32_t* idx,
                                          float* rho, int32_t* status, char* body, hipStream_t s) {
    if (method == GRASS_SEL_TOPR) {
        select_topr_kernel<<<1, kThreads, 0, s>>>(sumsq, m, r, idx, rho, status);
        return launch_status();
    }
    const int rescale =
        scale == GRASS_SCALE_INV_SQRT_RQ || (scale == GRASS_SCALE_PAPER && replacement);
    if (replacement) {
        unsigned long long* csum = reinterpret_cast<unsigned long long*>(body);
        uint32_t* hits = reinterpret_cast<uint32_t*>(body + static_cast<size_t>(m) * 8);
        select_repl_kernel<<<1, kThreads, 0, s>>>(sumsq, m, r, method, rescale, seed, refresh_id,
                                                  idx, rho, status, csum, hits);
        return launch_status();
    }
    const TreeShape shape = tree_shape(m);
    const size_t bytes = tree_bytes(shape);
    unsigned long long* ws_tree = reinterpret_cast<unsigned long long*>(body);
    if (bytes <= kLdsTreeBytes) {
        if (bytes > 48 * 1024 &&
            hipFuncSetAttribute(reinterpret_cast<const void*>(select_norepl_kernel<true>),
                                hipFuncAttributeMaxDynamicSharedMemorySize,
                                static_cast<int>(bytes)) != hipSuccess)
            return GRASS_ERR_DEVICE;
        select_norepl_kernel<true><<<1, kThreads, bytes, s>>>(
            sumsq, m, r, method, rescale, seed, refresh_id, idx, rho, status, ws_tree, shape);
    } else {
        select_norepl_kernel<false><<<1, kThreads, 0, s>>>(
            sumsq, m, r, method, rescale, seed, refresh_id, idx, rho, status, ws_tree, shape);
    }
    return launch_status();
}

grass_status launch_select(const float* sumsq, int64_t m, int64_t r, grass_method method,
                           int replacement, grass_scale scale, uint64_t seed, uint64_t refresh_id,
                           int32_t* idx, float* rho, void* ws, hipStream_t s) {
    return launch_select_kernels(sumsq, m, r, method, replacement, scale, seed, refresh_id, idx, rho,
                                 static_cast<int32_t*>(ws), static_cast<char*>(ws) + kHeaderBytes, s);
}

size_t select_static_scratch_bytes() { return kStaticScratchBytes; }

// Address of this device's copy of `scratch`, resolved once per device (with that device
// current) and kept; every later call only reads the table.
static grass_status static_scratch_address(char** out) {
    constexpr int kMaxDevices = 64;
    static std::atomic<char*> address[kMaxDevices];
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return GRASS_ERR_DEVICE;
    char* p = address[dev].load(std::memory_order_acquire);
    if (!p) {
        void* sym = nullptr;
        if (hipGetSymbolAddress(&sym, HIP_SYMBOL(scratch)) != hipSuccess || !sym)
            return GRASS_ERR_DEVICE;
        p = static_cast<char*>(sym);
        address[dev].store(p, std::memory_order_release);  // two first callers store the same value
    }
    *out = p;
    return GRASS_OK;
}

grass_status launch_select_static(const float* sumsq, int64_t m, int64_t r, grass_method method,
                                  int replacement, grass_scale scale, uint64_t seed,
                                  uint64_t refresh_id, int32_t* idx, float* rho, int32_t* status,
                                  hipStream_t s) {
    if (select_workspace_bytes(m, r, method, replacement) > kStaticScratchBytes)
        return GRASS_ERR_WORKSPACE;  // checked by the caller too; never launch past the array
    char* base = nullptr;
    const grass_status st = static_scratch_address(&base);
    if (st != GRASS_OK) return st;
    // Nothing in the scratch has to start at zero: the kernels initialise the prefix sums, the
    // hit counters and every level of the tree (padding included) before they read them, so
    // what the previous call left behind is never seen.
    return launch_select_kernels(sumsq, m, r, method, replacement, scale, seed, refresh_id, idx, rho,
                                 status ? status : reinterpret_cast<int32_t*>(base),
                                 base + kHeaderBytes, s);
}

}  // namespace grass
