// Device-wide integer primitives for graph construction: exclusive prefix sum, stable
// least-significant-digit radix sort (keys alone or keys with a payload), and ordered selection
// (of which the removal of equal neighbours is one use).  Hand-written for 64-wide wavefronts;
// all of them are used only while a matrix or a schedule is built, never inside an epoch.
//
// Every function here is synchronous with respect to its stream when it returns: temporary buffers
// are owned by the call and released before it ends.
#pragma once
#include <type_traits>

#include "common.h"

namespace gcn {
namespace prims {

constexpr int P_TPB = 256;                 // 4 wavefronts
constexpr int P_WAVES = P_TPB / 64;
constexpr int SCAN_ITEMS = 8;              // consecutive elements per thread
constexpr int SCAN_TILE = P_TPB * SCAN_ITEMS;
constexpr int RS_ROUNDS = 32;              // 256 keys per round
constexpr int RS_TILE = P_TPB * RS_ROUNDS;
constexpr int RS_RADIX = 256;              // 8-bit digits

struct NoValue {};

struct Scratch {   // frees on scope exit
    void* p = nullptr;
    ~Scratch() { device_free(p); }
    int alloc(size_t bytes) { device_free(p); p = nullptr; return device_alloc(&p, bytes ? bytes : 16); }
    template <typename T> T* as() const { return (T*)p; }
};

// ---- wavefront and workgroup scans -----------------------------------------------------------------

template <typename T> __device__ inline T shfl_up_any(T v, int d) {
    if constexpr (sizeof(T) == 8) return (T)__shfl_up((unsigned long long)v, d, 64);
    else return (T)__shfl_up((unsigned)v, d, 64);
}

template <typename T> __device__ inline T wave_inclusive_sum(T v) {
    const int lane = threadIdx.x & 63;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        T u = shfl_up_any(v, d);
        if (lane >= d) v += u;
    }
    return v;
}

// Exclusive prefix of v over the 256 threads of the workgroup; total receives the workgroup's sum.
// part is P_WAVES elements of LDS; the call ends with a barrier, so part may be reused at once.
template <typename T> __device__ inline T block_exclusive_sum(T v, T* part, T& total) {
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const T inc = wave_inclusive_sum(v);
    if (lane == 63) part[w] = inc;
    __syncthreads();
    T base = 0, all = 0;
#pragma unroll
    for (int i = 0; i < P_WAVES; ++i) {
        const T p = part[i];
        if (i < w) base += p;
        all += p;
    }
    __syncthreads();
    total = all;
    return base + inc - v;
}

// ---- exclusive prefix sum --------------------------------------------------------------------------

template <typename T>
__global__ __launch_bounds__(P_TPB) void k_scan_tile_sums(const T* __restrict__ in, size_t n, T* __restrict__ sums) {
    __shared__ T part[P_WAVES];
    const size_t base = (size_t)blockIdx.x * SCAN_TILE + (size_t)threadIdx.x * SCAN_ITEMS;
    T a = 0;
#pragma unroll
    for (int k = 0; k < SCAN_ITEMS; ++k)
        if (base + k < n) a += in[base + k];
    T total;
    block_exclusive_sum(a, part, total);
    if (threadIdx.x == 0) sums[blockIdx.x] = total;
}

// in == out is allowed: a workgroup reads its whole tile before it writes any of it.
template <typename T>
__global__ __launch_bounds__(P_TPB) void k_scan_tiles(const T* in, T* out, size_t n, const T* __restrict__ tile_off) {
    __shared__ T part[P_WAVES];
    const size_t base = (size_t)blockIdx.x * SCAN_TILE + (size_t)threadIdx.x * SCAN_ITEMS;
    T x[SCAN_ITEMS];
    T a = 0;
#pragma unroll
    for (int k = 0; k < SCAN_ITEMS; ++k) {
        x[k] = base + k < n ? in[base + k] : (T)0;
        a += x[k];
    }
    T total;
    T run = block_exclusive_sum(a, part, total) + (tile_off ? tile_off[blockIdx.x] : (T)0);
#pragma unroll
    for (int k = 0; k < SCAN_ITEMS; ++k) {
        if (base + k < n) out[base + k] = run;
        run += x[k];
    }
}

// out[i] = in[0] + ... + in[i-1]; in == out allowed.
template <typename T> int exclusive_scan(const T* in, T* out, size_t n, hipStream_t s) {
    if (n == 0) return GCN_OK;
    const size_t ntiles = (n + SCAN_TILE - 1) / SCAN_TILE;
    if (ntiles >= (1ull << 31)) return fail(GCN_ERR_RANGE, "exclusive_scan: %zu elements are too many", n);
    if (ntiles == 1) {
        hipLaunchKernelGGL(k_scan_tiles<T>, dim3(1), dim3(P_TPB), 0, s, in, out, n, (const T*)nullptr);
        GCN_LAUNCH_CHECK();
        GCN_HIP_TRY(hipStreamSynchronize(s));
        return GCN_OK;
    }
    Scratch sums;
    GCN_TRY(sums.alloc(ntiles * sizeof(T)));
    hipLaunchKernelGGL(k_scan_tile_sums<T>, dim3((unsigned)ntiles), dim3(P_TPB), 0, s, in, n, sums.as<T>());
    GCN_LAUNCH_CHECK();
    GCN_TRY(exclusive_scan<T>(sums.as<T>(), sums.as<T>(), ntiles, s));
    hipLaunchKernelGGL(k_scan_tiles<T>, dim3((unsigned)ntiles), dim3(P_TPB), 0, s, in, out, n, (const T*)sums.as<T>());
    GCN_LAUNCH_CHECK();
    GCN_HIP_TRY(hipStreamSynchronize(s));
    return GCN_OK;
}

// ---- ordered selection -----------------------------------------------------------------------------
// pred(i) decides whether index i is kept; emit(i, pos) stores it as the pos-th kept one.  Kept
// indices keep their order.  Both functors are called once per index in each of two passes.

template <typename Pred>
__global__ __launch_bounds__(P_TPB) void k_select_count(int64_t n, Pred pred, int64_t* __restrict__ tile_cnt) {
    __shared__ int part[P_WAVES];
    const int64_t base = (int64_t)blockIdx.x * SCAN_TILE + (int64_t)threadIdx.x * SCAN_ITEMS;
    int c = 0;
#pragma unroll
    for (int k = 0; k < SCAN_ITEMS; ++k)
        if (base + k < n && pred(base + k)) ++c;
    int total;
    block_exclusive_sum(c, part, total);
    if (threadIdx.x == 0) tile_cnt[blockIdx.x] = total;
}

template <typename Pred, typename Emit>
__global__ __launch_bounds__(P_TPB) void k_select_emit(int64_t n, Pred pred, Emit emit,
                                                      const int64_t* __restrict__ tile_off) {
    __shared__ int part[P_WAVES];
    const int64_t base = (int64_t)blockIdx.x * SCAN_TILE + (int64_t)threadIdx.x * SCAN_ITEMS;
    unsigned keep = 0;
    int c = 0;
#pragma unroll
    for (int k = 0; k < SCAN_ITEMS; ++k)
        if (base + k < n && pred(base + k)) { keep |= 1u << k; ++c; }
    int total;
    int64_t pos = tile_off[blockIdx.x] + block_exclusive_sum(c, part, total);
#pragma unroll
    for (int k = 0; k < SCAN_ITEMS; ++k)
        if (keep >> k & 1u) emit(base + k, pos++);
}

template <typename Pred, typename Emit> int select(int64_t n, Pred pred, Emit emit, int64_t* count, hipStream_t s) {
    if (count) *count = 0;
    if (n <= 0) return GCN_OK;
    const int64_t ntiles = (n + SCAN_TILE - 1) / SCAN_TILE;
    if (ntiles >= (1ll << 31)) return fail(GCN_ERR_RANGE, "select: %lld candidates are too many", (long long)n);
    Scratch cnt;
    GCN_TRY(cnt.alloc((size_t)(ntiles + 1) * 8));
    GCN_HIP_TRY(hipMemsetAsync(cnt.as<int64_t>() + ntiles, 0, 8, s));
    hipLaunchKernelGGL(k_select_count<Pred>, dim3((unsigned)ntiles), dim3(P_TPB), 0, s, n, pred, cnt.as<int64_t>());
    GCN_LAUNCH_CHECK();
    GCN_TRY(exclusive_scan<int64_t>(cnt.as<int64_t>(), cnt.as<int64_t>(), (size_t)ntiles + 1, s));
    hipLaunchKernelGGL((k_select_emit<Pred, Emit>), dim3((unsigned)ntiles), dim3(P_TPB), 0, s, n, pred, emit,
                       (const int64_t*)cnt.as<int64_t>());
    GCN_LAUNCH_CHECK();
    int64_t total = 0;
    GCN_HIP_TRY(hipMemcpyAsync(&total, cnt.as<int64_t>() + ntiles, 8, hipMemcpyDeviceToHost, s));
    GCN_HIP_TRY(hipStreamSynchronize(s));
    if (count) *count = total;
    return GCN_OK;
}

struct EmitIndex32 {   // out[pos] = i
    int32_t* out;
    __device__ void operator()(int64_t i, int64_t pos) const { out[pos] = (int32_t)i; }
};

// The indices 0 <= i < n (n below 2^31) with pred(i), ascending.
template <typename Pred> int select_indices(int64_t n, Pred pred, int32_t* out, int64_t* count, hipStream_t s) {
    if (n >= (1ll << 31)) return fail(GCN_ERR_RANGE, "select_indices: %lld candidates do not fit 32-bit ids", (long long)n);
    return select(n, pred, EmitIndex32{out}, count, s);
}

struct FirstOfRun {
    const uint64_t* in;
    __device__ bool operator()(int64_t i) const { return i == 0 || in[i] != in[i - 1]; }
};
struct EmitKey {
    const uint64_t* in;
    uint64_t* out;
    __device__ void operator()(int64_t i, int64_t pos) const { out[pos] = in[i]; }
};

// Keeps the first key of every run of equal neighbours (in and out must not overlap).
inline int unique_keys(const uint64_t* in, uint64_t* out, int64_t n, int64_t* count, hipStream_t s) {
    return select(n, FirstOfRun{in}, EmitKey{in, out}, count, s);
}

// ---- radix sort ------------------------------------------------------------------------------------
// One pass orders the keys by one 8-bit digit and keeps the order of equal digits, so passes from
// the lowest digit upwards sort the keys and equal keys keep their input order.  A pass takes three
// steps: every workgroup counts the digits of its tile of RS_TILE keys; an exclusive prefix sum of
// the counts laid out digit-major (digit d of tile t at d*ntiles + t) gives each (digit, tile) its
// first output position; the workgroup then reads the tile again, 256 keys at a time, ranks each
// key among the tile's earlier keys of the same digit and stores it (and its payload).

template <typename K> __device__ inline unsigned digit_of(K key, unsigned shift, unsigned mask, unsigned flip) {
    return ((unsigned)(key >> shift) & mask) ^ flip;
}

// Whole-key histograms of every digit position at once: hist[p*256 + d] = keys whose p-th byte is d.
template <typename K>
__global__ __launch_bounds__(P_TPB) void k_radix_byte_hist(const K* __restrict__ keys, size_t n,
                                                          unsigned long long* __restrict__ hist) {
    constexpr int NB = sizeof(K);
    __shared__ unsigned h[NB * RS_RADIX];
    for (int i = threadIdx.x; i < NB * RS_RADIX; i += P_TPB) h[i] = 0;
    __syncthreads();
    // a thread adds a run of equal bytes with one LDS atomic: positions at which all keys agree
    // (the unused high bytes of small ids) would otherwise serialise on one counter
    const size_t base = (size_t)blockIdx.x * RS_TILE;
    unsigned last[NB], run[NB];
#pragma unroll
    for (int p = 0; p < NB; ++p) { last[p] = 0; run[p] = 0; }
    for (int r = 0; r < RS_ROUNDS; ++r) {
        const size_t i = base + (size_t)r * P_TPB + threadIdx.x;
        if (i < n) {
            const K key = keys[i];
#pragma unroll
            for (int p = 0; p < NB; ++p) {
                const unsigned d = (unsigned)(key >> (8 * p)) & 255u;
                if (run[p] && d != last[p]) { atomicAdd(&h[p * RS_RADIX + last[p]], run[p]); run[p] = 0; }
                last[p] = d;
                ++run[p];
            }
        }
    }
#pragma unroll
    for (int p = 0; p < NB; ++p)
        if (run[p]) atomicAdd(&h[p * RS_RADIX + last[p]], run[p]);
    __syncthreads();
    for (int i = threadIdx.x; i < NB * RS_RADIX; i += P_TPB)
        if (h[i]) atomicAdd(&hist[i], (unsigned long long)h[i]);
}

template <typename K, typename Off>
__global__ __launch_bounds__(P_TPB) void k_radix_tile_hist(const K* __restrict__ keys, size_t n, unsigned shift,
                                                          unsigned mask, unsigned flip, size_t ntiles,
                                                          Off* __restrict__ hist) {
    __shared__ unsigned h[RS_RADIX];
    h[threadIdx.x] = 0;
    __syncthreads();
    const size_t base = (size_t)blockIdx.x * RS_TILE;
    unsigned last = 0, run = 0;
    for (int r = 0; r < RS_ROUNDS; ++r) {
        const size_t i = base + (size_t)r * P_TPB + threadIdx.x;
        if (i < n) {
            const unsigned d = digit_of(keys[i], shift, mask, flip);
            if (run && d != last) { atomicAdd(&h[last], run); run = 0; }
            last = d;
            ++run;
        }
    }
    if (run) atomicAdd(&h[last], run);
    __syncthreads();
    hist[(size_t)threadIdx.x * ntiles + blockIdx.x] = (Off)h[threadIdx.x];
}

template <typename K, typename V, typename Off>
__global__ __launch_bounds__(P_TPB) void k_radix_scatter(const K* __restrict__ kin, K* __restrict__ kout,
                                                        const V* __restrict__ vin, V* __restrict__ vout, size_t n,
                                                        unsigned shift, unsigned mask, unsigned flip, size_t ntiles,
                                                        const Off* __restrict__ first) {
    __shared__ Off next[RS_RADIX];                 // output position of the tile's next key of each digit
    __shared__ unsigned wcnt[P_WAVES][RS_RADIX];   // this round's keys of each digit, by wavefront
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    next[threadIdx.x] = first[(size_t)threadIdx.x * ntiles + blockIdx.x];
#pragma unroll
    for (int i = 0; i < P_WAVES; ++i) wcnt[i][threadIdx.x] = 0;
    __syncthreads();
    const size_t base = (size_t)blockIdx.x * RS_TILE;
    for (int r = 0; r < RS_ROUNDS; ++r) {
        const size_t i = base + (size_t)r * P_TPB + threadIdx.x;
        if (base + (size_t)r * P_TPB >= n) break;              // uniform over the workgroup
        const bool valid = i < n;
        K key = 0;
        unsigned d = 0;
        if (valid) { key = kin[i]; d = digit_of(key, shift, mask, flip); }
        // lanes of this wavefront that hold the same digit
        unsigned long long peers = __ballot(valid);
#pragma unroll
        for (int b = 0; b < 8; ++b) {
            const bool bit = d >> b & 1u;
            const unsigned long long have = __ballot(valid && bit);
            peers &= bit ? have : ~have;
        }
        const int rank = __popcll(peers & ((1ull << lane) - 1ull));
        if (valid && rank == 0) wcnt[w][d] = (unsigned)__popcll(peers);
        __syncthreads();
        Off pos = 0;
        if (valid) {
            pos = next[d] + (Off)rank;
            for (int i2 = 0; i2 < w; ++i2) pos += (Off)wcnt[i2][d];
        }
        __syncthreads();
        {
            unsigned t = 0;
#pragma unroll
            for (int i2 = 0; i2 < P_WAVES; ++i2) { t += wcnt[i2][threadIdx.x]; wcnt[i2][threadIdx.x] = 0; }
            next[threadIdx.x] += (Off)t;
        }
        __syncthreads();
        if (valid) {
            kout[pos] = key;
            if constexpr (!std::is_same<V, NoValue>::value) vout[pos] = vin[i];
        }
    }
}

template <typename K, typename V, typename Off>
int radix_passes(const K* kin, K* kout, const V* vin, V* vout, size_t n, const unsigned* shifts, const unsigned* masks,
                 int npass, bool descending, hipStream_t s) {
    constexpr bool HAS_V = !std::is_same<V, NoValue>::value;
    const size_t ntiles = (n + RS_TILE - 1) / RS_TILE;
    Scratch hist, tk, tv;
    GCN_TRY(hist.alloc(ntiles * RS_RADIX * sizeof(Off)));
    if (npass >= 2) {
        GCN_TRY(tk.alloc(n * sizeof(K)));
        if (HAS_V) GCN_TRY(tv.alloc(n * sizeof(V)));
    }
    const K* ksrc = kin;
    const V* vsrc = vin;
    for (int p = 0; p < npass; ++p) {
        const bool to_out = ((npass - 1 - p) % 2) == 0;      // the last pass lands in the caller's output
        K* kdst = to_out ? kout : tk.as<K>();
        V* vdst = to_out ? vout : tv.as<V>();
        const unsigned flip = descending ? masks[p] : 0u;
        hipLaunchKernelGGL((k_radix_tile_hist<K, Off>), dim3((unsigned)ntiles), dim3(P_TPB), 0, s, ksrc, n, shifts[p],
                           masks[p], flip, ntiles, hist.as<Off>());
        GCN_LAUNCH_CHECK();
        GCN_TRY(exclusive_scan<Off>(hist.as<Off>(), hist.as<Off>(), ntiles * RS_RADIX, s));
        hipLaunchKernelGGL((k_radix_scatter<K, V, Off>), dim3((unsigned)ntiles), dim3(P_TPB), 0, s, ksrc, kdst, vsrc,
                           vdst, n, shifts[p], masks[p], flip, ntiles, (const Off*)hist.as<Off>());
        GCN_LAUNCH_CHECK();
        ksrc = kdst;
        vsrc = vdst;
    }
    GCN_HIP_TRY(hipStreamSynchronize(s));
    return GCN_OK;
}

// Stable sort of n keys by their bits [0, end_bit), ascending or descending; the payload (if V is
// not NoValue) moves with its key.  The inputs are left as they were; outputs must not overlap them.
// Digit positions at which every key holds the same byte are skipped.
template <typename K, typename V>
int radix_sort(const K* kin, K* kout, const V* vin, V* vout, size_t n, unsigned end_bit, bool descending, hipStream_t s) {
    constexpr bool HAS_V = !std::is_same<V, NoValue>::value;
    constexpr int NB = sizeof(K);
    if (n == 0) return GCN_OK;
    if (end_bit > 8 * NB) end_bit = 8 * NB;
    const size_t ntiles = (n + RS_TILE - 1) / RS_TILE;
    if (ntiles >= (1ull << 31)) return fail(GCN_ERR_RANGE, "radix_sort: %zu keys are too many", n);
    Scratch bh;
    GCN_TRY(bh.alloc(NB * RS_RADIX * 8));
    GCN_HIP_TRY(hipMemsetAsync(bh.p, 0, NB * RS_RADIX * 8, s));
    hipLaunchKernelGGL(k_radix_byte_hist<K>, dim3((unsigned)ntiles), dim3(P_TPB), 0, s, kin, n,
                       bh.as<unsigned long long>());
    GCN_LAUNCH_CHECK();
    unsigned long long h[NB * RS_RADIX];
    GCN_HIP_TRY(hipMemcpyAsync(h, bh.p, sizeof(h), hipMemcpyDeviceToHost, s));
    GCN_HIP_TRY(hipStreamSynchronize(s));
    unsigned shifts[NB], masks[NB];
    int npass = 0;
    for (int p = 0; p * 8 < (int)end_bit; ++p) {
        const unsigned width = end_bit - 8 * p < 8 ? end_bit - 8 * p : 8;
        const unsigned mask = (1u << width) - 1u;
        // bins of the masked digit: fold the byte histogram
        bool trivial = false;
        for (unsigned d = 0; d <= mask && !trivial; ++d) {
            unsigned long long c = 0;
            for (unsigned hi = d; hi < RS_RADIX; hi += mask + 1) c += h[p * RS_RADIX + hi];
            trivial = (c == n);
        }
        if (trivial) continue;
        shifts[npass] = 8 * p;
        masks[npass] = mask;
        ++npass;
    }
    if (npass == 0) {
        GCN_HIP_TRY(hipMemcpyAsync(kout, kin, n * sizeof(K), hipMemcpyDeviceToDevice, s));
        if (HAS_V) GCN_HIP_TRY(hipMemcpyAsync((void*)vout, (const void*)vin, n * sizeof(V), hipMemcpyDeviceToDevice, s));
        GCN_HIP_TRY(hipStreamSynchronize(s));
        return GCN_OK;
    }
    // positions are 64-bit whatever n is (their table is 1/32 of the keys' size): one code path at every size
    return radix_passes<K, V, unsigned long long>(kin, kout, vin, vout, n, shifts, masks, npass, descending, s);
}

template <typename K> int sort_keys(const K* in, K* out, size_t n, unsigned end_bit, hipStream_t s) {
    return radix_sort<K, NoValue>(in, out, (const NoValue*)nullptr, (NoValue*)nullptr, n, end_bit, false, s);
}
template <typename K, typename V>
int sort_pairs(const K* kin, K* kout, const V* vin, V* vout, size_t n, unsigned end_bit, hipStream_t s) {
    return radix_sort<K, V>(kin, kout, vin, vout, n, end_bit, false, s);
}
template <typename K, typename V>
int sort_pairs_descending(const K* kin, K* kout, const V* vin, V* vout, size_t n, unsigned end_bit, hipStream_t s) {
    return radix_sort<K, V>(kin, kout, vin, vout, n, end_bit, true, s);
}

}  // namespace prims
}  // namespace gcn
