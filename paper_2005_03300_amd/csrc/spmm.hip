// SpMM: Z = op(A) X for a compressed-row matrix and a tall-skinny dense fp32 operand -- the
// "SpMM" of the paper's sections "Graph Neural Networks" and "A One-Dimensional (1D) Algorithm",
// the operation the paper calls the most time consuming.
//
// Main kernel: nonzero-split.  Every wavefront owns CHUNK = 512 consecutive stored entries no
// matter how they fall into rows, so a 20,000-entry row and 20,000 one-entry rows cost the same.
// The wavefront is cut into G = 64/LPR lane groups; a group of LPR lanes covers one gathered row
// of X (VEC floats per lane) and walks its own contiguous slice of the chunk.  Row boundaries come
// from one precomputed 32-bit flag word per 32 entries, so the walk never touches rowptr.
//   * a row that starts and ends inside one group's slice is written directly;
//   * pieces of a row spread over several groups are joined by a segmented suffix scan across the
//     groups (lane shuffles), in a fixed order;
//   * pieces spread over several wavefronts go through a per-chunk carry buffer and a small
//     second kernel that adds them in ascending chunk order.
// No floating-point atomics are used anywhere: results are bit-reproducible run to run.
// Column indices and values are read with coalesced 16-byte loads into LDS first and consumed
// from there; the gathered rows of X are read with one 16-byte load per lane.
#include <algorithm>
#include <mutex>
#include <string>

#include "common.h"

namespace gcn {

static constexpr int WAVES_PER_BLOCK = 4;
#ifndef SPLIT_UNROLL
#define SPLIT_UNROLL 4
#endif
static constexpr int SUB_STRIDE = SUB + 4;                         // LDS padding: groups hit different banks
static constexpr int LDS_PER_WAVE = SUBS_PER_CHUNK * SUB_STRIDE;   // ints

struct SplitArgs {
    const int32_t* colidx;
    const float* val;         // NULL: value-free product (every stored entry counts as 1)
    const float* row_scale;   // NULL, or one factor per output row applied before the epilogue
    const uint8_t* defer;     // NULL, or 1 for rows whose sum is stored raw (another pass finishes them)
    const uint32_t* flags;
    const int32_t* sub_row;
    const int32_t* ne_rows;   // NULL: row index == non-empty-row index
    const int64_t* rp;        // rowptr over non-empty rows
    const int32_t* fix_list;  // chunks with work for the fix-up kernel (n_fix of them), or n_fix < 0: all chunks
    int64_t n_fix;
    int64_t nnz, nsub, nchunks;
    int32_t f;
    const float* X;
    int64_t ldx;
    float* Z;
    int64_t ldz;
    const float* Zprev;
    int64_t ldzprev;
    float* carry;             // [nchunks][f]
    int lds_kb;               // host side: LDS per workgroup of the narrow kernel, padding included (settings)
};

// The index/value stream is read exactly once per product: load it with the non-temporal hint so
// it does not push the gathered rows of X out of L2.
typedef int intx4 __attribute__((ext_vector_type(4)));
typedef float fltx4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ int4 stream_load_i4(const int32_t* p) {
    const intx4 v = __builtin_nontemporal_load(reinterpret_cast<const intx4*>(p));
    return make_int4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ float4 stream_load_f4(const float* p) {
    const fltx4 v = __builtin_nontemporal_load(reinterpret_cast<const fltx4*>(p));
    return make_float4(v.x, v.y, v.z, v.w);
}

template <int VEC> struct Vec;
template <> struct Vec<4> { using T = float4; };
template <> struct Vec<1> { using T = float; };

template <int VEC>
__device__ __forceinline__ void load_vec(float (&d)[VEC], const float* p) {
    if constexpr (VEC == 4) {
        float4 v = *reinterpret_cast<const float4*>(p);
        d[0] = v.x; d[1] = v.y; d[2] = v.z; d[3] = v.w;
    } else {
        d[0] = *p;
    }
}

template <int VEC>
__device__ __forceinline__ void store_vec(float* p, const float (&d)[VEC]) {
    if constexpr (VEC == 4) {
        *reinterpret_cast<float4*>(p) = make_float4(d[0], d[1], d[2], d[3]);
    } else {
        *p = d[0];
    }
}

template <int VEC, int EPI>
__device__ __forceinline__ void epilogue_store(float* z, const float* zprev, float (&v)[VEC], float scale = 1.f,
                                               bool raw = false) {
    if (raw) {
        store_vec<VEC>(z, v);
        return;
    }
#pragma unroll
    for (int e = 0; e < VEC; ++e) v[e] *= scale;           // exact for scale = 1
    if constexpr (EPI == GCN_EPI_RELU) {
#pragma unroll
        for (int e = 0; e < VEC; ++e) v[e] = v[e] > 0.f ? v[e] : 0.f;
    } else if constexpr (EPI == GCN_EPI_MASK) {
        float m[VEC];
        load_vec<VEC>(m, zprev);
#pragma unroll
        for (int e = 0; e < VEC; ++e) v[e] = m[e] > 0.f ? v[e] : 0.f;
    }
    store_vec<VEC>(z, v);
}

// The work of one workgroup: the four chunks 4*grp .. 4*grp+3 of the matrix described by `a`.
// s_col / s_val: the workgroup's staging arrays, [WAVES_PER_BLOCK][LDS_PER_WAVE] each (owned by the kernel,
// so that two instantiations of this body in one kernel share them).
template <int LPR, int VEC, int EPI>
__device__ __forceinline__ void split_body(const SplitArgs& a, int64_t grp, int32_t (*s_col)[LDS_PER_WAVE],
                                           float (*s_val)[LDS_PER_WAVE]) {
    constexpr int G = 64 / LPR;                 // lane groups per wavefront
    constexpr int NW = SUBS_PER_CHUNK / G;      // flag words per group
    static_assert(NW >= 1, "a group needs at least one flag word");
    constexpr int UNR = SPLIT_UNROLL;           // gathers in flight per lane group

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t c = grp * WAVES_PER_BLOCK + wave;
    if (c >= a.nchunks) return;                 // whole wavefront leaves; no block-wide barrier below
    const int g = lane / LPR, li = lane % LPR;
    const int col0 = blockIdx.y * (LPR * VEC) + li * VEC;
    const bool col_ok = col0 < a.f;
    const int64_t k0 = c * CHUNK;

    // ---- stage the chunk's column indices and values in LDS (coalesced 16-byte loads) ----
    int32_t* lc = s_col[wave];
    float* lv = s_val[wave];
#pragma unroll
    for (int t = 0; t < CHUNK / 256; ++t) {
        const int i = t * 256 + lane * 4;
        const int64_t k = k0 + i;
        int4 cc = make_int4(0, 0, 0, 0);
        float4 vv = make_float4(0.f, 0.f, 0.f, 0.f);
        if (!a.val) {                           // value-free: only the column stream is read
            vv = make_float4(1.f, 1.f, 1.f, 1.f);
            if (k + 4 <= a.nnz) {
                cc = stream_load_i4(a.colidx + k);
            } else {
                if (k + 0 < a.nnz) cc.x = a.colidx[k + 0];
                if (k + 1 < a.nnz) cc.y = a.colidx[k + 1];
                if (k + 2 < a.nnz) cc.z = a.colidx[k + 2];
            }
        } else if (k + 4 <= a.nnz) {
            cc = stream_load_i4(a.colidx + k);
            vv = stream_load_f4(a.val + k);
        } else {
            if (k + 0 < a.nnz) { cc.x = a.colidx[k + 0]; vv.x = a.val[k + 0]; }
            if (k + 1 < a.nnz) { cc.y = a.colidx[k + 1]; vv.y = a.val[k + 1]; }
            if (k + 2 < a.nnz) { cc.z = a.colidx[k + 2]; vv.z = a.val[k + 2]; }
        }
        const int p = i + (i >> 5) * (SUB_STRIDE - SUB);
        *reinterpret_cast<int4*>(lc + p) = cc;
        *reinterpret_cast<float4*>(lv + p) = vv;
    }
    // each wavefront reads only what it wrote; LDS operations of one wavefront complete in order
    __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
    __builtin_amdgcn_wave_barrier();

    // ---- walk this group's slice ----
    const int64_t j0 = c * SUBS_PER_CHUNK + (int64_t)g * NW;
    int32_t q = a.sub_row[j0];
    uint32_t first = a.flags[j0];
    q -= (int32_t)(first & 1u);                 // a start bit at the very first entry re-increments q
    float acc[VEC], head[VEC];
#pragma unroll
    for (int e = 0; e < VEC; ++e) { acc[e] = 0.f; head[e] = 0.f; }
    bool owned = false;                         // has this group seen a row start yet?
    const float* xbase = a.X + col0;

    for (int w = 0; w < NW; ++w) {
        const int64_t j = j0 + w;
        uint32_t mask = (w == 0) ? first : a.flags[j];
        const int64_t left = a.nnz - j * SUB;
        const int cnt = left >= SUB ? SUB : (left > 0 ? (int)left : 0);
        const int base = (g * NW + w) * SUB_STRIDE;
        for (int b = 0; b < cnt; b += UNR) {
            int32_t cs[UNR];
            float vs[UNR];
#pragma unroll
            for (int h = 0; h < UNR / 4; ++h) {
                const int4 cc = *reinterpret_cast<const int4*>(lc + base + b + 4 * h);
                const float4 vv = *reinterpret_cast<const float4*>(lv + base + b + 4 * h);
                cs[4 * h] = cc.x; cs[4 * h + 1] = cc.y; cs[4 * h + 2] = cc.z; cs[4 * h + 3] = cc.w;
                vs[4 * h] = vv.x; vs[4 * h + 1] = vv.y; vs[4 * h + 2] = vv.z; vs[4 * h + 3] = vv.w;
            }
            float x[UNR][VEC];
#pragma unroll
            for (int e = 0; e < UNR; ++e) {
                if (b + e < cnt && col_ok) load_vec<VEC>(x[e], xbase + (int64_t)cs[e] * a.ldx);
                else {
#pragma unroll
                    for (int v = 0; v < VEC; ++v) x[e][v] = 0.f;
                }
            }
#pragma unroll
            for (int e = 0; e < UNR; ++e) {
                if (b + e < cnt) {
                    if (mask & 1u) {            // entry starts a row: close the fragment before it
                        if (owned) {
                            if (col_ok) {
                                const int64_t row = a.ne_rows ? a.ne_rows[q] : q;
                                epilogue_store<VEC, EPI>(a.Z + row * a.ldz + col0,
                                                         EPI == GCN_EPI_MASK ? a.Zprev + row * a.ldzprev + col0 : nullptr,
                                                         acc, a.row_scale ? a.row_scale[row] : 1.f,
                                                         a.defer && a.defer[row]);
                            }
                        } else {
#pragma unroll
                            for (int v = 0; v < VEC; ++v) head[v] = acc[v];
                            owned = true;
                        }
                        q += 1;
#pragma unroll
                        for (int v = 0; v < VEC; ++v) acc[v] = 0.f;
                    }
                    mask >>= 1;
#pragma unroll
                    for (int v = 0; v < VEC; ++v) acc[v] = fmaf(vs[e], x[e][v], acc[v]);
                }
            }
        }
    }
    if (!owned) {                               // the whole slice lies inside one row
#pragma unroll
        for (int v = 0; v < VEC; ++v) { head[v] = acc[v]; acc[v] = 0.f; }
    }

    // ---- join fragments across groups: R_g = head_g + (owned_g ? 0 : R_{g+1}) ----
    float R[VEC];
#pragma unroll
    for (int v = 0; v < VEC; ++v) R[v] = head[v];
    int stop = owned ? 1 : 0;
#pragma unroll
    for (int d = 1; d < G; d <<= 1) {
        float Rp[VEC];
#pragma unroll
        for (int v = 0; v < VEC; ++v) Rp[v] = __shfl_down(R[v], d * LPR, 64);
        const int sp = __shfl_down(stop, d * LPR, 64);
        if (g + d < G && !stop) {
#pragma unroll
            for (int v = 0; v < VEC; ++v) R[v] += Rp[v];
            stop = sp;
        }
    }
    float T[VEC];
    int stop_next = 0;
    if constexpr (G > 1) {
#pragma unroll
        for (int v = 0; v < VEC; ++v) T[v] = __shfl_down(R[v], LPR, 64);
        stop_next = __shfl_down(stop, LPR, 64);
    }
    if (G == 1 || g == G - 1) {
#pragma unroll
        for (int v = 0; v < VEC; ++v) T[v] = 0.f;
        stop_next = 0;
    }
    if (g == 0 && col_ok) store_vec<VEC>(a.carry + c * a.f + col0, R);

    if (owned && col_ok) {
        // the row opened last in this slice: add what later groups of this wavefront hold for it
#pragma unroll
        for (int v = 0; v < VEC; ++v) acc[v] += T[v];
        const int64_t knext = k0 + CHUNK;
        const bool runs_on = !stop_next && knext < a.nnz && !(a.flags[(c + 1) * SUBS_PER_CHUNK] & 1u);
        const int64_t row = a.ne_rows ? a.ne_rows[q] : q;
        if (runs_on) store_vec<VEC>(a.Z + row * a.ldz + col0, acc);     // finished by k_spmm_fixup
        else epilogue_store<VEC, EPI>(a.Z + row * a.ldz + col0,
                                      EPI == GCN_EPI_MASK ? a.Zprev + row * a.ldzprev + col0 : nullptr, acc,
                                      a.row_scale ? a.row_scale[row] : 1.f, a.defer && a.defer[row]);
    }
}

template <int LPR, int VEC, int EPI>
__global__ __launch_bounds__(64 * WAVES_PER_BLOCK) void k_spmm_split(SplitArgs a) {
    __shared__ int32_t s_col[WAVES_PER_BLOCK][LDS_PER_WAVE];
    __shared__ float s_val[WAVES_PER_BLOCK][LDS_PER_WAVE];
    split_body<LPR, VEC, EPI>(a, blockIdx.x, s_col, s_val);
}

// Two matrices in one launch: of every ra + rb consecutive workgroups the first ra work on `a` (with
// the epilogue) and the other rb on `b` (plain sums).  Used when one part is bound by line fills and
// the other by L2 hits, so that both kinds of work are resident on every compute unit together.
template <int LPR, int VEC, int EPI>
__global__ __launch_bounds__(64 * WAVES_PER_BLOCK) void k_spmm_split_pair(SplitArgs a, SplitArgs b, int ra, int rb) {
    // ra + rb == 8.  Workgroups go to the eight XCDs round-robin; the rotation by q lets every XCD see
    // both kinds of work in turn.
    __shared__ int32_t s_col[WAVES_PER_BLOCK][LDS_PER_WAVE];
    __shared__ float s_val[WAVES_PER_BLOCK][LDS_PER_WAVE];
    const unsigned q = blockIdx.x / 8, r = (blockIdx.x + q) % 8;
    if ((int)r < ra) split_body<LPR, VEC, EPI>(a, (int64_t)q * ra + r, s_col, s_val);
    else split_body<LPR, VEC, GCN_EPI_NONE>(b, (int64_t)q * rb + (r - ra), s_col, s_val);
}

// Adds, in ascending chunk order, the carries of the chunks a row runs on into, then applies the
// epilogue.  One LPR-lane group per chunk; only the first continuation chunk of a row acts.
template <int LPR, int VEC, int EPI>
__global__ __launch_bounds__(256) void k_spmm_fixup(SplitArgs a) {
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int li = (int)(t % LPR);
    int64_t c = t / LPR + 1;                    // chunk 0 starts a row by definition
    if (a.n_fix >= 0) {                         // only the listed chunks have work
        if (t / LPR >= a.n_fix) return;
        c = a.fix_list[t / LPR];
    }
    if (c >= a.nchunks) return;
    const int col0 = blockIdx.y * (LPR * VEC) + li * VEC;
    if (col0 >= a.f) return;
    const int64_t j0 = c * SUBS_PER_CHUNK;
    if (a.flags[j0] & 1u) return;               // the chunk starts on a row start: no carry-in
    const int32_t q = a.sub_row[j0];
    const int64_t rs = a.rp[q], re = a.rp[q + 1];
    if (c != rs / CHUNK + 1) return;            // an earlier chunk leads this row
    const int64_t c_last = (re - 1) / CHUNK;
    float sum[VEC];
#pragma unroll
    for (int v = 0; v < VEC; ++v) sum[v] = 0.f;
    for (int64_t cc = c; cc <= c_last; ++cc) {
        float part[VEC];
        load_vec<VEC>(part, a.carry + cc * a.f + col0);
#pragma unroll
        for (int v = 0; v < VEC; ++v) sum[v] += part[v];
    }
    const int64_t row = a.ne_rows ? a.ne_rows[q] : q;
    float* z = a.Z + row * a.ldz + col0;
    float cur[VEC];
    load_vec<VEC>(cur, z);
#pragma unroll
    for (int v = 0; v < VEC; ++v) cur[v] += sum[v];
    epilogue_store<VEC, EPI>(z, EPI == GCN_EPI_MASK ? a.Zprev + row * a.ldzprev + col0 : nullptr, cur,
                             a.row_scale ? a.row_scale[row] : 1.f, a.defer && a.defer[row]);
}

// Rows without stored entries produce zeros (any epilogue maps 0 to 0).
__global__ void k_zero_empty_rows(int64_t n, const int64_t* __restrict__ rowptr, int32_t f, float* __restrict__ Z,
                                  int64_t ldz) {
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t i = t / f;
    const int j = (int)(t % f);
    if (i >= n) return;
    if (rowptr[i + 1] == rowptr[i]) Z[i * ldz + j] = 0.f;
}

// The same from the list of empty rows that the schedule keeps (only their elements are touched).
__global__ void k_zero_listed_rows(int64_t count, const int32_t* __restrict__ rows, int32_t f, float* __restrict__ Z,
                                   int64_t ldz) {
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t q = t / f;
    if (q < count) Z[(int64_t)rows[q] * ldz + (int)(t % f)] = 0.f;
}

// Reference-shaped kernel: one thread per output element walks its row.  Kept as a selectable
// second implementation (GCN_CFG_SPMM_ALGO = 1) for cross-checks; never chosen automatically.
template <int EPI>
__global__ void k_spmm_rowwise(int64_t n, const int64_t* __restrict__ rowptr, const int32_t* __restrict__ colidx,
                               const float* __restrict__ val, const float* __restrict__ row_scale, int32_t f,
                               const float* __restrict__ X, int64_t ldx,
                               float* __restrict__ Z, int64_t ldz, const float* __restrict__ Zprev, int64_t ldzprev) {
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t i = t / f;
    const int j = (int)(t % f);
    if (i >= n) return;
    float acc = 0.f;
    for (int64_t k = rowptr[i]; k < rowptr[i + 1]; ++k)
        acc = fmaf(val ? val[k] : 1.f, X[(int64_t)colidx[k] * ldx + j], acc);
    if (row_scale) acc *= row_scale[i];
    if (EPI == GCN_EPI_RELU) acc = acc > 0.f ? acc : 0.f;
    if (EPI == GCN_EPI_MASK) acc = Zprev[i * ldzprev + j] > 0.f ? acc : 0.f;
    Z[i * ldz + j] = acc;
}

// Dynamic LDS on top of the kernel's own 18 KB, to lower the number of resident workgroups.  The kernels
// with 16 lane groups per wavefront (rows of up to 64 bytes) keep 64 gathers in flight per wavefront; at
// full occupancy they run slower than with about two thirds of it (measured on config 3: 18 KB per
// workgroup 0.66 / 0.57 ms valued / value-free, 28 KB 0.58 / 0.55 ms, 32 KB 0.61 / 0.58 ms; plain kernel
// on config 4 4.40 -> 4.10 ms; long rows of config 5 -0.1 ms).  The 8-group kernels (config 2: 1.44 ->
// 1.59 ms at half occupancy) and the paired launch (config 4: 3.15 -> 3.34 ms) want it all.
static size_t occupancy_pad(int lpr, int lds_kb) {
    if (lpr != 4) return 0;
    const size_t own = 2 * sizeof(int32_t) * WAVES_PER_BLOCK * LDS_PER_WAVE;     // s_col + s_val
    const size_t want = (size_t)lds_kb * 1024;
    return want > own ? want - own : 0;
}

template <int LPR, int VEC>
static int launch_split(const SplitArgs& args, int epilogue, hipStream_t s) {
    const int tile = LPR * VEC;
    const unsigned ytiles = (unsigned)((args.f + tile - 1) / tile);
    const dim3 grid((unsigned)((args.nchunks + WAVES_PER_BLOCK - 1) / WAVES_PER_BLOCK), ytiles);
    const int64_t fix_threads = (args.n_fix >= 0 ? args.n_fix : args.nchunks - 1) * LPR;
    const dim3 fgrid((unsigned)((fix_threads + 255) / 256), ytiles);
    timing_begin(s);
    switch (epilogue) {
        case GCN_EPI_NONE: hipLaunchKernelGGL((k_spmm_split<LPR, VEC, GCN_EPI_NONE>), grid, dim3(64 * WAVES_PER_BLOCK), occupancy_pad(LPR, args.lds_kb), s, args); break;
        case GCN_EPI_RELU: hipLaunchKernelGGL((k_spmm_split<LPR, VEC, GCN_EPI_RELU>), grid, dim3(64 * WAVES_PER_BLOCK), occupancy_pad(LPR, args.lds_kb), s, args); break;
        default: hipLaunchKernelGGL((k_spmm_split<LPR, VEC, GCN_EPI_MASK>), grid, dim3(64 * WAVES_PER_BLOCK), occupancy_pad(LPR, args.lds_kb), s, args); break;
    }
    timing_end(s);
    GCN_LAUNCH_CHECK();
    if (fix_threads > 0) {
        switch (epilogue) {
            case GCN_EPI_NONE: hipLaunchKernelGGL((k_spmm_fixup<LPR, VEC, GCN_EPI_NONE>), fgrid, dim3(256), 0, s, args); break;
            case GCN_EPI_RELU: hipLaunchKernelGGL((k_spmm_fixup<LPR, VEC, GCN_EPI_RELU>), fgrid, dim3(256), 0, s, args); break;
            default: hipLaunchKernelGGL((k_spmm_fixup<LPR, VEC, GCN_EPI_MASK>), fgrid, dim3(256), 0, s, args); break;
        }
        GCN_LAUNCH_CHECK();
    }
    return GCN_OK;
}

static inline bool aligned16(const void* p) { return ((uintptr_t)p & 15u) == 0; }

// Adds the partial rows of the column-blocked product in ascending block order, then the epilogue.
template <int VEC, int EPI>
__global__ __launch_bounds__(256) void k_block_reduce(int64_t n, int32_t f, int32_t lanes, const int64_t* __restrict__ rq_ptr,
                                                      const int32_t* __restrict__ rq_idx, const int32_t* __restrict__ row_map,
                                                      const float* __restrict__ row_scale, const float* __restrict__ P,
                                                      float* __restrict__ Z, int64_t ldz, const float* __restrict__ Zprev,
                                                      int64_t ldzprev, int accumulate) {
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t i = t / lanes;
    const int col0 = (int)(t % lanes) * VEC;
    if (i >= n) return;
    const int64_t row = row_map ? row_map[i] : i;    // a row-subset matrix writes only its own rows
    float acc[VEC];
#pragma unroll
    for (int v = 0; v < VEC; ++v) acc[v] = 0.f;
    if (accumulate) load_vec<VEC>(acc, Z + row * ldz + col0);   // what an earlier pass stored raw for this row
    for (int64_t k = rq_ptr[i]; k < rq_ptr[i + 1]; ++k) {
        float part[VEC];
        load_vec<VEC>(part, P + (int64_t)rq_idx[k] * f + col0);
#pragma unroll
        for (int v = 0; v < VEC; ++v) acc[v] += part[v];
    }
    epilogue_store<VEC, EPI>(Z + row * ldz + col0, EPI == GCN_EPI_MASK ? Zprev + row * ldzprev + col0 : nullptr, acc,
                             row_scale ? row_scale[row] : 1.f);
}

template <int VEC>
static int launch_block_reduce(int64_t n, int32_t f, const Blocked& b, const int32_t* row_map, const float* row_scale,
                               int accumulate, const float* P, float* Z,
                               int64_t ldz, int epilogue, const float* Zprev, int64_t ldzprev, hipStream_t s) {
    const int lanes = f / VEC;
    const int64_t threads = n * lanes;
    const dim3 grid((unsigned)((threads + 255) / 256));
    switch (epilogue) {
        case GCN_EPI_NONE: hipLaunchKernelGGL((k_block_reduce<VEC, GCN_EPI_NONE>), grid, dim3(256), 0, s, n, f, lanes, b.rq_ptr, b.rq_idx, row_map, row_scale, P, Z, ldz, Zprev, ldzprev, accumulate); break;
        case GCN_EPI_RELU: hipLaunchKernelGGL((k_block_reduce<VEC, GCN_EPI_RELU>), grid, dim3(256), 0, s, n, f, lanes, b.rq_ptr, b.rq_idx, row_map, row_scale, P, Z, ldz, Zprev, ldzprev, accumulate); break;
        default: hipLaunchKernelGGL((k_block_reduce<VEC, GCN_EPI_MASK>), grid, dim3(256), 0, s, n, f, lanes, b.rq_ptr, b.rq_idx, row_map, row_scale, P, Z, ldz, Zprev, ldzprev, accumulate); break;
    }
    GCN_LAUNCH_CHECK();
    return GCN_OK;
}

// ---- column sweep ---------------------------------------------------------------------------------------
// One wavefront owns a task: `rb` consecutive rows whose results live in LDS (rb x W floats, W = 16
// or 32) for the whole launch.  Its entries come in ascending column order, so it walks X left to
// right; all wavefronts of a launch start together and have about the same length, so at any moment
// the whole GPU gathers from a narrow band of X, which therefore stays in L2 even when X is far
// larger than every cache.  The stored order puts G entries of different rows into every step (see
// Sweep), so the G lane groups of one step always hold different rows: each multiplies its gathered row by the
// value and adds it to the task's row in LDS with a plain read-modify-write.  Only this wavefront
// touches these accumulators and its LDS operations complete in program order, so the sum order is
// fixed and the result reproducible.
struct SweepArgs {
    const int32_t* colidx;
    const float* val;            // NULL: value-free product
    const float* row_scale;      // NULL, or one factor per output row
    const uint8_t* lrow;
    const int64_t* task_base;
    const int32_t* task_len;
    const int32_t* task_order;
    int64_t n;
    int32_t f, rb;
    const float* X; int64_t ldx;
    float* Z; int64_t ldz;
    const float* Zprev; int64_t ldzprev;
};

template <int LPR, int EPI>
__global__ __launch_bounds__(64) void k_spmm_sweep(SweepArgs a, int64_t first_task) {
    constexpr int G = 64 / LPR;                  // entries per step (16 or 8), all of different rows
    constexpr int W = LPR * 4;                   // panel width in floats
    constexpr int SPT = 64 / G;                  // steps per 64 entries
    constexpr int U = 2;                         // 64-entry loads per trip
    constexpr int STEPS = SPT * U;
    extern __shared__ float acc[];               // [rb][W]
    const int lane = threadIdx.x;
    const int g = lane / LPR, li = lane % LPR;
    const int col0 = li * 4;
    const bool col_ok = col0 < a.f;
    const int64_t task = a.task_order[first_task + blockIdx.x];
    for (int i = lane * 4; i < a.rb * W; i += 256) *reinterpret_cast<float4*>(acc + i) = make_float4(0.f, 0.f, 0.f, 0.f);
    __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
    __builtin_amdgcn_wave_barrier();

    const int64_t e0 = a.task_base[task];        // multiple of 16
    const int len = a.task_len[task];            // multiple of G; padding entries have column -1
    const float* xbase = a.X + col0;
    // the entries of the next trip are fetched while the current one is gathered and added
    int32_t c[U]; float v[U]; int r[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int k = 64 * u + lane;
        c[u] = -1; v[u] = 0.f; r[u] = 0;
        if (k < len) {
            c[u] = __builtin_nontemporal_load(a.colidx + e0 + k);
            v[u] = a.val ? __builtin_nontemporal_load(a.val + e0 + k) : 1.f;
            r[u] = (int)__builtin_nontemporal_load(a.lrow + e0 + k);
        }
    }
    for (int base = 0; base < len; base += 64 * U) {
        int32_t nc[U]; float nv[U]; int nr[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int k = base + 64 * U + 64 * u + lane;
            nc[u] = -1; nv[u] = 0.f; nr[u] = 0;
            if (k < len) {
                nc[u] = __builtin_nontemporal_load(a.colidx + e0 + k);
                nv[u] = a.val ? __builtin_nontemporal_load(a.val + e0 + k) : 1.f;
                nr[u] = (int)__builtin_nontemporal_load(a.lrow + e0 + k);
            }
        }
        float x[STEPS][4];
        float vs[STEPS];
        int rs[STEPS];                           // row inside the task, or -1 for a padding entry
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int t = 0; t < SPT; ++t) {      // every gather of the trip is issued before any add
                const int q = u * SPT + t;
                const int src = t * G + g;
                const int32_t cs = __shfl(c[u], src, 64);
                vs[q] = __shfl(v[u], src, 64);
                const int rr = __shfl(r[u], src, 64);
                rs[q] = cs >= 0 ? rr : -1;
                if (rs[q] >= 0 && col_ok) {
                    const float4 w4 = *reinterpret_cast<const float4*>(xbase + (int64_t)cs * a.ldx);
                    x[q][0] = w4.x; x[q][1] = w4.y; x[q][2] = w4.z; x[q][3] = w4.w;
                } else {
                    x[q][0] = x[q][1] = x[q][2] = x[q][3] = 0.f;
                }
            }
#pragma unroll
        for (int q = 0; q < STEPS; ++q) {
            if (rs[q] >= 0 && col_ok) {          // the groups of a step hold different rows
                float4* dst = reinterpret_cast<float4*>(acc + rs[q] * W + col0);
                float4 cur = *dst;
                cur.x = fmaf(vs[q], x[q][0], cur.x);
                cur.y = fmaf(vs[q], x[q][1], cur.y);
                cur.z = fmaf(vs[q], x[q][2], cur.z);
                cur.w = fmaf(vs[q], x[q][3], cur.w);
                *dst = cur;
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u) { c[u] = nc[u]; v[u] = nv[u]; r[u] = nr[u]; }
    }
    __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
    __builtin_amdgcn_wave_barrier();
    // write the task's rows: G rows per pass, 16 bytes per lane
    const int64_t row0 = task * a.rb;
    for (int i = g; i < a.rb; i += G) {
        const int64_t row = row0 + i;
        if (row < a.n && col_ok) {
            const float4 w4 = *reinterpret_cast<const float4*>(acc + i * W + col0);
            float out[4] = {w4.x, w4.y, w4.z, w4.w};
            epilogue_store<4, EPI>(a.Z + row * a.ldz + col0, EPI == GCN_EPI_MASK ? a.Zprev + row * a.ldzprev + col0 : nullptr, out,
                                   a.row_scale ? a.row_scale[row] : 1.f);
        }
    }
}

template <int LPR>
static int launch_sweep(const SweepArgs& args, int64_t ntasks, int sweep_waves, int epilogue, hipStream_t s) {
    constexpr int W = LPR * 4;
    const size_t lds = (size_t)args.rb * W * sizeof(float);
    const unsigned ytiles = (unsigned)((args.f + W - 1) / W);
    // tasks that are resident at once; the launches get equal shares so that the last one is not a stub
    const int64_t cap = (int64_t)device_info().cus * sweep_waves;
    const int64_t nlaunch = (ntasks + cap - 1) / cap;
    const int64_t gen = (ntasks + nlaunch - 1) / nlaunch;
    timing_begin(s);
    for (unsigned y = 0; y < ytiles; ++y) {
        for (int64_t first = 0; first < ntasks; first += gen) {
            const int64_t count = ntasks - first < gen ? ntasks - first : gen;
            const dim3 grid((unsigned)count, 1);
            SweepArgs a = args;
            // one panel per launch: shift the column origin instead of using blockIdx.y
            a.X = args.X + (size_t)y * W;
            a.Z = args.Z + (size_t)y * W;
            a.Zprev = args.Zprev ? args.Zprev + (size_t)y * W : nullptr;
            a.f = args.f - (int32_t)(y * W) < W ? args.f - (int32_t)(y * W) : W;
            switch (epilogue) {
                case GCN_EPI_NONE: hipLaunchKernelGGL((k_spmm_sweep<LPR, GCN_EPI_NONE>), grid, dim3(64), lds, s, a, first); break;
                case GCN_EPI_RELU: hipLaunchKernelGGL((k_spmm_sweep<LPR, GCN_EPI_RELU>), grid, dim3(64), lds, s, a, first); break;
                default: hipLaunchKernelGGL((k_spmm_sweep<LPR, GCN_EPI_MASK>), grid, dim3(64), lds, s, a, first); break;
            }
        }
    }
    timing_end(s);
    GCN_LAUNCH_CHECK();
    return GCN_OK;
}

// Chooses the lane layout for one nonzero-split product and launches it.
static int run_split(const SplitArgs& args, int epilogue, hipStream_t s, bool l2_resident = false) {
    const int32_t f = args.f;
    const bool vec4 = (f % 4 == 0) && (args.ldx % 4 == 0) && (args.ldz % 4 == 0) && aligned16(args.X) && aligned16(args.Z) &&
                      (epilogue != GCN_EPI_MASK || ((args.ldzprev % 4 == 0) && aligned16(args.Zprev)));
    if (vec4) {
        // Wider operands are processed in panels of 32 columns (one 128-byte line per gathered row):
        // the panel of X that the gathers touch is 4x smaller than at f = 128, so far more of it stays
        // in L2, at the price of re-reading the index/value stream once per panel.
        // When the gathers are served by the L2 anyway (column-blocked copy) panels of 64 are better: half
        // the passes over the index/value stream and half the requests (config 3 at f = 128: 3.55 -> 3.27 ms;
        // config 2, bound by line fills: 1.46 -> 1.69 ms, so not there).
        if (f >= 64 && l2_resident) return launch_split<16, 4>(args, epilogue, s);
        if (f > 32) return launch_split<8, 4>(args, epilogue, s);
        const int lanes = f / 4;
        if (lanes <= 4) return launch_split<4, 4>(args, epilogue, s);
        return launch_split<8, 4>(args, epilogue, s);
    }
    if (f <= 4) return launch_split<4, 1>(args, epilogue, s);
    if (f <= 8) return launch_split<8, 1>(args, epilogue, s);
    if (f <= 16) return launch_split<16, 1>(args, epilogue, s);
    if (f <= 32) return launch_split<32, 1>(args, epilogue, s);
    return launch_split<64, 1>(args, epilogue, s);
}

// How many column blocks to cut X into so that one block of the gathered panel stays in one L2
// (4 MB per XCD on this GPU; the size is read from the device).  Blocking costs one partial row per
// non-empty (block,row) pair, so it only pays when rows are long compared with the number of blocks: at
// least `per_block` entries per partial row.  When half-L2 blocks would make the partial rows shorter than
// that, blocks of up to twice the L2 are still worth it (measured on the long rows of config 5: 5.6 MB
// blocks beat 2 MB ones); beyond that 1 (no blocking).
static int64_t choose_blocks(const Config& cfg, int64_t nrows, int64_t ncols, int64_t nnz, int32_t f, int64_t per_block) {
    const int forced = cfg.spmm_blocks;
    if (forced >= 1) return forced;
    const int64_t l2 = device_info().l2_bytes;
    const int64_t panel = f < 32 ? f : 32;
    const int64_t xbytes = ncols * panel * 4;
    if (xbytes <= l2 / 8 * 7) return 1;                    // already L2-resident
    const int64_t block = l2 / 2;
    const int64_t want = (xbytes + block - 1) / block;
    const int64_t cap = (nnz / (nrows > 0 ? nrows : 1)) / per_block;
    if (want <= cap) return want;
    return (cap >= 2 && 4 * cap >= want) ? cap : 1;
}

// The nonzero-split product of one stored matrix -- the whole matrix, or the heavy rows of a sweep
// copy (then row_map gives the row each of its rows stands for) -- with or without column blocks.
static int run_matrix(gcn_csr* a, Matrix& mm, const int32_t* row_map, int64_t nnz, int64_t nblocks, int32_t f,
                      const float* X, int64_t ldx, float* Z, int64_t ldz, int epilogue, const float* Zprev,
                      int64_t ldzprev, const SpmmOpt& o, hipStream_t s, float* carry_given = nullptr) {
    if ((mm.nchunks + WAVES_PER_BLOCK - 1) / WAVES_PER_BLOCK >= (1ll << 31))
        return fail(GCN_ERR_RANGE, "gcn_spmm: too many chunks for one launch");
    // carry_given: a buffer of at least nchunks * f floats that the caller of this function provides
    // (only without column blocks); otherwise the handle's own buffer, grown on demand
    if (!carry_given) GCN_TRY(grow_retire(a, &a->carry, &a->carry_bytes, (size_t)mm.nchunks * (size_t)f * sizeof(float)));
    SplitArgs args;
    args.lds_kb = cfg_of(a).split_lds_kb;
    args.nnz = nnz; args.nsub = mm.nsub; args.nchunks = mm.nchunks; args.f = f;
    args.X = X; args.ldx = ldx; args.carry = carry_given ? carry_given : a->carry;
    args.defer = nullptr;
    if (nblocks >= 2) {
        int64_t cpb = (mm.ncols + nblocks - 1) / nblocks;
        cpb = (cpb + 1023) & ~1023ll;
        GCN_TRY(want_blocked(mm, nnz, cpb, s));
        const Blocked& b = mm.blk;
        GCN_TRY(grow_retire(a, &a->partial, &a->partial_bytes, (size_t)b.nrows * (size_t)f * sizeof(float)));
        if (o.describe) {
            char t[160];
            snprintf(t, sizeof t, "blocked(blocks=%d,cols_per_block=%lld,partial_rows=%lld,chunks=%lld)", (int)b.nblocks,
                     (long long)b.cols_per_block, (long long)b.nrows, (long long)mm.nchunks);
            *o.describe += t;
        }
        if (o.dry) return GCN_OK;
        args.colidx = b.colidx; args.val = o.pattern ? nullptr : b.val; args.flags = b.flags; args.sub_row = b.sub_row;
        args.ne_rows = nullptr; args.rp = b.rp; args.row_scale = nullptr;     // the scale belongs to the reduced row
        args.fix_list = b.fix_list; args.n_fix = b.n_fix;
        args.Z = a->partial; args.ldz = f; args.Zprev = nullptr; args.ldzprev = 0;
        GCN_TRY(run_split(args, GCN_EPI_NONE, s, true));
        const bool vec4 = (f % 4 == 0) && (ldz % 4 == 0) && aligned16(Z) &&
                          (epilogue != GCN_EPI_MASK || ((ldzprev % 4 == 0) && aligned16(Zprev)));
        if (vec4) return launch_block_reduce<4>(mm.nrows, f, b, row_map, o.row_scale, o.accumulate ? 1 : 0, a->partial, Z, ldz, epilogue, Zprev, ldzprev, s);
        return launch_block_reduce<1>(mm.nrows, f, b, row_map, o.row_scale, o.accumulate ? 1 : 0, a->partial, Z, ldz, epilogue, Zprev, ldzprev, s);
    }
    if (o.describe) {
        char t[96];
        snprintf(t, sizeof t, "split(chunks=%lld)", (long long)mm.nchunks);
        *o.describe += t;
    }
    if (o.dry) return GCN_OK;
    args.colidx = mm.colidx; args.val = o.pattern ? nullptr : mm.val; args.flags = mm.flags; args.sub_row = mm.sub_row;
    args.row_scale = o.row_scale;
    args.defer = o.defer;
    args.ne_rows = row_map ? row_map : mm.ne_rows;
    args.rp = mm.ne_rowptr ? mm.ne_rowptr : mm.rowptr;
    args.fix_list = mm.fix_list; args.n_fix = mm.n_fix;
    args.Z = Z; args.ldz = ldz; args.Zprev = Zprev; args.ldzprev = ldzprev;
    return run_split(args, epilogue, s);
}

static int zero_empty_rows(const Matrix& m, int32_t f, float* Z, int64_t ldz, hipStream_t s) {
    const int64_t n_empty = m.nrows - m.n_ne;
    if (m.empty_rows && n_empty > 0) {
        const int64_t work = n_empty * f;
        hipLaunchKernelGGL(k_zero_listed_rows, dim3((unsigned)((work + 255) / 256)), dim3(256), 0, s, n_empty, m.empty_rows, f, Z, ldz);
    } else {
        const int64_t work = m.nrows * f;
        hipLaunchKernelGGL(k_zero_empty_rows, dim3((unsigned)((work + 255) / 256)), dim3(256), 0, s, m.nrows, m.rowptr, f, Z, ldz);
    }
    GCN_LAUNCH_CHECK();
    return GCN_OK;
}

// ---- hub schedule -----------------------------------------------------------------------------------------
// xhot[r,:] = X[hot_col[r],:], 16 bytes per thread.
__global__ __launch_bounds__(256) void k_pack_rows(int64_t H, int32_t lanes, const float* __restrict__ X, int64_t ldx,
                                                   const int32_t* __restrict__ hot_col, float* __restrict__ xhot) {
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t r = t / lanes;
    const int j = (int)(t % lanes) * 4;
    if (r >= H) return;
    *reinterpret_cast<float4*>(xhot + r * (int64_t)lanes * 4 + j) =
        *reinterpret_cast<const float4*>(X + (int64_t)hot_col[r] * ldx + j);
}

// Packed-buffer size and block width of the hub copy for operands of width f: blocks of about 2 MB
// of the gathered panel, as many hot columns as fit `budget` bytes (a multiple of the block width).
static void hub_shape(const Config& cfg, int64_t ncols, int32_t f, int64_t* H, int64_t* cpb) {
    const int64_t panel = f < 32 ? f : 32;
    *cpb = cfg.hub_block_cols > 0 ? cfg.hub_block_cols : (device_info().l2_bytes / 2) / (panel * 4);
    const int64_t budget = (int64_t)cfg.hub_mb << 20;
    int64_t h = budget / ((int64_t)f * 4);
    if (h > ncols) h = ncols;
    *H = h / *cpb * *cpb;
}

template <int LPR>
static int launch_pair(const SplitArgs& ra_args, const SplitArgs& rb_args, int epilogue, hipStream_t s) {
    const int tile = LPR * 4;
    const unsigned ytiles = (unsigned)((ra_args.f + tile - 1) / tile);
    const int64_t ga = (ra_args.nchunks + WAVES_PER_BLOCK - 1) / WAVES_PER_BLOCK;
    const int64_t gb = (rb_args.nchunks + WAVES_PER_BLOCK - 1) / WAVES_PER_BLOCK;
    // shares of the two matrices among eight consecutive workgroups, in proportion to their chunk groups
    int ra = (int)((8 * ga + (ga + gb) / 2) / (ga + gb));
    ra = ra < 1 ? 1 : (ra > 7 ? 7 : ra);
    const int rb = 8 - ra;
    const int64_t periods = std::max((ga + ra - 1) / ra, (gb + rb - 1) / rb);
    if (periods * 8 >= (1ll << 31)) return fail(GCN_ERR_RANGE, "gcn_spmm: too many chunks for one launch");
    const dim3 grid((unsigned)(periods * 8), ytiles);
    timing_begin(s);
    switch (epilogue) {
        case GCN_EPI_NONE: hipLaunchKernelGGL((k_spmm_split_pair<LPR, 4, GCN_EPI_NONE>), grid, dim3(64 * WAVES_PER_BLOCK), 0, s, ra_args, rb_args, ra, rb); break;
        case GCN_EPI_RELU: hipLaunchKernelGGL((k_spmm_split_pair<LPR, 4, GCN_EPI_RELU>), grid, dim3(64 * WAVES_PER_BLOCK), 0, s, ra_args, rb_args, ra, rb); break;
        default: hipLaunchKernelGGL((k_spmm_split_pair<LPR, 4, GCN_EPI_MASK>), grid, dim3(64 * WAVES_PER_BLOCK), 0, s, ra_args, rb_args, ra, rb); break;
    }
    timing_end(s);
    GCN_LAUNCH_CHECK();
    const SplitArgs* both[2] = {&ra_args, &rb_args};
    for (int k = 0; k < 2; ++k) {
        const SplitArgs& args = *both[k];
        const int64_t fix_threads = (args.n_fix >= 0 ? args.n_fix : args.nchunks - 1) * LPR;
        if (fix_threads <= 0) continue;
        const dim3 fgrid((unsigned)((fix_threads + 255) / 256), ytiles);
        const int epi = k == 0 ? epilogue : GCN_EPI_NONE;
        switch (epi) {
            case GCN_EPI_NONE: hipLaunchKernelGGL((k_spmm_fixup<LPR, 4, GCN_EPI_NONE>), fgrid, dim3(256), 0, s, args); break;
            case GCN_EPI_RELU: hipLaunchKernelGGL((k_spmm_fixup<LPR, 4, GCN_EPI_RELU>), fgrid, dim3(256), 0, s, args); break;
            default: hipLaunchKernelGGL((k_spmm_fixup<LPR, 4, GCN_EPI_MASK>), fgrid, dim3(256), 0, s, args); break;
        }
        GCN_LAUNCH_CHECK();
    }
    return GCN_OK;
}

// Z = A_rest X (long rows stored raw) and the partial rows of A_hot X_hot in one paired launch, then
// the long rows get their partial rows added, are scaled and finished.  Needs 16-byte aligned operands.
static int run_hub(gcn_csr* a, Matrix& m, int32_t f, const float* X, int64_t ldx, float* Z, int64_t ldz, int epilogue,
                   const float* Zprev, int64_t ldzprev, const SpmmOpt& o, hipStream_t s) {
    Hub& h = m.hub;
    GCN_TRY(grow_retire(a, &h.xhot, &h.xhot_bytes, (size_t)h.H * (size_t)f * sizeof(float)));
    Matrix& rest = *h.rest;
    Matrix& hot = *h.hot;
    const Blocked& b = hot.blk;
    if ((rest.nchunks + hot.nchunks) / WAVES_PER_BLOCK + 16 >= (1ll << 31))
        return fail(GCN_ERR_RANGE, "gcn_spmm: too many chunks for one launch");
    GCN_TRY(grow_retire(a, &a->carry, &a->carry_bytes, (size_t)rest.nchunks * (size_t)f * sizeof(float)));
    GCN_TRY(grow_retire(a, &a->carry2, &a->carry2_bytes, (size_t)hot.nchunks * (size_t)f * sizeof(float)));
    GCN_TRY(grow_retire(a, &a->partial, &a->partial_bytes, (size_t)b.nrows * (size_t)f * sizeof(float)));
    if (o.describe) {
        char t[200];
        snprintf(t, sizeof t, "hub(hot_cols=%lld,cols_per_block=%lld,long_row>=%d,nnz_hot=%lld,nnz_rest=%lld,partial_rows=%lld)",
                 (long long)h.H, (long long)h.cpb, (int)h.dmin, (long long)h.nnz_hot, (long long)h.nnz_rest, (long long)b.nrows);
        *o.describe += t;
    }
    if (o.dry) return GCN_OK;
    const int lanes = f / 4;
    hipLaunchKernelGGL(k_pack_rows, dim3((unsigned)((h.H * lanes + 255) / 256)), dim3(256), 0, s, h.H, lanes, X, ldx,
                       h.hot_col, h.xhot);
    GCN_LAUNCH_CHECK();
    if (rest.n_ne < rest.nrows) GCN_TRY(zero_empty_rows(rest, f, Z, ldz, s));

    SplitArgs ar;                                  // A_rest over X, into Z
    ar.lds_kb = cfg_of(a).split_lds_kb;
    ar.colidx = rest.colidx; ar.val = o.pattern ? nullptr : rest.val; ar.flags = rest.flags; ar.sub_row = rest.sub_row;
    ar.row_scale = o.row_scale; ar.defer = h.defer;
    ar.ne_rows = rest.ne_rows; ar.rp = rest.ne_rowptr ? rest.ne_rowptr : rest.rowptr;
    ar.fix_list = rest.fix_list; ar.n_fix = rest.n_fix;
    ar.nnz = h.nnz_rest; ar.nsub = rest.nsub; ar.nchunks = rest.nchunks; ar.f = f;
    ar.X = X; ar.ldx = ldx; ar.Z = Z; ar.ldz = ldz; ar.Zprev = Zprev; ar.ldzprev = ldzprev; ar.carry = a->carry;
    SplitArgs ah;                                  // A_hot over the packed rows, into the partial rows
    ah.lds_kb = ar.lds_kb;
    ah.colidx = b.colidx; ah.val = o.pattern ? nullptr : b.val; ah.flags = b.flags; ah.sub_row = b.sub_row;
    ah.row_scale = nullptr; ah.defer = nullptr; ah.ne_rows = nullptr; ah.rp = b.rp;
    ah.fix_list = b.fix_list; ah.n_fix = b.n_fix;
    ah.nnz = h.nnz_hot; ah.nsub = hot.nsub; ah.nchunks = hot.nchunks; ah.f = f;
    ah.X = h.xhot; ah.ldx = f; ah.Z = a->partial; ah.ldz = f; ah.Zprev = nullptr; ah.ldzprev = 0; ah.carry = a->carry2;
    if (f > 16) GCN_TRY(launch_pair<8>(ar, ah, epilogue, s));
    else GCN_TRY(launch_pair<4>(ar, ah, epilogue, s));
    return launch_block_reduce<4>(hot.nrows, f, b, h.heavy_rows, o.row_scale, 1, a->partial, Z, ldz, epilogue, Zprev,
                                  ldzprev, s);
}

// ---- stored orders kept per key ------------------------------------------------------------------------
int want_blocked(Matrix& m, int64_t nnz, int64_t cpb, hipStream_t s) {
    if (m.blk.cols_per_block == cpb) return GCN_OK;
    if (m.blk.cols_per_block != 0) {
        m.blk_parked.push_back(m.blk);
        m.blk = Blocked();
    }
    for (size_t i = 0; i < m.blk_parked.size(); ++i)
        if (m.blk_parked[i].cols_per_block == cpb) {
            m.blk = m.blk_parked[i];
            m.blk_parked.erase(m.blk_parked.begin() + (long)i);
            return GCN_OK;
        }
    return build_blocked(m, nnz, cpb, s);
}

int want_sweep(Matrix& m, int64_t nnz, int32_t groups, int32_t rb, int32_t th, hipStream_t s) {
    auto is = [&](const Sweep& w) { return w.groups == groups && w.rb == rb && w.heavy_threshold == th; };
    if (is(m.swp)) return GCN_OK;
    if (m.swp.groups != 0) {
        m.swp_parked.push_back(m.swp);
        m.swp = Sweep();
    }
    for (size_t i = 0; i < m.swp_parked.size(); ++i)
        if (is(m.swp_parked[i])) {
            m.swp = m.swp_parked[i];
            m.swp_parked.erase(m.swp_parked.begin() + (long)i);
            return GCN_OK;
        }
    return build_sweep(m, nnz, groups, rb, th, s);
}

// The hub copy for the current settings: the one in use, a parked one, or a new attempt (state 1 built,
// -1 rejected for these settings).  A change of operand width reuses the copy.
static int want_hub(Matrix& m, const Config& cfg, int64_t nnz, int64_t H, int64_t cpb, bool forced, hipStream_t s) {
    auto is = [&](const Hub& h) {
        return h.state != 0 && h.dmin == cfg.hub_dmin && h.cfg_mb == cfg.hub_mb && h.cfg_block_cols == cfg.hub_block_cols;
    };
    if (is(m.hub)) return GCN_OK;
    if (m.hub.state != 0) {
        m.hub_parked.push_back(m.hub);
        m.hub = Hub();
    }
    for (size_t i = 0; i < m.hub_parked.size(); ++i)
        if (is(m.hub_parked[i])) {
            m.hub = m.hub_parked[i];
            m.hub_parked.erase(m.hub_parked.begin() + (long)i);
            return GCN_OK;
        }
    const int rc = build_hub(m, nnz, H, cpb, cfg.hub_dmin, s);
    if (rc != GCN_OK) {
        // the copy is an optimisation: without it (for instance out of memory) the plain kernel runs
        if (forced) return rc;
        free_hub(m.hub);
        m.hub.state = -1;
    }
    m.hub.dmin = cfg.hub_dmin;
    m.hub.cfg_mb = cfg.hub_mb;
    m.hub.cfg_block_cols = cfg.hub_block_cols;
    return GCN_OK;
}

static void took(gcn_csr* a, int sched) {
    g_last_schedule = sched;
    a->last_schedule = sched;
}

int spmm_launch(gcn_csr* a, Matrix& m, int32_t f, const float* X, int64_t ldx, float* Z, int64_t ldz,
                int epilogue, const float* Zprev, int64_t ldzprev, hipStream_t s, const SpmmOpt& o) {
    const int64_t n = m.nrows, ncols = m.ncols, nnz = a->nnz;
    const Config& cfg = cfg_of(a);
    if (nnz == 0) {
        if (o.describe) *o.describe += "empty";
        if (o.dry) return GCN_OK;
        const int64_t work = n * f;
        hipLaunchKernelGGL(k_zero_empty_rows, dim3((unsigned)((work + 255) / 256)), dim3(256), 0, s, n, m.rowptr, f, Z, ldz);
        GCN_LAUNCH_CHECK();
        return GCN_OK;
    }
    int algo = cfg.spmm_algo;
    const bool vec4_all = (f % 4 == 0) && (ldx % 4 == 0) && (ldz % 4 == 0) && aligned16(X) && aligned16(Z) &&
                          (epilogue != GCN_EPI_MASK || ((ldzprev % 4 == 0) && aligned16(Zprev)));
    const int64_t nblocks = choose_blocks(cfg, n, ncols, nnz, f, 24);
    if (algo == 0) {
        // Column sweep when X is far beyond the caches, rows are long enough to give every task a
        // real walk over the columns, and too short for partial-row blocking; else nonzero-split.
        const int64_t panel = f < 32 ? f : 32;
        const bool huge = ncols * panel * 4 > (64ll << 20);
        // one step of a task spans about groups^2 * ncols * rowbytes / (rows_per_task * mean_degree) bytes
        // of X (64 * ncols / degree at width 16); the sweep pays while that stays within an L2
        const int64_t deg = nnz / n;
        const bool narrow_steps = deg >= 64 && 64 * ncols / deg <= (6ll << 20);
        algo = (huge && vec4_all && nblocks < 2 && narrow_steps) ? 3 : 2;
    }
    if (algo == 3 && !vec4_all) algo = 2;
    if ((algo == 2 && cfg.spmm_algo == 0) || algo == 4) {
        // Hub schedule: for operands beyond the L2s when most entries sit in long rows and hot columns
        // (decided from the matrix itself when the copy is built; a rejected shape is remembered).
        const bool forced = algo == 4;
        algo = 2;
        const int64_t panel = f < 32 ? f : 32;
        int64_t H = 0, cpb = 0;
        hub_shape(cfg, ncols, f, &H, &cpb);
        // Measured: it pays when a gathered row is narrower than a 128-byte line (packing then also puts
        // two hot rows into one line: config 4, width 16, 4.33 -> 3.15 ms) and not at 128 bytes per row
        // (config 2: 1.44 -> 1.48 ms), so the automatic choice is limited to panels below 32 floats.
        const bool eligible = vec4_all && nblocks < 2 && H >= 2 * cpb && nnz >= (forced ? 1 : (4ll << 20)) &&
                              (forced || (panel < 32 && ncols * panel * 4 > (32ll << 20)));
        if (eligible) {
            // built once per matrix and settings for the width of the first product that qualifies
            GCN_TRY(want_hub(m, cfg, nnz, H, cpb, forced, s));
            if (m.hub.state == 1) {
                took(a, GCN_SCHED_HUB);
                return run_hub(a, m, f, X, ldx, Z, ldz, epilogue, Zprev, ldzprev, o, s);
            }
        }
    }
    if (algo == 3) {
        took(a, GCN_SCHED_SWEEP);
        const int LPRs = f <= 16 ? 4 : 8;
        const int W = LPRs * 4;
        const int32_t rb = 4096 / W;                       // 16 KB of accumulators per wavefront
        GCN_TRY(want_sweep(m, nnz, 64 / LPRs, rb, cfg.sweep_heavy, s));
        const Sweep& w = m.swp;
        if (o.describe) {
            const int64_t cap = (int64_t)device_info().cus * cfg.sweep_waves;
            char t[200];
            snprintf(t, sizeof t, "sweep(entries_per_step=%d,rows_per_task=%d,long_row>%d,tasks=%lld,launches=%lld,stored=%lld)",
                     64 / LPRs, (int)rb, (int)cfg.sweep_heavy, (long long)w.ntasks,
                     (long long)(((w.ntasks + cap - 1) / cap) * ((f + W - 1) / W)), (long long)w.padded);
            *o.describe += t;
        }
        if (!o.dry) {
            SweepArgs sa;
            sa.colidx = w.colidx; sa.val = o.pattern ? nullptr : w.val; sa.row_scale = o.row_scale; sa.lrow = w.lrow; sa.task_base = w.task_base; sa.task_len = w.task_len; sa.task_order = w.task_order;
            sa.n = n; sa.f = f; sa.rb = rb; sa.X = X; sa.ldx = ldx; sa.Z = Z; sa.ldz = ldz; sa.Zprev = Zprev; sa.ldzprev = ldzprev;
            if (LPRs == 4) GCN_TRY(launch_sweep<4>(sa, w.ntasks, cfg.sweep_waves, epilogue, s));
            else GCN_TRY(launch_sweep<8>(sa, w.ntasks, cfg.sweep_waves, epilogue, s));
        }
        if (w.heavy) {
            // long rows: nonzero-split kernel over the row subset; their rows are long enough for the
            // column-blocked form to pay even with many blocks
            Matrix& h = *w.heavy;
            const int64_t hb = choose_blocks(cfg, h.nrows, ncols, w.nnz_heavy, f, 30);
            if (o.describe) *o.describe += "+long_rows:";
            GCN_TRY(run_matrix(a, h, h.ne_rows, w.nnz_heavy, hb, f, X, ldx, Z, ldz, epilogue, Zprev, ldzprev, o, s));
        }
        return GCN_OK;
    }
    if (algo == 1) {
        took(a, GCN_SCHED_ROWWISE);
        if (o.describe) *o.describe += "rowwise";
        if (o.dry) return GCN_OK;
        const int64_t work = n * f;
        const dim3 grid((unsigned)((work + 255) / 256));
        if (work / 256 >= (1ll << 31)) return fail(GCN_ERR_RANGE, "gcn_spmm: n*f too large for the row-wise kernel");
        timing_begin(s);
        switch (epilogue) {
            case GCN_EPI_NONE: hipLaunchKernelGGL(k_spmm_rowwise<GCN_EPI_NONE>, grid, dim3(256), 0, s, n, m.rowptr, m.colidx, o.pattern ? nullptr : m.val, o.row_scale, f, X, ldx, Z, ldz, Zprev, ldzprev); break;
            case GCN_EPI_RELU: hipLaunchKernelGGL(k_spmm_rowwise<GCN_EPI_RELU>, grid, dim3(256), 0, s, n, m.rowptr, m.colidx, o.pattern ? nullptr : m.val, o.row_scale, f, X, ldx, Z, ldz, Zprev, ldzprev); break;
            default: hipLaunchKernelGGL(k_spmm_rowwise<GCN_EPI_MASK>, grid, dim3(256), 0, s, n, m.rowptr, m.colidx, o.pattern ? nullptr : m.val, o.row_scale, f, X, ldx, Z, ldz, Zprev, ldzprev); break;
        }
        timing_end(s);
        GCN_LAUNCH_CHECK();
        return GCN_OK;
    }
    took(a, nblocks >= 2 ? GCN_SCHED_BLOCKED : GCN_SCHED_SPLIT);
    if (!o.dry && nblocks < 2 && m.n_ne < n) GCN_TRY(zero_empty_rows(m, f, Z, ldz, s));
    return run_matrix(a, m, nullptr, nnz, nblocks, f, X, ldx, Z, ldz, epilogue, Zprev, ldzprev, o, s);
}

// For a matrix this library normalised symmetrically, D^-1/2 (A+I) D^-1/2 X = D^-1/2 ((A+I) (D^-1/2 X))
// (section "Graph Neural Networks"): the product can skip the stored values, which halves the
// index/value stream.  It pays when rows are long (the pre-scaling pass over X is amortised).
bool use_value_free(const gcn_csr* a) {
    const int mode = cfg_of(a).pattern_spmm;
    if (!a->inv_sqrt_deg || mode == 0) return false;
    return mode == 1 || a->nnz / (a->n > 0 ? a->n : 1) >= 64;
}

int spmm_prepare(gcn_csr* a, Matrix& m, int32_t f, hipStream_t s) {
    SpmmOpt o;
    o.dry = true;
    return spmm_launch(a, m, f, nullptr, f, nullptr, f, GCN_EPI_NONE, nullptr, 0, s, o);
}

}  // namespace gcn

using namespace gcn;

static inline hipStream_t s_of(void* stream) { return (hipStream_t)stream; }

static int check_spmm_args(const char* who, const gcn_csr* a, int trans, int32_t f, const float* X, int64_t ldx,
                           const float* Z, int64_t ldz, int epilogue, const float* Zprev, int64_t ldzprev) {
    if (!a || !X || !Z) return fail(GCN_ERR_BADARG, "%s: NULL argument", who);
    if (f <= 0 || ldx < f || ldz < f) return fail(GCN_ERR_BADARG, "%s: need f > 0, ldx >= f, ldz >= f", who);
    if (epilogue < GCN_EPI_NONE || epilogue > GCN_EPI_MASK) return fail(GCN_ERR_BADARG, "%s: unknown epilogue", who);
    if (epilogue == GCN_EPI_MASK && (!Zprev || ldzprev < f)) return fail(GCN_ERR_BADARG, "%s: mask epilogue needs Zprev with ld >= f", who);
    if (trans && !a->has_t) return fail(GCN_ERR_NOTRANSPOSE, "%s: trans=1 needs GCN_BUILD_TRANSPOSE", who);
    // X and Z must not overlap: the product gathers rows of X while rows of Z are written
    const int64_t xrows = trans ? a->n : a->ncols, zrows = trans ? a->ncols : a->n;
    const char* xb = (const char*)X; const char* xe = xb + ((size_t)(xrows - 1) * ldx + f) * sizeof(float);
    const char* zb = (const char*)Z; const char* ze = zb + ((size_t)(zrows - 1) * ldz + f) * sizeof(float);
    if (xb < ze && zb < xe) return fail(GCN_ERR_BADARG, "%s: X and Z overlap", who);
    return GCN_OK;
}

extern "C" int gcn_spmm(gcn_csr* a, int trans, int32_t f, const float* X, int64_t ldx, float* Z, int64_t ldz,
                        int epilogue, const float* Zprev, int64_t ldzprev, void* stream) {
    GCN_TRY(check_spmm_args("gcn_spmm", a, trans, f, X, ldx, Z, ldz, epilogue, Zprev, ldzprev));
    PhaseTimer whole(s_of(stream), GCN_PHASE_SPMM);           // the whole product: every kernel it queues
    if (use_value_free(a)) {
        // value-free form: a pre-scaled copy of X in the handle (n x f), then sums of gathered rows, the output
        // rows scaled in the kernels' store path; differs from the valued product by fp32 roundings only
        GCN_TRY(grow_retire(a, &a->xs, &a->xs_bytes, (size_t)a->n * (size_t)f * sizeof(float)));
        GCN_TRY(scale_rows_launch(a->n, f, X, ldx, a->inv_sqrt_deg, a->xs, f, s_of(stream)));
        SpmmOpt o;
        o.pattern = true;
        o.row_scale = a->inv_sqrt_deg;
        return spmm_launch(a, trans ? a->At : a->A, f, a->xs, f, Z, ldz, epilogue, Zprev, ldzprev, s_of(stream), o);
    }
    return spmm_launch(a, trans ? a->At : a->A, f, X, ldx, Z, ldz, epilogue, Zprev, ldzprev, (hipStream_t)stream);
}

extern "C" int gcn_spmm_prepare(gcn_csr* a, int trans, int32_t f, void* stream) {
    if (!a || f <= 0) return fail(GCN_ERR_BADARG, "gcn_spmm_prepare: NULL matrix or f <= 0");
    if (trans && !a->has_t) return fail(GCN_ERR_NOTRANSPOSE, "gcn_spmm_prepare: trans=1 needs GCN_BUILD_TRANSPOSE");
    if (use_value_free(a)) GCN_TRY(grow_retire(a, &a->xs, &a->xs_bytes, (size_t)a->n * (size_t)f * sizeof(float)));
    return spmm_prepare(a, trans ? a->At : a->A, f, (hipStream_t)stream);
}

extern "C" int gcn_spmm_describe(gcn_csr* a, int trans, int32_t f, char* out, size_t out_bytes, void* stream) {
    if (!a || f <= 0 || !out || out_bytes == 0) return fail(GCN_ERR_BADARG, "gcn_spmm_describe: bad argument");
    if (trans && !a->has_t) return fail(GCN_ERR_NOTRANSPOSE, "gcn_spmm_describe: trans=1 needs GCN_BUILD_TRANSPOSE");
    std::string text;
    SpmmOpt o;
    o.dry = true;
    o.describe = &text;
    o.pattern = use_value_free(a);
    GCN_TRY(spmm_launch(a, trans ? a->At : a->A, f, nullptr, f, nullptr, f, GCN_EPI_NONE, nullptr, 0, (hipStream_t)stream, o));
    if (o.pattern) text += "; value-free (operand rows pre-scaled by d^-1/2, output rows scaled)";
    snprintf(out, out_bytes, "%s", text.c_str());
    return GCN_OK;
}

// ---- the product for callers that cannot allocate --------------------------------------------------------
// The nonzero-split kernel needs one row of f floats per 512 stored entries for the pieces of rows that
// cross wavefronts.  gcn_spmm keeps that buffer in the handle and grows it with hipMalloc; this entry point
// keeps it in a fixed array in the library's device image instead, so that it never allocates.  Each GPU
// has its own copy of the array at its own address; the address is looked up once per device.
static constexpr size_t STATIC_SCRATCH_BYTES = GCN_SPMM_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[STATIC_SCRATCH_BYTES];
static constexpr int STATIC_MAX_DEVICES = 64;
static std::mutex g_static_mu;
static void* g_static_ptr[STATIC_MAX_DEVICES] = {};

static int static_scratch(float** out) {
    int dev = -1;
    GCN_HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= STATIC_MAX_DEVICES) return fail(GCN_ERR_RANGE, "gcn_spmm_static: device index %d not supported", dev);
    std::lock_guard<std::mutex> lk(g_static_mu);
    if (!g_static_ptr[dev]) {
        void* ptr = nullptr;
        GCN_HIP_TRY(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));      // with `dev` current: this device's copy
        if (!ptr) return fail(GCN_ERR_HIP, "gcn_spmm_static: no address for the scratch array on device %d", dev);
        g_static_ptr[dev] = ptr;
    }
    *out = (float*)g_static_ptr[dev];
    return GCN_OK;
}

extern "C" int gcn_spmm_static(gcn_csr* a, int trans, int32_t f, const float* X, int64_t ldx, float* Z, int64_t ldz,
                               int epilogue, const float* Zprev, int64_t ldzprev, void* stream) {
    GCN_TRY(check_spmm_args("gcn_spmm_static", a, trans, f, X, ldx, Z, ldz, epilogue, Zprev, ldzprev));
    int dev = -1;
    GCN_HIP_TRY(hipGetDevice(&dev));
    if (dev != a->device) return fail(GCN_ERR_BADARG, "gcn_spmm_static: the matrix lives on device %d, current device is %d", a->device, dev);
    Matrix& m = trans ? a->At : a->A;
    const size_t need = (size_t)m.nchunks * (size_t)f * sizeof(float);
    if (need > STATIC_SCRATCH_BYTES)
        return fail(GCN_ERR_WORKSPACE, "gcn_spmm_static: needs %zu bytes of scratch (%lld stored entries / 512, rounded up, x %d floats), the fixed "
                    "array holds %zu; use gcn_spmm", need, (long long)a->nnz, (int)f, STATIC_SCRATCH_BYTES);
    hipStream_t s = (hipStream_t)stream;
    if (a->nnz == 0 || m.n_ne < m.nrows) GCN_TRY(zero_empty_rows(m, f, Z, ldz, s));
    if (a->nnz == 0) return GCN_OK;
    float* carry = nullptr;
    GCN_TRY(static_scratch(&carry));
    took(a, GCN_SCHED_SPLIT);
    return run_matrix(a, m, nullptr, a->nnz, 1, f, X, ldx, Z, ldz, epilogue, Zprev, ldzprev, SpmmOpt(), s, carry);
}

extern "C" int gcn_spmm_pattern(gcn_csr* a, int trans, int32_t f, const float* X, int64_t ldx, float* Z, int64_t ldz,
                                const float* row_scale, int epilogue, const float* Zprev, int64_t ldzprev,
                                void* stream) {
    GCN_TRY(check_spmm_args("gcn_spmm_pattern", a, trans, f, X, ldx, Z, ldz, epilogue, Zprev, ldzprev));
    SpmmOpt o;
    o.pattern = true;
    o.row_scale = row_scale;
    PhaseTimer whole(s_of(stream), GCN_PHASE_SPMM);
    return spmm_launch(a, trans ? a->At : a->A, f, X, ldx, Z, ldz, epilogue, Zprev, ldzprev, (hipStream_t)stream, o);
}
