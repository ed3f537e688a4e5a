// fp32 MFMA kernels for the dense products around the SpMM (v_mfma_f32_16x16x4_f32; full fp32
// multiply-add, so the 1e-4 bound against the double oracle holds):
//   k_gemm_tall   C[M x N] = A[M x K] op(B)            M = n (millions), K and N small: H W of
//                 "Forward Propagation", S W^T of Equation 2.  Streams A once from HBM; op(B) sits
//                 in LDS; one wavefront owns a 16-row strip and up to four 16-column tiles.
//   k_gemm_tn     C[M x N] = A[K x M]^T B[K x N]        K = n: the weight gradient of Equation 3.
//                 Split over K across workgroups; partial results are reduced in a fixed order.
// At hidden width 16 both are bandwidth-bound (8 flops per byte of A): the matrix cores keep the
// arithmetic off the critical path.
//
// Operand layout of the 16x16x4 instruction (64 lanes): lane l supplies A[i = l%16][k = l/16] and
// B[k = l/16][j = l%16], and holds D[i = 4*(l/16) + v][j = l%16] in element v of its accumulator.
#include "common.h"

namespace gcn {

typedef float floatx4 __attribute__((ext_vector_type(4)));

struct __attribute__((packed, aligned(4))) f4u { float x, y, z, w; };   // 16 bytes at 4-byte alignment

// 16-byte load of data that is read once: the non-temporal hint keeps the stream from displacing what other
// wavefronts still need in the caches.  Measured on 14 M rows: +10 % on the A^T B kernel when every row of A is
// whole 128-byte lines (256 floats: 2.67 -> 2.39 ms, 128 floats: 1.62 -> 1.42 ms), +2 % on the strip kernel; a loss
// where neighbouring wavefronts share lines (A^T B at 300 floats per row: 4.13 -> 4.22 ms), so the callers decide.
__device__ __forceinline__ float4 stream4(const float* p) {
    const floatx4 v = __builtin_nontemporal_load(reinterpret_cast<const floatx4*>(p));
    return make_float4(v[0], v[1], v[2], v[3]);
}

__device__ __forceinline__ float4 load4(const float* p, bool aligned, bool nt = false) {
    if (aligned) return nt ? stream4(p) : *reinterpret_cast<const float4*>(p);
    f4u v = *reinterpret_cast<const f4u*>(p);
    return make_float4(v.x, v.y, v.z, v.w);
}

template <int EPI>
__device__ __forceinline__ float epi(float v, const float* zprev_elem) {
    if (EPI == GCN_EPI_RELU) return v > 0.f ? v : 0.f;
    if (EPI == GCN_EPI_MASK) return *zprev_elem > 0.f ? v : 0.f;
    return v;
}

struct TallArgs {
    int64_t M;
    int32_t N, K;
    const float* A; int64_t lda;
    const float* B; int64_t ldb; int tb;
    float* C; int64_t ldc;
    const float* bias;
    const float* Zprev; int64_t ldzprev;
    int32_t Kpad;      // K rounded up to 16
    int32_t S;         // LDS row stride in floats: 16*NT + 4 (bank-conflict-free B reads)
    int a_aligned;     // A rows are 16-byte aligned
    const float* row_scale;   // NULL, or one factor per row of C, applied after bias and epilogue (wide store path only)
};

// TR: the two MFMA operands are swapped, so a lane ends up with four consecutive columns of one
// row of C (element v of tile t is C[row0 + l%16][16t + 4*(l/16) + v]) and stores them with one
// 16-byte instruction; needs N % 4 == 0 and 16-byte aligned rows of C (and of Zprev for the mask).
template <int NT, int EPI, bool TR>
__global__ __launch_bounds__(256) void k_gemm_tall(TallArgs a) {
    extern __shared__ float Bs[];                       // [Kpad][S]
    const int n0 = blockIdx.y * (NT * 16);
    const int ncols = NT * 16;
    for (int idx = threadIdx.x; idx < a.Kpad * ncols; idx += 256) {
        const int k = idx / ncols, j = idx % ncols;
        float v = 0.f;
        if (k < a.K && n0 + j < a.N) v = a.tb ? a.B[(int64_t)(n0 + j) * a.ldb + k] : a.B[(int64_t)k * a.ldb + n0 + j];
        Bs[k * a.S + j] = v;
    }
    __syncthreads();

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int r = lane & 15, kq = lane >> 4;
    const int64_t ntiles = (a.M + 15) / 16;
    for (int64_t tile = (int64_t)blockIdx.x * 4 + wave; tile < ntiles; tile += (int64_t)gridDim.x * 4) {
        const int64_t row0 = tile * 16;
        int64_t arow = row0 + r;
        if (arow >= a.M) arow = a.M - 1;                // clamp: loads stay in bounds, stores are masked
        const float* ap = a.A + arow * a.lda + 4 * kq;
        floatx4 acc[NT];
#pragma unroll
        for (int t = 0; t < NT; ++t) acc[t] = (floatx4){0.f, 0.f, 0.f, 0.f};
        const int kfull = a.K & ~15;
        int k0 = 0;
        for (; k0 + 64 <= kfull; k0 += 64) {            // four 16-deep steps per trip: 4 loads in flight
            float4 av[4];
#pragma unroll
            for (int s = 0; s < 4; ++s) av[s] = load4(ap + k0 + 16 * s, a.a_aligned);
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                const float ae[4] = {av[s].x, av[s].y, av[s].z, av[s].w};
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const float* bp = Bs + (k0 + 16 * s + 4 * kq + e) * a.S + r;
#pragma unroll
                    for (int t = 0; t < NT; ++t)
                        acc[t] = TR ? __builtin_amdgcn_mfma_f32_16x16x4f32(bp[16 * t], ae[e], acc[t], 0, 0, 0)
                                    : __builtin_amdgcn_mfma_f32_16x16x4f32(ae[e], bp[16 * t], acc[t], 0, 0, 0);
                }
            }
        }
        for (; k0 < kfull; k0 += 16) {
            const float4 av = load4(ap + k0, a.a_aligned);
            const float ae[4] = {av.x, av.y, av.z, av.w};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float* bp = Bs + (k0 + 4 * kq + e) * a.S + r;
#pragma unroll
                for (int t = 0; t < NT; ++t)
                    acc[t] = TR ? __builtin_amdgcn_mfma_f32_16x16x4f32(bp[16 * t], ae[e], acc[t], 0, 0, 0)
                                : __builtin_amdgcn_mfma_f32_16x16x4f32(ae[e], bp[16 * t], acc[t], 0, 0, 0);
            }
        }
        if (k0 < a.K) {                                 // ragged tail (fewer than 16 columns left)
            // whole 16-byte pieces when K is a multiple of 4 (300 = 18*16 + 12), else element-wise guarded loads
            float tail[4] = {0.f, 0.f, 0.f, 0.f};
            if ((a.K & 3) == 0) {
                if (k0 + 4 * kq + 4 <= a.K) {
                    const float4 av = load4(ap + k0, a.a_aligned);
                    tail[0] = av.x; tail[1] = av.y; tail[2] = av.z; tail[3] = av.w;
                }
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e) tail[e] = k0 + 4 * kq + e < a.K ? ap[k0 + e] : 0.f;
            }
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int k = k0 + 4 * kq + e;
                const float ae = tail[e];
                const float* bp = Bs + k * a.S + r;     // rows K..Kpad-1 of Bs are zero
#pragma unroll
                for (int t = 0; t < NT; ++t)
                    acc[t] = TR ? __builtin_amdgcn_mfma_f32_16x16x4f32(bp[16 * t], ae, acc[t], 0, 0, 0)
                                : __builtin_amdgcn_mfma_f32_16x16x4f32(ae, bp[16 * t], acc[t], 0, 0, 0);
            }
        }
        if constexpr (TR) {
            const int64_t row = row0 + r;
#pragma unroll
            for (int t = 0; t < NT; ++t) {
                const int col = n0 + 16 * t + 4 * kq;           // N % 4 == 0: the four columns exist together
                if (col >= a.N || row >= a.M) continue;
                float4 o = make_float4(acc[t][0], acc[t][1], acc[t][2], acc[t][3]);
                if (a.bias) {
                    o.x += a.bias[col]; o.y += a.bias[col + 1]; o.z += a.bias[col + 2]; o.w += a.bias[col + 3];
                }
                if (EPI == GCN_EPI_RELU) {
                    o.x = o.x > 0.f ? o.x : 0.f; o.y = o.y > 0.f ? o.y : 0.f;
                    o.z = o.z > 0.f ? o.z : 0.f; o.w = o.w > 0.f ? o.w : 0.f;
                } else if (EPI == GCN_EPI_MASK) {
                    const float4 m = *reinterpret_cast<const float4*>(a.Zprev + row * a.ldzprev + col);
                    o.x = m.x > 0.f ? o.x : 0.f; o.y = m.y > 0.f ? o.y : 0.f;
                    o.z = m.z > 0.f ? o.z : 0.f; o.w = m.w > 0.f ? o.w : 0.f;
                }
                if (a.row_scale) {
                    const float rs = a.row_scale[row];
                    o.x *= rs; o.y *= rs; o.z *= rs; o.w *= rs;
                }
                *reinterpret_cast<float4*>(a.C + row * a.ldc + col) = o;
            }
            continue;
        }
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            const int col = n0 + 16 * t + r;
            if (col >= a.N) continue;
            const float b = a.bias ? a.bias[col] : 0.f;
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int64_t row = row0 + 4 * kq + v;
                if (row < a.M)
                    a.C[row * a.ldc + col] =
                        epi<EPI>(acc[t][v] + b, EPI == GCN_EPI_MASK ? a.Zprev + row * a.ldzprev + col : nullptr);
            }
        }
    }
}

// ---- the same product for dense rows that are not a multiple of a 128-byte line (300 floats = 1200 bytes) ----
// With such rows the strided 64-byte pieces of k_gemm_tall straddle lines and every line is touched by several
// instructions.  Here a wavefront instead copies its whole 16-row strip, which is one contiguous run of 16 K
// floats when lda == K, with fully coalesced 16-byte loads (1 KB per instruction, like a plain copy) into its own
// LDS buffer and takes the MFMA operands from there; the loads of the next strip are in flight (in registers)
// while the current strip is multiplied.  Needs lda == K, K % 4 == 0, 16-byte aligned A, and the wide store path
// (N % 4 == 0, aligned C).  KV = 16-byte loads per lane and strip = ceil(K / 16).
template <int NT, int EPI, int KV>
__global__ __launch_bounds__(512) void k_gemm_tall_flat(TallArgs a) {
    extern __shared__ float lds[];
    float* Bs = lds;                                    // [Kpad][S]
    const int strip_floats = 16 * a.K;
    float* As = lds + a.Kpad * a.S + (threadIdx.x >> 6) * (KV * 256);    // this wavefront's strip, flat
    const int n0 = blockIdx.y * (NT * 16);
    const int ncols = NT * 16;
    for (int idx = threadIdx.x; idx < a.Kpad * ncols; idx += blockDim.x) {
        const int k = idx / ncols, j = idx % ncols;
        float v = 0.f;
        if (k < a.K && n0 + j < a.N) v = a.tb ? a.B[(int64_t)(n0 + j) * a.ldb + k] : a.B[(int64_t)k * a.ldb + n0 + j];
        Bs[k * a.S + j] = v;
    }
    __syncthreads();

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, waves = blockDim.x >> 6;
    const int r = lane & 15, kq = lane >> 4;
    const int64_t ntiles = (a.M + 15) / 16;
    const int64_t total = a.M * (int64_t)a.K;           // floats of A
    const int64_t stride = (int64_t)gridDim.x * waves;
    float4 pre[KV];
    auto fetch = [&](int64_t tile) {
        const int64_t base = tile * strip_floats;
#pragma unroll
        for (int q = 0; q < KV; ++q) {
            const int64_t off = base + (int64_t)(q * 64 + lane) * 4;
            pre[q] = (q * 256 + lane * 4 < strip_floats && off + 4 <= total) ? stream4(a.A + off)
                                                                             : make_float4(0.f, 0.f, 0.f, 0.f);
        }
    };
    int64_t tile = (int64_t)blockIdx.x * waves + wave;
    if (tile < ntiles) fetch(tile);
    for (; tile < ntiles; tile += stride) {
#pragma unroll
        for (int q = 0; q < KV; ++q) *reinterpret_cast<float4*>(As + (q * 64 + lane) * 4) = pre[q];
        __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
        __builtin_amdgcn_wave_barrier();
        if (tile + stride < ntiles) fetch(tile + stride);      // in flight while this strip is multiplied

        const int64_t row0 = tile * 16;
        const float* ap = As + r * a.K + 4 * kq;
        floatx4 acc[NT];
#pragma unroll
        for (int t = 0; t < NT; ++t) acc[t] = (floatx4){0.f, 0.f, 0.f, 0.f};
        const int kfull = a.K & ~15;
        int k0 = 0;
        for (; k0 < kfull; k0 += 16) {
            const float4 av = *reinterpret_cast<const float4*>(ap + k0);
            const float ae[4] = {av.x, av.y, av.z, av.w};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float* bp = Bs + (k0 + 4 * kq + e) * a.S + r;
#pragma unroll
                for (int t = 0; t < NT; ++t) acc[t] = __builtin_amdgcn_mfma_f32_16x16x4f32(bp[16 * t], ae[e], acc[t], 0, 0, 0);
            }
        }
        if (k0 < a.K) {                                 // K % 16 is 4, 8 or 12: whole 16-byte pieces
            float4 av = make_float4(0.f, 0.f, 0.f, 0.f);
            if (k0 + 4 * kq + 4 <= a.K) av = *reinterpret_cast<const float4*>(ap + k0);
            const float ae[4] = {av.x, av.y, av.z, av.w};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float* bp = Bs + (k0 + 4 * kq + e) * a.S + r;     // rows K..Kpad-1 of Bs are zero
#pragma unroll
                for (int t = 0; t < NT; ++t) acc[t] = __builtin_amdgcn_mfma_f32_16x16x4f32(bp[16 * t], ae[e], acc[t], 0, 0, 0);
            }
        }
        const int64_t row = row0 + r;
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            const int col = n0 + 16 * t + 4 * kq;               // N % 4 == 0: the four columns exist together
            if (col >= a.N || row >= a.M) continue;
            float4 o = make_float4(acc[t][0], acc[t][1], acc[t][2], acc[t][3]);
            if (a.bias) {
                o.x += a.bias[col]; o.y += a.bias[col + 1]; o.z += a.bias[col + 2]; o.w += a.bias[col + 3];
            }
            if (EPI == GCN_EPI_RELU) {
                o.x = o.x > 0.f ? o.x : 0.f; o.y = o.y > 0.f ? o.y : 0.f;
                o.z = o.z > 0.f ? o.z : 0.f; o.w = o.w > 0.f ? o.w : 0.f;
            } else if (EPI == GCN_EPI_MASK) {
                const float4 m = *reinterpret_cast<const float4*>(a.Zprev + row * a.ldzprev + col);
                o.x = m.x > 0.f ? o.x : 0.f; o.y = m.y > 0.f ? o.y : 0.f;
                o.z = m.z > 0.f ? o.z : 0.f; o.w = m.w > 0.f ? o.w : 0.f;
            }
            if (a.row_scale) {
                const float rs = a.row_scale[row];
                o.x *= rs; o.y *= rs; o.z *= rs; o.w *= rs;
            }
            *reinterpret_cast<float4*>(a.C + row * a.ldc + col) = o;
        }
        // the next strip overwrites As: this wavefront's LDS operations complete in order
        __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
        __builtin_amdgcn_wave_barrier();
    }
}

// ---- C = A^T B over a long K ---------------------------------------------------------------------
// A workgroup takes the rows [kb, ke) of A and B.  Wavefront w owns the 64-wide column groups
// w, w+4, w+8, ... of A (at most MG of them); inside a group lane i covers columns 4i..4i+3 with one
// 16-byte load, which makes four M-tiles {4i+t : i} for t = 0..3.  Each step consumes four rows
// (one per lane quarter).  The partial M x N results go to part[block][M][N].
struct TnArgs {
    int64_t K;
    int32_t M, N;
    const float* A; int64_t lda;
    const float* B; int64_t ldb;
    float* part;
    int64_t k_per_block;
    int a_aligned;
    int a_stream;      // rows of A are whole 128-byte lines: non-temporal loads
    int waves;         // wavefronts per workgroup (the column groups are dealt to them round-robin); 4 when NARROW
};

template <int MG, int NT, bool NARROW>   // NARROW: MG counts 16-column tiles of A (M <= 16*MG)
__global__ __launch_bounds__(512) void k_gemm_tn(TnArgs a) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int i = lane & 15, kq = lane >> 4;
    const int64_t kb = (int64_t)blockIdx.x * a.k_per_block;
    const int64_t ke = kb + a.k_per_block < a.K ? kb + a.k_per_block : a.K;
    constexpr int TT = NARROW ? 1 : 4;                  // M-tiles per column group
    floatx4 acc[MG][TT][NT];
#pragma unroll
    for (int g = 0; g < MG; ++g)
#pragma unroll
        for (int t = 0; t < TT; ++t)
#pragma unroll
            for (int u = 0; u < NT; ++u) acc[g][t][u] = (floatx4){0.f, 0.f, 0.f, 0.f};

    // NARROW (M <= 32): lane i covers columns i, i+16 of A with 4-byte loads (one M-tile each), and
    // the four wavefronts split the rows instead of the columns.
    int mcol[MG];
    int mvalid[MG];                                     // how many of the lane's 4 columns exist
#pragma unroll
    for (int g = 0; g < MG; ++g) {
        mcol[g] = NARROW ? i + 16 * g : (wave + a.waves * g) * 64 + 4 * i;
        const int left = a.M - mcol[g];
        mvalid[g] = left >= (NARROW ? 1 : 4) ? (NARROW ? 1 : 4) : (left > 0 ? left : 0);
    }
    bool nok[NT];
#pragma unroll
    for (int u = 0; u < NT; ++u) nok[u] = 16 * u + i < a.N;
    const int kstep = NARROW ? 64 : 16;                 // rows per trip of the whole workgroup
    const int koff = NARROW ? 16 * wave : 0;
    for (int64_t k0 = kb + koff; k0 < ke; k0 += kstep) {
        float av[4][MG][TT];
        float bv[4][NT];
#pragma unroll
        for (int s = 0; s < 4; ++s) {                   // issue every load of the trip first
            const int64_t k = k0 + 4 * s + kq;
            const bool kok = k < ke;
            const float* arow = a.A + (kok ? k : kb) * a.lda;
            const float* brow = a.B + (kok ? k : kb) * a.ldb;
#pragma unroll
            for (int u = 0; u < NT; ++u) bv[s][u] = (kok && nok[u]) ? brow[16 * u + i] : 0.f;
#pragma unroll
            for (int g = 0; g < MG; ++g) {
                if constexpr (NARROW) {
                    av[s][g][0] = (kok && mvalid[g]) ? arow[mcol[g]] : 0.f;
                } else {
                    if (kok && mvalid[g] == 4) {
                        const float4 v = load4(arow + mcol[g], a.a_aligned, a.a_stream);
                        av[s][g][0] = v.x; av[s][g][1] = v.y; av[s][g][2] = v.z; av[s][g][3] = v.w;
                    } else {
#pragma unroll
                        for (int t = 0; t < 4; ++t) av[s][g][t] = (kok && t < mvalid[g]) ? arow[mcol[g] + t] : 0.f;
                    }
                }
            }
        }
#pragma unroll
        for (int s = 0; s < 4; ++s)
#pragma unroll
            for (int g = 0; g < MG; ++g)
#pragma unroll
                for (int t = 0; t < TT; ++t)
#pragma unroll
                    for (int u = 0; u < NT; ++u)
                        acc[g][t][u] = __builtin_amdgcn_mfma_f32_16x16x4f32(av[s][g][t], bv[s][u], acc[g][t][u], 0, 0, 0);
    }
    float* out = a.part + (int64_t)blockIdx.x * a.M * a.N;
    if constexpr (NARROW) {
        // the four wavefronts hold partial sums of the same tiles: add them in LDS, fixed order
        __shared__ float s_red[4][MG][NT][64][4];
#pragma unroll
        for (int g = 0; g < MG; ++g)
#pragma unroll
            for (int u = 0; u < NT; ++u)
#pragma unroll
                for (int v = 0; v < 4; ++v) s_red[wave][g][u][lane][v] = acc[g][0][u][v];
        __syncthreads();
        if (wave == 0) {
#pragma unroll
            for (int g = 0; g < MG; ++g)
#pragma unroll
                for (int u = 0; u < NT; ++u)
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        const float sum = ((s_red[0][g][u][lane][v] + s_red[1][g][u][lane][v]) + s_red[2][g][u][lane][v]) +
                                          s_red[3][g][u][lane][v];
                        const int m = 16 * g + 4 * kq + v, n = 16 * u + i;
                        if (m < a.M && n < a.N) out[(int64_t)m * a.N + n] = sum;
                    }
        }
    } else {
        // D[ii = 4*kq + v][j = i] of tile (g, t) is C[m = (wave + waves*g)*64 + 4*ii + t][n = 16u + j]
#pragma unroll
        for (int g = 0; g < MG; ++g)
#pragma unroll
            for (int t = 0; t < 4; ++t)
#pragma unroll
                for (int u = 0; u < NT; ++u)
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        const int m = (wave + a.waves * g) * 64 + 4 * (4 * kq + v) + t;
                        const int n = 16 * u + i;
                        if (m < a.M && n < a.N) out[(int64_t)m * a.N + n] = acc[g][t][u][v];
                    }
    }
}

// Stage 1 of the reduction: group g of `groups` sums the partials g, g+groups, g+2*groups, ... in
// ascending order (coalesced over the output index).
__global__ void k_tn_fold(int64_t count, int parts, int groups, const float* __restrict__ part, float* __restrict__ out) {
    const int64_t o = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int g = blockIdx.y;
    if (o >= count) return;
    float s = 0.f;
    for (int p = g; p < parts; p += groups) s += part[(int64_t)p * count + o];
    out[(int64_t)g * count + o] = s;
}

// Stage 2: sum the (few) groups in ascending order, add the bias, apply the epilogue and store;
// `transposed` means part holds C^T (N x M row-major).
template <int EPI>
__global__ void k_tn_reduce(int32_t M, int32_t N, int parts, int transposed, const float* __restrict__ part,
                            float* __restrict__ C, int64_t ldc, const float* __restrict__ bias,
                            const float* __restrict__ Zprev, int64_t ldzprev) {
    const int64_t o = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t count = (int64_t)M * N;
    if (o >= count) return;
    const int m = (int)(o / N), n = (int)(o % N);
    const int64_t src = transposed ? (int64_t)n * M + m : o;
    float s = 0.f;
    for (int p = 0; p < parts; ++p) s += part[(int64_t)p * count + src];
    if (bias) s += bias[n];
    C[(int64_t)m * ldc + n] = epi<EPI>(s, EPI == GCN_EPI_MASK ? Zprev + (int64_t)m * ldzprev + n : nullptr);
}

static inline bool al16(const void* p) { return ((uintptr_t)p & 15u) == 0; }

template <int NT, bool TR>
static void launch_tall_tr(const TallArgs& args, int epilogue, dim3 grid, size_t lds, hipStream_t s) {
    switch (epilogue) {
        case GCN_EPI_NONE: hipLaunchKernelGGL((k_gemm_tall<NT, GCN_EPI_NONE, TR>), grid, dim3(256), lds, s, args); break;
        case GCN_EPI_RELU: hipLaunchKernelGGL((k_gemm_tall<NT, GCN_EPI_RELU, TR>), grid, dim3(256), lds, s, args); break;
        default: hipLaunchKernelGGL((k_gemm_tall<NT, GCN_EPI_MASK, TR>), grid, dim3(256), lds, s, args); break;
    }
}

template <int NT>
static void launch_tall(const TallArgs& args, int epilogue, dim3 grid, size_t lds, hipStream_t s) {
    // 16-byte stores when every row of C (and of the mask operand) allows them
    const bool wide = (args.N % 4 == 0) && (args.ldc % 4 == 0) && al16(args.C) &&
                      (epilogue != GCN_EPI_MASK || ((args.ldzprev % 4 == 0) && al16(args.Zprev)));
    if (wide) launch_tall_tr<NT, true>(args, epilogue, grid, lds, s);
    else launch_tall_tr<NT, false>(args, epilogue, grid, lds, s);
}

template <int NT, int KV>
static void launch_flat_epi(const TallArgs& args, int waves, int epilogue, dim3 grid, size_t lds, hipStream_t s) {
    // more than 64 KB of LDS per workgroup has to be asked for
    switch (epilogue) {
        case GCN_EPI_NONE:
            (void)hipFuncSetAttribute((const void*)k_gemm_tall_flat<NT, GCN_EPI_NONE, KV>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
            hipLaunchKernelGGL((k_gemm_tall_flat<NT, GCN_EPI_NONE, KV>), grid, dim3(64 * waves), lds, s, args); break;
        case GCN_EPI_RELU:
            (void)hipFuncSetAttribute((const void*)k_gemm_tall_flat<NT, GCN_EPI_RELU, KV>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
            hipLaunchKernelGGL((k_gemm_tall_flat<NT, GCN_EPI_RELU, KV>), grid, dim3(64 * waves), lds, s, args); break;
        default:
            (void)hipFuncSetAttribute((const void*)k_gemm_tall_flat<NT, GCN_EPI_MASK, KV>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
            hipLaunchKernelGGL((k_gemm_tall_flat<NT, GCN_EPI_MASK, KV>), grid, dim3(64 * waves), lds, s, args); break;
    }
}

// KV is a compile-time bound of the per-lane loads: the instantiations cover K <= 112 (7), <= 208 (13), <= 304 (19)
static bool launch_tall_flat(const TallArgs& args, int NT, int KV, int waves, int epilogue, dim3 grid, size_t lds, hipStream_t s) {
    if (NT == 1 && KV <= 7) launch_flat_epi<1, 7>(args, waves, epilogue, grid, lds, s);
    else if (NT == 1 && KV <= 13) launch_flat_epi<1, 13>(args, waves, epilogue, grid, lds, s);
    else if (NT == 1 && KV <= 19) launch_flat_epi<1, 19>(args, waves, epilogue, grid, lds, s);
    else if (NT == 2 && KV <= 7) launch_flat_epi<2, 7>(args, waves, epilogue, grid, lds, s);
    else if (NT == 2 && KV <= 13) launch_flat_epi<2, 13>(args, waves, epilogue, grid, lds, s);
    else if (NT == 2 && KV <= 19) launch_flat_epi<2, 19>(args, waves, epilogue, grid, lds, s);
    else return false;
    return true;
}

template <int MG, int NT, bool NARROW>
static void launch_tn(const TnArgs& args, int blocks, hipStream_t s) {
    hipLaunchKernelGGL((k_gemm_tn<MG, NT, NARROW>), dim3(blocks), dim3(64 * args.waves), 0, s, args);
}

// Launch geometry of the MFMA A^T B product (K long): which operand goes on the 64-column groups, wavefronts
// per workgroup, split of K, partial buffers.  Returns false when the shape is left to the plain kernel.
struct TnShape {
    bool swap, narrow;
    int64_t Mw, Nw, blocks, kpb;
    int NTn, W, MG, fold;
    size_t scratch_bytes;
};

static bool tn_shape(int64_t M, int64_t N, int64_t K, TnShape* g) {
    if (K < 1024) return false;
    // Put the wider of (M, N) on the 64-column groups: if N > M compute C^T = B^T A and let the
    // reduction write it back transposed.
    g->swap = N > M;
    g->Mw = g->swap ? N : M;
    g->Nw = g->swap ? M : N;
    if (g->Nw > 32 || g->Mw > 1024) return false;        // narrow side up to 32, wide side up to 1024
    g->NTn = (int)((g->Nw + 15) / 16);
    g->narrow = g->Mw <= 32;
    const int groups = (int)((g->Mw + 63) / 64);
    // wavefronts per workgroup: one per column group up to 8, else the count in 4..8 that leaves the
    // fewest idle slots (300 columns: 5 groups on 5 wavefronts instead of 2+1+1+1 on 4)
    int W = 4;
    if (!g->narrow) {
        if (groups <= 8) W = groups < 2 ? 2 : groups;
        else {
            int best = 1 << 30;
            for (int w = 4; w <= 8; ++w) {
                const int idle = (groups + w - 1) / w * w - groups;
                if (idle < best) { best = idle; W = w; }
            }
        }
    }
    g->W = W;
    g->MG = g->narrow ? (int)((g->Mw + 15) / 16) : (groups + W - 1) / W;   // tiles (narrow) or column groups per wavefront
    int64_t blocks = K / 256;                             // at least 256 rows per workgroup
    // measured: more, shorter workgroups pay when a workgroup has five or more wavefronts (300 columns:
    // 4.13 ms with 2048 workgroups, 3.84 ms with 8192), fewer otherwise (256 columns: 2.69 vs 2.84 ms)
    // and when it has two or three, so that enough wavefronts exist (128 columns: 1.74 vs 1.47 ms)
    const int64_t max_blocks = g->narrow ? 2048 : (W >= 5 ? 8192 : (W <= 3 ? 16384 / W : 2048));
    if (blocks > max_blocks) blocks = max_blocks;
    if (blocks < 1) blocks = 1;
    int64_t kpb = (K + blocks - 1) / blocks;
    kpb = (kpb + 63) & ~63ll;
    blocks = (K + kpb - 1) / kpb;
    g->blocks = blocks;
    g->kpb = kpb;
    g->fold = blocks > 64 ? 32 : 0;                       // two-stage reduction when there are many partials
    g->scratch_bytes = (size_t)(blocks + g->fold) * g->Mw * g->Nw * sizeof(float);
    return true;
}

size_t gemm_mfma_tn_scratch_bytes(int64_t M, int64_t N, int64_t K) {
    TnShape g;
    return tn_shape(M, N, K, &g) ? g.scratch_bytes : 0;
}

int gemm_mfma_launch(int ta, int tb, int64_t M, int64_t N, int64_t K, const float* A, int64_t lda, const float* B,
                     int64_t ldb, float* C, int64_t ldc, const float* bias, int epilogue, const float* Zprev,
                     int64_t ldzprev, hipStream_t s, bool* handled, const float* row_scale, bool* scaled) {
    *handled = false;
    *scaled = false;
    if (!ta) {
        if (K > 4096 || N > 4096 || M < 64) return GCN_OK;
        const int nt_total = (int)((N + 15) / 16);
        // tiles per wavefront: as many as fit (whole rows of C from one wavefront when N <= 256), while
        // op(B) for them stays within 40 KB of LDS
        const int64_t kpad = (K + 15) & ~15ll;
        int NT = nt_total >= 4 ? 4 : nt_total;
        if (nt_total >= 16 && kpad * (16 * 16 + 4) * 4 <= 40 * 1024) NT = 16;
        else if (nt_total >= 8 && kpad * (16 * 8 + 4) * 4 <= 40 * 1024) NT = 8;
        TallArgs args;
        args.M = M; args.N = (int32_t)N; args.K = (int32_t)K;
        args.A = A; args.lda = lda; args.B = B; args.ldb = ldb; args.tb = tb;
        args.C = C; args.ldc = ldc; args.bias = bias; args.Zprev = Zprev; args.ldzprev = ldzprev;
        args.Kpad = (int32_t)((K + 15) & ~15ll);
        args.S = 16 * NT + 4;
        args.a_aligned = (lda % 4 == 0) && al16(A);
        const bool wide_c = (N % 4 == 0) && (ldc % 4 == 0) && al16(C) &&
                            (epilogue != GCN_EPI_MASK || ((ldzprev % 4 == 0) && al16(Zprev)));
        args.row_scale = wide_c ? row_scale : nullptr;       // the 16-byte store path applies it; else the caller does
        *scaled = args.row_scale != nullptr;
        const size_t lds = (size_t)args.Kpad * args.S * sizeof(float);
        if (lds > 64 * 1024) { *scaled = false; return GCN_OK; }
        const int64_t ntiles = (M + 15) / 16;
        {   // rows that are not whole 128-byte lines, and short rows (up to 208 floats, where the coalesced copy also beats
            // the strided 64-byte pieces: 128 floats 1.02 -> 0.96 ms on 8.7 M rows; at 256 floats it loses, 3.14 -> 3.23 ms):
            // contiguous strips through LDS (see k_gemm_tall_flat)
            const bool wide = (N % 4 == 0) && (ldc % 4 == 0) && al16(C) &&
                              (epilogue != GCN_EPI_MASK || ((ldzprev % 4 == 0) && al16(Zprev)));
            const int kv_need = (int)((K + 15) / 16);
            const int KV = kv_need <= 7 ? 7 : (kv_need <= 13 ? 13 : 19);     // the compiled per-lane load counts
            // wavefronts per workgroup: up to four, as the strips leave room beside op(B); measured on 14 M rows of
            // 300 floats: 2: 4.15, 3: 4.29, 4: 3.57, 5: 3.87, 6: 3.74 ms (the same ranking at 64, 128 and 192 floats)
            int fw = (int)((150 * 1024 - (int64_t)lds) / ((int64_t)KV * 256 * sizeof(float)));
            fw = fw > 4 ? 4 : fw;
            const size_t lds_flat = lds + (size_t)(fw > 0 ? fw : 1) * KV * 256 * sizeof(float);
            if (fw >= 2 && wide && lda == K && (K % 4) == 0 && (((K * 4) % 128) != 0 || K <= 208) && K >= 64 && kv_need <= 19 && NT <= 2 && al16(A) &&
                lds_flat <= 150 * 1024 && M >= 4096) {
                int64_t fb = (ntiles + fw - 1) / fw;
                const int per_cu = (int)((160 * 1024) / lds_flat);
                const int64_t fcap = 256 * (int64_t)(per_cu < 1 ? 1 : per_cu);
                if (fb > fcap) fb = fcap;
                const dim3 fgrid((unsigned)fb, (unsigned)((nt_total + NT - 1) / NT));
                if (launch_tall_flat(args, NT, KV, fw, epilogue, fgrid, lds_flat, s)) {
                    GCN_LAUNCH_CHECK();
                    *handled = true;
                    return GCN_OK;
                }
            }
        }
        int64_t bx = (ntiles + 3) / 4;
        const int64_t cap = 256 * (lds > 40 * 1024 ? 3 : (lds > 20 * 1024 ? 6 : 8));
        if (bx > cap) bx = cap;
        const dim3 grid((unsigned)bx, (unsigned)((nt_total + NT - 1) / NT));
        switch (NT) {
            case 1: launch_tall<1>(args, epilogue, grid, lds, s); break;
            case 2: launch_tall<2>(args, epilogue, grid, lds, s); break;
            case 3: launch_tall<3>(args, epilogue, grid, lds, s); break;
            case 4: launch_tall<4>(args, epilogue, grid, lds, s); break;
            case 8: launch_tall<8>(args, epilogue, grid, lds, s); break;
            default: launch_tall<16>(args, epilogue, grid, lds, s); break;
        }
        GCN_LAUNCH_CHECK();
        *handled = true;
        return GCN_OK;
    }
    // ta: C = A^T B with K long
    if (tb) return GCN_OK;
    TnShape g;
    if (!tn_shape(M, N, K, &g)) return GCN_OK;
    const bool swap = g.swap, narrow = g.narrow;
    const float* Aw = swap ? B : A;
    const float* Bw = swap ? A : B;
    const int64_t ldaw = swap ? ldb : lda, ldbw = swap ? lda : ldb;
    const int64_t Mw = g.Mw, Nw = g.Nw, blocks = g.blocks, kpb = g.kpb;
    const int NTn = g.NTn, W = g.W, MG = g.MG, fold = g.fold;
    void* scratch = nullptr;
    GCN_TRY(scratch_get(&scratch, g.scratch_bytes, s));
    TnArgs args;
    args.K = K; args.M = (int32_t)Mw; args.N = (int32_t)Nw;
    args.A = Aw; args.lda = ldaw; args.B = Bw; args.ldb = ldbw;
    args.part = (float*)scratch; args.k_per_block = kpb;
    args.a_aligned = (ldaw % 4 == 0) && al16(Aw);
    args.a_stream = args.a_aligned && (ldaw % 32 == 0) && (((uintptr_t)Aw & 127u) == 0);
    args.waves = W;
#define GCN_TN_CASE(mg, nt) if (!narrow && MG == mg && NTn == nt) launch_tn<mg, nt, false>(args, (int)blocks, s)
    GCN_TN_CASE(1, 1); GCN_TN_CASE(2, 1); GCN_TN_CASE(3, 1); GCN_TN_CASE(4, 1);
    GCN_TN_CASE(1, 2); GCN_TN_CASE(2, 2); GCN_TN_CASE(3, 2); GCN_TN_CASE(4, 2);
    if (narrow && MG == 1 && NTn == 1) launch_tn<1, 1, true>(args, (int)blocks, s);
    if (narrow && MG == 2 && NTn == 1) launch_tn<2, 1, true>(args, (int)blocks, s);
    if (narrow && MG == 2 && NTn == 2) launch_tn<2, 2, true>(args, (int)blocks, s);
#undef GCN_TN_CASE
    GCN_LAUNCH_CHECK();
    const int64_t count = M * N;
    const float* red_src = (const float*)scratch;
    int red_parts = (int)blocks;
    if (fold) {
        float* folded = (float*)scratch + blocks * count;
        hipLaunchKernelGGL(k_tn_fold, dim3((unsigned)((count + 255) / 256), (unsigned)fold), dim3(256), 0, s, count,
                           (int)blocks, fold, (const float*)scratch, folded);
        GCN_LAUNCH_CHECK();
        red_src = folded;
        red_parts = fold;
    }
    const dim3 rgrid((unsigned)((count + 255) / 256));
    switch (epilogue) {
        case GCN_EPI_NONE: hipLaunchKernelGGL(k_tn_reduce<GCN_EPI_NONE>, rgrid, dim3(256), 0, s, (int32_t)M, (int32_t)N, red_parts, (int)swap, red_src, C, ldc, bias, Zprev, ldzprev); break;
        case GCN_EPI_RELU: hipLaunchKernelGGL(k_tn_reduce<GCN_EPI_RELU>, rgrid, dim3(256), 0, s, (int32_t)M, (int32_t)N, red_parts, (int)swap, red_src, C, ldc, bias, Zprev, ldzprev); break;
        default: hipLaunchKernelGGL(k_tn_reduce<GCN_EPI_MASK>, rgrid, dim3(256), 0, s, (int32_t)M, (int32_t)N, red_parts, (int)swap, red_src, C, ldc, bias, Zprev, ldzprev); break;
    }
    GCN_LAUNCH_CHECK();
    *handled = true;
    return GCN_OK;
}

}  // namespace gcn
