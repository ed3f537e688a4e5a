// The last layer of the epoch in SpMM-first order, fused.  With T = A^T H^{L-1} (n x 16) at hand, everything
// that follows is local to a row of T: the logits Z^L = T W^L ("Forward Propagation"), the row-wise
// log-softmax and its loss (section "Block Two-Dimensional (2D) Algorithms" names the activation), Equation 1
// G^L = (softmax(Z^L) - onehot(y)) / m, the weight gradient Y^L = T^T G^L (Equation 3 in this association
// order) and the operand S = G^L (W^L)^T of Equation 2's sparse product.  One kernel does all of it per
// 16-row strip, so the n x C matrices Z^L and G^L are never written to memory (unless the caller wants to
// look at them): per row it reads 64 bytes of T and a label and writes 64 bytes of S.
//
// Matrix instruction: v_mfma_f32_16x16x4_f32 (full fp32).  Lane l supplies A[i = l%16][k = l/16] and
// B[k = l/16][j = l%16] and holds D[i = 4*(l/16) + v][j = l%16] in element v.  Let r = l%16, g = l/16.
// The three products are arranged so that each result is already the next one's operand:
//   1. Z^T tiles:  A = W[k = feature][c = 16t + r], B = T[row r][k = feature]   -> the lane holds
//      Z[row r][c = 16t + 4g + v]: a quarter of the row's logits; the softmax joins the four g by shuffles.
//      (The k index of instruction e is 4g' + e for lane group g', so B is element e of the lane's
//      16-byte load of T[row r][4g .. 4g+3].)
//   2. S^T = W G^T:  A = W[feature r][c = 16t + 4g + v], B = the lane's own G[row r][16t + 4g + v]
//      -> the lane holds S[row r][4g + v], stored with one 16-byte store.
//   3. Y tiles += T^T G over the 16 rows of the strip: here the row index is the contraction index, which
//      both operand layouts keep in l/16, so G goes through 16 x 16 transpositions in LDS, four tiles at a time.
// Y accumulates in registers over all strips of a wavefront; the wavefronts of a workgroup are added in a fixed
// order in LDS, the workgroups by two small kernels in a fixed order: bit-reproducible.
#include "common.h"

namespace gcn {

typedef float floatx4 __attribute__((ext_vector_type(4)));

static constexpr int FUSED_BLOCKS_MAX = 2048;
static constexpr int FUSED_FOLD = 32;

struct FusedArgs {
    int64_t n;
    int32_t C;                // classes
    const float* T;           // n x 16, contiguous rows, 16-byte aligned
    const float* W;           // 16 x C row-major
    const int32_t* labels;    // n; negative: outside the training split
    float inv_m;              // 1 / labelled vertices
    float* S;                 // n x 16 = G W^T, or NULL when no earlier layer needs it
    const float* s_scale;     // NULL, or one factor per row of S (the pre-scaling of the value-free sparse product)
    float* Zout;              // n x C (ld C) or NULL
    float* Gout;              // n x C (ld C) or NULL
    float* ypart;             // [gridDim.x][16][16*NT]
    double* lpart;            // [gridDim.x]
};

// FULL: C == 16 NT, no padding columns (their tests are compiled out)
template <int NT, bool FULL>
__global__ __launch_bounds__(256) void k_fused_last(FusedArgs a) {
    constexpr int CP = 16 * NT;            // padded class count
    constexpr int SW = CP + 4;             // row stride of Ws
    constexpr int ST = 20;                 // row stride of Wt and of the per-wavefront tiles
    constexpr int GT = NT < 4 ? NT : 4;    // tiles of G that go through LDS together (NT is 1, 2, 3, 4, 8 or 16; measured at
                                           // 256 classes: 1 tile 3.03 ms, 4 tiles 2.82 ms, 8 tiles 2.95 ms, all 16 slower still)
    extern __shared__ float lds[];
    float* Ws = lds;                       // [16][SW]   W[feature][c]
    float* Wt = Ws + 16 * SW;              // [CP][ST]   W[feature][c] stored as [c][feature]
    float* tiles = Wt + CP * ST;           // per wavefront: Ts[16][ST], Gs[GT][16][ST]
    for (int idx = threadIdx.x; idx < 16 * CP; idx += 256) {
        const int k = idx / CP, c = idx % CP;
        const float v = c < a.C ? a.W[k * a.C + c] : 0.f;
        Ws[k * SW + c] = v;
        Wt[c * ST + k] = v;
    }
    __syncthreads();

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int r = lane & 15, g = lane >> 4;
    float* Ts = tiles + wave * ((1 + GT) * 16 * ST);
    float* Gs = Ts + 16 * ST;
    floatx4 yacc[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) yacc[t] = (floatx4){0.f, 0.f, 0.f, 0.f};
    double lmine = 0.0;
    const int64_t nstrips = (a.n + 15) / 16;
    // The strip's inputs (16 bytes of T per lane, the row's label and the factor of its row of S) are fetched one
    // strip ahead: with one wavefront per SIMD nothing else hides the latency of these loads.
    float4 tv_next = make_float4(0.f, 0.f, 0.f, 0.f);
    int32_t y_next = -1;
    float rs_next = 1.f;
    auto fetch = [&](int64_t strip) {
        const int64_t row = strip * 16 + r;
        tv_next = make_float4(0.f, 0.f, 0.f, 0.f);
        y_next = -1;
        rs_next = 1.f;
        if (row < a.n) {
            tv_next = *reinterpret_cast<const float4*>(a.T + row * 16 + 4 * g);
            y_next = a.labels[row];
            if (a.s_scale) rs_next = a.s_scale[row];
        }
    };
    const int64_t stride = (int64_t)gridDim.x * 4;
    if ((int64_t)blockIdx.x * 4 + wave < nstrips) fetch((int64_t)blockIdx.x * 4 + wave);
    for (int64_t strip = (int64_t)blockIdx.x * 4 + wave; strip < nstrips; strip += stride) {
        const int64_t row = strip * 16 + r;
        const bool valid = row < a.n;
        const float4 tv = tv_next;
        const int32_t y = y_next;
        const float rs = rs_next;
        if (strip + stride < nstrips) fetch(strip + stride);
        // (The operands from W do not depend on the strip: the compiler keeps them in registers across the
        // loop, 128 of them at 256 classes, which leaves one wavefront per SIMD; forcing two by re-reading them
        // from LDS made the register allocator spill, so this is the faster form.)
        const bool labelled = y >= 0;
        const int yc = y < 0 ? 0 : (y >= a.C ? a.C - 1 : y);       // labels >= C are the caller's error; stay in bounds
        *reinterpret_cast<float4*>(Ts + r * ST + 4 * g) = tv;
        const float te[4] = {tv.x, tv.y, tv.z, tv.w};

        // 1. logits: the lane gets Z[row r][16t + 4g + v]
        floatx4 z[NT];
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            z[t] = (floatx4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int e = 0; e < 4; ++e)
                z[t] = __builtin_amdgcn_mfma_f32_16x16x4f32(Ws[(4 * g + e) * SW + 16 * t + r], te[e], z[t], 0, 0, 0);
        }
        if (a.Zout && valid) {
#pragma unroll
            for (int t = 0; t < NT; ++t)
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const int c = 16 * t + 4 * g + v;
                    if (FULL || c < a.C) a.Zout[row * a.C + c] = z[t][v];
                }
        }
        // row-wise log-softmax over the C real columns (padding columns are left out)
        float m = -INFINITY;
#pragma unroll
        for (int t = 0; t < NT; ++t)
#pragma unroll
            for (int v = 0; v < 4; ++v)
                if (FULL || 16 * t + 4 * g + v < a.C) m = fmaxf(m, z[t][v]);
        m = fmaxf(m, __shfl_xor(m, 16, 64));
        m = fmaxf(m, __shfl_xor(m, 32, 64));
        // e = exp(z - max) is computed once per logit and reused: softmax = e / sum(e); the lane that holds
        // column y keeps z_y for the loss
        float ssum = 0.f, zy = 0.f;
#pragma unroll
        for (int t = 0; t < NT; ++t)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int c = 16 * t + 4 * g + v;
                const float zv = z[t][v];
                zy = c == yc ? zv : zy;
                const float e = (FULL || c < a.C) ? __expf(zv - m) : 0.f;
                ssum += e;
                z[t][v] = e;
            }
        ssum += __shfl_xor(ssum, 16, 64);
        ssum += __shfl_xor(ssum, 32, 64);
        const float lse = m + logf(ssum);
        if (labelled && yc >= 4 * g && ((yc - 4 * g) & 15) < 4) lmine += (double)lse - (double)zy;   // column y is this lane's
        // Equation 1 for this loss
        const float scale = labelled ? a.inv_m / ssum : 0.f;
        const float minus = labelled ? a.inv_m : 0.f;
#pragma unroll
        for (int t = 0; t < NT; ++t)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int c = 16 * t + 4 * g + v;
                z[t][v] = z[t][v] * scale - (c == yc ? minus : 0.f);
            }
        if (a.Gout && valid) {
#pragma unroll
            for (int t = 0; t < NT; ++t)
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const int c = 16 * t + 4 * g + v;
                    if (FULL || c < a.C) a.Gout[row * a.C + c] = z[t][v];
                }
        }
        // 2. S = G W^T: the lane gets S[row r][4g + v]
        if (a.S) {
            floatx4 sacc[4];                       // four independent chains, joined at the end
#pragma unroll
            for (int v = 0; v < 4; ++v) sacc[v] = (floatx4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int t = 0; t < NT; ++t) {
#pragma unroll
                for (int v = 0; v < 4; ++v)
                    sacc[v] = __builtin_amdgcn_mfma_f32_16x16x4f32(Wt[(16 * t + 4 * g + v) * ST + r], z[t][v], sacc[v], 0, 0, 0);
            }
            const floatx4 sum = (sacc[0] + sacc[1]) + (sacc[2] + sacc[3]);
            if (valid) *reinterpret_cast<float4*>(a.S + row * 16 + 4 * g) = make_float4(sum[0] * rs, sum[1] * rs, sum[2] * rs, sum[3] * rs);
        }
        // 3. Y += T^T G: the row index is the contraction index, so G goes through a transposition in this
        //    wavefront's LDS, GT tiles at a time (one round trip through LDS per group instead of per tile, and the
        //    tiles' accumulation chains are independent).  The wavefront's LDS operations complete in program order;
        //    the barriers only keep the compiler from reordering them.
        __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
        __builtin_amdgcn_wave_barrier();
        float tk[4];                               // T[row 4kk + g][feature r]: the same for every tile
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) tk[kk] = Ts[(4 * kk + g) * ST + r];
#pragma unroll
        for (int t0 = 0; t0 < NT; t0 += GT) {
#pragma unroll
            for (int u = 0; u < GT; ++u)
                *reinterpret_cast<float4*>(Gs + u * (16 * ST) + r * ST + 4 * g) =
                    make_float4(z[t0 + u][0], z[t0 + u][1], z[t0 + u][2], z[t0 + u][3]);
            __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
            __builtin_amdgcn_wave_barrier();
#pragma unroll
            for (int kk = 0; kk < 4; ++kk) {
                const int rs4 = 4 * kk + g;        // the strip's row this lane contributes to instruction kk
#pragma unroll
                for (int u = 0; u < GT; ++u)
                    yacc[t0 + u] = __builtin_amdgcn_mfma_f32_16x16x4f32(tk[kk], Gs[u * (16 * ST) + rs4 * ST + r], yacc[t0 + u], 0, 0, 0);
            }
            __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
            __builtin_amdgcn_wave_barrier();
        }
    }

    // the workgroup's Y: wavefronts added in order 0, 1, 2, 3 in LDS (the lane holds Y[4g + v][16t + r])
    __syncthreads();
    float* Yr = Ws;
    for (int w = 0; w < 4; ++w) {
        if (wave == w) {
#pragma unroll
            for (int t = 0; t < NT; ++t)
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const int idx = (4 * g + v) * SW + 16 * t + r;
                    Yr[idx] = (w == 0 ? 0.f : Yr[idx]) + yacc[t][v];
                }
        }
        __syncthreads();
    }
    float* yp = a.ypart + (size_t)blockIdx.x * 16 * CP;
    for (int idx = threadIdx.x; idx < 16 * CP; idx += 256) yp[idx] = Yr[(idx / CP) * SW + idx % CP];
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) lmine += __shfl_xor(lmine, d, 64);
    __shared__ double s_w[4];
    if (lane == 0) s_w[wave] = lmine;
    __syncthreads();
    if (threadIdx.x == 0) a.lpart[blockIdx.x] = (s_w[0] + s_w[1]) + (s_w[2] + s_w[3]);
}

// ---- the same layer for more than 64 classes ------------------------------------------------------------------
// With many classes the kernel above keeps 8 registers of W per class tile and runs one wavefront per SIMD, whose
// matrix, vector and LDS phases follow each other with nothing to overlap them.  Here the four wavefronts of a
// workgroup share one strip and each takes a quarter of the class tiles (tile t = wavefront + 4u, u < TW): a quarter of
// the registers (the operands from W come straight from memory, once), so that four workgroups are resident per
// compute unit and fill each other's gaps.  What the wavefronts have to exchange per strip goes through LDS with
// one workgroup barrier: the maxima and sums of the softmax (combined in wavefront order), and the four partial
// tiles of S = G W^T, which one wavefront adds in wavefront order after the barrier of the next strip.  Every
// wavefront owns the Y tiles of its own classes, so the workgroup's partial Y needs no addition.
// Measured at 256 classes on 8.7 M rows: 3.03 ms with S and 2.54 ms without, against 3.59 and 2.83 ms for the kernel
// above; the time falls with the number of resident workgroups per compute unit (1: 4.1, 2: 2.8, 3: 2.5 ms without S),
// three are what the registers allow without spilling (a limit of 128 registers for four made the compiler spill 57 of
// them: 5.1 ms).
template <int TW>      // class tiles per wavefront: up to 64 TW classes
__global__ __launch_bounds__(256, 3) void k_fused_last_wide(FusedArgs a) {
    constexpr int NT = 4 * TW;
    constexpr int CP = 16 * NT;            // padded class count
    constexpr int ST = 20;                 // row stride of the tiles
    extern __shared__ float lds[];
    float* tiles = lds;                    // per wavefront: Ts[16][ST], Gs[TW][16][ST]
    float* red = tiles + 4 * (1 + TW) * 16 * ST;   // two sets of [2][4][16]: row maxima, row sums per wavefront
    float* Sp = red + 2 * 128;             // two sets of [4][64][4]: partial S per wavefront, in lane order

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int r = lane & 15, g = lane >> 4;
    // The operands from W do not depend on the strip: 8 registers per tile, read once from memory.
    //   w1[u][e] = W[feature 4g + e][class 16 (wave + 4u) + r]        (logits)
    //   w2[u][v] = W[feature r][class 16 (wave + 4u) + 4g + v]        (S = G W^T)
    float w1[TW][4], w2[TW][4];
#pragma unroll
    for (int u = 0; u < TW; ++u)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int c1 = 16 * (wave + 4 * u) + r, c2 = 16 * (wave + 4 * u) + 4 * g + e;
            w1[u][e] = c1 < a.C ? a.W[(4 * g + e) * a.C + c1] : 0.f;
            w2[u][e] = c2 < a.C ? a.W[r * a.C + c2] : 0.f;
        }
    float* Ts = tiles + wave * ((1 + TW) * 16 * ST);
    float* Gs = Ts + 16 * ST;
    floatx4 yacc[TW];
#pragma unroll
    for (int u = 0; u < TW; ++u) yacc[u] = (floatx4){0.f, 0.f, 0.f, 0.f};
    double lmine = 0.0;
    const int64_t nstrips = (a.n + 15) / 16;
    float4 tv_next = make_float4(0.f, 0.f, 0.f, 0.f);
    int32_t y_next = -1;
    float rs_next = 1.f;
    auto fetch = [&](int64_t strip) {
        const int64_t row = strip * 16 + r;
        tv_next = make_float4(0.f, 0.f, 0.f, 0.f);
        y_next = -1;
        rs_next = 1.f;
        if (row < a.n) {
            tv_next = *reinterpret_cast<const float4*>(a.T + row * 16 + 4 * g);
            y_next = a.labels[row];
            if (a.s_scale) rs_next = a.s_scale[row];
        }
    };
    if ((int64_t)blockIdx.x < nstrips) fetch(blockIdx.x);
    int trip = 0;
    int64_t prev_row = 0;
    float prev_rs = 1.f;
    bool prev_valid = false;
    for (int64_t strip = blockIdx.x; strip < nstrips; strip += gridDim.x, ++trip) {   // the same trip count for all four wavefronts
        const int64_t row = strip * 16 + r;
        const bool valid = row < a.n;
        const float4 tv = tv_next;
        const int32_t y = y_next;
        const float rs = rs_next;
        if (strip + gridDim.x < nstrips) fetch(strip + gridDim.x);
        const bool labelled = y >= 0;
        const int yc = y < 0 ? 0 : (y >= a.C ? a.C - 1 : y);       // labels >= C are the caller's error; stay in bounds
        *reinterpret_cast<float4*>(Ts + r * ST + 4 * g) = tv;
        const float te[4] = {tv.x, tv.y, tv.z, tv.w};

        // 1. logits of this wavefront's tiles: the lane gets Z[row r][16 (wave + 4u) + 4g + v]
        floatx4 z[TW];
#pragma unroll
        for (int u = 0; u < TW; ++u) {
            z[u] = (floatx4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int e = 0; e < 4; ++e)
                z[u] = __builtin_amdgcn_mfma_f32_16x16x4f32(w1[u][e], te[e], z[u], 0, 0, 0);
        }
        if (a.Zout && valid) {
#pragma unroll
            for (int u = 0; u < TW; ++u)
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const int c = 16 * (wave + 4 * u) + 4 * g + v;
                    if (c < a.C) a.Zout[row * a.C + c] = z[u][v];
                }
        }
        // Row-wise log-softmax over the C real columns with one exchange between the wavefronts: every wavefront takes
        // maximum m_w and sum s_w = sum exp(z - m_w) over its own columns; with m = max m_w the row's sum is
        // sum_w s_w exp(m_w - m) (added in wavefront order) and this wavefront's exp(z - m) are its exp(z - m_w) times
        // exp(m_w - m), a factor that goes into the scale of Equation 1.  The lane that holds column y keeps z_y.
        float mw = -INFINITY;
#pragma unroll
        for (int u = 0; u < TW; ++u)
#pragma unroll
            for (int v = 0; v < 4; ++v)
                if (16 * (wave + 4 * u) + 4 * g + v < a.C) mw = fmaxf(mw, z[u][v]);
        mw = fmaxf(mw, __shfl_xor(mw, 16, 64));
        mw = fmaxf(mw, __shfl_xor(mw, 32, 64));
        float sw = 0.f, zy = 0.f;
#pragma unroll
        for (int u = 0; u < TW; ++u)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int c = 16 * (wave + 4 * u) + 4 * g + v;
                const float zv = z[u][v];
                zy = c == yc ? zv : zy;
                const float e = c < a.C ? __expf(zv - mw) : 0.f;      // a wavefront without real columns: all 0
                sw += e;
                z[u][v] = e;
            }
        sw += __shfl_xor(sw, 16, 64);
        sw += __shfl_xor(sw, 32, 64);
        float* const redb = red + (trip & 1) * 128;          // two sets of slots: a fast wavefront writes the next
        float* const Spb = Sp + (trip & 1) * 1024;           // strip's while a slow one still reads this strip's
        if (g == 0) {
            redb[wave * 16 + r] = mw;
            redb[64 + wave * 16 + r] = sw;
        }
        __syncthreads();                                     // the one workgroup barrier of a strip
        // the strip before this one left its four partial tiles of S in the other set of slots: one wavefront (they take
        // turns) adds them in wavefront order and stores the rows
        if (a.S && trip > 0 && ((trip - 1) & 3) == wave && prev_valid) {
            const float* q = Sp + ((trip - 1) & 1) * 1024;
            const float4 p0 = *reinterpret_cast<const float4*>(q + lane * 4);
            const float4 p1 = *reinterpret_cast<const float4*>(q + (64 + lane) * 4);
            const float4 p2 = *reinterpret_cast<const float4*>(q + (128 + lane) * 4);
            const float4 p3 = *reinterpret_cast<const float4*>(q + (192 + lane) * 4);
            *reinterpret_cast<float4*>(a.S + prev_row * 16 + 4 * g) =
                make_float4((((p0.x + p1.x) + p2.x) + p3.x) * prev_rs, (((p0.y + p1.y) + p2.y) + p3.y) * prev_rs,
                            (((p0.z + p1.z) + p2.z) + p3.z) * prev_rs, (((p0.w + p1.w) + p2.w) + p3.w) * prev_rs);
        }
        const float m0 = redb[r], m1 = redb[16 + r], m2 = redb[32 + r], m3 = redb[48 + r];
        const float m = fmaxf(fmaxf(m0, m1), fmaxf(m2, m3));
        const float ssum = ((redb[64 + r] * __expf(m0 - m) + redb[64 + 16 + r] * __expf(m1 - m)) +
                            redb[64 + 32 + r] * __expf(m2 - m)) + redb[64 + 48 + r] * __expf(m3 - m);
        const float lse = m + logf(ssum);
        if (labelled && ((yc >> 4) & 3) == wave && ((yc & 15) >> 2) == g) lmine += (double)lse - (double)zy;   // column y is this lane's
        // Equation 1 for this loss
        const float scale = labelled ? a.inv_m * __expf(mw - m) / ssum : 0.f;
        const float minus = labelled ? a.inv_m : 0.f;
#pragma unroll
        for (int u = 0; u < TW; ++u)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int c = 16 * (wave + 4 * u) + 4 * g + v;
                z[u][v] = z[u][v] * scale - (c == yc ? minus : 0.f);
            }
        if (a.Gout && valid) {
#pragma unroll
            for (int u = 0; u < TW; ++u)
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const int c = 16 * (wave + 4 * u) + 4 * g + v;
                    if (c < a.C) a.Gout[row * a.C + c] = z[u][v];
                }
        }
        // 2. S = G W^T: this wavefront's classes give a partial S[row r][4g + v], left in LDS for the next trip
        if (a.S) {
            floatx4 sacc[4];
#pragma unroll
            for (int v = 0; v < 4; ++v) sacc[v] = (floatx4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int u = 0; u < TW; ++u)
#pragma unroll
                for (int v = 0; v < 4; ++v)
                    sacc[v] = __builtin_amdgcn_mfma_f32_16x16x4f32(w2[u][v], z[u][v], sacc[v], 0, 0, 0);
            const floatx4 part = (sacc[0] + sacc[1]) + (sacc[2] + sacc[3]);
            *reinterpret_cast<float4*>(Spb + (wave * 64 + lane) * 4) = make_float4(part[0], part[1], part[2], part[3]);
        }
        prev_row = row; prev_rs = rs; prev_valid = valid;
        // 3. Y += T^T G for this wavefront's tiles, all of them through one transposition in its own LDS (its LDS
        //    operations complete in program order; the barriers only keep the compiler from reordering them)
        __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
        __builtin_amdgcn_wave_barrier();
        float tk[4];                               // T[row 4kk + g][feature r]
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) tk[kk] = Ts[(4 * kk + g) * ST + r];
#pragma unroll
        for (int u = 0; u < TW; ++u)
            *reinterpret_cast<float4*>(Gs + u * (16 * ST) + r * ST + 4 * g) = make_float4(z[u][0], z[u][1], z[u][2], z[u][3]);
        __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            const int rs4 = 4 * kk + g;
#pragma unroll
            for (int u = 0; u < TW; ++u)
                yacc[u] = __builtin_amdgcn_mfma_f32_16x16x4f32(tk[kk], Gs[u * (16 * ST) + rs4 * ST + r], yacc[u], 0, 0, 0);
        }
        __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
        __builtin_amdgcn_wave_barrier();
    }

    __syncthreads();
    if (a.S && trip > 0 && ((trip - 1) & 3) == wave && prev_valid) {              // the last strip's rows of S
        const float* q = Sp + ((trip - 1) & 1) * 1024;
        const float4 p0 = *reinterpret_cast<const float4*>(q + lane * 4);
        const float4 p1 = *reinterpret_cast<const float4*>(q + (64 + lane) * 4);
        const float4 p2 = *reinterpret_cast<const float4*>(q + (128 + lane) * 4);
        const float4 p3 = *reinterpret_cast<const float4*>(q + (192 + lane) * 4);
        *reinterpret_cast<float4*>(a.S + prev_row * 16 + 4 * g) =
            make_float4((((p0.x + p1.x) + p2.x) + p3.x) * prev_rs, (((p0.y + p1.y) + p2.y) + p3.y) * prev_rs,
                        (((p0.z + p1.z) + p2.z) + p3.z) * prev_rs, (((p0.w + p1.w) + p2.w) + p3.w) * prev_rs);
    }
    // the workgroup's Y: the lane holds Y[feature 4g + v][class 16 (wave + 4u) + r] of its own tiles
    float* yp = a.ypart + (size_t)blockIdx.x * 16 * CP;
#pragma unroll
    for (int u = 0; u < TW; ++u)
#pragma unroll
        for (int v = 0; v < 4; ++v) yp[(4 * g + v) * CP + 16 * (wave + 4 * u) + r] = yacc[u][v];
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) lmine += __shfl_xor(lmine, d, 64);
    __shared__ double s_w[4];
    if (lane == 0) s_w[wave] = lmine;
    __syncthreads();
    if (threadIdx.x == 0) a.lpart[blockIdx.x] = (s_w[0] + s_w[1]) + (s_w[2] + s_w[3]);
}

// folded[j][e] = sum over the workgroups b = j, j + FOLD, j + 2 FOLD, ... of part[b][e], in that order
__global__ __launch_bounds__(256) void k_fused_fold(int count, int blocks, const float* __restrict__ part,
                                                    float* __restrict__ folded) {
    const int e = blockIdx.x * 256 + threadIdx.x;
    const int j = blockIdx.y;
    if (e >= count) return;
    float acc = 0.f;
    for (int b = j; b < blocks; b += FUSED_FOLD) acc += part[(size_t)b * count + e];
    folded[(size_t)j * count + e] = acc;
}

// Y[k][c] = sum over j of folded[j][k][c] for the C real columns
__global__ __launch_bounds__(256) void k_fused_y(int C, int CP, int parts, const float* __restrict__ folded,
                                                 float* __restrict__ Y) {
    const int e = blockIdx.x * 256 + threadIdx.x;
    if (e >= 16 * C) return;
    const int k = e / C, c = e % C;
    float acc = 0.f;
    for (int j = 0; j < parts; ++j) acc += folded[(size_t)j * 16 * CP + k * CP + c];
    Y[k * C + c] = acc;
}

int loss_final_launch(int64_t parts, const double* part, double inv_n, float* loss, hipStream_t s);

static int fused_nt(int32_t C) {
    const int need = (C + 15) / 16;
    const int have[6] = {1, 2, 3, 4, 8, 16};
    for (int i = 0; i < 6; ++i)
        if (have[i] >= need) return have[i];
    return 0;
}

static int64_t fused_blocks(int64_t n) {
    int64_t blocks = ((n + 15) / 16 + 3) / 4;
    return blocks > FUSED_BLOCKS_MAX ? FUSED_BLOCKS_MAX : (blocks < 1 ? 1 : blocks);
}

bool fused_last_supported(int32_t f_in, int32_t C) { return f_in == 16 && C >= 1 && fused_nt(C) != 0; }

size_t fused_last_scratch_bytes(int64_t n, int32_t C) {
    const int NT = fused_nt(C);
    if (!NT) return 0;
    const size_t per = (size_t)16 * 16 * NT * sizeof(float);
    return (size_t)(fused_blocks(n) + FUSED_FOLD) * per + (size_t)FUSED_BLOCKS_MAX * sizeof(double);
}

template <int NT>
static void launch_fused(const FusedArgs& a, int64_t blocks, hipStream_t s) {
    const int GT = NT < 4 ? NT : 4;
    const size_t lds = (size_t)(16 * (16 * NT + 4) + 16 * NT * 20 + 4 * (1 + GT) * 16 * 20) * sizeof(float);
    // (a variant with the padding tests compiled out for C == 16 NT made the register allocator spill: not used)
    hipLaunchKernelGGL((k_fused_last<NT, false>), dim3((unsigned)blocks), dim3(256), lds, s, a);
}

template <int TW>
static void launch_fused_wide(const FusedArgs& a, int64_t blocks, hipStream_t s) {
    // per wavefront Ts and TW tiles of G, two sets of softmax slots, two sets of partial S tiles
    const size_t lds = (size_t)(4 * (1 + TW) * 16 * 20 + 2 * 128 + 2 * 4 * 64 * 4) * sizeof(float);
    hipLaunchKernelGGL((k_fused_last_wide<TW>), dim3((unsigned)blocks), dim3(256), lds, s, a);
}

// T: n x 16 contiguous; W: 16 x C; Y: 16 x C; S: n x 16 or NULL, its rows multiplied by s_scale when that is given;
// Zout / Gout: n x C or NULL; scratch: at least fused_last_scratch_bytes(n, C).
int fused_last_launch(int64_t n, int32_t C, const float* T, const float* W, const int32_t* labels, int64_t n_labelled,
                      float* loss, float* Y, float* S, const float* s_scale, float* Zout, float* Gout, void* scratch,
                      hipStream_t s) {
    const int NT = fused_nt(C);
    if (!NT) return fail(GCN_ERR_BADARG, "fused last layer: more than 256 classes");
    if (((uintptr_t)T & 15u) || (S && ((uintptr_t)S & 15u))) return fail(GCN_ERR_BADARG, "fused last layer: unaligned operand");
    const int64_t blocks = fused_blocks(n);
    const int count = 16 * 16 * NT;
    FusedArgs a;
    a.n = n; a.C = C; a.T = T; a.W = W; a.labels = labels; a.inv_m = 1.0f / (float)n_labelled;
    a.S = S; a.s_scale = s_scale; a.Zout = Zout; a.Gout = Gout;
    a.ypart = (float*)scratch;
    float* folded = a.ypart + (size_t)blocks * count;
    a.lpart = (double*)(folded + (size_t)FUSED_FOLD * count);
    switch (NT) {
        case 1: launch_fused<1>(a, blocks, s); break;
        case 2: launch_fused<2>(a, blocks, s); break;
        case 3: launch_fused<3>(a, blocks, s); break;
        case 4: launch_fused<4>(a, blocks, s); break;
        case 8: launch_fused_wide<2>(a, blocks, s); break;
        default: launch_fused_wide<4>(a, blocks, s); break;
    }
    GCN_LAUNCH_CHECK();
    const int parts = blocks < FUSED_FOLD ? (int)blocks : FUSED_FOLD;
    hipLaunchKernelGGL(k_fused_fold, dim3((unsigned)((count + 255) / 256), (unsigned)parts), dim3(256), 0, s, count,
                       (int)blocks, (const float*)a.ypart, folded);
    GCN_LAUNCH_CHECK();
    hipLaunchKernelGGL(k_fused_y, dim3((unsigned)((16 * C + 255) / 256)), dim3(256), 0, s, (int)C, 16 * NT, parts,
                       (const float*)folded, Y);
    GCN_LAUNCH_CHECK();
    return loss_final_launch(blocks, a.lpart, 1.0 / (double)n_labelled, loss, s);
}

}  // namespace gcn
