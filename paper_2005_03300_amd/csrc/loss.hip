// Last-layer activation and loss: row-wise log-softmax (the non-elementwise activation the paper
// discusses under "Block Two-Dimensional (2D) Algorithms", Equation H = sigma(Z)) with the mean
// negative log-likelihood over all vertices, and Equation 1 specialised to it:
//   G = (softmax(Z) - onehot(y)) / n.
// L lanes share a row and keep its logits in registers (VEC per lane, C <= L*VEC): one read of Z,
// one write of G.  Row maxima and sums are butterfly reductions inside the L lanes.  Workgroups
// stride over the rows; every thread adds its rows' losses in double in a fixed order, then a
// fixed tree joins threads and workgroups, so the loss is reproducible bit for bit.
#include "common.h"

namespace gcn {

static constexpr int LOSS_BLOCKS_MAX = 2048;

template <int L, int VEC>
__global__ __launch_bounds__(256) void k_softmax_nll(int64_t n, int32_t C, const float* __restrict__ Z, int64_t ldz,
                                                     const int32_t* __restrict__ labels, float* __restrict__ G,
                                                     int64_t ldg, float inv_n, double* __restrict__ part) {
    constexpr int ROWS = 256 / L;
    const int li = threadIdx.x % L;
    const int c0 = li * VEC;
    double mine = 0.0;
    for (int64_t i = (int64_t)blockIdx.x * ROWS + threadIdx.x / L; i < n; i += (int64_t)gridDim.x * ROWS) {
        const float* z = Z + i * ldz;
        float v[VEC];
        if constexpr (VEC == 4) {
            if (c0 < C) {
                const float4 t = *reinterpret_cast<const float4*>(z + c0);
                v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w;
            } else {
                v[0] = v[1] = v[2] = v[3] = -INFINITY;
            }
        } else {
            v[0] = c0 < C ? z[c0] : -INFINITY;
        }
        float m = v[0];
#pragma unroll
        for (int e = 1; e < VEC; ++e) m = fmaxf(m, v[e]);
#pragma unroll
        for (int d = L / 2; d >= 1; d >>= 1) m = fmaxf(m, __shfl_xor(m, d, 64));
        float ssum = 0.f;
#pragma unroll
        for (int e = 0; e < VEC; ++e) ssum += expf(v[e] - m);          // exp(-inf) = 0 for padding lanes
#pragma unroll
        for (int d = L / 2; d >= 1; d >>= 1) ssum += __shfl_xor(ssum, d, 64);
        const float lse = m + logf(ssum);
        int32_t y = labels[i];
        const bool labelled = y >= 0;           // negative label: vertex outside the training split
        y = y < 0 ? 0 : (y >= C ? C - 1 : y);   // labels >= C are the caller's error; stay in bounds
        if (G && c0 < C) {
            float g[VEC];
#pragma unroll
            for (int e = 0; e < VEC; ++e)
                g[e] = labelled ? (expf(v[e] - lse) - (c0 + e == y ? 1.f : 0.f)) * inv_n : 0.f;
            if constexpr (VEC == 4) *reinterpret_cast<float4*>(G + i * ldg + c0) = make_float4(g[0], g[1], g[2], g[3]);
            else G[i * ldg + c0] = g[0];
        }
        // the lane that holds column y contributes lse - z_y
        float zy = 0.f;
#pragma unroll
        for (int e = 0; e < VEC; ++e) zy = (c0 + e == y) ? v[e] : zy;
        if (labelled && y >= c0 && y < c0 + VEC) mine += (double)lse - (double)zy;
    }
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) mine += __shfl_xor(mine, d, 64);
    __shared__ double s_w[4];
    if ((threadIdx.x & 63) == 0) s_w[threadIdx.x >> 6] = mine;
    __syncthreads();
    if (threadIdx.x == 0) part[blockIdx.x] = (s_w[0] + s_w[1]) + (s_w[2] + s_w[3]);
}

// Any C: lanes loop over the columns and re-read the row (three passes, served by the caches).
__global__ __launch_bounds__(256) void k_softmax_nll_wide(int64_t n, int32_t C, const float* __restrict__ Z,
                                                          int64_t ldz, const int32_t* __restrict__ labels,
                                                          float* __restrict__ G, int64_t ldg, float inv_n,
                                                          double* __restrict__ part) {
    const int li = threadIdx.x & 63;
    double mine = 0.0;
    for (int64_t i = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6); i < n; i += (int64_t)gridDim.x * 4) {
        const float* z = Z + i * ldz;
        float m = -INFINITY;
        for (int j = li; j < C; j += 64) m = fmaxf(m, z[j]);
#pragma unroll
        for (int d = 32; d >= 1; d >>= 1) m = fmaxf(m, __shfl_xor(m, d, 64));
        float ssum = 0.f;
        for (int j = li; j < C; j += 64) ssum += expf(z[j] - m);
#pragma unroll
        for (int d = 32; d >= 1; d >>= 1) ssum += __shfl_xor(ssum, d, 64);
        const float lse = m + logf(ssum);
        int32_t y = labels[i];
        const bool labelled = y >= 0;
        y = y < 0 ? 0 : (y >= C ? C - 1 : y);
        if (G) {
            float* g = G + i * ldg;
            for (int j = li; j < C; j += 64) g[j] = labelled ? (expf(z[j] - lse) - (j == y ? 1.f : 0.f)) * inv_n : 0.f;
        }
        if (li == 0 && labelled) mine += (double)lse - (double)z[y];
    }
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) mine += __shfl_xor(mine, d, 64);
    __shared__ double s_w[4];
    if ((threadIdx.x & 63) == 0) s_w[threadIdx.x >> 6] = mine;
    __syncthreads();
    if (threadIdx.x == 0) part[blockIdx.x] = (s_w[0] + s_w[1]) + (s_w[2] + s_w[3]);
}

// Single block: strided sums per thread, then a fixed shared-memory tree.
__global__ __launch_bounds__(256) void k_loss_final(int64_t parts, const double* __restrict__ part, double inv_n,
                                                    float* __restrict__ loss) {
    __shared__ double s[256];
    double acc = 0.0;
    for (int64_t p = threadIdx.x; p < parts; p += 256) acc += part[p];
    s[threadIdx.x] = acc;
    __syncthreads();
    for (int d = 128; d >= 1; d >>= 1) {
        if ((int)threadIdx.x < d) s[threadIdx.x] += s[threadIdx.x + d];
        __syncthreads();
    }
    if (threadIdx.x == 0) *loss = (float)(s[0] * inv_n);
}

template <int L, int VEC>
static void launch_rows(int64_t blocks, int64_t n, int32_t C, const float* Z, int64_t ldz, const int32_t* labels,
                        float* G, int64_t ldg, double* part, float inv_m, hipStream_t s) {
    hipLaunchKernelGGL((k_softmax_nll<L, VEC>), dim3((unsigned)blocks), dim3(256), 0, s, n, C, Z, ldz, labels, G, ldg,
                       inv_m, part);
}

template <int VEC>
static void dispatch_rows(int lanes, int64_t n, int32_t C, const float* Z, int64_t ldz, const int32_t* labels,
                          float* G, int64_t ldg, double* part, int64_t* blocks_out, float inv_m, hipStream_t s) {
    int L = 2;
    while (L < lanes) L <<= 1;
    const int64_t rows_per_block = 256 / L;
    int64_t blocks = (n + rows_per_block - 1) / rows_per_block;
    if (blocks > LOSS_BLOCKS_MAX) blocks = LOSS_BLOCKS_MAX;
    *blocks_out = blocks;
    switch (L) {
        case 2: launch_rows<2, VEC>(blocks, n, C, Z, ldz, labels, G, ldg, part, inv_m, s); break;
        case 4: launch_rows<4, VEC>(blocks, n, C, Z, ldz, labels, G, ldg, part, inv_m, s); break;
        case 8: launch_rows<8, VEC>(blocks, n, C, Z, ldz, labels, G, ldg, part, inv_m, s); break;
        case 16: launch_rows<16, VEC>(blocks, n, C, Z, ldz, labels, G, ldg, part, inv_m, s); break;
        case 32: launch_rows<32, VEC>(blocks, n, C, Z, ldz, labels, G, ldg, part, inv_m, s); break;
        default: launch_rows<64, VEC>(blocks, n, C, Z, ldz, labels, G, ldg, part, inv_m, s); break;
    }
}

int loss_final_launch(int64_t parts, const double* part, double inv_n, float* loss, hipStream_t s) {
    hipLaunchKernelGGL(k_loss_final, dim3(1), dim3(256), 0, s, parts, part, inv_n, loss);
    GCN_LAUNCH_CHECK();
    return GCN_OK;
}

size_t loss_scratch_bytes() { return (size_t)LOSS_BLOCKS_MAX * sizeof(double); }

}  // namespace gcn

using namespace gcn;

static int softmax_nll_impl(int64_t n, int32_t C, const float* Z, int64_t ldz, const int32_t* labels, int64_t n_labelled,
                            float* loss, float* G, int64_t ldg, hipStream_t s) {
    void* scratch = nullptr;
    GCN_TRY(scratch_get(&scratch, loss_scratch_bytes(), s));
    double* part = (double*)scratch;
    int64_t blocks = 0;
    const float inv_m = 1.0f / (float)n_labelled;
    const bool vec4 = (C % 4 == 0) && (ldz % 4 == 0) && (((uintptr_t)Z & 15u) == 0) &&
                      (!G || ((ldg % 4 == 0) && (((uintptr_t)G & 15u) == 0)));
    if (vec4 && C <= 256) {
        dispatch_rows<4>(C / 4, n, C, Z, ldz, labels, G, ldg, part, &blocks, inv_m, s);
    } else if (C <= 64) {
        dispatch_rows<1>(C, n, C, Z, ldz, labels, G, ldg, part, &blocks, inv_m, s);
    } else {
        blocks = (n + 3) / 4;
        if (blocks > LOSS_BLOCKS_MAX) blocks = LOSS_BLOCKS_MAX;
        hipLaunchKernelGGL(k_softmax_nll_wide, dim3((unsigned)blocks), dim3(256), 0, s, n, C, Z, ldz, labels, G, ldg,
                           inv_m, part);
    }
    GCN_LAUNCH_CHECK();
    hipLaunchKernelGGL(k_loss_final, dim3(1), dim3(256), 0, s, blocks, (const double*)part, 1.0 / (double)n_labelled, loss);
    GCN_LAUNCH_CHECK();
    return GCN_OK;
}

extern "C" int gcn_softmax_nll(int64_t n, int32_t C, const float* Z, int64_t ldz, const int32_t* labels, float* loss,
                               float* G, int64_t ldg, void* stream) {
    if (!Z || !labels || !loss) return fail(GCN_ERR_BADARG, "gcn_softmax_nll: NULL argument");
    if (n <= 0 || C <= 0 || ldz < C || (G && ldg < C)) return fail(GCN_ERR_BADARG, "gcn_softmax_nll: bad size");
    return softmax_nll_impl(n, C, Z, ldz, labels, n, loss, G, ldg, (hipStream_t)stream);
}

extern "C" int gcn_softmax_nll_masked(int64_t n, int32_t C, const float* Z, int64_t ldz, const int32_t* labels,
                                      int64_t n_labelled, float* loss, float* G, int64_t ldg, void* stream) {
    if (!Z || !labels || !loss) return fail(GCN_ERR_BADARG, "gcn_softmax_nll_masked: NULL argument");
    if (n <= 0 || C <= 0 || ldz < C || (G && ldg < C)) return fail(GCN_ERR_BADARG, "gcn_softmax_nll_masked: bad size");
    if (n_labelled <= 0 || n_labelled > n) return fail(GCN_ERR_BADARG, "gcn_softmax_nll_masked: n_labelled must be in [1, n]");
    return softmax_nll_impl(n, C, Z, ldz, labels, n_labelled, loss, G, ldg, (hipStream_t)stream);
}
