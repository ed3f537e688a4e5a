// Last-layer activation and loss: row-wise log-softmax (the non-elementwise activation the paper
// discusses under "Block Two-Dimensional (2D) Algorithms", Equation H = sigma(Z)) with the mean
// negative log-likelihood over all vertices, and Equation 1 specialised to it:
//   G = (softmax(Z) - onehot(y)) / n.
// L lanes share a row (L = power of two >= min(C, 64)); row maxima and sums are butterfly
// reductions inside the L lanes; the per-row losses are summed in double in a fixed tree.
#include "common.h"

namespace gcn {

template <int L>
__global__ __launch_bounds__(256) void k_softmax_nll(int64_t n, int32_t C, const float* __restrict__ Z, int64_t ldz,
                                                     const int32_t* __restrict__ labels, float* __restrict__ G,
                                                     int64_t ldg, float inv_n, double* __restrict__ part) {
    constexpr int ROWS = 256 / L;
    const int li = threadIdx.x % L;
    const int64_t i = (int64_t)blockIdx.x * ROWS + threadIdx.x / L;
    const bool row_ok = i < n;
    const float* z = Z + (row_ok ? i : 0) * ldz;
    float m = -INFINITY;
    for (int j = li; j < C; j += L) m = fmaxf(m, z[j]);
#pragma unroll
    for (int d = L / 2; d >= 1; d >>= 1) m = fmaxf(m, __shfl_xor(m, d, 64));
    float ssum = 0.f;
    for (int j = li; j < C; j += L) ssum += expf(z[j] - m);
#pragma unroll
    for (int d = L / 2; d >= 1; d >>= 1) ssum += __shfl_xor(ssum, d, 64);
    const float lse = m + logf(ssum);
    int32_t y = row_ok ? labels[i] : 0;
    y = y < 0 ? 0 : (y >= C ? C - 1 : y);   // out-of-range labels are the caller's error; stay in bounds
    if (row_ok && G) {
        float* g = G + i * ldg;
        for (int j = li; j < C; j += L) g[j] = (expf(z[j] - lse) - (j == y ? 1.f : 0.f)) * inv_n;
    }
    double contrib = (row_ok && li == 0) ? (double)lse - (double)z[y] : 0.0;
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) contrib += __shfl_xor(contrib, d, 64);
    __shared__ double s_w[4];
    if ((threadIdx.x & 63) == 0) s_w[threadIdx.x >> 6] = contrib;
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

template <int L>
static int launch(int64_t n, int32_t C, const float* Z, int64_t ldz, const int32_t* labels, float* loss, float* G,
                  int64_t ldg, hipStream_t s) {
    constexpr int ROWS = 256 / L;
    const int64_t blocks = (n + ROWS - 1) / ROWS;
    if (blocks >= (1ll << 31)) return fail(GCN_ERR_RANGE, "gcn_softmax_nll: too many rows");
    void* scratch = nullptr;
    GCN_TRY(scratch_get(&scratch, (size_t)blocks * sizeof(double)));
    hipLaunchKernelGGL(k_softmax_nll<L>, dim3((unsigned)blocks), dim3(256), 0, s, n, C, Z, ldz, labels, G, ldg,
                       1.0f / (float)n, (double*)scratch);
    GCN_LAUNCH_CHECK();
    hipLaunchKernelGGL(k_loss_final, dim3(1), dim3(256), 0, s, blocks, (const double*)scratch, 1.0 / (double)n, loss);
    GCN_LAUNCH_CHECK();
    return GCN_OK;
}

}  // namespace gcn

using namespace gcn;

extern "C" int gcn_softmax_nll(int64_t n, int32_t C, const float* Z, int64_t ldz, const int32_t* labels, float* loss,
                               float* G, int64_t ldg, void* stream) {
    if (!Z || !labels || !loss) return fail(GCN_ERR_BADARG, "gcn_softmax_nll: NULL argument");
    if (n <= 0 || C <= 0 || ldz < C || (G && ldg < C)) return fail(GCN_ERR_BADARG, "gcn_softmax_nll: bad size");
    hipStream_t s = (hipStream_t)stream;
    if (C <= 4) return launch<4>(n, C, Z, ldz, labels, loss, G, ldg, s);
    if (C <= 8) return launch<8>(n, C, Z, ldz, labels, loss, G, ldg, s);
    if (C <= 16) return launch<16>(n, C, Z, ldz, labels, loss, G, ldg, s);
    if (C <= 32) return launch<32>(n, C, Z, ldz, labels, loss, G, ldg, s);
    return launch<64>(n, C, Z, ldz, labels, loss, G, ldg, s);
}
