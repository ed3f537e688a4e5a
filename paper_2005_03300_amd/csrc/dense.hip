// Dense products and element-wise kernels around the SpMM: H W of "Forward Propagation", S W^T of
// Equation 2, the weight gradient H^T S of Equation 3, ReLU and its derivative mask, column sums
// for an optional bias gradient, and the gradient step.
#include "common.h"

namespace gcn {

template <int EPI>
__device__ __forceinline__ float apply_epi(float v, const float* zprev_elem) {
    if (EPI == GCN_EPI_RELU) return v > 0.f ? v : 0.f;
    if (EPI == GCN_EPI_MASK) return *zprev_elem > 0.f ? v : 0.f;
    return v;
}

// ---- generic fallback: one thread per output element (any shape, any leading dimension) ----
template <int EPI>
__global__ void k_gemm_naive(int tb, int64_t M, int64_t N, int64_t K, const float* __restrict__ A, int64_t lda,
                             const float* __restrict__ B, int64_t ldb, float* __restrict__ C, int64_t ldc,
                             const float* __restrict__ bias, const float* __restrict__ Zprev, int64_t ldzprev) {
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t i = t / N, j = t % N;
    if (i >= M) return;
    float acc = 0.f;
    if (tb) for (int64_t k = 0; k < K; ++k) acc = fmaf(A[i * lda + k], B[j * ldb + k], acc);
    else for (int64_t k = 0; k < K; ++k) acc = fmaf(A[i * lda + k], B[k * ldb + j], acc);
    if (bias) acc += bias[j];
    C[i * ldc + j] = apply_epi<EPI>(acc, EPI == GCN_EPI_MASK ? Zprev + i * ldzprev + j : nullptr);
}

// ---- C = A^T B with a long K: each block sums one K range into a partial M x N --------------
__global__ void k_gemm_tn_partial(int64_t M, int64_t N, int64_t K, int64_t k_per_block, const float* __restrict__ A,
                                  int64_t lda, const float* __restrict__ B, int64_t ldb, float* __restrict__ part) {
    const int64_t kb = (int64_t)blockIdx.x * k_per_block;
    const int64_t ke = kb + k_per_block < K ? kb + k_per_block : K;
    float* out = part + (int64_t)blockIdx.x * M * N;
    for (int64_t o = threadIdx.x; o < M * N; o += blockDim.x) {
        const int64_t i = o / N, j = o % N;
        float acc = 0.f;
        for (int64_t k = kb; k < ke; ++k) acc = fmaf(A[k * lda + i], B[k * ldb + j], acc);
        out[o] = acc;
    }
}

template <int EPI>
__global__ void k_reduce_partials(int64_t count, int64_t N, int parts, const float* __restrict__ part,
                                  float* __restrict__ C, int64_t ldc, const float* __restrict__ bias,
                                  const float* __restrict__ Zprev, int64_t ldzprev) {
    const int64_t o = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (o >= count) return;
    float acc = 0.f;
    for (int p = 0; p < parts; ++p) acc += part[(int64_t)p * count + o];   // fixed order
    const int64_t i = o / N, j = o % N;
    if (bias) acc += bias[j];
    C[i * ldc + j] = apply_epi<EPI>(acc, EPI == GCN_EPI_MASK ? Zprev + i * ldzprev + j : nullptr);
}

// ---- element-wise -----------------------------------------------------------------------------
__global__ void k_relu(int64_t rows, int32_t cols, const float* __restrict__ Z, int64_t ldz, float* __restrict__ H,
                       int64_t ldh) {
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t i = t / cols;
    const int j = (int)(t % cols);
    if (i >= rows) return;
    const float z = Z[i * ldz + j];
    H[i * ldh + j] = z > 0.f ? z : 0.f;
}

__global__ void k_relu_mask(int64_t rows, int32_t cols, const float* __restrict__ G, int64_t ldg,
                            const float* __restrict__ Zp, int64_t ldzp, float* __restrict__ out, int64_t ldo) {
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t i = t / cols;
    const int j = (int)(t % cols);
    if (i >= rows) return;
    out[i * ldo + j] = Zp[i * ldzp + j] > 0.f ? G[i * ldg + j] : 0.f;
}

__global__ void k_colsum_partial(int64_t rows, int32_t cols, int64_t rows_per_block, const float* __restrict__ G,
                                 int64_t ldg, float* __restrict__ part) {
    const int64_t rb = (int64_t)blockIdx.x * rows_per_block;
    const int64_t re = rb + rows_per_block < rows ? rb + rows_per_block : rows;
    for (int j = threadIdx.x; j < cols; j += blockDim.x) {
        float acc = 0.f;
        for (int64_t i = rb; i < re; ++i) acc += G[i * ldg + j];
        part[(int64_t)blockIdx.x * cols + j] = acc;
    }
}

__global__ void k_bias_add(int64_t rows, int32_t cols, float* __restrict__ Z, int64_t ldz, const float* __restrict__ bias,
                           int relu) {
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t i = t / cols;
    const int j = (int)(t % cols);
    if (i >= rows) return;
    float v = Z[i * ldz + j] + bias[j];
    Z[i * ldz + j] = (relu && !(v > 0.f)) ? 0.f : v;
}

// Y[i,:] = scale[i] * X[i,:]; 16 bytes per thread when the layout allows it.
template <int VEC>
__global__ __launch_bounds__(256) void k_scale_rows(int64_t rows, int32_t lanes, const float* __restrict__ X, int64_t ldx,
                                                    const float* __restrict__ scale, float* __restrict__ Y, int64_t ldy) {
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t i = t / lanes;
    const int j = (int)(t % lanes) * VEC;
    if (i >= rows) return;
    const float sc = scale[i];
    if constexpr (VEC == 4) {
        float4 v = *reinterpret_cast<const float4*>(X + i * ldx + j);
        v.x *= sc; v.y *= sc; v.z *= sc; v.w *= sc;
        *reinterpret_cast<float4*>(Y + i * ldy + j) = v;
    } else {
        Y[i * ldy + j] = sc * X[i * ldx + j];
    }
}

// out[i] = (float)(1 / sqrt((double)deg[i])), 0 for an empty row.
__global__ void k_inv_sqrt_deg(int64_t n, const int32_t* __restrict__ deg, float* __restrict__ out) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) out[i] = deg[i] > 0 ? (float)__ddiv_rn(1.0, __dsqrt_rn((double)deg[i])) : 0.f;
}

__global__ void k_axpy(int64_t count, float* __restrict__ W, const float* __restrict__ Y, float lr) {
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t < count) W[t] = W[t] - lr * Y[t];
}

static inline unsigned nblocks(int64_t work) { return (unsigned)((work + 255) / 256 > 0 ? (work + 255) / 256 : 1); }

int gemm_mfma_launch(int ta, int tb, int64_t M, int64_t N, int64_t K, const float* A, int64_t lda, const float* B,
                     int64_t ldb, float* C, int64_t ldc, const float* bias, int epilogue, const float* Zprev,
                     int64_t ldzprev, hipStream_t s, bool* handled, const float* row_scale, bool* scaled);

// split of the long dimension of the plain (non-MFMA) A^T B kernel
static void naive_tn_split(int64_t K, int64_t* parts_out, int64_t* kpb_out) {
    int64_t parts = (K + 1023) / 1024;
    if (parts > 1024) parts = 1024;
    if (parts < 1) parts = 1;
    const int64_t kpb = (K + parts - 1) / parts;
    parts = (K + kpb - 1) / kpb;
    if (parts < 1) parts = 1;
    *parts_out = parts;
    *kpb_out = kpb;
}

size_t gemm_mfma_tn_scratch_bytes(int64_t M, int64_t N, int64_t K);

size_t gemm_tn_scratch_bytes(int64_t M, int64_t N, int64_t K) {
    int64_t parts = 0, kpb = 0;
    naive_tn_split(K, &parts, &kpb);
    const size_t plain = (size_t)parts * M * N * sizeof(float);
    const size_t mfma = gemm_mfma_tn_scratch_bytes(M, N, K);
    return plain > mfma ? plain : mfma;              // whichever kernel the operands' alignment selects
}

static void colsum_split(int64_t rows, int64_t* parts_out, int64_t* rpb_out) {
    int64_t parts = (rows + 4095) / 4096;
    if (parts > 512) parts = 512;
    if (parts < 1) parts = 1;
    const int64_t rpb = (rows + parts - 1) / parts;
    *parts_out = (rows + rpb - 1) / rpb;
    *rpb_out = rpb;
}

size_t colsum_scratch_bytes(int64_t rows, int32_t cols) {
    int64_t parts = 0, rpb = 0;
    colsum_split(rows, &parts, &rpb);
    return (size_t)parts * cols * sizeof(float);
}

int gemm_launch(int ta, int tb, int64_t M, int64_t N, int64_t K, const float* A, int64_t lda, const float* B,
                int64_t ldb, float* C, int64_t ldc, const float* bias, int epilogue, const float* Zprev,
                int64_t ldzprev, hipStream_t s, const float* row_scale) {
    bool handled = false, scaled = false;
    GCN_TRY(gemm_mfma_launch(ta, tb, M, N, K, A, lda, B, ldb, C, ldc, bias, epilogue, Zprev, ldzprev, s, &handled,
                             row_scale, &scaled));
    // kernels without a scaling store path leave the row factors to a pass of their own
    auto finish = [&]() { return (row_scale && !scaled) ? scale_rows_launch(M, (int32_t)N, C, ldc, row_scale, C, ldc, s) : (int)GCN_OK; };
    if (handled) return finish();
    if (!ta) {
        const int64_t work = M * N;
        if ((work + 255) / 256 >= (1ll << 31)) return fail(GCN_ERR_RANGE, "gcn_gemm: output too large");
        switch (epilogue) {
            case GCN_EPI_NONE: hipLaunchKernelGGL(k_gemm_naive<GCN_EPI_NONE>, dim3(nblocks(work)), dim3(256), 0, s, tb, M, N, K, A, lda, B, ldb, C, ldc, bias, Zprev, ldzprev); break;
            case GCN_EPI_RELU: hipLaunchKernelGGL(k_gemm_naive<GCN_EPI_RELU>, dim3(nblocks(work)), dim3(256), 0, s, tb, M, N, K, A, lda, B, ldb, C, ldc, bias, Zprev, ldzprev); break;
            default: hipLaunchKernelGGL(k_gemm_naive<GCN_EPI_MASK>, dim3(nblocks(work)), dim3(256), 0, s, tb, M, N, K, A, lda, B, ldb, C, ldc, bias, Zprev, ldzprev); break;
        }
        GCN_LAUNCH_CHECK();
        return finish();
    }
    // ta: split K
    int64_t parts = 0, kpb = 0;
    naive_tn_split(K, &parts, &kpb);
    void* scratch = nullptr;
    GCN_TRY(scratch_get(&scratch, (size_t)parts * M * N * sizeof(float), s));
    hipLaunchKernelGGL(k_gemm_tn_partial, dim3((unsigned)parts), dim3(256), 0, s, M, N, K, kpb, A, lda, B, ldb, (float*)scratch);
    GCN_LAUNCH_CHECK();
    const int64_t count = M * N;
    switch (epilogue) {
        case GCN_EPI_NONE: hipLaunchKernelGGL(k_reduce_partials<GCN_EPI_NONE>, dim3(nblocks(count)), dim3(256), 0, s, count, N, (int)parts, (const float*)scratch, C, ldc, bias, Zprev, ldzprev); break;
        case GCN_EPI_RELU: hipLaunchKernelGGL(k_reduce_partials<GCN_EPI_RELU>, dim3(nblocks(count)), dim3(256), 0, s, count, N, (int)parts, (const float*)scratch, C, ldc, bias, Zprev, ldzprev); break;
        default: hipLaunchKernelGGL(k_reduce_partials<GCN_EPI_MASK>, dim3(nblocks(count)), dim3(256), 0, s, count, N, (int)parts, (const float*)scratch, C, ldc, bias, Zprev, ldzprev); break;
    }
    GCN_LAUNCH_CHECK();
    return finish();
}

int colsum_launch(int64_t rows, int32_t cols, const float* G, int64_t ldg, float* out, hipStream_t s) {
    int64_t parts = 0, rpb = 0;
    colsum_split(rows, &parts, &rpb);
    void* scratch = nullptr;
    GCN_TRY(scratch_get(&scratch, (size_t)parts * cols * sizeof(float), s));
    hipLaunchKernelGGL(k_colsum_partial, dim3((unsigned)parts), dim3(64), 0, s, rows, cols, rpb, G, ldg, (float*)scratch);
    GCN_LAUNCH_CHECK();
    hipLaunchKernelGGL(k_reduce_partials<GCN_EPI_NONE>, dim3(nblocks(cols)), dim3(256), 0, s, (int64_t)cols, (int64_t)cols,
                       (int)parts, (const float*)scratch, out, (int64_t)cols, (const float*)nullptr, (const float*)nullptr, (int64_t)0);
    GCN_LAUNCH_CHECK();
    return GCN_OK;
}

int relu_launch(int64_t rows, int32_t cols, const float* Z, int64_t ldz, float* H, int64_t ldh, hipStream_t s) {
    hipLaunchKernelGGL(k_relu, dim3(nblocks(rows * cols)), dim3(256), 0, s, rows, cols, Z, ldz, H, ldh);
    GCN_LAUNCH_CHECK();
    return GCN_OK;
}

int bias_add_launch(int64_t rows, int32_t cols, float* Z, int64_t ldz, const float* bias, int relu, hipStream_t s) {
    hipLaunchKernelGGL(k_bias_add, dim3(nblocks(rows * cols)), dim3(256), 0, s, rows, cols, Z, ldz, bias, relu);
    GCN_LAUNCH_CHECK();
    return GCN_OK;
}

int scale_rows_launch(int64_t rows, int32_t cols, const float* X, int64_t ldx, const float* scale, float* Y, int64_t ldy,
                      hipStream_t s) {
    const bool vec4 = (cols % 4 == 0) && (ldx % 4 == 0) && (ldy % 4 == 0) && (((uintptr_t)X & 15u) == 0) &&
                      (((uintptr_t)Y & 15u) == 0);
    if (vec4) {
        const int lanes = cols / 4;
        hipLaunchKernelGGL(k_scale_rows<4>, dim3(nblocks(rows * lanes)), dim3(256), 0, s, rows, lanes, X, ldx, scale, Y, ldy);
    } else {
        hipLaunchKernelGGL(k_scale_rows<1>, dim3(nblocks(rows * cols)), dim3(256), 0, s, rows, cols, X, ldx, scale, Y, ldy);
    }
    GCN_LAUNCH_CHECK();
    return GCN_OK;
}

int inv_sqrt_deg_launch(int64_t n, const int32_t* deg, float* out, hipStream_t s) {
    hipLaunchKernelGGL(k_inv_sqrt_deg, dim3(nblocks(n)), dim3(256), 0, s, n, deg, out);
    GCN_LAUNCH_CHECK();
    return GCN_OK;
}

int axpy_launch(int64_t count, float* W, const float* Y, float lr, hipStream_t s) {
    hipLaunchKernelGGL(k_axpy, dim3(nblocks(count)), dim3(256), 0, s, count, W, Y, lr);
    GCN_LAUNCH_CHECK();
    return GCN_OK;
}

}  // namespace gcn

using namespace gcn;

extern "C" {

int gcn_gemm(int ta, int tb, int64_t M, int64_t N, int64_t K, const float* A, int64_t lda, const float* B,
             int64_t ldb, float* C, int64_t ldc, const float* bias, int epilogue, const float* Zprev,
             int64_t ldzprev, void* stream) {
    if (!A || !B || !C) return fail(GCN_ERR_BADARG, "gcn_gemm: NULL matrix");
    if (M <= 0 || N <= 0 || K <= 0) return fail(GCN_ERR_BADARG, "gcn_gemm: sizes must be positive");
    if (ta && tb) return fail(GCN_ERR_BADARG, "gcn_gemm: ta and tb together are not supported");
    if (lda < (ta ? M : K) || ldb < (tb ? K : N) || ldc < N) return fail(GCN_ERR_BADARG, "gcn_gemm: leading dimension too small");
    if (epilogue < GCN_EPI_NONE || epilogue > GCN_EPI_MASK) return fail(GCN_ERR_BADARG, "gcn_gemm: unknown epilogue");
    if (epilogue == GCN_EPI_MASK && (!Zprev || ldzprev < N)) return fail(GCN_ERR_BADARG, "gcn_gemm: mask epilogue needs Zprev with ld >= N");
    return gemm_launch(ta, tb, M, N, K, A, lda, B, ldb, C, ldc, bias, epilogue, Zprev, ldzprev, (hipStream_t)stream);
}

int gcn_relu(int64_t rows, int32_t cols, const float* Z, int64_t ldz, float* H, int64_t ldh, void* stream) {
    if (!Z || !H || rows <= 0 || cols <= 0 || ldz < cols || ldh < cols) return fail(GCN_ERR_BADARG, "gcn_relu: bad argument");
    return relu_launch(rows, cols, Z, ldz, H, ldh, (hipStream_t)stream);
}

int gcn_relu_mask(int64_t rows, int32_t cols, const float* G, int64_t ldg, const float* Zprev, int64_t ldzprev,
                  float* out, int64_t ldo, void* stream) {
    if (!G || !Zprev || !out || rows <= 0 || cols <= 0 || ldg < cols || ldzprev < cols || ldo < cols)
        return fail(GCN_ERR_BADARG, "gcn_relu_mask: bad argument");
    hipLaunchKernelGGL(k_relu_mask, dim3(nblocks(rows * cols)), dim3(256), 0, (hipStream_t)stream, rows, cols, G, ldg,
                       Zprev, ldzprev, out, ldo);
    GCN_LAUNCH_CHECK();
    return GCN_OK;
}

int gcn_scale_rows(int64_t rows, int32_t cols, const float* X, int64_t ldx, const float* scale, float* Y, int64_t ldy,
                   void* stream) {
    if (!X || !scale || !Y || rows <= 0 || cols <= 0 || ldx < cols || ldy < cols)
        return fail(GCN_ERR_BADARG, "gcn_scale_rows: bad argument");
    return scale_rows_launch(rows, cols, X, ldx, scale, Y, ldy, (hipStream_t)stream);
}

int gcn_csr_inv_sqrt_degrees(const gcn_csr* a, float* out, void* stream) {
    if (!a || !out) return fail(GCN_ERR_BADARG, "gcn_csr_inv_sqrt_degrees: NULL argument");
    if (a->n != a->ncols) return fail(GCN_ERR_BADARG, "gcn_csr_inv_sqrt_degrees: the matrix must be square");
    return inv_sqrt_deg_launch(a->n, a->deg, out, (hipStream_t)stream);
}

}  // extern "C"
