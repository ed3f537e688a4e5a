// One GCN layer forward / backward and the full-batch epoch, composed from the SpMM, the dense
// products and the loss kernel in the order of the paper's "Forward Propagation" and
// "Backpropagation Derivations" (Equations 1-3).  A G is computed once per layer and used for both
// the weight gradient and the propagated gradient, as the paper's 1D analysis notes.
#include <vector>

#include "common.h"

namespace gcn {

static int resolve_order(int order, int32_t f_in, int32_t f_out) {
    if (order == GCN_ORDER_GEMM_FIRST || order == GCN_ORDER_SPMM_FIRST) return order;
    // The SpMM costs in proportion to its width: run it at min(f_in, f_out).
    return f_out <= f_in ? GCN_ORDER_GEMM_FIRST : GCN_ORDER_SPMM_FIRST;
}

// Z = epilogue(op(A) X) with the handle's normalised matrix.  `xs` (n x f, ld f) receives the
// pre-scaled operand of the value-free form; it may be X itself when X is a temporary with ld f,
// or NULL to force the valued product.  `prescaled`: the producer of X already applied the row factors
// (only passed when pre_scale() said so for this operand).
static int norm_spmm(gcn_csr* a, Matrix& m, int32_t f, const float* X, int64_t ldx, float* xs, float* Z, int64_t ldz,
                     int epilogue, const float* Zprev, int64_t ldzprev, hipStream_t s, bool prescaled = false) {
    PhaseTimer pt(s, GCN_PHASE_SPMM);
    if (!xs || !use_value_free(a)) return spmm_launch(a, m, f, X, ldx, Z, ldz, epilogue, Zprev, ldzprev, s);
    if (!prescaled) GCN_TRY(scale_rows_launch(a->n, f, X, ldx, a->inv_sqrt_deg, xs, f, s));
    SpmmOpt o;
    o.pattern = true;
    o.row_scale = a->inv_sqrt_deg;
    return spmm_launch(a, m, f, prescaled ? X : xs, prescaled ? ldx : f, Z, ldz, epilogue, Zprev, ldzprev, s, o);
}

// The row factors that the kernel producing a temporary operand of norm_spmm should apply itself (the value-free
// form pre-scales its operand; when the operand is a temporary the producer's store path does it for free), or NULL.
static const float* pre_scale(const gcn_csr* a, bool operand_is_temporary) {
    return (operand_is_temporary && use_value_free(a)) ? a->inv_sqrt_deg : nullptr;
}

static int timed_gemm(int ta, int tb, int64_t M, int64_t N, int64_t K, const float* A, int64_t lda, const float* B,
                      int64_t ldb, float* C, int64_t ldc, const float* bias, int epilogue, const float* Zprev,
                      int64_t ldzprev, hipStream_t s, const float* row_scale = nullptr) {
    PhaseTimer pt(s, GCN_PHASE_GEMM);
    return gemm_launch(ta, tb, M, N, K, A, lda, B, ldb, C, ldc, bias, epilogue, Zprev, ldzprev, s, row_scale);
}

// `xs`: scratch for the value-free product (n x the SpMM width) or NULL; `t_scratch` says that T is
// a pure temporary which may be overwritten by its scaled copy.
static int layer_forward_impl(gcn_csr* a, int32_t f_in, int32_t f_out, const float* Hin, int64_t ldh, const float* W,
                              const float* bias, float* Z, float* Hout, float* T, int order, int act, hipStream_t s,
                              float* xs = nullptr, bool t_scratch = false, bool t_given = false) {
    const int64_t n = a->n;
    order = resolve_order(order, f_in, f_out);
    // When the caller passes Hout == Z only the activated matrix is wanted and ReLU is fused into
    // the kernel that produces Z; otherwise Z is kept (backward needs it) and H is a second pass.
    const bool in_place = (act == GCN_ACT_RELU) && Hout == Z;
    if (order == GCN_ORDER_GEMM_FIRST) {
        const float* ps = pre_scale(a, t_scratch);
        GCN_TRY(timed_gemm(0, 0, n, f_out, f_in, Hin, ldh, W, f_out, T, f_out, nullptr, GCN_EPI_NONE, nullptr, 0, s, ps));
        GCN_TRY(norm_spmm(a, a->At, f_out, T, f_out, t_scratch ? T : xs, Z, f_out,
                          (in_place && !bias) ? GCN_EPI_RELU : GCN_EPI_NONE, nullptr, 0, s, ps != nullptr));
        if (bias) {
            PhaseTimer pt(s, GCN_PHASE_OTHER);
            GCN_TRY(bias_add_launch(n, f_out, Z, f_out, bias, in_place ? 1 : 0, s));
        }
    } else {
        // t_given: T already holds A^T Hin (aggregated once by the caller; Hin itself is not read)
        if (!t_given) GCN_TRY(norm_spmm(a, a->At, f_in, Hin, ldh, xs, T, f_in, GCN_EPI_NONE, nullptr, 0, s));
        GCN_TRY(timed_gemm(0, 0, n, f_out, f_in, T, f_in, W, f_out, Z, f_out, bias,
                            in_place ? GCN_EPI_RELU : GCN_EPI_NONE, nullptr, 0, s));
    }
    PhaseTimer pt(s, GCN_PHASE_OTHER);
    if (act == GCN_ACT_RELU && !in_place) GCN_TRY(relu_launch(n, f_out, Z, f_out, Hout, f_out, s));
    if (act == GCN_ACT_NONE && Hout && Hout != Z)
        GCN_HIP_TRY(hipMemcpyAsync(Hout, Z, (size_t)n * f_out * sizeof(float), hipMemcpyDeviceToDevice, s));
    return GCN_OK;
}

static int layer_backward_impl(gcn_csr* a, int32_t f_in, int32_t f_out, const float* Hin, int64_t ldh,
                               const float* Zprev, const float* W, const float* G, const float* T, float* S, float* Y,
                               float* dbias, float* Gprev, int order, hipStream_t s, float* xs = nullptr,
                               bool s_scratch = false) {
    const int64_t n = a->n;
    order = resolve_order(order, f_in, f_out);
    if (dbias) {
        PhaseTimer pt(s, GCN_PHASE_OTHER);
        GCN_TRY(colsum_launch(n, f_out, G, f_out, dbias, s));
    }
    if (order == GCN_ORDER_GEMM_FIRST) {
        // S = A G;  Y = Hin^T S;  Gprev = (S W^T) (.) sigma'(Zprev)
        GCN_TRY(norm_spmm(a, a->A, f_out, G, f_out, xs, S, f_out, GCN_EPI_NONE, nullptr, 0, s));
        GCN_TRY(timed_gemm(1, 0, f_in, f_out, n, Hin, ldh, S, f_out, Y, f_out, nullptr, GCN_EPI_NONE, nullptr, 0, s));
        if (Gprev)
            GCN_TRY(timed_gemm(0, 1, n, f_in, f_out, S, f_out, W, f_out, Gprev, f_in, nullptr, GCN_EPI_MASK, Zprev, f_in, s));
    } else {
        // Y = (A^T Hin)^T G = T^T G;  Gprev = (A (G W^T)) (.) sigma'(Zprev): the same matrices, with the
        // SpMM at width f_in.
        GCN_TRY(timed_gemm(1, 0, f_in, f_out, n, T, f_in, G, f_out, Y, f_out, nullptr, GCN_EPI_NONE, nullptr, 0, s));
        if (Gprev) {
            const float* ps = pre_scale(a, s_scratch);
            GCN_TRY(timed_gemm(0, 1, n, f_in, f_out, G, f_out, W, f_out, S, f_in, nullptr, GCN_EPI_NONE, nullptr, 0, s, ps));
            GCN_TRY(norm_spmm(a, a->A, f_in, S, f_in, s_scratch ? S : xs, Gprev, f_in, GCN_EPI_MASK, Zprev, f_in, s,
                              ps != nullptr));
        }
    }
    return GCN_OK;
}

// ---- epoch workspace layout -------------------------------------------------------------------
struct EpochLayout {
    std::vector<size_t> Z, H, T, G;   // byte offsets per layer index 0..L_w-1 (layer l = index + 1)
    size_t S = 0, XS = 0, total = 0;  // XS: pre-scaled SpMM operand of the value-free product
    size_t scratch = 0, scratch_bytes = 0;   // split-K partials of the weight gradients, loss partials
    std::vector<int> order;
};

static size_t round256(size_t b) { return (b + 255) & ~(size_t)255; }

static EpochLayout epoch_layout(int64_t n, int32_t L, const int32_t* dims, int order) {
    EpochLayout lay;
    size_t off = 0, smax = 0;
    auto take = [&](size_t elems) { size_t o = off; off += round256(elems * sizeof(float)); return o; };
    for (int l = 0; l < L; ++l) {
        const int32_t fi = dims[l], fo = dims[l + 1];
        const int ord = resolve_order(order, fi, fo);
        lay.order.push_back(ord);
        // Hidden layers keep only H = ReLU(Z): the ReLU is fused into the kernel that produces Z, and
        // sigma'(Z) = [Z > 0] = [H > 0], so backward never needs Z itself.  The last layer keeps Z.
        lay.Z.push_back(take((size_t)n * fo));
        lay.H.push_back(lay.Z.back());
        lay.T.push_back(take((size_t)n * (ord == GCN_ORDER_GEMM_FIRST ? fo : fi)));
        lay.G.push_back(take((size_t)n * fo));
        const size_t sneed = (size_t)n * (ord == GCN_ORDER_GEMM_FIRST ? fo : fi);
        if (sneed > smax) smax = sneed;
    }
    lay.S = take(smax);
    lay.XS = take(smax);
    // the partial sums of the reductions over n live in the caller's workspace too, so that an epoch never
    // touches library-owned scratch (which is per stream and would have to exist before a graph capture)
    size_t sc = loss_scratch_bytes();
    for (int l = 0; l < L; ++l) {
        const size_t need = gemm_tn_scratch_bytes(dims[l], dims[l + 1], n);
        if (need > sc) sc = need;
    }
    // the fused last layer (SpMM-first order; a single layer can be put into that order by the pre-aggregated epoch)
    if ((lay.order[L - 1] == GCN_ORDER_SPMM_FIRST || L == 1) && fused_last_supported(dims[L - 1], dims[L])) {
        const size_t need = fused_last_scratch_bytes(n, dims[L]);
        if (need > sc) sc = need;
    }
    lay.scratch_bytes = sc;
    lay.scratch = take((sc + sizeof(float) - 1) / sizeof(float));
    lay.total = off;
    return lay;
}

static int check_dims(int64_t n, int32_t L, const int32_t* dims) {
    if (n <= 0 || L <= 0 || L > 64 || !dims) return fail(GCN_ERR_BADARG, "epoch: need n > 0, 1 <= L_w <= 64, dims non-NULL");
    for (int l = 0; l <= L; ++l)
        if (dims[l] <= 0 || dims[l] > 65536) return fail(GCN_ERR_BADARG, "epoch: dims[%d] = %d out of range", l, dims[l]);
    return GCN_OK;
}

}  // namespace gcn

using namespace gcn;

extern "C" {

int gcn_layer_forward(gcn_csr* a, int32_t f_in, int32_t f_out, const float* Hin, int64_t ldh, const float* W,
                      const float* bias, float* Z, float* Hout, float* T, int order, int act, void* stream) {
    if (!a || !Hin || !W || !Z || !T) return fail(GCN_ERR_BADARG, "gcn_layer_forward: NULL argument");
    if (f_in <= 0 || f_out <= 0 || ldh < f_in) return fail(GCN_ERR_BADARG, "gcn_layer_forward: bad sizes");
    if (order < GCN_ORDER_AUTO || order > GCN_ORDER_SPMM_FIRST) return fail(GCN_ERR_BADARG, "gcn_layer_forward: unknown order");
    if (act != GCN_ACT_NONE && act != GCN_ACT_RELU) return fail(GCN_ERR_BADARG, "gcn_layer_forward: unknown activation");
    if (act == GCN_ACT_RELU && !Hout) return fail(GCN_ERR_BADARG, "gcn_layer_forward: ReLU needs Hout");
    if (!a->has_t) return fail(GCN_ERR_NOTRANSPOSE, "gcn_layer_forward needs GCN_BUILD_TRANSPOSE");
    if (a->n != a->ncols) return fail(GCN_ERR_BADARG, "gcn_layer_forward needs a square matrix");
    return layer_forward_impl(a, f_in, f_out, Hin, ldh, W, bias, Z, Hout, T, order, act, (hipStream_t)stream);
}

int gcn_layer_backward(gcn_csr* a, int32_t f_in, int32_t f_out, const float* Hin, int64_t ldh, const float* Zprev,
                       const float* W, const float* G, const float* T, float* S, float* Y, float* dbias,
                       float* Gprev, int order, void* stream) {
    if (!a || !W || !G || !S || !Y) return fail(GCN_ERR_BADARG, "gcn_layer_backward: NULL argument");
    if (f_in <= 0 || f_out <= 0) return fail(GCN_ERR_BADARG, "gcn_layer_backward: bad sizes");
    if (order < GCN_ORDER_AUTO || order > GCN_ORDER_SPMM_FIRST) return fail(GCN_ERR_BADARG, "gcn_layer_backward: unknown order");
    if (a->n != a->ncols) return fail(GCN_ERR_BADARG, "gcn_layer_backward needs a square matrix");
    const int ord = resolve_order(order, f_in, f_out);
    if (ord == GCN_ORDER_GEMM_FIRST && (!Hin || ldh < f_in)) return fail(GCN_ERR_BADARG, "gcn_layer_backward: Hin needed");
    if (ord == GCN_ORDER_SPMM_FIRST && !T) return fail(GCN_ERR_BADARG, "gcn_layer_backward: SpMM-first order needs the forward T");
    if (Gprev && !Zprev) return fail(GCN_ERR_BADARG, "gcn_layer_backward: Gprev needs Zprev");
    return layer_backward_impl(a, f_in, f_out, Hin, ldh, Zprev, W, G, T, S, Y, dbias, Gprev, order, (hipStream_t)stream);
}

size_t gcn_epoch_workspace_bytes(int64_t n, int32_t L_w, const int32_t* dims, int order) {
    if (check_dims(n, L_w, dims) != GCN_OK) return 0;
    return epoch_layout(n, L_w, dims, order).total;
}

int gcn_epoch_view(int64_t n, int32_t L_w, const int32_t* dims, int order, void* workspace, int32_t l, float** Z,
                   float** G) {
    GCN_TRY(check_dims(n, L_w, dims));
    if (!workspace || l < 1 || l > L_w) return fail(GCN_ERR_BADARG, "gcn_epoch_view: bad layer or workspace");
    EpochLayout lay = epoch_layout(n, L_w, dims, order);
    if (Z) *Z = (float*)((char*)workspace + lay.Z[l - 1]);
    if (G) *G = (float*)((char*)workspace + lay.G[l - 1]);
    return GCN_OK;
}

int gcn_epoch(gcn_csr* a, int32_t L_w, const int32_t* dims, const float* H0, const int32_t* labels, float* const* W,
              float* const* Y, float lr, float* loss, void* workspace, size_t workspace_bytes, int order, void* stream) {
    if (!a) return fail(GCN_ERR_BADARG, "gcn_epoch: NULL argument");
    return gcn_epoch_masked(a, L_w, dims, H0, labels, a->n, W, Y, lr, loss, workspace, workspace_bytes, order, stream);
}

static int epoch_impl(gcn_csr* a, int32_t L_w, const int32_t* dims, const float* H0, const float* P0,
                      const int32_t* labels, int64_t n_labelled, float* const* W, float* const* Y, float lr, float* loss,
                      void* workspace, size_t workspace_bytes, int order, void* stream) {
    if (!a || !(H0 || P0) || !labels || !W || !Y || !loss || !workspace) return fail(GCN_ERR_BADARG, "gcn_epoch: NULL argument");
    if (n_labelled <= 0 || n_labelled > a->n) return fail(GCN_ERR_BADARG, "gcn_epoch: n_labelled must be in [1, n]");
    GCN_TRY(check_dims(a->n, L_w, dims));
    if (order < GCN_ORDER_AUTO || order > GCN_ORDER_SPMM_FIRST) return fail(GCN_ERR_BADARG, "gcn_epoch: unknown order");
    if (!a->has_t) return fail(GCN_ERR_NOTRANSPOSE, "gcn_epoch needs GCN_BUILD_TRANSPOSE");
    if (a->n != a->ncols) return fail(GCN_ERR_BADARG, "gcn_epoch needs a square matrix");
    for (int l = 0; l < L_w; ++l)
        if (!W[l] || !Y[l]) return fail(GCN_ERR_BADARG, "gcn_epoch: NULL weight or gradient pointer at layer %d", l + 1);
    if (((uintptr_t)workspace & 255u) != 0) return fail(GCN_ERR_BADARG, "gcn_epoch: workspace must be 256-byte aligned");
    const int64_t n = a->n;
    EpochLayout lay = epoch_layout(n, L_w, dims, order);
    if (workspace_bytes < lay.total)
        return fail(GCN_ERR_WORKSPACE, "gcn_epoch: workspace has %zu bytes, %zu needed", workspace_bytes, lay.total);
    hipStream_t s = (hipStream_t)stream;
    char* ws = (char*)workspace;
    auto at = [&](size_t off) { return (float*)(ws + off); };
    ScratchScope scratch_scope(ws + lay.scratch, lay.scratch_bytes);
    // With P0 = A^T H0 given, layer 1 runs in SpMM-first order on it: Z^1 = P0 W^1, Y^1 = P0^T G^1, and
    // neither direction needs a sparse product.
    auto layer_order = [&](int l) { return (l == 0 && P0) ? (int)GCN_ORDER_SPMM_FIRST : lay.order[l]; };
    auto layer_T = [&](int l) { return (l == 0 && P0) ? const_cast<float*>(P0) : at(lay.T[l]); };

    // Last layer in SpMM-first order at hidden width 16: logits, loss, Equation 1, the weight gradient and
    // the operand of Equation 2's sparse product come from one kernel per 16-row strip of T = A^T H^{L-1}.
    const int last = L_w - 1;
    const int fuse_mode = cfg_of(a).fused_last;
    const bool fuse = fuse_mode != 0 && layer_order(last) == GCN_ORDER_SPMM_FIRST &&
                      fused_last_supported(dims[last], dims[L_w]);
    const float* Hin = H0;
    for (int l = 0; l < L_w; ++l) {
        const bool is_last = (l == last);
        if (is_last && fuse) {
            if (!(l == 0 && P0))
                GCN_TRY(norm_spmm(a, a->At, dims[l], Hin, dims[l], at(lay.XS), layer_T(l), dims[l], GCN_EPI_NONE, nullptr, 0, s));
            break;
        }
        GCN_TRY(layer_forward_impl(a, dims[l], dims[l + 1], Hin, dims[l], W[l], nullptr, at(lay.Z[l]),
                                   is_last ? nullptr : at(lay.Z[l]), layer_T(l), layer_order(l),
                                   is_last ? GCN_ACT_NONE : GCN_ACT_RELU, s, at(lay.XS), true, l == 0 && P0));
        Hin = at(lay.H[l]);
    }
    if (fuse) {
        PhaseTimer pt(s, GCN_PHASE_GEMM);
        const bool keep = fuse_mode == 2;
        GCN_TRY(fused_last_launch(n, dims[L_w], layer_T(last), W[last], labels, n_labelled, loss, Y[last],
                                  last > 0 ? at(lay.S) : nullptr, pre_scale(a, true), keep ? at(lay.Z[last]) : nullptr,
                                  keep ? at(lay.G[last]) : nullptr, ws + lay.scratch, s));
    } else {
        PhaseTimer pt(s, GCN_PHASE_OTHER);
        GCN_TRY(gcn_softmax_nll_masked(n, dims[L_w], at(lay.Z[L_w - 1]), dims[L_w], labels, n_labelled, loss,
                                       at(lay.G[L_w - 1]), dims[L_w], stream));
    }
    for (int l = L_w - 1; l >= 0; --l) {
        if (l == last && fuse) {
            // Y^L and S = G^L (W^L)^T are done; what is left of Equation 2 is the sparse product
            if (l > 0)
                GCN_TRY(norm_spmm(a, a->A, dims[l], at(lay.S), dims[l], at(lay.S), at(lay.G[l - 1]), dims[l], GCN_EPI_MASK,
                                  at(lay.Z[l - 1]), dims[l], s, pre_scale(a, true) != nullptr));
            continue;
        }
        const float* Hl = l > 0 ? at(lay.H[l - 1]) : H0;
        GCN_TRY(layer_backward_impl(a, dims[l], dims[l + 1], Hl, dims[l], l > 0 ? at(lay.Z[l - 1]) : nullptr, W[l],
                                    at(lay.G[l]), layer_T(l), at(lay.S), Y[l], nullptr, l > 0 ? at(lay.G[l - 1]) : nullptr,
                                    layer_order(l), s, at(lay.XS), true));
    }
    PhaseTimer pt(s, GCN_PHASE_OTHER);
    if (lr != 0.f)
        for (int l = 0; l < L_w; ++l) GCN_TRY(axpy_launch((int64_t)dims[l] * dims[l + 1], W[l], Y[l], lr, s));
    return GCN_OK;
}

int gcn_epoch_prepare(gcn_csr* a, int32_t L_w, const int32_t* dims, int order, void* stream) {
    if (!a) return fail(GCN_ERR_BADARG, "gcn_epoch_prepare: NULL matrix");
    GCN_TRY(check_dims(a->n, L_w, dims));
    if (order < GCN_ORDER_AUTO || order > GCN_ORDER_SPMM_FIRST) return fail(GCN_ERR_BADARG, "gcn_epoch_prepare: unknown order");
    if (!a->has_t) return fail(GCN_ERR_NOTRANSPOSE, "gcn_epoch_prepare needs GCN_BUILD_TRANSPOSE");
    if (a->n != a->ncols) return fail(GCN_ERR_BADARG, "gcn_epoch_prepare needs a square matrix");
    hipStream_t s = (hipStream_t)stream;
    for (int l = 0; l < L_w; ++l) {
        const int ord = resolve_order(order, dims[l], dims[l + 1]);
        const int32_t fw = ord == GCN_ORDER_GEMM_FIRST ? dims[l + 1] : dims[l];     // width of this layer's sparse products
        GCN_TRY(spmm_prepare(a, a->At, fw, s));                                      // forward: A^T
        if (ord == GCN_ORDER_GEMM_FIRST || l > 0) GCN_TRY(spmm_prepare(a, a->A, fw, s));   // backward: A
    }
    GCN_HIP_TRY(hipStreamSynchronize(s));
    return GCN_OK;
}

int gcn_epoch_masked(gcn_csr* a, int32_t L_w, const int32_t* dims, const float* H0, const int32_t* labels,
                     int64_t n_labelled, float* const* W, float* const* Y, float lr, float* loss, void* workspace,
                     size_t workspace_bytes, int order, void* stream) {
    if (!H0) return fail(GCN_ERR_BADARG, "gcn_epoch: NULL argument");
    return epoch_impl(a, L_w, dims, H0, nullptr, labels, n_labelled, W, Y, lr, loss, workspace, workspace_bytes, order,
                      stream);
}

int gcn_epoch_preaggregated(gcn_csr* a, int32_t L_w, const int32_t* dims, const float* P0, const int32_t* labels,
                            int64_t n_labelled, float* const* W, float* const* Y, float lr, float* loss,
                            void* workspace, size_t workspace_bytes, int order, void* stream) {
    if (!P0) return fail(GCN_ERR_BADARG, "gcn_epoch_preaggregated: NULL argument");
    return epoch_impl(a, L_w, dims, nullptr, P0, labels, n_labelled, W, Y, lr, loss, workspace, workspace_bytes, order,
                      stream);
}

}  // extern "C"
