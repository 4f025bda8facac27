// CPU oracle for fused linear cross-entropy (FLCE) forward + backward.
//
// TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the
// HIP path is checked against; nothing on the product path may call it, and it
// shares no code with the HIP kernels.
//
// What it computes (paper section 3.2, paragraphs "CrossEntropy (CE)" and
// "FusedLinearCrossEntropy (FLCE)"), all arithmetic in fp64:
//   logits      z_i  = W h_i                       (Eq. FLCE-backward, line 1;
//                                                    W stored [V x H] row-major)
//   probabilities y_i = softmax(z_i)               (Eq. CE-forward)
//   loss        L    = -(1/N) sum_{valid i} log y_i[t_i]
//                                                   (CE loss, mean over the N
//                                                    rows whose target is not
//                                                    ignore_index)
//   dlogits     g_i  = (y_i - onehot(t_i)) / N      (Eq. CE-backward), 0 for
//                                                    ignored rows
//   dX_i = W^T g_i,   dW = sum_i g_i h_i^T          (Eq. FLCE-backward, lines
//                                                    2-3 and the sum over rows)
// Chunking only reorders the sum over rows, so the oracle is the unfused
// definition.  Rows are visited in blocks solely to bound the RAM held by the
// logits; every logit is one plain dot product.  The dot products carry
// `omp simd reduction`, so the compiler may keep one partial sum per vector lane
// and add the lanes at the end (a different association of the same fp64 sum, a
// few 1e-16 relative); all other sums run in index order.  N = 0 gives loss = 0
// and zero gradients (a reading: the paper does not cover it).  "Safe log": log is only ever taken of sum exp(z - max) >= 1.
//
// Optional row / vocabulary selections return dX only for the listed rows and
// dW only for the listed vocabulary ids; the arithmetic per returned element is
// the same code as the full result (selection = all indices).
#include <cmath>
#include <cstdint>
#include <cstdlib>
#include <vector>
#include <algorithm>
#include <omp.h>

namespace {

constexpr int64_t ROW_BLOCK = 64;

// Row-wise cross entropy on a block of logits, in place (paper: CE paragraph).
// z: [rows x V] logits in, dlogits out.  Returns the sum of the per-row losses
// of valid rows; lse (optional) receives log-sum-exp per row.
double ce_rows_inplace(double* z, const int64_t* t, int64_t rows, int64_t V,
                       int64_t ignore_index, double inv_n, double* lse_out,
                       std::vector<double>& row_loss) {
    row_loss.assign(rows, 0.0);
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r) {
        double* zr = z + r * V;
        double m = zr[0];
        for (int64_t v = 1; v < V; ++v) m = std::max(m, zr[v]);
        double s = 0.0;
        for (int64_t v = 0; v < V; ++v) s += std::exp(zr[v] - m);
        const double lse = m + std::log(s);
        if (lse_out) lse_out[r] = lse;
        if (t[r] == ignore_index) {
            for (int64_t v = 0; v < V; ++v) zr[v] = 0.0;
            continue;
        }
        row_loss[r] = lse - zr[t[r]];
        for (int64_t v = 0; v < V; ++v) zr[v] = std::exp(zr[v] - lse) * inv_n;
        zr[t[r]] -= inv_n;
    }
    double sum = 0.0;
    for (int64_t r = 0; r < rows; ++r) sum += row_loss[r];
    return sum;
}

template <typename T>
int flce_impl(const T* X, const T* W, const int64_t* targets, int64_t BT, int64_t H, int64_t V,
              int64_t ignore_index, const int64_t* rows_sel, int64_t n_rows_sel,
              const int64_t* vocab_sel, int64_t n_vocab_sel, double* loss, double* lse,
              double* dX, double* dW, double* G_out) {
    if (!X || !W || !targets || !loss || BT < 0 || H <= 0 || V <= 0) return 1;
    for (int64_t i = 0; i < BT; ++i)
        if (targets[i] != ignore_index && (targets[i] < 0 || targets[i] >= V)) return 2;

    int64_t n_valid = 0;
    for (int64_t i = 0; i < BT; ++i) n_valid += (targets[i] != ignore_index);
    const double inv_n = n_valid > 0 ? 1.0 / (double)n_valid : 0.0;

    const int64_t n_dx = rows_sel ? n_rows_sel : BT;
    const int64_t n_dw = vocab_sel ? n_vocab_sel : V;
    if (dX) std::fill(dX, dX + n_dx * H, 0.0);
    if (dW) std::fill(dW, dW + n_dw * H, 0.0);

    std::vector<double> z((size_t)std::min<int64_t>(ROW_BLOCK, std::max<int64_t>(BT, 1)) * V);
    std::vector<double> row_loss;
    double loss_sum = 0.0;

    for (int64_t i0 = 0; i0 < BT; i0 += ROW_BLOCK) {
        const int64_t rows = std::min(ROW_BLOCK, BT - i0);

        // logits of this row block: z[r][v] = <h_{i0+r}, W_v>.  Four rows share one
        // sweep over W_v; each logit is still its own dot product in k order.
#pragma omp parallel for schedule(static)
        for (int64_t v = 0; v < V; ++v) {
            const T* wv = W + v * H;
            int64_t r = 0;
            for (; r + 4 <= rows; r += 4) {
                const T* x0 = X + (i0 + r) * H;
                const T *x1 = x0 + H, *x2 = x0 + 2 * H, *x3 = x0 + 3 * H;
                double a0 = 0.0, a1 = 0.0, a2 = 0.0, a3 = 0.0;
#pragma omp simd reduction(+ : a0, a1, a2, a3)
                for (int64_t k = 0; k < H; ++k) {
                    const double w = (double)wv[k];
                    a0 += (double)x0[k] * w;
                    a1 += (double)x1[k] * w;
                    a2 += (double)x2[k] * w;
                    a3 += (double)x3[k] * w;
                }
                z[(r + 0) * V + v] = a0;
                z[(r + 1) * V + v] = a1;
                z[(r + 2) * V + v] = a2;
                z[(r + 3) * V + v] = a3;
            }
            for (; r < rows; ++r) {
                const T* xr = X + (i0 + r) * H;
                double acc = 0.0;
#pragma omp simd reduction(+ : acc)
                for (int64_t k = 0; k < H; ++k) acc += (double)xr[k] * (double)wv[k];
                z[r * V + v] = acc;
            }
        }

        loss_sum += ce_rows_inplace(z.data(), targets + i0, rows, V, ignore_index, inv_n,
                                    lse ? lse + i0 : nullptr, row_loss);
        if (G_out) std::copy(z.begin(), z.begin() + rows * V, G_out + i0 * V);

        // dX_i = sum_v g_i[v] W_v   for the requested rows of this block
        if (dX) {
            std::vector<std::pair<int64_t, int64_t>> todo;  // (row in block, row in dX)
            if (rows_sel) {
                for (int64_t j = 0; j < n_rows_sel; ++j)
                    if (rows_sel[j] >= i0 && rows_sel[j] < i0 + rows)
                        todo.emplace_back(rows_sel[j] - i0, j);
            } else {
                for (int64_t r = 0; r < rows; ++r) todo.emplace_back(r, i0 + r);
            }
            constexpr int64_t STRIP = 64;
            const int64_t n_strips = (H + STRIP - 1) / STRIP;
            if (!todo.empty()) {
#pragma omp parallel for schedule(static)
                for (int64_t s = 0; s < n_strips; ++s) {
                    const int64_t h0 = s * STRIP, h1 = std::min(H, h0 + STRIP);
                    for (int64_t v = 0; v < V; ++v) {
                        const T* wv = W + v * H;
                        for (const auto& rj : todo) {
                            const double g = z[rj.first * V + v];
                            double* out = dX + rj.second * H;
                            for (int64_t h = h0; h < h1; ++h) out[h] += g * (double)wv[h];
                        }
                    }
                }
            }
        }

        // dW_v += sum_{i in block} g_i[v] h_i   for the requested vocabulary ids
        if (dW) {
#pragma omp parallel for schedule(static)
            for (int64_t j = 0; j < n_dw; ++j) {
                const int64_t v = vocab_sel ? vocab_sel[j] : j;
                double* out = dW + j * H;
                for (int64_t r = 0; r < rows; ++r) {
                    const double g = z[r * V + v];
                    const T* xr = X + (i0 + r) * H;
                    for (int64_t h = 0; h < H; ++h) out[h] += g * (double)xr[h];
                }
            }
        }
    }
    *loss = n_valid > 0 ? loss_sum * inv_n : 0.0;
    return 0;
}

}  // namespace

extern "C" {

// Inputs already widened to fp64.
int flce_oracle_f64(const double* X, const double* W, const int64_t* targets, int64_t BT,
                    int64_t H, int64_t V, int64_t ignore_index, const int64_t* rows_sel,
                    int64_t n_rows_sel, const int64_t* vocab_sel, int64_t n_vocab_sel,
                    double* loss, double* lse, double* dX, double* dW, double* G) {
    return flce_impl(X, W, targets, BT, H, V, ignore_index, rows_sel, n_rows_sel, vocab_sel,
                     n_vocab_sel, loss, lse, dX, dW, G);
}

// Inputs held as fp32 (bf16 and fp32 values widen to fp64 exactly, element by
// element, inside the dot products); halves the memory the big shapes need.
int flce_oracle_f32in(const float* X, const float* W, const int64_t* targets, int64_t BT,
                      int64_t H, int64_t V, int64_t ignore_index, const int64_t* rows_sel,
                      int64_t n_rows_sel, const int64_t* vocab_sel, int64_t n_vocab_sel,
                      double* loss, double* lse, double* dX, double* dW, double* G) {
    return flce_impl(X, W, targets, BT, H, V, ignore_index, rows_sel, n_rows_sel, vocab_sel,
                     n_vocab_sel, loss, lse, dX, dW, G);
}

// Stand-alone cross entropy on given logits (paper: CE paragraph): loss (mean
// over valid rows) and dlogits written over z.
int ce_oracle_f64(double* z, const int64_t* targets, int64_t BT, int64_t V,
                  int64_t ignore_index, double* loss, double* lse) {
    if (!z || !targets || !loss || BT < 0 || V <= 0) return 1;
    int64_t n_valid = 0;
    for (int64_t i = 0; i < BT; ++i) {
        if (targets[i] != ignore_index && (targets[i] < 0 || targets[i] >= V)) return 2;
        n_valid += (targets[i] != ignore_index);
    }
    const double inv_n = n_valid > 0 ? 1.0 / (double)n_valid : 0.0;
    std::vector<double> row_loss;
    const double s = ce_rows_inplace(z, targets, BT, V, ignore_index, inv_n, lse, row_loss);
    *loss = n_valid > 0 ? s * inv_n : 0.0;
    return 0;
}

int flce_oracle_threads(void) { return omp_get_max_threads(); }

}  // extern "C"
