// CPU oracle of the MoE-layer hot path.  TEST INFRASTRUCTURE ONLY: nothing on
// the product path may call, link or import this file; it shares no code with
// the HIP kernels.
//
// What it computes (paper, Preliminary section): y = sum_i g(x)_i * f_i(x) with
// the gate g(x) = Softmax(TopK(x * W_g)); the experts f_i are SwiGLU MLPs
// without biases (overlap analysis of section 3.1: three H x H' matrices,
// 6*H*H' FLOPs per routed token); training is dropless (experimental setup), so
// an expert takes however many tokens the gate gives it, possibly none.
//
// Two forms that must agree:
//   * the dense definition (oracle_dense_layer_fwd): every token visits every
//     expert, weighted by a gate vector that is zero off the top-k;
//   * the staged form: gate -> stable permutation by expert -> per-expert FFN
//     -> weighted combine, and the exact derivatives of those stages with the
//     selected expert ids held constant.
//
// Everything is written as plain loops over the definitions.  The only
// concurrency is an OpenMP "parallel for" over independent output rows; the
// order of every floating-point sum is the plain loop order.  `real` is float or
// double (both instantiations are exported, suffix _f32 / _f64); gate logits are
// always accumulated in double so that the oracle is the accurate side of any
// near-tie between two experts.
//
// Readings where the paper is silent (also listed in the design notes):
//   slot order of TopK = descending logit; equal logits -> lower expert index;
//   rows of one expert keep their (token, slot) order (stable counting sort);
//   SwiGLU: H = silu(X*W1) (.) (X*W3), Y = H*W2, silu(a) = a / (1 + exp(-a));
//   no gradient flows through the selection itself.
//
// Pins: tests/test_oracle_*.py (closed forms, numpy/scipy special cases, brute
// force, finite differences in the fp64 instantiation, adjoint identities).

#include <cmath>
#include <cstdint>
#include <cstring>
#include <vector>

namespace {

template <class real>
inline real silu(real a) { return a / (real(1) + std::exp(-a)); }

template <class real>
inline real silu_grad(real a) {
    real s = real(1) / (real(1) + std::exp(-a));
    return s * (real(1) + a * (real(1) - s));
}

// ---- gate: logits, top-k (descending, lower index wins ties), softmax over the k
template <class real>
void gate_topk(int T, int d, int E, int k, const real* X, const real* Wg, const real* bias,
               int32_t* ids, real* w, double* logits_out) {
#pragma omp parallel for schedule(static)
    for (int t = 0; t < T; ++t) {
        std::vector<double> L(E);
        for (int e = 0; e < E; ++e) {
            double acc = 0.0;
            for (int c = 0; c < d; ++c) acc += double(X[(size_t)t * d + c]) * double(Wg[(size_t)c * E + e]);
            L[e] = acc + (bias ? double(bias[e]) : 0.0);
        }
        if (logits_out) for (int e = 0; e < E; ++e) logits_out[(size_t)t * E + e] = L[e];
        std::vector<char> taken(E, 0);
        for (int s = 0; s < k; ++s) {
            int best = -1;
            for (int e = 0; e < E; ++e)
                if (!taken[e] && (best < 0 || L[e] > L[best])) best = e;  // strict >: lower index wins
            taken[best] = 1;
            ids[(size_t)t * k + s] = best;
        }
        double m = L[ids[(size_t)t * k]];
        double z = 0.0;
        for (int s = 0; s < k; ++s) z += std::exp(L[ids[(size_t)t * k + s]] - m);
        for (int s = 0; s < k; ++s) w[(size_t)t * k + s] = real(std::exp(L[ids[(size_t)t * k + s]] - m) / z);
    }
}

// ---- permutation: counting sort of the flat pair index p = t*k + s by expert id
template <class elem>
void permute(int T, int d, int E, int k, const elem* X, const int32_t* ids, int32_t* counts,
             int32_t* offsets, int32_t* row_of_pair, int32_t* pair_of_row, elem* Xp) {
    const int R = T * k;
    for (int e = 0; e < E; ++e) counts[e] = 0;
    for (int p = 0; p < R; ++p) counts[ids[p]]++;
    offsets[0] = 0;
    for (int e = 0; e < E; ++e) offsets[e + 1] = offsets[e] + counts[e];
    std::vector<int32_t> next(offsets, offsets + E);
    for (int p = 0; p < R; ++p) {
        int32_t r = next[ids[p]]++;
        row_of_pair[p] = r;
        pair_of_row[r] = p;
    }
    if (Xp)
        for (int p = 0; p < R; ++p)
            std::memcpy(Xp + (size_t)row_of_pair[p] * d, X + (size_t)(p / k) * d, sizeof(elem) * d);
}

// ---- per-expert SwiGLU FFN on the permuted rows
template <class real>
void ffn_fwd(int R, int d, int f, int E, const real* Xp, const int32_t* offsets, const real* W1,
             const real* W3, const real* W2, real* Yp, real* A_out, real* B_out, real* H_out) {
    for (int e = 0; e < E; ++e) {
        const real* w1 = W1 + (size_t)e * d * f;
        const real* w3 = W3 + (size_t)e * d * f;
        const real* w2 = W2 + (size_t)e * f * d;
#pragma omp parallel for schedule(dynamic, 4)
        for (int r = offsets[e]; r < offsets[e + 1]; ++r) {
            std::vector<real> A(f, real(0)), B(f, real(0)), Y(d, real(0));
            const real* x = Xp + (size_t)r * d;
            for (int c = 0; c < d; ++c) {
                const real xc = x[c];
                const real* r1 = w1 + (size_t)c * f;
                const real* r3 = w3 + (size_t)c * f;
                for (int j = 0; j < f; ++j) { A[j] += xc * r1[j]; B[j] += xc * r3[j]; }
            }
            for (int j = 0; j < f; ++j) {
                const real h = silu(A[j]) * B[j];
                if (A_out) A_out[(size_t)r * f + j] = A[j];
                if (B_out) B_out[(size_t)r * f + j] = B[j];
                if (H_out) H_out[(size_t)r * f + j] = h;
                const real* r2 = w2 + (size_t)j * d;
                for (int c = 0; c < d; ++c) Y[c] += h * r2[c];
            }
            std::memcpy(Yp + (size_t)r * d, Y.data(), sizeof(real) * d);
        }
    }
}

// ---- weighted combine: Y[t] = sum_s w[t,s] * Yp[row_of_pair[t*k+s]]  (w == NULL: all ones)
template <class real>
void unpermute_combine(int T, int d, int k, const real* Yp, const int32_t* row_of_pair,
                       const real* w, real* Y) {
#pragma omp parallel for schedule(static)
    for (int t = 0; t < T; ++t)
        for (int c = 0; c < d; ++c) {
            real acc = 0;
            for (int s = 0; s < k; ++s) {
                const real ws = w ? w[(size_t)t * k + s] : real(1);
                acc += ws * Yp[(size_t)row_of_pair[(size_t)t * k + s] * d + c];
            }
            Y[(size_t)t * d + c] = acc;
        }
}

// ---- derivative of the combine: dYp[row] = w * dY[t],  dw[t,s] = <dY[t], Yp[row]>
template <class real>
void combine_bwd(int T, int d, int k, const real* dY, const real* Yp, const int32_t* row_of_pair,
                 const real* w, real* dYp, real* dw) {
#pragma omp parallel for schedule(static)
    for (int t = 0; t < T; ++t)
        for (int s = 0; s < k; ++s) {
            const size_t r = (size_t)row_of_pair[(size_t)t * k + s];
            const real ws = w[(size_t)t * k + s];
            real acc = 0;
            for (int c = 0; c < d; ++c) {
                dYp[r * d + c] = ws * dY[(size_t)t * d + c];
                acc += dY[(size_t)t * d + c] * Yp[r * d + c];
            }
            dw[(size_t)t * k + s] = acc;
        }
}

// ---- derivative of the grouped FFN (recomputes A, B, H from Xp)
template <class real>
void ffn_bwd(int R, int d, int f, int E, const real* Xp, const int32_t* offsets, const real* W1,
             const real* W3, const real* W2, const real* dYp, real* dXp, real* dW1, real* dW3,
             real* dW2) {
    std::vector<real> Hs((size_t)R * f), dAs((size_t)R * f), dBs((size_t)R * f);
    for (int e = 0; e < E; ++e) {
        const real* w1 = W1 + (size_t)e * d * f;
        const real* w3 = W3 + (size_t)e * d * f;
        const real* w2 = W2 + (size_t)e * f * d;
        const int r0 = offsets[e], r1 = offsets[e + 1];
        // per row: A, B, H, dH = dYp*W2^T, dA, dB, dXp = dA*W1^T + dB*W3^T
#pragma omp parallel for schedule(dynamic, 4)
        for (int r = r0; r < r1; ++r) {
            std::vector<real> A(f, real(0)), B(f, real(0));
            const real* x = Xp + (size_t)r * d;
            const real* g = dYp + (size_t)r * d;
            for (int c = 0; c < d; ++c) {
                const real xc = x[c];
                for (int j = 0; j < f; ++j) {
                    A[j] += xc * w1[(size_t)c * f + j];
                    B[j] += xc * w3[(size_t)c * f + j];
                }
            }
            for (int j = 0; j < f; ++j) {
                real dh = 0;
                for (int c = 0; c < d; ++c) dh += g[c] * w2[(size_t)j * d + c];
                Hs[(size_t)r * f + j] = silu(A[j]) * B[j];
                dAs[(size_t)r * f + j] = dh * B[j] * silu_grad(A[j]);
                dBs[(size_t)r * f + j] = dh * silu(A[j]);
            }
            for (int c = 0; c < d; ++c) {
                real acc = 0;
                for (int j = 0; j < f; ++j)
                    acc += dAs[(size_t)r * f + j] * w1[(size_t)c * f + j] +
                           dBs[(size_t)r * f + j] * w3[(size_t)c * f + j];
                dXp[(size_t)r * d + c] = acc;
            }
        }
        // weight gradients: sums over the expert's rows (zero rows -> exact zeros)
        real* g1 = dW1 + (size_t)e * d * f;
        real* g3 = dW3 + (size_t)e * d * f;
        real* g2 = dW2 + (size_t)e * f * d;
#pragma omp parallel for schedule(static)
        for (int c = 0; c < d; ++c) {
            for (int j = 0; j < f; ++j) { g1[(size_t)c * f + j] = 0; g3[(size_t)c * f + j] = 0; }
            for (int r = r0; r < r1; ++r) {
                const real xc = Xp[(size_t)r * d + c];
                for (int j = 0; j < f; ++j) {
                    g1[(size_t)c * f + j] += xc * dAs[(size_t)r * f + j];
                    g3[(size_t)c * f + j] += xc * dBs[(size_t)r * f + j];
                }
            }
        }
#pragma omp parallel for schedule(static)
        for (int j = 0; j < f; ++j) {
            for (int c = 0; c < d; ++c) g2[(size_t)j * d + c] = 0;
            for (int r = r0; r < r1; ++r) {
                const real h = Hs[(size_t)r * f + j];
                for (int c = 0; c < d; ++c) g2[(size_t)j * d + c] += h * dYp[(size_t)r * d + c];
            }
        }
    }
}

// ---- derivative of the gate w.r.t. X and W_g through the k selected logits
//      dl_s = w_s * (dw_s - sum_j w_j dw_j);  dW_g = X^T dL;  dX += dL W_g^T
template <class real>
void gate_bwd(int T, int d, int E, int k, const real* X, const real* Wg, const int32_t* ids,
              const real* w, const real* dw, real* dX_accum, real* dWg, real* dlogits_out) {
    std::vector<real> dL((size_t)T * E, real(0));
    for (int t = 0; t < T; ++t) {
        real dot = 0;
        for (int s = 0; s < k; ++s) dot += w[(size_t)t * k + s] * dw[(size_t)t * k + s];
        for (int s = 0; s < k; ++s)
            dL[(size_t)t * E + ids[(size_t)t * k + s]] = w[(size_t)t * k + s] * (dw[(size_t)t * k + s] - dot);
    }
    if (dlogits_out) std::memcpy(dlogits_out, dL.data(), sizeof(real) * dL.size());
    // dWg[c,e] = sum over t (in order) of X[t,c] * dL[t,e]; columns are walked in blocks of 16 so
    // that the token rows are read as contiguous pieces (the sum of each output is unchanged)
#pragma omp parallel for schedule(static)
    for (int c0 = 0; c0 < d; c0 += 16) {
        const int c1 = c0 + 16 < d ? c0 + 16 : d;
        std::vector<real> acc((size_t)(c1 - c0) * E, real(0));
        for (int t = 0; t < T; ++t)
            for (int c = c0; c < c1; ++c) {
                const real xv = X[(size_t)t * d + c];
                for (int e = 0; e < E; ++e) acc[(size_t)(c - c0) * E + e] += xv * dL[(size_t)t * E + e];
            }
        for (int c = c0; c < c1; ++c)
            for (int e = 0; e < E; ++e) dWg[(size_t)c * E + e] = acc[(size_t)(c - c0) * E + e];
    }
    if (dX_accum) {
#pragma omp parallel for schedule(static)
        for (int t = 0; t < T; ++t)
            for (int c = 0; c < d; ++c) {
                real acc = 0;
                for (int e = 0; e < E; ++e) acc += dL[(size_t)t * E + e] * Wg[(size_t)c * E + e];
                dX_accum[(size_t)t * d + c] += acc;
            }
    }
}

// ---- the dense definition: no permutation, no grouping, every expert evaluated
template <class real>
void dense_layer_fwd(int T, int d, int f, int E, int k, const real* X, const real* Wg,
                     const real* bias, const real* W1, const real* W3, const real* W2, real* Y,
                     real* gate_out) {
#pragma omp parallel for schedule(dynamic, 1)
    for (int t = 0; t < T; ++t) {
        const real* x = X + (size_t)t * d;
        std::vector<double> L(E), g(E, 0.0);
        for (int e = 0; e < E; ++e) {
            double acc = 0;
            for (int c = 0; c < d; ++c) acc += double(x[c]) * double(Wg[(size_t)c * E + e]);
            L[e] = acc + (bias ? double(bias[e]) : 0.0);
        }
        // expert i is among the top k iff fewer than k experts precede it in
        // the order (logit descending, index ascending)
        double z = 0;
        for (int i = 0; i < E; ++i) {
            int before = 0;
            for (int j = 0; j < E; ++j)
                if (L[j] > L[i] || (L[j] == L[i] && j < i)) ++before;
            if (before < k) { g[i] = 1.0; }
        }
        double m = -INFINITY;
        for (int i = 0; i < E; ++i) if (g[i] != 0.0 && L[i] > m) m = L[i];
        for (int i = 0; i < E; ++i) if (g[i] != 0.0) { g[i] = std::exp(L[i] - m); z += g[i]; }
        for (int i = 0; i < E; ++i) g[i] /= z;
        if (gate_out) for (int i = 0; i < E; ++i) gate_out[(size_t)t * E + i] = real(g[i]);
        std::vector<real> y(d, real(0));
        for (int i = 0; i < E; ++i) {
            const real* w1 = W1 + (size_t)i * d * f;
            const real* w3 = W3 + (size_t)i * d * f;
            const real* w2 = W2 + (size_t)i * f * d;
            const real gi = real(g[i]);
            for (int j = 0; j < f; ++j) {
                real a = 0, b = 0;
                for (int c = 0; c < d; ++c) { a += x[c] * w1[(size_t)c * f + j]; b += x[c] * w3[(size_t)c * f + j]; }
                const real h = silu(a) * b;
                for (int c = 0; c < d; ++c) y[c] += gi * (h * w2[(size_t)j * d + c]);
            }
        }
        std::memcpy(Y + (size_t)t * d, y.data(), sizeof(real) * d);
    }
}

}  // namespace

#define EXPORT_FOR(real, sfx)                                                                         \
    extern "C" void oracle_gate_topk_##sfx(int T, int d, int E, int k, const real* X, const real* Wg, \
                                           const real* bias, int32_t* ids, real* w, double* logits) { \
        gate_topk<real>(T, d, E, k, X, Wg, bias, ids, w, logits);                                     \
    }                                                                                                 \
    extern "C" void oracle_permute_##sfx(int T, int d, int E, int k, const real* X,                   \
                                         const int32_t* ids, int32_t* counts, int32_t* offsets,       \
                                         int32_t* row_of_pair, int32_t* pair_of_row, real* Xp) {      \
        permute<real>(T, d, E, k, X, ids, counts, offsets, row_of_pair, pair_of_row, Xp);             \
    }                                                                                                 \
    extern "C" void oracle_ffn_fwd_##sfx(int R, int d, int f, int E, const real* Xp,                  \
                                         const int32_t* offsets, const real* W1, const real* W3,      \
                                         const real* W2, real* Yp, real* A, real* B, real* H) {       \
        ffn_fwd<real>(R, d, f, E, Xp, offsets, W1, W3, W2, Yp, A, B, H);                              \
    }                                                                                                 \
    extern "C" void oracle_unpermute_combine_##sfx(int T, int d, int k, const real* Yp,               \
                                                   const int32_t* row_of_pair, const real* w,         \
                                                   real* Y) {                                         \
        unpermute_combine<real>(T, d, k, Yp, row_of_pair, w, Y);                                      \
    }                                                                                                 \
    extern "C" void oracle_combine_bwd_##sfx(int T, int d, int k, const real* dY, const real* Yp,     \
                                             const int32_t* row_of_pair, const real* w, real* dYp,    \
                                             real* dw) {                                              \
        combine_bwd<real>(T, d, k, dY, Yp, row_of_pair, w, dYp, dw);                                  \
    }                                                                                                 \
    extern "C" void oracle_ffn_bwd_##sfx(int R, int d, int f, int E, const real* Xp,                  \
                                         const int32_t* offsets, const real* W1, const real* W3,      \
                                         const real* W2, const real* dYp, real* dXp, real* dW1,       \
                                         real* dW3, real* dW2) {                                      \
        ffn_bwd<real>(R, d, f, E, Xp, offsets, W1, W3, W2, dYp, dXp, dW1, dW3, dW2);                  \
    }                                                                                                 \
    extern "C" void oracle_gate_bwd_##sfx(int T, int d, int E, int k, const real* X, const real* Wg,  \
                                          const int32_t* ids, const real* w, const real* dw,          \
                                          real* dX_accum, real* dWg, real* dlogits) {                 \
        gate_bwd<real>(T, d, E, k, X, Wg, ids, w, dw, dX_accum, dWg, dlogits);                        \
    }                                                                                                 \
    extern "C" void oracle_dense_layer_fwd_##sfx(int T, int d, int f, int E, int k, const real* X,    \
                                                 const real* Wg, const real* bias, const real* W1,    \
                                                 const real* W3, const real* W2, real* Y,             \
                                                 real* gate) {                                        \
        dense_layer_fwd<real>(T, d, f, E, k, X, Wg, bias, W1, W3, W2, Y, gate);                       \
    }

EXPORT_FOR(float, f32)
EXPORT_FOR(double, f64)

extern "C" int oracle_abi_version(void) { return 1; }
