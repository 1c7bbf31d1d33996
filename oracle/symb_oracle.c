/*
 * CPU oracle for the segmented base+adapter linear layer.  TEST INFRASTRUCTURE ONLY:
 * it exists to check the GPU library and to be timed beside it; no product path may
 * call it.  It shares no code with the GPU path.
 *
 * What it is: the plain definition, written as nested loops in fp64 over inputs that
 * are bf16 bit patterns (widened exactly), with no blocking, fusion or reordering.
 * Outputs stay in fp64.  Rows are independent, so the outer row (or column) loop is
 * spread over host threads with OpenMP; each output element is still one sequential
 * fp64 sum.
 *
 * What it follows (Symbiosis, arXiv 2507.03220):
 *   - Sec. 3.2 "Base Executor": requests of many clients for one frozen layer are
 *     batched, executed once, and the output is split per client.
 *   - Sec. 3.7: for nn.Linear / Conv1D the token position is irrelevant, so all
 *     clients' tokens are flattened into one padding-free token sequence; client i
 *     owns rows off[i] .. off[i+1]-1.
 *   - Sec. 3.6: the layer is frozen, so backward is the output gradient times the
 *     parameters (no weight gradient, nothing saved from forward), and the backward
 *     batch is any batch of its own.
 *   - Sec. 3.8 eqs. (1)-(3): y = Linear(x, W) + b, with a bias-free variant.
 *   - Sec. 1 / Sec. 3.2 "Client": each client picks its own PEFT method and
 *     parameters (LoRA rank/alpha, IA3).  The paper does not restate LoRA or IA3; the
 *     standard definitions are used: LoRA adds s*(x A)B to the base output, IA3
 *     rescales the layer output (or, for IA3_IN, the layer input) elementwise by a
 *     learned vector.
 *
 * Storage layouts (row-major):  X [T][d_in], W [d_out][d_in], bias [d_out],
 *   LoRA A [r][d_in] (so mathematically A_i[k][p] = A[p][k]), LoRA B [d_out][r]
 *   (B_i[p][j] = B[j][p]), IA3 l [d_out], IA3_IN l [d_in].  Gradients use the layout
 *   of the tensor they belong to.
 *
 * Parity pins (tests/test_oracle_*.py): brute-force Python loops on tiny shapes,
 * merged-weight closed forms via a library fp64 matmul, B=0 / l=1 reductions,
 * segment-permutation and batched-vs-alone invariance, exact central finite
 * differences of <dY,Y>, noise linearity, and an exact integer-valued index probe; the two roundings
 * the paper's flow fixes (the client's x + n and its IA3 product, orc_noise_add and orc_client_scale)
 * against exact rational arithmetic rounded by the definition of round-to-nearest-even.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORC_NONE = 0, ORC_LORA = 1, ORC_IA3 = 2, ORC_IA3_IN = 3 };

typedef struct {
    int32_t kind;
    int32_t rank;
    double scale;
    const uint16_t* A; /* LoRA A, or the IA3 vector */
    const uint16_t* B; /* LoRA B */
} orc_adapter;

static inline double bf(uint16_t b) {
    union { uint32_t u; float f; } v;
    v.u = ((uint32_t)b) << 16;
    return (double)v.f;
}

int orc_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Offsets are valid when off[0] = 0 and they never decrease. */
int orc_check_offsets(int32_t S, const int32_t* off) {
    if (S < 0 || !off || off[0] != 0) return 1;
    for (int32_t i = 0; i < S; ++i)
        if (off[i + 1] < off[i]) return 1;
    return 0;
}

/* seg(t) = i  <=>  off[i] <= t < off[i+1]  (Sec. 3.7 flattening; Sec. 3.2 split). */
static int32_t seg_of(int32_t S, const int32_t* off, int32_t t) {
    for (int32_t i = 0; i < S; ++i)
        if (off[i] <= t && t < off[i + 1]) return i;
    return -1;
}

int orc_row_segment_map(int32_t S, const int32_t* off, int32_t* out) {
    if (orc_check_offsets(S, off)) return 1;
    int32_t T = off[S];
    for (int32_t t = 0; t < T; ++t) out[t] = seg_of(S, off, t);
    return 0;
}

/*
 * Forward for the listed rows (rows == NULL: rows 0..nrows-1).
 *   Y0[t][j] = sum_k X[t][k] W[j][k] (+ b[j])
 *   NONE:   Y = Y0
 *   LORA:   H[t][p] = sum_k X[t][k] A[p][k];  Y[t][j] = Y0[t][j] + s * sum_p H[t][p] B[j][p]
 *   IA3:    Y[t][j] = l[j] * Y0[t][j]
 *   IA3_IN: Y[t][j] = sum_k (l[k] X[t][k]) W[j][k] (+ b[j]);  Y0 stays the unscaled base output
 * Y0_out / Y_out: [nrows][d_out] fp64, either may be NULL.
 */
int orc_forward_rows(int32_t d_in, int32_t d_out, int32_t S, const int32_t* off,
                     const orc_adapter* ad, const uint16_t* X, const uint16_t* W,
                     const uint16_t* bias, int32_t nrows, const int32_t* rows,
                     double* Y0_out, double* Y_out) {
    if (orc_check_offsets(S, off)) return 1;
    int bad = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int32_t q = 0; q < nrows; ++q) {
        int32_t t = rows ? rows[q] : q;
        int32_t i = seg_of(S, off, t);
        if (i < 0) {
#pragma omp atomic write
            bad = 1;
            continue;
        }
        const orc_adapter* a = &ad[i];
        const uint16_t* x = X + (size_t)t * d_in;
        double* H = NULL;
        if (a->kind == ORC_LORA) {
            H = (double*)malloc(sizeof(double) * (size_t)a->rank);
            for (int32_t p = 0; p < a->rank; ++p) {
                double h = 0.0;
                for (int32_t k = 0; k < d_in; ++k) h += bf(x[k]) * bf(a->A[(size_t)p * d_in + k]);
                H[p] = h;
            }
        }
        for (int32_t j = 0; j < d_out; ++j) {
            const uint16_t* w = W + (size_t)j * d_in;
            double y0 = 0.0;
            for (int32_t k = 0; k < d_in; ++k) y0 += bf(x[k]) * bf(w[k]);
            if (bias) y0 += bf(bias[j]);
            double y = y0;
            if (a->kind == ORC_LORA) {
                double u = 0.0;
                for (int32_t p = 0; p < a->rank; ++p) u += H[p] * bf(a->B[(size_t)j * a->rank + p]);
                y = y0 + a->scale * u;
            } else if (a->kind == ORC_IA3) {
                y = bf(a->A[j]) * y0;
            } else if (a->kind == ORC_IA3_IN) {
                double v = 0.0;
                for (int32_t k = 0; k < d_in; ++k) v += bf(a->A[k]) * bf(x[k]) * bf(w[k]);
                if (bias) v += bf(bias[j]);
                y = v;
            }
            if (Y0_out) Y0_out[(size_t)q * d_out + j] = y0;
            if (Y_out) Y_out[(size_t)q * d_out + j] = y;
        }
        free(H);
    }
    return bad;
}

/*
 * Activation privacy (Sec. 3.8, eqs. (1)-(3)).  A segment's noise: noise[i] NULL = none, else
 * rows[i] rows of bf16, one broadcast row (rows[i] == 1) or one per token of the segment.
 *
 * orc_noise_add: the client's prepass  xn = x + n.  Activations are 16-bit (Sec. 4), so the sum
 * is rounded to bf16, nearest-even (reading: formed in fp32, rounded once).
 */
static uint16_t to_bf16_rne(float f) {
    uint32_t u;
    memcpy(&u, &f, 4);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40u);   /* NaN */
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

int orc_noise_add(int32_t width, int32_t S, const int32_t* off, const uint16_t* X,
                  const uint16_t* const* noise, const int32_t* rows, uint16_t* out) {
    if (orc_check_offsets(S, off)) return 1;
    for (int32_t i = 0; i < S; ++i) {
        if (noise[i] && rows[i] != 1 && rows[i] != off[i + 1] - off[i]) return 1;
        for (int32_t t = off[i]; t < off[i + 1]; ++t)
            for (int32_t k = 0; k < width; ++k) {
                uint16_t x = X[(size_t)t * width + k];
                if (noise[i]) {
                    const uint16_t n = noise[i][(size_t)(rows[i] == 1 ? 0 : t - off[i]) * width + k];
                    uint32_t xu = (uint32_t)x << 16, nu = (uint32_t)n << 16;
                    float xf, nf;
                    memcpy(&xf, &xu, 4);
                    memcpy(&nf, &nu, 4);
                    x = to_bf16_rne(xf + nf);
                }
                out[(size_t)t * width + k] = x;
            }
    }
    return 0;
}

/*
 * orc_client_scale: the elementwise product an IA3 client forms itself, in 16 bits, before the tensor
 * crosses to the executor (Sec. 3.2: the adapters run at the client; Sec. 4: 16-bit precision):
 * out[t][c] = bf16(in[t][c] * l_i[c]) for the rows of every segment of kind `kind` (ORC_IA3: in = dY,
 * the gradient entering the frozen layer's backward; ORC_IA3_IN: in = x, the layer's input), rows of
 * other segments copied.  The product of two bf16 values is exact in fp32, so this is one rounding,
 * nearest-even.  Feeding the result to orc_backward_input_rows / orc_forward_rows with those segments'
 * adapters set to NONE gives the layer's result as the paper's unfused flow computes it.
 */
int orc_client_scale(int32_t width, int32_t S, const int32_t* off, const orc_adapter* ad, int32_t kind,
                     const uint16_t* in, uint16_t* out) {
    if (orc_check_offsets(S, off)) return 1;
    if (kind != ORC_IA3 && kind != ORC_IA3_IN) return 1;
    for (int32_t i = 0; i < S; ++i)
        for (int32_t t = off[i]; t < off[i + 1]; ++t)
            for (int32_t c = 0; c < width; ++c) {
                uint16_t v = in[(size_t)t * width + c];
                if (ad[i].kind == kind) {
                    uint32_t vu = (uint32_t)v << 16, lu = (uint32_t)ad[i].A[c] << 16;
                    float vf, lf;
                    memcpy(&vf, &vu, 4);
                    memcpy(&lf, &lu, 4);
                    v = to_bf16_rne(vf * lf);
                }
                out[(size_t)t * width + c] = v;
            }
    return 0;
}

/*
 * orc_forward_private_rows: for the listed rows,
 *   (1) n_eff   = layer(n), bias nullified, the row's own adapter applied;
 *   (2) y_noisy = layer(xn) + b, the same adapter applied;
 *   (3) y       = y_noisy - n_eff.
 * Xn is what the executor receives (the output of orc_noise_add).  Both layer evaluations are
 * orc_forward_rows; nothing is rounded.
 */
int orc_forward_private_rows(int32_t d_in, int32_t d_out, int32_t S, const int32_t* off,
                             const orc_adapter* ad, const uint16_t* Xn, const uint16_t* W,
                             const uint16_t* bias, const uint16_t* const* noise, const int32_t* rows_of,
                             int32_t nrows, const int32_t* rows, double* Y_out) {
    if (orc_check_offsets(S, off)) return 1;
    const int32_t T = off[S];
    /* the noise as a flattened batch of its own: broadcast rows written out per token */
    uint16_t* Nfull = (uint16_t*)calloc((size_t)(T > 0 ? T : 1) * d_in, sizeof(uint16_t));
    double* neff = (double*)malloc(sizeof(double) * (size_t)(nrows > 0 ? nrows : 1) * d_out);
    if (!Nfull || !neff) { free(Nfull); free(neff); return 2; }
    for (int32_t i = 0; i < S; ++i) {
        if (!noise[i]) continue;
        if (rows_of[i] != 1 && rows_of[i] != off[i + 1] - off[i]) { free(Nfull); free(neff); return 1; }
        for (int32_t t = off[i]; t < off[i + 1]; ++t)
            memcpy(Nfull + (size_t)t * d_in, noise[i] + (size_t)(rows_of[i] == 1 ? 0 : t - off[i]) * d_in,
                   sizeof(uint16_t) * (size_t)d_in);
    }
    int rc = orc_forward_rows(d_in, d_out, S, off, ad, Nfull, W, NULL, nrows, rows, NULL, neff);      /* (1) */
    if (!rc) rc = orc_forward_rows(d_in, d_out, S, off, ad, Xn, W, bias, nrows, rows, NULL, Y_out);   /* (2) */
    if (!rc)
        for (size_t e = 0; e < (size_t)nrows * d_out; ++e) Y_out[e] -= neff[e];                       /* (3) */
    free(Nfull);
    free(neff);
    return rc;
}

/*
 * orc_forward_denoise_rows: steps (2) and (3) alone, with the noise effect given.  The client
 * computes n_eff once per noise value and keeps it for later iterations (Sec. 3.8); what it keeps
 * is a 16-bit activation tensor like any other it holds (Sec. 4), so here neff[i] is bf16,
 * rows_of[i] rows of width d_out (one broadcast row or one per token; NULL = nothing to take
 * off), and for the listed rows
 *   y = (layer(xn) + b, the row's adapter applied) - neff,
 * the layer evaluated by orc_forward_rows, the stored value widened exactly, nothing rounded.
 */
int orc_forward_denoise_rows(int32_t d_in, int32_t d_out, int32_t S, const int32_t* off,
                             const orc_adapter* ad, const uint16_t* Xn, const uint16_t* W,
                             const uint16_t* bias, const uint16_t* const* neff, const int32_t* rows_of,
                             int32_t nrows, const int32_t* rows, double* Y_out) {
    if (orc_check_offsets(S, off)) return 1;
    for (int32_t i = 0; i < S; ++i)
        if (neff[i] && rows_of[i] != 1 && rows_of[i] != off[i + 1] - off[i]) return 1;
    int rc = orc_forward_rows(d_in, d_out, S, off, ad, Xn, W, bias, nrows, rows, NULL, Y_out);        /* (2) */
    if (rc) return rc;
    for (int32_t q = 0; q < nrows; ++q) {                                                            /* (3) */
        const int32_t t = rows ? rows[q] : q, i = seg_of(S, off, t);
        if (!neff[i]) continue;
        const uint16_t* n = neff[i] + (size_t)(rows_of[i] == 1 ? 0 : t - off[i]) * d_out;
        for (int32_t j = 0; j < d_out; ++j) Y_out[(size_t)q * d_out + j] -= bf(n[j]);
    }
    return 0;
}

/*
 * Input gradient for the listed rows of a backward batch (its own offsets/adapters).
 *   NONE:   dX[t][k] = sum_j dY[t][j] W[j][k]
 *   LORA:   dH[t][p] = s * sum_j dY[t][j] B[j][p]
 *           dX[t][k] = sum_j dY[t][j] W[j][k] + sum_p dH[t][p] A[p][k]   (base_only drops the 2nd sum)
 *   IA3:    dX[t][k] = sum_j dY[t][j] l[j] W[j][k]
 *   IA3_IN: dX[t][k] = l[k] * sum_j dY[t][j] W[j][k]
 * base_only != 0 gives what the paper's executor returns (Sec. 3.6): dY times W only.
 */
int orc_backward_input_rows(int32_t d_in, int32_t d_out, int32_t S, const int32_t* off,
                            const orc_adapter* ad, const uint16_t* dY, const uint16_t* W,
                            int32_t nrows, const int32_t* rows, int32_t base_only,
                            double* dX_out) {
    if (orc_check_offsets(S, off)) return 1;
    int bad = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int32_t q = 0; q < nrows; ++q) {
        int32_t t = rows ? rows[q] : q;
        int32_t i = seg_of(S, off, t);
        if (i < 0) {
#pragma omp atomic write
            bad = 1;
            continue;
        }
        const orc_adapter* a = &ad[i];
        int kind = base_only ? ORC_NONE : a->kind;
        const uint16_t* g = dY + (size_t)t * d_out;
        double* dH = NULL;
        if (kind == ORC_LORA) {
            dH = (double*)malloc(sizeof(double) * (size_t)a->rank);
            for (int32_t p = 0; p < a->rank; ++p) {
                double h = 0.0;
                for (int32_t j = 0; j < d_out; ++j) h += bf(g[j]) * bf(a->B[(size_t)j * a->rank + p]);
                dH[p] = a->scale * h;
            }
        }
        /* Base term, accumulated j-outermost so W is read along its rows; every dX[t][k]
         * is still the sum over j = 0..d_out-1 taken in that order. */
        double* o = dX_out + (size_t)q * d_in;
        for (int32_t k = 0; k < d_in; ++k) o[k] = 0.0;
        for (int32_t j = 0; j < d_out; ++j) {
            double gj = bf(g[j]);
            if (kind == ORC_IA3) gj *= bf(a->A[j]);
            const uint16_t* w = W + (size_t)j * d_in;
            for (int32_t k = 0; k < d_in; ++k) o[k] += gj * bf(w[k]);
        }
        if (kind == ORC_LORA) {
            for (int32_t k = 0; k < d_in; ++k) {
                double u = 0.0;
                for (int32_t p = 0; p < a->rank; ++p) u += dH[p] * bf(a->A[(size_t)p * d_in + k]);
                o[k] += u;
            }
        } else if (kind == ORC_IA3_IN) {
            for (int32_t k = 0; k < d_in; ++k) o[k] = bf(a->A[k]) * o[k];
        }
        free(dH);
    }
    return bad;
}

/*
 * LoRA parameter gradients of segment i (sum over the segment's own tokens only):
 *   dA[p][k] = sum_t X[t][k] dH[t][p],  dH[t][p] = s * sum_j dY[t][j] B[j][p]
 *   dB[j][p] = s * sum_t H[t][p] dY[t][j],  H[t][p] = sum_k X[t][k] A[p][k]
 * dA_out [r][d_in], dB_out [d_out][r]; either may be NULL.  An empty segment gives zeros.
 */
int orc_lora_grad_segment(int32_t d_in, int32_t d_out, int32_t S, const int32_t* off,
                          const orc_adapter* ad, const uint16_t* X, const uint16_t* dY,
                          int32_t i, double* dA_out, double* dB_out) {
    if (orc_check_offsets(S, off) || i < 0 || i >= S || ad[i].kind != ORC_LORA) return 1;
    const orc_adapter* a = &ad[i];
    const int32_t r = a->rank, lo = off[i], n = off[i + 1] - off[i];
    double* H = (double*)malloc(sizeof(double) * (size_t)(n > 0 ? n : 1) * r);
    double* dH = (double*)malloc(sizeof(double) * (size_t)(n > 0 ? n : 1) * r);
#pragma omp parallel for schedule(static)
    for (int32_t u = 0; u < n; ++u) {
        const uint16_t* x = X + (size_t)(lo + u) * d_in;
        const uint16_t* g = dY + (size_t)(lo + u) * d_out;
        for (int32_t p = 0; p < r; ++p) {
            double h = 0.0;
            for (int32_t k = 0; k < d_in; ++k) h += bf(x[k]) * bf(a->A[(size_t)p * d_in + k]);
            H[(size_t)u * r + p] = h;
            double e = 0.0;
            for (int32_t j = 0; j < d_out; ++j) e += bf(g[j]) * bf(a->B[(size_t)j * r + p]);
            dH[(size_t)u * r + p] = a->scale * e;
        }
    }
    if (dA_out) {
#pragma omp parallel for schedule(static)
        for (int32_t k = 0; k < d_in; ++k)
            for (int32_t p = 0; p < r; ++p) {
                double v = 0.0;
                for (int32_t u = 0; u < n; ++u)
                    v += bf(X[(size_t)(lo + u) * d_in + k]) * dH[(size_t)u * r + p];
                dA_out[(size_t)p * d_in + k] = v;
            }
    }
    if (dB_out) {
#pragma omp parallel for schedule(static)
        for (int32_t j = 0; j < d_out; ++j)
            for (int32_t p = 0; p < r; ++p) {
                double v = 0.0;
                for (int32_t u = 0; u < n; ++u)
                    v += H[(size_t)u * r + p] * bf(dY[(size_t)(lo + u) * d_out + j]);
                dB_out[(size_t)j * r + p] = a->scale * v;
            }
    }
    free(H);
    free(dH);
    return 0;
}

/*
 * IA3 vector gradient of segment i for the listed channels (cols == NULL: 0..ncols-1).
 *   IA3:    dl[j] = sum_t dY[t][j] * Y0[t][j],   Y0[t][j] = sum_k X[t][k] W[j][k] (+ b[j])
 *   IA3_IN: dl[k] = sum_t X[t][k] * G[t][k],     G[t][k]  = sum_j dY[t][j] W[j][k]
 * Y0_saved (IA3 only, may be NULL): the [T][d_out] bf16 base output the client kept from
 * its forward pass (Sec. 3.2: a fine-tuning client saves the layer's input and output
 * tensors for the backward pass; Sec. 4: they are 16-bit).  When given, it stands for
 * Y0[t][j] in the sum above instead of the value recomputed from X and W.
 * G_saved (IA3_IN only, may be NULL): likewise the [T][d_in] bf16 input gradient dY W the
 * executor returned to the client (Sec. 3.6), standing for G[t][k].
 */
int orc_ia3_grad_segment(int32_t d_in, int32_t d_out, int32_t S, const int32_t* off,
                         const orc_adapter* ad, const uint16_t* X, const uint16_t* dY,
                         const uint16_t* W, const uint16_t* bias, const uint16_t* Y0_saved,
                         int32_t i, int32_t ncols, const int32_t* cols, double* dl_out,
                         const uint16_t* G_saved) {
    if (orc_check_offsets(S, off) || i < 0 || i >= S) return 1;
    const int kind = ad[i].kind;
    if (kind != ORC_IA3 && kind != ORC_IA3_IN) return 1;
    const int32_t lo = off[i], n = off[i + 1] - off[i];
#pragma omp parallel for schedule(dynamic, 1)
    for (int32_t q = 0; q < ncols; ++q) {
        int32_t c = cols ? cols[q] : q;
        double v = 0.0;
        for (int32_t u = 0; u < n; ++u) {
            const uint16_t* x = X + (size_t)(lo + u) * d_in;
            const uint16_t* g = dY + (size_t)(lo + u) * d_out;
            if (kind == ORC_IA3 && Y0_saved) {
                v += bf(g[c]) * bf(Y0_saved[(size_t)(lo + u) * d_out + c]);
            } else if (kind == ORC_IA3) {
                double y0 = 0.0;
                for (int32_t k = 0; k < d_in; ++k) y0 += bf(x[k]) * bf(W[(size_t)c * d_in + k]);
                if (bias) y0 += bf(bias[c]);
                v += bf(g[c]) * y0;
            } else if (G_saved) {
                v += bf(x[c]) * bf(G_saved[(size_t)(lo + u) * d_in + c]);
            } else {
                double G = 0.0;
                for (int32_t j = 0; j < d_out; ++j) G += bf(g[j]) * bf(W[(size_t)j * d_in + c]);
                v += bf(x[c]) * G;
            }
        }
        dl_out[q] = v;
    }
    return 0;
}
