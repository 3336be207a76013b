/*
 * CPU oracle for Independent Subnet Training (IST).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition of what the
 * GPU library must compute.  It shares no code, header, table or helper with the
 * HIP path; only tests, the smoke check and the bench's cpu_baseline leg may
 * call it.  The product never routes through it.
 *
 * What it follows (paper: "Distributed Learning of Fully Connected Neural
 * Networks using Independent Subnet Training"):
 *   - Section 2.1 "Constructing Subnets" and Appendix A (membership indicators
 *     m^{(s)}_{l,i}, one subnet per hidden neuron, input and output neurons in
 *     every subnet): ist_oracle_block, ist_oracle_gather.
 *   - Section 2.1 "Training Subnets": J (= k) iterations of local mini-batch SGD
 *     on each narrow subnet with no communication, then parameters copied back
 *     into the full network without collisions: ist_oracle_subnet_sgd,
 *     ist_oracle_scatter.
 *   - Appendix B, third bullet: the local step is w <- z - eta * grad l(z).
 *   - Section 2.2: the n^2 factor is dropped; the hot path is the plain narrow
 *     MLP, optionally with the per-neuron standardisation of that section
 *     (ist_oracle_subnet_sgd_norm).
 *
 * Readings where the paper is silent (all restated in the design notes):
 *   ReLU hidden activations with ReLU'(0) = 0, mean softmax cross-entropy loss,
 *   hidden biases travel with their neuron, the shared output bias is replicated
 *   and averaged on merge, blocks of a uniform random permutation that are as
 *   equal in size as the layer width allows.
 *
 * Arithmetic is fp64.  "mode" selects where values are rounded to a storage
 * type, emulating a device that keeps parameters, activations and activation
 * gradients in that type while accumulating in higher precision:
 *   mode 0: exact  (no rounding anywhere)
 *   mode 1: f32    (W, b, h_l, dz_l rounded to IEEE binary32, nearest-even)
 *   mode 2: bf16   (same tensors rounded to bfloat16, nearest-even)
 *
 * Pins (tests/test_oracle_*.py): disjoint cover, masked-network equivalence,
 * closed-form parameter counts, NumPy fancy-index cross-check, merge/partition
 * round trip, S = 1 equals a full-network SGD step, central finite differences,
 * subnet independence, hand-computed 2-2-2 network.  k-step parameters at the
 * full benchmark shapes have no printed values in the paper: parity unpinned
 * beyond that chain.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ---------------------------------------------------------------- rounding */

static double round_store(double x, int mode)
{
    if (mode == 0 || x == 0.0 || !isfinite(x)) return x;
    if (mode == 1) return (double)(float)x;
    /* bfloat16: 8 significant bits, same exponent range as binary32.
       x = m * 2^e with 0.5 <= |m| < 1, so one unit in the last place is
       2^(e-8); below the normal range the quantum stays at 2^-133. */
    int e;
    (void)frexp(x, &e);
    int q = e - 8;
    if (q < -133) q = -133;
    return ldexp(nearbyint(ldexp(x, -q)), q);
}

double ist_oracle_round(double x, int32_t mode) { return round_store(x, mode); }
void ist_oracle_round_array(double *x, int64_t n, int32_t mode)
{
    for (int64_t i = 0; i < n; ++i) x[i] = round_store(x[i], mode);
}

/* ------------------------------------------------- blocks, partition, merge */

/* Neurons of hidden layer l owned by subnet s: the s-th block of the layer's
   permutation, order kept (Section 2.1 "Constructing Subnets": every hidden neuron is
   assigned to exactly one of the n subnets; Appendix A: sum_s m^{(s)}_{l,i} = 1).  The
   blocks are as equal as N allows: with N = q*S + r, the first r subnets own q + 1
   neurons and the others q (equal blocks when S divides N), so subnet s starts at
   position s*q + min(s, r).  Writes the block to out and returns its width, or -1 on
   a bad argument. */
int64_t ist_oracle_block(const int32_t *perm, int64_t N, int32_t S, int32_t s, int32_t *out)
{
    if (S <= 0 || N < 0 || s < 0 || s >= S) return -1;
    int64_t q = N / S, r = N % S;
    int64_t start = (int64_t)s * q + (s < r ? s : r);
    int64_t w = q + (s < r ? 1 : 0);
    for (int64_t i = 0; i < w; ++i) out[i] = perm[start + i];
    return w;
}

/* sub[i][j] = W[ridx[i]][cidx[j]] on raw elements of esz bytes; a NULL index
   list means "all, in order" (input and output neurons are shared by every
   subnet).  A weight is in the subnet iff both endpoint neurons are. */
void ist_oracle_gather(const uint8_t *W, int64_t ncols_full, int64_t esz,
                       const int32_t *ridx, int64_t nr, const int32_t *cidx, int64_t nc,
                       uint8_t *sub)
{
    for (int64_t i = 0; i < nr; ++i) {
        int64_t r = ridx ? ridx[i] : i;
        for (int64_t j = 0; j < nc; ++j) {
            int64_t c = cidx ? cidx[j] : j;
            memcpy(sub + (i * nc + j) * esz, W + (r * ncols_full + c) * esz, (size_t)esz);
        }
    }
}

/* W[ridx[i]][cidx[j]] = sub[i][j]; every other entry of W is left untouched
   (Section 2.1 "Training Subnets": copied back, no collisions). */
void ist_oracle_scatter(uint8_t *W, int64_t ncols_full, int64_t esz,
                        const int32_t *ridx, int64_t nr, const int32_t *cidx, int64_t nc,
                        const uint8_t *sub)
{
    for (int64_t i = 0; i < nr; ++i) {
        int64_t r = ridx ? ridx[i] : i;
        for (int64_t j = 0; j < nc; ++j) {
            int64_t c = cidx ? cidx[j] : j;
            memcpy(W + (r * ncols_full + c) * esz, sub + (i * nc + j) * esz, (size_t)esz);
        }
    }
}

/* Output bias after merge: every subnet holds a copy of the shared output
   neurons' bias; the merged value is their mean.  The S values are added in
   binary32 as a balanced pairwise tree over the subnet index (neighbours first,
   then pairs of pairs, ...), multiplied by 1/S in binary32 and rounded to the
   storage type.  With S a power of two and S identical copies every addition
   and the scaling are exact, so merge(partition(b)) == b bit for bit. */
void ist_oracle_merge_out_bias(const double *bsub /* [S][n] */, int32_t S, int64_t n,
                               int32_t mode, double *out)
{
    float inv = 1.0f / (float)S;
    float *v = (float *)malloc((size_t)S * sizeof(float));
    for (int64_t i = 0; i < n; ++i) {
        for (int32_t s = 0; s < S; ++s) v[s] = (float)bsub[(int64_t)s * n + i];
        for (int32_t d = 1; d < S; d *= 2)
            for (int32_t s = 0; s + d < S; s += 2 * d) v[s] = v[s] + v[s + d];
        out[i] = round_store((double)(v[0] * inv), mode == 0 ? 1 : mode);
    }
    free(v);
}

/* ------------------------------------------------------ local SGD on a subnet */

/*
 * k steps of mini-batch SGD on one narrow fully connected net.
 *
 *   t        number of weight matrices; n[0..t] layer widths of THIS subnet
 *   W[l-1]   [n_l][n_{l-1}] row-major, updated in place   (f_l = W_l f_{l-1})
 *   b[l-1]   [n_l] or NULL (b == NULL: no biases at all)
 *   input    dense: X [k][B][n_0]
 *            CSR:   rowptr [k*B+1] (absolute offsets), colidx, vals
 *   y        [k][B] class ids
 *   lr       learning rate eta
 *   loss_out [k] mean cross-entropy of each step's batch before its update
 *
 * Per step j (Section 2.1 / Appendix B): forward through the narrow net with
 * ReLU hidden units, mean softmax cross-entropy, back-propagation, and
 * w <- w - eta * grad.  dh_{l-1} is formed with the weights before their update.
 * Returns 0, or -1 on a bad argument.
 */
int32_t ist_oracle_subnet_sgd_norm(int32_t t, const int64_t *n, double **W, double **b,
                                   int32_t is_csr, const double *X, const int32_t *rowptr,
                                   const int32_t *colidx, const double *vals, const int32_t *y,
                                   int32_t B, int32_t k, double lr, int32_t mode, int32_t normalize,
                                   double eps, double *loss_out);

int32_t ist_oracle_subnet_sgd(int32_t t, const int64_t *n, double **W, double **b,
                              int32_t is_csr, const double *X, const int32_t *rowptr,
                              const int32_t *colidx, const double *vals, const int32_t *y,
                              int32_t B, int32_t k, double lr, int32_t mode, double *loss_out)
{
    return ist_oracle_subnet_sgd_norm(t, n, W, b, is_csr, X, rowptr, colidx, vals, y, B, k, lr, mode, 0, 0.0,
                                      loss_out);
}

/*
 * The same with the correction of Section 2.2 ("Correcting Distributional Shift"):
 * with normalize != 0 every hidden neuron's input is standardised over the mini-batch
 * before the activation,
 *     mu_r = mean_b z[b][r],  sigma_r = sqrt(mean_b (z[b][r] - mu_r)^2 + eps),
 *     zh = (z - mu) / sigma,  h = ReLU(zh),
 * (no n^2 factor, no learned scale or shift; the statistics are those of the batch
 * and the gradient flows through them, as in batch normalisation, to which the
 * paper likens the step).  Back-propagation through the standardisation:
 *     dz = (dzh - mean_b dzh - zh * mean_b(dzh * zh)) / sigma,   dzh = dh * [zh > 0].
 * Storage rounding (mode 1/2): zh and dzh and dz are rounded where they are stored;
 * z, mu, sigma are not.
 */
int32_t ist_oracle_subnet_sgd_scaled(int32_t t, const int64_t *n, double **W, double **b,
                                     int32_t is_csr, const double *X, const int32_t *rowptr,
                                     const int32_t *colidx, const double *vals, const int32_t *y,
                                     int32_t B, int32_t k, double lr, int32_t mode, int32_t normalize,
                                     double eps, const double *scale, double *loss_out);

int32_t ist_oracle_subnet_sgd_norm(int32_t t, const int64_t *n, double **W, double **b,
                                   int32_t is_csr, const double *X, const int32_t *rowptr,
                                   const int32_t *colidx, const double *vals, const int32_t *y,
                                   int32_t B, int32_t k, double lr, int32_t mode, int32_t normalize,
                                   double eps, double *loss_out)
{
    return ist_oracle_subnet_sgd_scaled(t, n, W, b, is_csr, X, rowptr, colidx, vals, y, B, k, lr, mode, normalize,
                                        eps, NULL, loss_out);
}

/*
 * The same with the subnet forward pass of Appendix A, equation (4): the product of layer l is
 * multiplied by a factor gamma_l = scale[l-1] (the paper's n^2, which makes the sum over subnets
 * of the masked products an unbiased estimate of W_l f_{l-1}),
 *     z_l = gamma_l * (W_l h_{l-1}) + b_l,
 * hence dh_{l-1} = gamma_l * (dz_l W_l) and dW_l = gamma_l * dz_l^T h_{l-1}; the bias is not
 * scaled.  scale == NULL: every gamma_l = 1.
 */
int32_t ist_oracle_subnet_sgd_scaled(int32_t t, const int64_t *n, double **W, double **b,
                                     int32_t is_csr, const double *X, const int32_t *rowptr,
                                     const int32_t *colidx, const double *vals, const int32_t *y,
                                     int32_t B, int32_t k, double lr, int32_t mode, int32_t normalize,
                                     double eps, const double *scale, double *loss_out)
{
    if (t < 1 || B <= 0 || k < 0) return -1;
    double **zh = (double **)calloc((size_t)t + 1, sizeof(double *));
    double **isg = (double **)calloc((size_t)t + 1, sizeof(double *));
    if (normalize)
        for (int32_t l = 1; l < t; ++l) {
            zh[l] = (double *)malloc(sizeof(double) * (size_t)B * (size_t)n[l]);
            isg[l] = (double *)malloc(sizeof(double) * (size_t)n[l]);
        }
    /* activations h[l] [B][n_l] for l = 1..t-1, logits z [B][n_t], gradients */
    double **h = (double **)calloc((size_t)t + 1, sizeof(double *));
    double **dz = (double **)calloc((size_t)t + 1, sizeof(double *));
    for (int32_t l = 1; l <= t; ++l) {
        h[l] = (double *)malloc(sizeof(double) * (size_t)B * (size_t)n[l]);
        dz[l] = (double *)malloc(sizeof(double) * (size_t)B * (size_t)n[l]);
    }
    double *rowloss = (double *)malloc(sizeof(double) * (size_t)B);

    for (int32_t j = 0; j < k; ++j) {
        const double *x = is_csr ? NULL : X + (int64_t)j * B * n[0];
        const int32_t *rp = is_csr ? rowptr + (int64_t)j * B : NULL;
        const int32_t *yy = y + (int64_t)j * B;

        /* ---- forward: z_l = W_l h_{l-1} + b_l, h_l = ReLU(z_l) for l < t ---- */
        for (int32_t l = 1; l <= t; ++l) {
            const double *Wl = W[l - 1];
            const double *bl = b ? b[l - 1] : NULL;
            const int64_t nin = n[l - 1], nout = n[l];
            const double *hin = (l == 1) ? x : h[l - 1];
            double *hout = h[l];
#pragma omp parallel for schedule(static)
            for (int64_t q = 0; q < (int64_t)B * nout; ++q) {
                int64_t bi = q / nout, r = q % nout;
                double acc = 0.0;
                if (l == 1 && is_csr) {
                    for (int32_t p = rp[bi]; p < rp[bi + 1]; ++p)
                        acc += vals[p] * Wl[r * nin + colidx[p]];
                } else {
                    const double *hr = hin + bi * nin;
                    const double *wr = Wl + r * nin;
#pragma omp simd reduction(+ : acc)
                    for (int64_t c = 0; c < nin; ++c) acc += hr[c] * wr[c];
                }
                if (scale) acc *= scale[l - 1];
                if (bl) acc += bl[r];
                if (l < t && !normalize) acc = round_store(acc > 0.0 ? acc : 0.0, mode);
                hout[bi * nout + r] = acc; /* logits (and inputs of the standardisation) stay unrounded */
            }
            if (l < t && normalize) {
#pragma omp parallel for schedule(static)
                for (int64_t r = 0; r < nout; ++r) {
                    double mu = 0.0, var = 0.0;
                    for (int64_t bi = 0; bi < B; ++bi) mu += hout[bi * nout + r];
                    mu /= (double)B;
                    for (int64_t bi = 0; bi < B; ++bi) {
                        double d = hout[bi * nout + r] - mu;
                        var += d * d;
                    }
                    var /= (double)B;
                    double inv = 1.0 / sqrt(var + eps);
                    isg[l][r] = inv;
                    for (int64_t bi = 0; bi < B; ++bi) {
                        double v = round_store((hout[bi * nout + r] - mu) * inv, mode);
                        zh[l][bi * nout + r] = v;
                        hout[bi * nout + r] = v > 0.0 ? v : 0.0;
                    }
                }
            }
        }

        /* ---- loss and dz_t = (softmax(z_t) - onehot(y)) / B ---- */
        {
            const int64_t C = n[t];
            const double *z = h[t];
            double *g = dz[t];
#pragma omp parallel for schedule(static)
            for (int64_t bi = 0; bi < B; ++bi) {
                const double *zr = z + bi * C;
                double mx = zr[0];
                for (int64_t c = 1; c < C; ++c) mx = zr[c] > mx ? zr[c] : mx;
                double se = 0.0;
                for (int64_t c = 0; c < C; ++c) se += exp(zr[c] - mx);
                rowloss[bi] = log(se) + mx - zr[yy[bi]];
                for (int64_t c = 0; c < C; ++c) {
                    double p = exp(zr[c] - mx) / se;
                    if (c == yy[bi]) p -= 1.0;
                    g[bi * C + c] = round_store(p / (double)B, mode);
                }
            }
            double tot = 0.0;
            for (int64_t bi = 0; bi < B; ++bi) tot += rowloss[bi];
            if (loss_out) loss_out[j] = tot / (double)B;
        }

        /* ---- backward and update, top layer first ---- */
        for (int32_t l = t; l >= 1; --l) {
            double *Wl = W[l - 1];
            double *bl = b ? b[l - 1] : NULL;
            const int64_t nin = n[l - 1], nout = n[l];
            const double *g = dz[l];

            /* dz_{l-1} = (dz_l W_l) masked by h_{l-1} > 0, with the old W_l */
            if (l > 1) {
                const double *hprev = h[l - 1];
                double *gp = dz[l - 1];
#pragma omp parallel for schedule(static)
                for (int64_t bi = 0; bi < B; ++bi) {
                    double *row = gp + bi * nin;
                    for (int64_t c = 0; c < nin; ++c) row[c] = 0.0;
                    for (int64_t r = 0; r < nout; ++r) {
                        double gv = g[bi * nout + r];
                        const double *wr = Wl + r * nin;
#pragma omp simd
                        for (int64_t c = 0; c < nin; ++c) row[c] += gv * wr[c];
                    }
                    if (scale)
                        for (int64_t c = 0; c < nin; ++c) row[c] *= scale[l - 1];
                    for (int64_t c = 0; c < nin; ++c)
                        row[c] = round_store(hprev[bi * nin + c] > 0.0 ? row[c] : 0.0, mode);
                }
                if (normalize) {
                    const double *zz = zh[l - 1];
                    const double *inv = isg[l - 1];
#pragma omp parallel for schedule(static)
                    for (int64_t c = 0; c < nin; ++c) {
                        double s1 = 0.0, s2 = 0.0;
                        for (int64_t bi = 0; bi < B; ++bi) {
                            s1 += gp[bi * nin + c];
                            s2 += gp[bi * nin + c] * zz[bi * nin + c];
                        }
                        s1 /= (double)B;
                        s2 /= (double)B;
                        for (int64_t bi = 0; bi < B; ++bi)
                            gp[bi * nin + c] = round_store(
                                (gp[bi * nin + c] - s1 - zz[bi * nin + c] * s2) * inv[c], mode);
                    }
                }
            }

            /* dW_l = gamma_l dz_l^T h_{l-1};  W_l <- W_l - lr dW_l;  b_l <- b_l - lr sum_b dz_l */
            const double gam = scale ? scale[l - 1] : 1.0;
#pragma omp parallel
            {
                double *dwrow = (double *)calloc((size_t)nin, sizeof(double));
#pragma omp for schedule(static)
                for (int64_t r = 0; r < nout; ++r) {
                    double db = 0.0;
                    double *wr = Wl + r * nin;
                    if (l == 1 && is_csr) {
                        for (int64_t bi = 0; bi < B; ++bi) {
                            double gv = g[bi * nout + r];
                            db += gv;
                            for (int32_t p = rp[bi]; p < rp[bi + 1]; ++p)
                                dwrow[colidx[p]] += gv * vals[p];
                        }
                        /* only columns present in the batch carry a gradient */
                        for (int64_t bi = 0; bi < B; ++bi)
                            for (int32_t p = rp[bi]; p < rp[bi + 1]; ++p) {
                                int32_t c = colidx[p];
                                if (dwrow[c] != 0.0) {
                                    wr[c] = round_store(wr[c] - lr * (gam * dwrow[c]), mode);
                                    dwrow[c] = 0.0;
                                }
                            }
                    } else {
                        const double *hin = (l == 1) ? x : h[l - 1];
                        for (int64_t c = 0; c < nin; ++c) dwrow[c] = 0.0;
                        for (int64_t bi = 0; bi < B; ++bi) {
                            double gv = g[bi * nout + r];
                            db += gv;
                            const double *hr = hin + bi * nin;
#pragma omp simd
                            for (int64_t c = 0; c < nin; ++c) dwrow[c] += gv * hr[c];
                        }
                        for (int64_t c = 0; c < nin; ++c)
                            wr[c] = round_store(wr[c] - lr * (gam * dwrow[c]), mode);
                    }
                    if (bl) bl[r] = round_store(bl[r] - lr * db, mode);
                }
                free(dwrow);
            }
        }
    }

    for (int32_t l = 1; l <= t; ++l) { free(h[l]); free(dz[l]); free(zh[l]); free(isg[l]); }
    free(h); free(dz); free(zh); free(isg); free(rowloss);
    return 0;
}
