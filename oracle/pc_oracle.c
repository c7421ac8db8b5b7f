/*
 * CPU oracle for the pattern-sparse 3x3 convolution path (test infrastructure).
 *
 * Plain, slow, host-only C. It is the checker the HIP kernels are compared
 * against and must never be called from the product path. It shares no code
 * with the HIP library: no headers, no tables, no helpers.
 *
 * What it follows (ClickTrain, arXiv 2011.10170):
 *   - Section 4.1: per-weight importance (g*w)^2, Eq. 1 (pattern importance = sum of the
 *     importances of the taps a pattern keeps, best pattern = arg max over the pool),
 *     Eq. 2 (kernel importance = the same sum over all 9 taps).
 *   - Section 2 "Fine-grained pattern-based pruning": 4 of 9 taps kept in every kept kernel,
 *     whole kernels removed by connectivity pruning; Section 5.2: every filter of a layer
 *     keeps the same number of weights.
 *   - Section 5.2 "Backward phase acceleration": z = a (*) W, delta_prev = delta (*) rot180(W),
 *     dE/dW = a_prev (*) delta. "(*)" is the deep-learning cross-correlation: the rot180 in the
 *     backward formula is what fixes that the forward pass does not flip the kernel.
 *
 * The convolution passes are exact definitions: a direct loop nest over the dense
 * masked weight tensor Wm = W (.) M with zero padding 1, stride 1 or 2, NHWC
 * activations, double accumulation, one rounding to float at the end.
 *
 * The selection step has discrete output, so its float32 operation order is
 * part of its definition (compile with -ffp-contract=off):
 *   s_t   = (g_t*w_t)*(g_t*w_t)            two rounded multiplies; without G: s_t = w_t*w_t
 *   I_p   = ((s_a+s_b)+s_c)+s_d            taps a<b<c<d of pattern p, ascending tap order
 *   pid   = first p attaining max I_p
 *   R     = I_pid  (score mode 0)  or  ((((((((s0+s1)+s2)+s3)+s4)+s5)+s6)+s7)+s8  (mode 1, Eq. 2)
 *   keep  = R among the n_keep largest of its filter row (keep mode 0) or of the layer
 *           (keep mode 1); equal scores are ordered by lower index first.
 *
 * Layouts: W, G, M, dW: [F][C][9] with tap t = 3*r + s (kernel row r, column s,
 * offset (r-1, s-1)); x: [N][H][W][C]; y, dy: [N][Ho][Wo][F]; Ho = (H-1)/stride + 1.
 *
 * Pins (tests/test_oracle_*.py): PyTorch-CPU conv2d and autograd in float64 on the masked
 * weights; a separately written im2col product; closed forms (all-ones, impulse);
 * adjoint identities; P=126 equals textbook top-4; brute force on tiny inputs; mask
 * invariants. No function here is unpinned.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#include <math.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int orc_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* ---- bf16 storage rounding (round to nearest, ties to even; finite inputs) ---- */
static float bf16_rne(float v)
{
    uint32_t b;
    memcpy(&b, &v, 4);
    b += 0x7FFFu + ((b >> 16) & 1u);
    b &= 0xFFFF0000u;
    memcpy(&v, &b, 4);
    return v;
}

void orc_bf16_round(const float *in, int64_t n, float *out)
{
    for (int64_t i = 0; i < n; ++i) out[i] = bf16_rne(in[i]);
}

/* ---- selection (Section 4.1, Eq. 1 and Eq. 2) ---- */

static void tap_scores(const float *w, const float *g, float s[9])
{
    for (int t = 0; t < 9; ++t) {
        if (g) {
            float gw = g[t] * w[t];
            s[t] = gw * gw;
        } else {
            s[t] = w[t] * w[t];
        }
    }
}

static float pattern_score(const float s[9], unsigned mask)
{
    float acc = 0.0f;
    int first = 1;
    for (int t = 0; t < 9; ++t) {
        if (mask & (1u << t)) {
            if (first) { acc = s[t]; first = 0; }
            else acc = acc + s[t];
        }
    }
    return acc;
}

typedef struct { float r; int64_t idx; } rank_item;

static int rank_cmp(const void *pa, const void *pb)
{
    const rank_item *a = (const rank_item *)pa, *b = (const rank_item *)pb;
    if (a->r > b->r) return -1;
    if (a->r < b->r) return 1;
    return (a->idx < b->idx) ? -1 : (a->idx > b->idx);
}

/* returns 0 on success, 1 on a bad argument */
int orc_select(const float *W, const float *G, int F, int C,
               const uint16_t *lib, int P, int keep_mode, int64_t n_keep, int score_mode,
               uint8_t *pid, uint8_t *keep)
{
    if (!W || !lib || !pid || !keep || F < 1 || C < 1 || P < 1 || P > 126 || n_keep < 0) return 1;
    if (keep_mode == 0 && n_keep > C) return 1;
    if (keep_mode == 1 && n_keep > (int64_t)F * C) return 1;
    int64_t nk = (int64_t)F * C;
    float *R = (float *)malloc(sizeof(float) * (size_t)nk);
    if (!R) return 1;
    for (int64_t k = 0; k < nk; ++k) {
        float s[9];
        tap_scores(W + 9 * k, G ? G + 9 * k : NULL, s);
        int best = 0;
        float best_score = pattern_score(s, lib[0]);
        for (int p = 1; p < P; ++p) {
            float sc = pattern_score(s, lib[p]);
            if (sc > best_score) { best_score = sc; best = p; }
        }
        pid[k] = (uint8_t)best;
        R[k] = (score_mode == 0) ? best_score : pattern_score(s, 0x1FFu);
    }
    memset(keep, 0, (size_t)nk);
    int64_t seg = (keep_mode == 0) ? C : nk;
    rank_item *items = (rank_item *)malloc(sizeof(rank_item) * (size_t)seg);
    if (!items) { free(R); return 1; }
    for (int64_t base = 0; base < nk; base += seg) {
        for (int64_t i = 0; i < seg; ++i) { items[i].r = R[base + i]; items[i].idx = i; }
        qsort(items, (size_t)seg, sizeof(rank_item), rank_cmp);
        for (int64_t i = 0; i < n_keep; ++i) keep[base + items[i].idx] = 1;
    }
    free(items);
    free(R);
    return 0;
}

/* ---- masks and hard prune (W (.) M) ---- */

void orc_mask(const uint8_t *pid, const uint8_t *keep, const uint16_t *lib, int F, int C, uint8_t *M)
{
    for (int64_t k = 0; k < (int64_t)F * C; ++k)
        for (int t = 0; t < 9; ++t)
            M[9 * k + t] = (uint8_t)((keep[k] != 0) && ((lib[pid[k]] >> t) & 1u));
}

void orc_apply_mask(const float *W, const uint8_t *M, int64_t n, float *Wm)
{
    for (int64_t i = 0; i < n; ++i) Wm[i] = M[i] ? W[i] : 0.0f;
}

/* Compact order of the kept kernels: filters ascending; inside a filter by pattern id,
 * then by channel. Slot i of a compact [nnzk][4] array belongs to kernel (slot_f[i],
 * slot_c[i]) and its 4 entries are that kernel's kept taps in ascending tap index.
 * Returns nnzk. slot_f / slot_c may be NULL to count only. */
int64_t orc_compact_order(const uint8_t *pid, const uint8_t *keep, int F, int C, int P,
                          int32_t *slot_f, int32_t *slot_c)
{
    int64_t n = 0;
    for (int f = 0; f < F; ++f)
        for (int p = 0; p < P; ++p)
            for (int c = 0; c < C; ++c) {
                int64_t k = (int64_t)f * C + c;
                if (keep[k] && pid[k] == p) {
                    if (slot_f) slot_f[n] = f;
                    if (slot_c) slot_c[n] = c;
                    ++n;
                }
            }
    return n;
}

/* dense [F][C][9] -> compact [nnzk][4] in the order above */
void orc_gather_compact(const float *dense, const uint8_t *pid, const uint16_t *lib,
                        const int32_t *slot_f, const int32_t *slot_c, int64_t nnzk, int C,
                        float *compact)
{
    for (int64_t i = 0; i < nnzk; ++i) {
        int64_t k = (int64_t)slot_f[i] * C + slot_c[i];
        unsigned m = lib[pid[k]];
        int j = 0;
        for (int t = 0; t < 9; ++t)
            if (m & (1u << t)) compact[4 * i + j++] = dense[9 * k + t];
    }
}

/* ---- the three passes (Section 5.2) ---- */

static int out_dim(int in, int stride) { return (in - 1) / stride + 1; }

/* y[n,oy,ox,f] = sum_{c,r,s} x[n, oy*stride + r - 1, ox*stride + s - 1, c] * Wm[f,c,r,s] */
void orc_conv_fwd(const float *x, const float *Wm, int N, int H, int Wd, int C, int F, int stride, float *y)
{
    int Ho = out_dim(H, stride), Wo = out_dim(Wd, stride);
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n)
        for (int oy = 0; oy < Ho; ++oy)
            for (int ox = 0; ox < Wo; ++ox)
                for (int f = 0; f < F; ++f) {
                    double acc = 0.0;
                    for (int c = 0; c < C; ++c)
                        for (int r = 0; r < 3; ++r)
                            for (int s = 0; s < 3; ++s) {
                                float w = Wm[((int64_t)f * C + c) * 9 + 3 * r + s];
                                if (w == 0.0f) continue;
                                int iy = oy * stride + r - 1, ix = ox * stride + s - 1;
                                if (iy < 0 || iy >= H || ix < 0 || ix >= Wd) continue;
                                acc += (double)x[(((int64_t)n * H + iy) * Wd + ix) * C + c] * (double)w;
                            }
                    y[(((int64_t)n * Ho + oy) * Wo + ox) * F + f] = (float)acc;
                }
}

/* One output element of the forward pass, addressed by its flat NHWC index. */
void orc_conv_fwd_at(const float *x, const float *Wm, int N, int H, int Wd, int C, int F, int stride,
                     const int64_t *idx, int64_t n_idx, float *out)
{
    int Ho = out_dim(H, stride), Wo = out_dim(Wd, stride);
    (void)N;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n_idx; ++i) {
        int64_t q = idx[i];
        int f = (int)(q % F); q /= F;
        int ox = (int)(q % Wo); q /= Wo;
        int oy = (int)(q % Ho); q /= Ho;
        int n = (int)q;
        double acc = 0.0;
        for (int c = 0; c < C; ++c)
            for (int r = 0; r < 3; ++r)
                for (int s = 0; s < 3; ++s) {
                    int iy = oy * stride + r - 1, ix = ox * stride + s - 1;
                    if (iy < 0 || iy >= H || ix < 0 || ix >= Wd) continue;
                    acc += (double)x[(((int64_t)n * H + iy) * Wd + ix) * C + c] *
                           (double)Wm[((int64_t)f * C + c) * 9 + 3 * r + s];
                }
        out[i] = (float)acc;
    }
}

/* Adjoint of the forward pass in x, written as the transpose of its loop nest:
 * every forward term x[n,iy,ix,c]*Wm[f,c,r,s] -> y[n,oy,ox,f] sends dy[n,oy,ox,f]*Wm[f,c,r,s]
 * back to dx[n,iy,ix,c]. This equals delta (*) rot180(W). */
void orc_conv_bwd_data(const float *dy, const float *Wm, int N, int H, int Wd, int C, int F, int stride, float *dx)
{
    int Ho = out_dim(H, stride), Wo = out_dim(Wd, stride);
#pragma omp parallel for schedule(static)
    for (int n = 0; n < N; ++n) {
        double *acc = (double *)calloc((size_t)H * Wd * C, sizeof(double));
        for (int oy = 0; oy < Ho; ++oy)
            for (int ox = 0; ox < Wo; ++ox)
                for (int f = 0; f < F; ++f) {
                    double d = (double)dy[(((int64_t)n * Ho + oy) * Wo + ox) * F + f];
                    for (int c = 0; c < C; ++c)
                        for (int r = 0; r < 3; ++r)
                            for (int s = 0; s < 3; ++s) {
                                float w = Wm[((int64_t)f * C + c) * 9 + 3 * r + s];
                                if (w == 0.0f) continue;
                                int iy = oy * stride + r - 1, ix = ox * stride + s - 1;
                                if (iy < 0 || iy >= H || ix < 0 || ix >= Wd) continue;
                                acc[((int64_t)iy * Wd + ix) * C + c] += d * (double)w;
                            }
                }
        for (int64_t i = 0; i < (int64_t)H * Wd * C; ++i) dx[(int64_t)n * H * Wd * C + i] = (float)acc[i];
        free(acc);
    }
}

/* One element of dx by the gather form of the same sum (flat NHWC index of dx). */
void orc_conv_bwd_data_at(const float *dy, const float *Wm, int N, int H, int Wd, int C, int F, int stride,
                          const int64_t *idx, int64_t n_idx, float *out)
{
    int Ho = out_dim(H, stride), Wo = out_dim(Wd, stride);
    (void)N;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n_idx; ++i) {
        int64_t q = idx[i];
        int c = (int)(q % C); q /= C;
        int ix = (int)(q % Wd); q /= Wd;
        int iy = (int)(q % H); q /= H;
        int n = (int)q;
        double acc = 0.0;
        for (int oy = 0; oy < Ho; ++oy)
            for (int ox = 0; ox < Wo; ++ox) {
                int r = iy - oy * stride + 1, s = ix - ox * stride + 1;
                if (r < 0 || r > 2 || s < 0 || s > 2) continue;
                for (int f = 0; f < F; ++f)
                    acc += (double)dy[(((int64_t)n * Ho + oy) * Wo + ox) * F + f] *
                           (double)Wm[((int64_t)f * C + c) * 9 + 3 * r + s];
            }
        out[i] = (float)acc;
    }
}

/* dW[f,c,r,s] = M[f,c,r,s] * sum_{n,oy,ox} dy[n,oy,ox,f] * x[n, oy*stride+r-1, ox*stride+s-1, c] */
void orc_conv_bwd_weight(const float *x, const float *dy, const uint8_t *M,
                         int N, int H, int Wd, int C, int F, int stride, float *dW)
{
    int Ho = out_dim(H, stride), Wo = out_dim(Wd, stride);
#pragma omp parallel for collapse(2) schedule(static)
    for (int f = 0; f < F; ++f)
        for (int c = 0; c < C; ++c)
            for (int r = 0; r < 3; ++r)
                for (int s = 0; s < 3; ++s) {
                    int64_t wi = ((int64_t)f * C + c) * 9 + 3 * r + s;
                    if (!M[wi]) { dW[wi] = 0.0f; continue; }
                    double acc = 0.0;
                    for (int n = 0; n < N; ++n)
                        for (int oy = 0; oy < Ho; ++oy) {
                            int iy = oy * stride + r - 1;
                            if (iy < 0 || iy >= H) continue;
                            for (int ox = 0; ox < Wo; ++ox) {
                                int ix = ox * stride + s - 1;
                                if (ix < 0 || ix >= Wd) continue;
                                acc += (double)dy[(((int64_t)n * Ho + oy) * Wo + ox) * F + f] *
                                       (double)x[(((int64_t)n * H + iy) * Wd + ix) * C + c];
                            }
                        }
                    dW[wi] = (float)acc;
                }
}

/* Selected entries of dW only: widx are flat [F][C][9] indices (the mask is not applied here). */
void orc_conv_bwd_weight_at(const float *x, const float *dy, int N, int H, int Wd, int C, int F, int stride,
                            const int64_t *widx, int64_t n_idx, float *out)
{
    int Ho = out_dim(H, stride), Wo = out_dim(Wd, stride);
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t i = 0; i < n_idx; ++i) {
        int64_t q = widx[i];
        int t = (int)(q % 9); q /= 9;
        int c = (int)(q % C); q /= C;
        int f = (int)q;
        int r = t / 3, s = t % 3;
        double acc = 0.0;
        for (int n = 0; n < N; ++n)
            for (int oy = 0; oy < Ho; ++oy) {
                int iy = oy * stride + r - 1;
                if (iy < 0 || iy >= H) continue;
                for (int ox = 0; ox < Wo; ++ox) {
                    int ix = ox * stride + s - 1;
                    if (ix < 0 || ix >= Wd) continue;
                    acc += (double)dy[(((int64_t)n * Ho + oy) * Wo + ox) * F + f] *
                           (double)x[(((int64_t)n * H + iy) * Wd + ix) * C + c];
                }
            }
        out[i] = (float)acc;
    }
}
