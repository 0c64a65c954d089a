/*
 * CPU oracle for the quantised-expert MoE forward with low-rank compensation.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the plain definition of what the HIP library must
 * compute, written for checking, not for speed: fp64 arithmetic over the exact values of the
 * fp16 / bf16 / integer inputs, no blocking, no fusion, no reordering beyond the definition.
 * It shares no code with the HIP path and must never be linked into, or called from, the
 * product library.  Only the tests, the smoke check and the benchmark's cpu_baseline leg use it.
 *
 * What each function follows in the paper (TileQ, arXiv 2605.09281):
 *   - routing and the weighted combination over the selected top-K experts: the MoE forward,
 *     Eq. 3 (Section 3, "Model"), with G(x) the routing scores and g_{b,t} the routing weights
 *     of Section 3.2;
 *   - a projection on "quantised weights + rank-r term": Eq. 2 (Section 2.2) and Eq. 4
 *     (Section 3.1), W ~ Q(W - W_r) + U V, evaluated per expert in the per-expert
 *     ("element-wise") form of Appendix A.3 / A.4, with the input-side scaling s_k and Sigma
 *     already folded into the left factor offline (Algorithm 1);
 *   - group-wise scalar quantisation with one scale per group of g weights: Appendix A.3
 *     ("Basic Quantization");
 *   - orc_moe_forward_shared: the same layer on SHARED 2D-tiled factors (Eq. 4 with the placement table phi),
 *     every projection's low-rank term in the accumulator form of Section 3.2;
 *   - orc_moe_forward_fp8: the layer with fp8 E4M3 factors and an fp16 diagonal Sigma, per-expert or shared tiled;
 *   - orc_lotile_forward: the fused low-rank path over shared 2D-tiled factors, LoTileMoE of
 *     Section 3.2 in its defining three-dimensional accumulator form (the construction that ends
 *     in Eq. 15), NOT the compact buffer of Eq. 16 that an implementation would use;
 *   - orc_lotile_forward_fp8: the same on mixed-precision factors, U and V in fp8 with Sigma kept
 *     in fp16 (end of Section 3.1; Appendix A.3, d_low); the paper names no fp8 format: E4M3 of
 *     the OCP specification is taken.
 * Readings taken where the paper is silent (stated once more in the repository's design notes):
 *   - routing weights are the softmax over the k selected logits (equal to softmax over all
 *     experts renormalised over the selected ones);
 *   - ties between equal logits go to the lower expert index, output in descending score;
 *   - an expert is a SwiGLU MLP: h = silu(gate(x)) * up(x), y = down(h), each of the three
 *     projections independently "quantised + low-rank", the low-rank term added before SiLU;
 *   - row-vector convention y = x W^T with W stored [out, in]; A is [in, r], B is [r, out];
 *   - asymmetric codes: deq = (q - zero) * scale with fp16 scale and fp16 zero per (row, group);
 *   - shared experts see every token with weight exactly 1, outside the top-k normalisation.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

typedef struct {
    int32_t n_experts; /* E, routed */
    int32_t n_shared;  /* S, always on */
    int32_t top_k;
    int32_t hidden;    /* H */
    int32_t ffn;       /* F */
    int32_t group;     /* g */
    int32_t bits;      /* 3 or 4 (informational; codes arrive one per byte) */
    int32_t rank;      /* r, may be 0 */
} orc_layer;

/* IEEE binary16 -> double, written out from the format definition. */
double orc_half_to_double(uint16_t h)
{
    int sign = (h >> 15) & 1;
    int expo = (h >> 10) & 0x1F;
    int mant = h & 0x3FF;
    double v;
    if (expo == 0)
        v = ldexp((double)mant, -24);             /* subnormal: mant * 2^-10 * 2^-14 */
    else if (expo == 31)
        v = mant ? NAN : INFINITY;
    else
        v = ldexp((double)(mant + 1024), expo - 25); /* (1 + mant/1024) * 2^(expo-15) */
    return sign ? -v : v;
}

/* ---------------------------------------------------------------------------------------------
 * Routing (Eq. 3: the selected top-K set and the routing scores).
 * For each token: l = logits (+ bias) in fp32; the k largest by the key (-l, index); weights
 * w_j = exp(l_j - l_max) / sum over the selected k, evaluated in double, stored as fp32.
 * idx is [T, k] in descending score order; w is [T, k].
 */
void orc_route(const float *logits, const float *bias, int32_t T, int32_t E, int32_t k,
               int32_t *idx, float *w)
{
    float *l = (float *)malloc(sizeof(float) * (size_t)E);
    char *taken = (char *)malloc((size_t)E);
    for (int32_t t = 0; t < T; ++t) {
        for (int32_t e = 0; e < E; ++e) {
            float v = logits[(size_t)t * E + e];
            if (bias) v = v + bias[e];     /* one fp32 addition, as the selection is made on fp32 scores */
            l[e] = v;
        }
        memset(taken, 0, (size_t)E);
        /* selection by repeated maximum: the first maximum found scanning upward is the lowest index */
        for (int32_t j = 0; j < k; ++j) {
            int32_t best = -1;
            for (int32_t e = 0; e < E; ++e) {
                if (taken[e]) continue;
                if (best < 0 || l[e] > l[best]) best = e;
            }
            taken[best] = 1;
            idx[(size_t)t * k + j] = best;
        }
        double lmax = (double)l[idx[(size_t)t * k]];
        double den = 0.0;
        for (int32_t j = 0; j < k; ++j) den += exp((double)l[idx[(size_t)t * k + j]] - lmax);
        for (int32_t j = 0; j < k; ++j)
            w[(size_t)t * k + j] = (float)(exp((double)l[idx[(size_t)t * k + j]] - lmax) / den);
    }
    free(l);
    free(taken);
}

/* ---------------------------------------------------------------------------------------------
 * Token -> expert permutation.  Assignment a = t*k + j goes to expert idx[a].  offsets[E+1] is
 * the exclusive prefix sum of the per-expert counts; within one expert, assignments keep their
 * order in a (stable).  slot_of[a] is the position of assignment a in expert-sorted order and
 * src_of[slot] its inverse.
 */
void orc_permute(const int32_t *idx, int32_t T, int32_t E, int32_t k, int32_t *offsets,
                 int32_t *slot_of, int32_t *src_of)
{
    int64_t n = (int64_t)T * k;
    for (int32_t e = 0; e <= E; ++e) offsets[e] = 0;
    for (int64_t a = 0; a < n; ++a) offsets[idx[a] + 1] += 1;
    for (int32_t e = 0; e < E; ++e) offsets[e + 1] += offsets[e];
    int32_t *cursor = (int32_t *)malloc(sizeof(int32_t) * (size_t)E);
    for (int32_t e = 0; e < E; ++e) cursor[e] = offsets[e];
    for (int64_t a = 0; a < n; ++a) {
        int32_t s = cursor[idx[a]]++;
        slot_of[a] = s;
        src_of[s] = (int32_t)a;
    }
    free(cursor);
}

/* ---------------------------------------------------------------------------------------------
 * Dequantisation of one [N, K] matrix: W[n, kk] = (q[n, kk] - zero[n, kk/g]) * scale[n, kk/g].
 */
void orc_dequant(const uint8_t *q, const uint16_t *scale, const uint16_t *zero, int32_t N,
                 int32_t K, int32_t g, double *W)
{
    int32_t G = K / g;
    for (int32_t n = 0; n < N; ++n)
        for (int32_t kk = 0; kk < K; ++kk) {
            double s = orc_half_to_double(scale[(size_t)n * G + kk / g]);
            double z = orc_half_to_double(zero[(size_t)n * G + kk / g]);
            W[(size_t)n * K + kk] = ((double)q[(size_t)n * K + kk] - z) * s;
        }
}

/* ---------------------------------------------------------------------------------------------
 * One projection of one vector (Eq. 2 / Eq. 4 applied to a row vector):
 *   out[n] = sum_kk v[kk] * deq(W)[n, kk]  +  sum_rho ( sum_kk v[kk] * A[kk, rho] ) * B[rho, n]
 * A is [K, r], B is [r, N], both fp16 bit patterns; r may be 0 (then A, B are not read).
 */
void orc_project(const double *v, const uint8_t *q, const uint16_t *scale, const uint16_t *zero,
                 const uint16_t *A, const uint16_t *B, int32_t N, int32_t K, int32_t g, int32_t r,
                 double *out)
{
    int32_t G = K / g;
    double *t = (double *)malloc(sizeof(double) * (size_t)(r > 0 ? r : 1));
    for (int32_t rho = 0; rho < r; ++rho) {
        double acc = 0.0;
        for (int32_t kk = 0; kk < K; ++kk) acc += v[kk] * orc_half_to_double(A[(size_t)kk * r + rho]);
        t[rho] = acc;
    }
#pragma omp parallel for schedule(static)
    for (int32_t n = 0; n < N; ++n) {
        double acc = 0.0;
        for (int32_t gi = 0; gi < G; ++gi) {
            double s = orc_half_to_double(scale[(size_t)n * G + gi]);
            double z = orc_half_to_double(zero[(size_t)n * G + gi]);
            for (int32_t kk = gi * g; kk < (gi + 1) * g; ++kk)
                acc += v[kk] * (((double)q[(size_t)n * K + kk] - z) * s);
        }
        double lr = 0.0;
        for (int32_t rho = 0; rho < r; ++rho) lr += t[rho] * orc_half_to_double(B[(size_t)rho * N + n]);
        out[n] = acc + lr;
    }
    free(t);
}

static double orc_silu(double v) { return v / (1.0 + exp(-v)); }
double orc_silu_export(double v) { return orc_silu(v); }

/* Canonical weight arrays of a whole layer, expert-major (see the layout in the header comment of
 * orc_moe_forward).  Offsets of expert e, projection p (0 gate, 1 up, 2 down). */
typedef struct {
    const uint8_t *codes;  /* [E+S][3][H*F] */
    const uint16_t *scale; /* [E+S][3][H*F/g] */
    const uint16_t *zero;  /* [E+S][3][H*F/g] */
    const uint16_t *A;     /* [E+S][(2H+F)*r]: gate [H,r] | up [H,r] | down [F,r] */
    const uint16_t *B;     /* [E+S][(2F+H)*r]: gate [r,F] | up [r,F] | down [r,H] */
} orc_weights;

/* ---------------------------------------------------------------------------------------------
 * One expert applied to one token: G = proj(x; gate), U = proj(x; up), h = silu(G) * U,
 * y = proj(h; down).  Nothing is rounded in between.
 */
void orc_expert(const orc_layer *L, const orc_weights *Wt, int32_t e, const double *x, double *y,
                double *scratch /* 3*F doubles */)
{
    int32_t H = L->hidden, F = L->ffn, g = L->group, r = L->rank;
    size_t HF = (size_t)H * F, HFg = HF / g;
    const uint8_t *cq = Wt->codes + (size_t)e * 3 * HF;
    const uint16_t *cs = Wt->scale + (size_t)e * 3 * HFg;
    const uint16_t *cz = Wt->zero + (size_t)e * 3 * HFg;
    const uint16_t *Ae = r ? Wt->A + (size_t)e * (2 * (size_t)H + F) * r : NULL;
    const uint16_t *Be = r ? Wt->B + (size_t)e * (2 * (size_t)F + H) * r : NULL;
    double *Gv = scratch, *Uv = scratch + F, *hv = scratch + 2 * (size_t)F;
    orc_project(x, cq, cs, cz, Ae, Be, F, H, g, r, Gv);
    orc_project(x, cq + HF, cs + HFg, cz + HFg, r ? Ae + (size_t)H * r : NULL,
                r ? Be + (size_t)F * r : NULL, F, H, g, r, Uv);
    for (int32_t f = 0; f < F; ++f) hv[f] = orc_silu(Gv[f]) * Uv[f];
    orc_project(hv, cq + 2 * HF, cs + 2 * HFg, cz + 2 * HFg, r ? Ae + 2 * (size_t)H * r : NULL,
                r ? Be + 2 * (size_t)F * r : NULL, H, F, g, r, y);
}

/* ---------------------------------------------------------------------------------------------
 * The MoE layer (Eq. 3) for a list of tokens:
 *   y[t] = sum_j w[t, j] * Expert_{idx[t, j]}(x[t])  +  sum over shared experts s of Expert_s(x[t])
 * x is [T, H] fp32 (the exact values of the bf16 or fp32 activations), idx/w are [T, k].
 * tokens[n_tokens] selects which rows to evaluate (NULL = all T, then n_tokens must equal T);
 * y is [n_tokens, H] in double.  The k terms are added in slot order j = 0..k-1, then the shared
 * experts in index order.  Returns 0, or -1 on an expert index outside [0, E).
 */
int32_t orc_moe_forward(const orc_layer *L, const orc_weights *Wt, const float *x, const int32_t *idx,
                        const float *w, int32_t T, const int32_t *tokens, int32_t n_tokens, double *y)
{
    int32_t H = L->hidden, F = L->ffn, k = L->top_k, E = L->n_experts, S = L->n_shared;
    double *xv = (double *)malloc(sizeof(double) * (size_t)H);
    double *ye = (double *)malloc(sizeof(double) * (size_t)H);
    double *scratch = (double *)malloc(sizeof(double) * 3 * (size_t)F);
    int32_t rc = 0;
    for (int32_t i = 0; i < n_tokens && rc == 0; ++i) {
        int32_t t = tokens ? tokens[i] : i;
        if (t < 0 || t >= T) { rc = -1; break; }
        for (int32_t c = 0; c < H; ++c) xv[c] = (double)x[(size_t)t * H + c];
        double *yt = y + (size_t)i * H;
        for (int32_t c = 0; c < H; ++c) yt[c] = 0.0;
        for (int32_t j = 0; j < k; ++j) {
            int32_t e = idx[(size_t)t * k + j];
            if (e < 0 || e >= E) { rc = -1; break; }
            orc_expert(L, Wt, e, xv, ye, scratch);
            double wj = (double)w[(size_t)t * k + j];
            for (int32_t c = 0; c < H; ++c) yt[c] += wj * ye[c];
        }
        for (int32_t s = 0; s < S && rc == 0; ++s) {
            orc_expert(L, Wt, E + s, xv, ye, scratch);
            for (int32_t c = 0; c < H; ++c) yt[c] += ye[c];
        }
    }
    free(xv);
    free(ye);
    free(scratch);
    return rc;
}

/* ---------------------------------------------------------------------------------------------
 * The layer on SHARED 2D-tiled factors (Section 3.1, Eq. 4: W_k = U_p Sigma V_q + quantised residual,
 * {p, q} = phi(k)), each projection's low-rank term evaluated the way Section 3.2 defines the fused path
 * (the construction ending in Eq. 15), for one vector and one selected expert at a time:
 *   X_proj = v (U Sigma)_reshape, i.e. the vector projected on EVERY row tile's factor   [M][r]
 *   accumulator A [M][r N]: zero, except block n of row m, (m, n) = phi(e), which receives X_proj[m]
 *   out_lr = sum over m of A[m] V_reshape, V_reshape = the N right factors stacked   [r N][N_out]
 * (the routing weight of the selection is applied by the caller, Eq. 3, exactly as for per-expert factors).
 * us is [M][K][r], vv is [N][r][N_out], fp16 bit patterns.
 */
typedef struct {
    const uint16_t *us[3]; /* per projection (gate, up, down): [M][K_p][r] */
    const uint16_t *v[3];  /* per projection: [N][r][N_p] */
    const int32_t *phi;    /* [E+S][2] */
    int32_t M, N;
} orc_shared;

void orc_project_shared(const double *v, const uint8_t *q, const uint16_t *scale, const uint16_t *zero,
                        const uint16_t *us, const uint16_t *vv, int32_t M, int32_t Nt, int32_t m_e, int32_t n_e,
                        int32_t Nout, int32_t K, int32_t g, int32_t r, double *out)
{
    int32_t G = K / g;
    const size_t rN = (size_t)r * Nt;
    double *xproj = (double *)malloc(sizeof(double) * (size_t)M * r);
    double *acc = (double *)calloc((size_t)M * rN, sizeof(double));
    for (int32_t m = 0; m < M; ++m)
        for (int32_t rho = 0; rho < r; ++rho) {
            double a = 0.0;
            for (int32_t kk = 0; kk < K; ++kk) a += v[kk] * orc_half_to_double(us[((size_t)m * K + kk) * r + rho]);
            xproj[(size_t)m * r + rho] = a;
        }
    for (int32_t rho = 0; rho < r; ++rho) acc[(size_t)m_e * rN + (size_t)n_e * r + rho] += xproj[(size_t)m_e * r + rho];
#pragma omp parallel for schedule(static)
    for (int32_t n = 0; n < Nout; ++n) {
        double a = 0.0;
        for (int32_t gi = 0; gi < G; ++gi) {
            double s = orc_half_to_double(scale[(size_t)n * G + gi]);
            double z = orc_half_to_double(zero[(size_t)n * G + gi]);
            for (int32_t kk = gi * g; kk < (gi + 1) * g; ++kk)
                a += v[kk] * (((double)q[(size_t)n * K + kk] - z) * s);
        }
        double lr = 0.0;
        for (int32_t m = 0; m < M; ++m)
            for (int32_t nt = 0; nt < Nt; ++nt)
                for (int32_t rho = 0; rho < r; ++rho)
                    lr += acc[(size_t)m * rN + (size_t)nt * r + rho] * orc_half_to_double(vv[((size_t)nt * r + rho) * Nout + n]);
        out[n] = a + lr;
    }
    free(xproj);
    free(acc);
}

/* Eq. 3 over experts whose three projections use the shared factors; same conventions as orc_moe_forward
 * (Wt->A and Wt->B are not read). */
int32_t orc_moe_forward_shared(const orc_layer *L, const orc_weights *Wt, const orc_shared *Sh, const float *x,
                               const int32_t *idx, const float *w, int32_t T, const int32_t *tokens,
                               int32_t n_tokens, double *y)
{
    int32_t H = L->hidden, F = L->ffn, k = L->top_k, E = L->n_experts, S = L->n_shared, g = L->group, r = L->rank;
    size_t HF = (size_t)H * F, HFg = HF / g;
    double *xv = (double *)malloc(sizeof(double) * (size_t)H);
    double *ye = (double *)malloc(sizeof(double) * (size_t)H);
    double *Gv = (double *)malloc(sizeof(double) * 3 * (size_t)F), *Uv = Gv + F, *hv = Gv + 2 * (size_t)F;
    int32_t rc = 0;
    for (int32_t i = 0; i < n_tokens && rc == 0; ++i) {
        int32_t t = tokens ? tokens[i] : i;
        if (t < 0 || t >= T) { rc = -1; break; }
        for (int32_t c = 0; c < H; ++c) xv[c] = (double)x[(size_t)t * H + c];
        double *yt = y + (size_t)i * H;
        for (int32_t c = 0; c < H; ++c) yt[c] = 0.0;
        for (int32_t j = 0; j < k + S; ++j) {
            int32_t e = j < k ? idx[(size_t)t * k + j] : E + (j - k);
            if (j < k && (e < 0 || e >= E)) { rc = -1; break; }
            int32_t m_e = Sh->phi[2 * e], n_e = Sh->phi[2 * e + 1];
            if (m_e < 0 || m_e >= Sh->M || n_e < 0 || n_e >= Sh->N) { rc = -1; break; }
            const uint8_t *cq = Wt->codes + (size_t)e * 3 * HF;
            const uint16_t *cs = Wt->scale + (size_t)e * 3 * HFg, *cz = Wt->zero + (size_t)e * 3 * HFg;
            orc_project_shared(xv, cq, cs, cz, Sh->us[0], Sh->v[0], Sh->M, Sh->N, m_e, n_e, F, H, g, r, Gv);
            orc_project_shared(xv, cq + HF, cs + HFg, cz + HFg, Sh->us[1], Sh->v[1], Sh->M, Sh->N, m_e, n_e, F, H, g, r, Uv);
            for (int32_t f = 0; f < F; ++f) hv[f] = orc_silu(Gv[f]) * Uv[f];
            orc_project_shared(hv, cq + 2 * HF, cs + 2 * HFg, cz + 2 * HFg, Sh->us[2], Sh->v[2], Sh->M, Sh->N, m_e, n_e, H, F, g, r, ye);
            double wj = j < k ? (double)w[(size_t)t * k + j] : 1.0;
            for (int32_t c = 0; c < H; ++c) yt[c] += wj * ye[c];
        }
    }
    free(xv);
    free(ye);
    free(Gv);
    return rc;
}

/* ---------------------------------------------------------------------------------------------
 * The layer with mixed-precision factors (end of Section 3.1; Appendix A.3 with d_low = 8): the factors are fp8 E4M3
 * codes and a diagonal Sigma in fp16 carries the magnitude.  A projection's low-rank term is
 *     ((v fp8(A8)) * sigma) fp8(B8),
 * everything else as orc_moe_forward.  One routine for both factor formats: per projection p the left factors are
 * a8[p] [nA][K_p][r] and the right factors b8[p] [nB][r][N_p]; with phi == NULL expert e uses block e of both and
 * sigma [E+S][3][r] (per-expert factors), otherwise blocks phi[e] = (m, n) and one sigma [3][r] (shared tiled factors).
 */
double orc_fp8_e4m3_to_double(uint8_t b);      /* the format's decode, defined with the shared-factor operator below */

static void orc_project_fp8(const double *v, const uint8_t *q, const uint16_t *scale, const uint16_t *zero,
                            const uint8_t *A8, const uint16_t *sigma, const uint8_t *B8, int32_t N, int32_t K, int32_t g,
                            int32_t r, double *out)
{
    int32_t G = K / g;
    double *t = (double *)malloc(sizeof(double) * (size_t)r);
    for (int32_t rho = 0; rho < r; ++rho) {
        double acc = 0.0;
        for (int32_t kk = 0; kk < K; ++kk) acc += v[kk] * orc_fp8_e4m3_to_double(A8[(size_t)kk * r + rho]);
        t[rho] = acc * orc_half_to_double(sigma[rho]);
    }
#pragma omp parallel for schedule(static)
    for (int32_t n = 0; n < N; ++n) {
        double acc = 0.0;
        for (int32_t gi = 0; gi < G; ++gi) {
            double s = orc_half_to_double(scale[(size_t)n * G + gi]);
            double z = orc_half_to_double(zero[(size_t)n * G + gi]);
            for (int32_t kk = gi * g; kk < (gi + 1) * g; ++kk)
                acc += v[kk] * (((double)q[(size_t)n * K + kk] - z) * s);
        }
        double lr = 0.0;
        for (int32_t rho = 0; rho < r; ++rho) lr += t[rho] * orc_fp8_e4m3_to_double(B8[(size_t)rho * N + n]);
        out[n] = acc + lr;
    }
    free(t);
}

int32_t orc_moe_forward_fp8(const orc_layer *L, const uint8_t *codes, const uint16_t *scale, const uint16_t *zero,
                            const uint8_t *const *a8, const uint8_t *const *b8, const uint16_t *sigma,
                            const int32_t *phi, int32_t M, int32_t Nt, const float *x, const int32_t *idx, const float *w,
                            int32_t T, const int32_t *tokens, int32_t n_tokens, double *y)
{
    int32_t H = L->hidden, F = L->ffn, k = L->top_k, E = L->n_experts, S = L->n_shared, g = L->group, r = L->rank;
    size_t HF = (size_t)H * F, HFg = HF / g;
    const int32_t Kp[3] = {H, H, F}, Np[3] = {F, F, H};
    double *xv = (double *)malloc(sizeof(double) * (size_t)H);
    double *ye = (double *)malloc(sizeof(double) * (size_t)H);
    double *buf = (double *)malloc(sizeof(double) * 3 * (size_t)F);
    double *Gv = buf, *Uv = buf + F, *hv = buf + 2 * (size_t)F;
    int32_t rc = 0;
    if (r < 1) rc = -1;
    for (int32_t i = 0; i < n_tokens && rc == 0; ++i) {
        int32_t t = tokens ? tokens[i] : i;
        if (t < 0 || t >= T) { rc = -1; break; }
        for (int32_t c = 0; c < H; ++c) xv[c] = (double)x[(size_t)t * H + c];
        double *yt = y + (size_t)i * H;
        for (int32_t c = 0; c < H; ++c) yt[c] = 0.0;
        for (int32_t j = 0; j < k + S; ++j) {
            int32_t e = j < k ? idx[(size_t)t * k + j] : E + (j - k);
            if (j < k && (e < 0 || e >= E)) { rc = -1; break; }
            int32_t ma = e, nb = e;
            if (phi) {
                ma = phi[2 * e]; nb = phi[2 * e + 1];
                if (ma < 0 || ma >= M || nb < 0 || nb >= Nt) { rc = -1; break; }
            }
            double *dst[3] = {Gv, Uv, ye};
            for (int32_t p = 0; p < 3; ++p) {
                const uint8_t *A8 = a8[p] + (size_t)ma * Kp[p] * r;
                const uint8_t *B8 = b8[p] + (size_t)nb * r * Np[p];
                const uint16_t *sg = phi ? sigma + (size_t)p * r : sigma + ((size_t)e * 3 + p) * r;
                if (p == 2)
                    for (int32_t f = 0; f < F; ++f) hv[f] = orc_silu(Gv[f]) * Uv[f];
                orc_project_fp8(p == 2 ? hv : xv, codes + ((size_t)e * 3 + p) * HF, scale + ((size_t)e * 3 + p) * HFg,
                                zero + ((size_t)e * 3 + p) * HFg, A8, sg, B8, Np[p], Kp[p], g, r, dst[p]);
            }
            double wj = j < k ? (double)w[(size_t)t * k + j] : 1.0;
            for (int32_t c = 0; c < H; ++c) yt[c] += wj * ye[c];
        }
    }
    free(xv);
    free(ye);
    free(buf);
    return rc;
}

#ifdef _OPENMP
#include <omp.h>
int32_t orc_num_threads(void) { return omp_get_max_threads(); }
void orc_set_num_threads(int32_t n) { omp_set_num_threads(n); }
#else
int32_t orc_num_threads(void) { return 1; }
void orc_set_num_threads(int32_t n) { (void)n; }
#endif

/*
 * LoTileMoE (Section 3.2, the construction ending in Eq. 15; complexity in Appendix A.4), one linear
 * map with an input shared by all experts:
 *   x     [T][in]            activations (fp32 holding the values)
 *   us    [M][in][r]  fp16   row-tile factors U_m Sigma  (the "(U Sigma)_reshape" of step one is us
 *                            viewed as [in][M r])
 *   v     [N][r][out] fp16   column-tile factors V_n     ("V_flat" is v viewed as [N r][out])
 *   phi   [E][2]             expert -> (m, n)
 *   idx,w [T][k]             selected experts and routing weights g_{b,t}
 *   y     [T][out]           LoTileMoE(x)
 * Steps, in the paper's order: X_proj = x (U Sigma)_reshape; X_tile = X_proj reshaped [T][M][r] and
 * repeated N times along the last axis; the accumulator A [T][M][r N] is zero except that, for every
 * (b, t), block n_{b,t} of row m_{b,t} receives g_{b,t} times the same block of X_tile (a second
 * selection of the same tile by the same token adds to it - the paper's arrow leaves this open;
 * with distinct top-k experts it cannot happen); Y3 = A V_reshape per row tile; y = sum over m.
 */
void orc_lotile_forward(int32_t T, int32_t n_in, int32_t n_out, int32_t M, int32_t N, int32_t r, int32_t k,
                        const float *x, const uint16_t *us, const uint16_t *v, const int32_t *phi,
                        const int32_t *idx, const float *w, double *y)
{
    const size_t Mr = (size_t)M * r, rN = (size_t)r * N;
    double *xproj = (double *)malloc(sizeof(double) * Mr);
    double *acc = (double *)malloc(sizeof(double) * (size_t)M * rN);
    for (int32_t b = 0; b < T; ++b) {
        /* step one: projection on every row tile's factor */
        for (int32_t m = 0; m < M; ++m)
            for (int32_t rho = 0; rho < r; ++rho) {
                double a = 0.0;
                for (int32_t i = 0; i < n_in; ++i)
                    a += (double)x[(size_t)b * n_in + i] * orc_half_to_double(us[((size_t)m * n_in + i) * r + rho]);
                xproj[(size_t)m * r + rho] = a;
            }
        /* the accumulator: routing-weighted copies of X_tile at the active tiles only */
        memset(acc, 0, sizeof(double) * (size_t)M * rN);
        for (int32_t t = 0; t < k; ++t) {
            const int32_t e = idx[(size_t)b * k + t];
            const int32_t m = phi[2 * e], n = phi[2 * e + 1];
            for (int32_t rho = 0; rho < r; ++rho)
                acc[(size_t)m * rN + (size_t)n * r + rho] += (double)w[(size_t)b * k + t] * xproj[(size_t)m * r + rho];
        }
        /* batched product with the reshaped V, then the sum over row tiles */
        for (int32_t o = 0; o < n_out; ++o) y[(size_t)b * n_out + o] = 0.0;
        for (int32_t m = 0; m < M; ++m)
            for (int32_t n = 0; n < N; ++n)
                for (int32_t rho = 0; rho < r; ++rho) {
                    const double a = acc[(size_t)m * rN + (size_t)n * r + rho];
                    if (a == 0.0) continue;       /* zero entries add nothing (keeps the brute force usable) */
                    for (int32_t o = 0; o < n_out; ++o)
                        y[(size_t)b * n_out + o] += a * orc_half_to_double(v[((size_t)n * r + rho) * n_out + o]);
                }
    }
    free(xproj);
    free(acc);
}


/*
 * fp8 E4M3 as published in the OCP 8-bit floating point specification ("E4M3", the variant without
 * infinities): 1 sign, 4 exponent (bias 7), 3 mantissa bits; exponent 0 is subnormal (m / 8 * 2^-6);
 * S.1111.111 is NaN; the largest finite value is 448.
 */
double orc_fp8_e4m3_to_double(uint8_t b)
{
    const int sign = b >> 7, e = (b >> 3) & 15, m = b & 7;
    double v;
    if (e == 15 && m == 7) return NAN;
    if (e == 0) v = ldexp((double)m, -9);
    else v = ldexp(1.0 + (double)m / 8.0, e - 7);
    return sign ? -v : v;
}

/*
 * LoTileMoE on mixed-precision factors (end of Section 3.1: U and V stored in fp8, Sigma kept in fp16;
 * Appendix A.3 d_low = 8 bits).  Same construction and order as orc_lotile_forward with
 *   u8    [M][in][r]  fp8    row-tile factors U_m
 *   sigma [r]         fp16   the diagonal of the rank-r factorisation, shared by all tiles
 *   v8    [N][r][out] fp8    column-tile factors V_n
 * and U_m Sigma formed in fp64 from the decoded values: X_proj = x (U diag(sigma))_reshape.
 */
void orc_lotile_forward_fp8(int32_t T, int32_t n_in, int32_t n_out, int32_t M, int32_t N, int32_t r, int32_t k,
                            const float *x, const uint8_t *u8, const uint16_t *sigma, const uint8_t *v8,
                            const int32_t *phi, const int32_t *idx, const float *w, double *y)
{
    const size_t Mr = (size_t)M * r, rN = (size_t)r * N;
    double *xproj = (double *)malloc(sizeof(double) * Mr);
    double *acc = (double *)malloc(sizeof(double) * (size_t)M * rN);
    for (int32_t b = 0; b < T; ++b) {
        for (int32_t m = 0; m < M; ++m)
            for (int32_t rho = 0; rho < r; ++rho) {
                const double sg = orc_half_to_double(sigma[rho]);
                double a = 0.0;
                for (int32_t i = 0; i < n_in; ++i)
                    a += (double)x[(size_t)b * n_in + i] * (orc_fp8_e4m3_to_double(u8[((size_t)m * n_in + i) * r + rho]) * sg);
                xproj[(size_t)m * r + rho] = a;
            }
        memset(acc, 0, sizeof(double) * (size_t)M * rN);
        for (int32_t t = 0; t < k; ++t) {
            const int32_t e = idx[(size_t)b * k + t];
            const int32_t m = phi[2 * e], n = phi[2 * e + 1];
            for (int32_t rho = 0; rho < r; ++rho)
                acc[(size_t)m * rN + (size_t)n * r + rho] += (double)w[(size_t)b * k + t] * xproj[(size_t)m * r + rho];
        }
        for (int32_t o = 0; o < n_out; ++o) y[(size_t)b * n_out + o] = 0.0;
        for (int32_t m = 0; m < M; ++m)
            for (int32_t n = 0; n < N; ++n)
                for (int32_t rho = 0; rho < r; ++rho) {
                    const double a = acc[(size_t)m * rN + (size_t)n * r + rho];
                    if (a == 0.0) continue;
                    for (int32_t o = 0; o < n_out; ++o)
                        y[(size_t)b * n_out + o] += a * orc_fp8_e4m3_to_double(v8[((size_t)n * r + rho) * n_out + o]);
                }
    }
    free(xproj);
    free(acc);
}
