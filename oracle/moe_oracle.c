/*
 * moe_oracle.c -- TEST INFRASTRUCTURE, not part of the product.
 *
 * A plain, slow, fp64 CPU statement of what one Mixture-of-Experts FFN layer
 * computes and of the two prefill schedules (chunked, layered) that drive a
 * contiguous layer group over a mixed decode+prefill batch.  It exists only so
 * that tests, the smoke check and the benchmark's cpu_baseline leg can compare
 * the GPU library against the definition.  It shares no code with the GPU
 * library and nothing in the product path may call it.
 *
 * Passages followed (layered-prefill paper):
 *   - MoE layer = a router that assigns each token to a small subset (top-k)
 *     of independent expert FFNs: Sec. 1 and Sec. 2.4 ("Mixture of Experts").
 *   - Expert FFN = fully connected layers with a SwiGLU non-linearity, the
 *     first expanding the hidden size, the last projecting back: Sec. 2.1.
 *   - Hybrid batch of decode tokens plus prefill tokens: Sec. 2.3, Sec. 3.1.
 *   - Chunked prefill (one token chunk per iteration through all layers of
 *     the group, together with the decode batch): Sec. 2.3, Fig. 1 (upper).
 *   - Layered prefill (the whole prompt crosses the layer group once, decode
 *     tokens riding along): Sec. 4.1, Sec. 4.2, Fig. 1 (lower).
 *   - Expert-weight load bytes (an expert's parameters are counted every time
 *     they are brought in for execution, prefill or decode): Sec. 5.4.
 *   - A whole layer stack cut into contiguous layer groups, one group per
 *     iteration doing prefill and decode while the others do decode only:
 *     Sec. 4.1, Sec. 4.2; combined with chunking along the tokens: Sec. 4.3;
 *     the number of groups for a prompt length: Sec. 4.4.
 *
 * The paper does not print the layer's arithmetic.  The readings used here:
 * selection on raw logits, ties to the lower expert index, selected experts
 * ordered by (logit descending, index ascending); mixing weights = softmax
 * over all E logits, restricted to the selected k and (optionally) divided by
 * their sum; gate_up rows [0,I) are the gate, [I,2I) the up projection;
 * silu(v) = v / (1 + exp(-v)); layers inside a group are linked by
 * x <- x + MoE(x) when `residual` is set.
 *
 * Every function is the definition written out token by token, with every sum
 * taken in ascending index order; there is no blocking, fusion or permutation
 * on the value path.
 *
 * parity unpinned by the paper: it prints no worked numerical example of a
 * layer output.  The functions are pinned instead by closed forms, special
 * cases that reduce to library routines, invariants and brute force (see the
 * CPU tests).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORC_F64 = 0, ORC_F32 = 1, ORC_BF16 = 2, ORC_MXFP4 = 3 /* expert weights only */ };
enum { ORC_OK = 0, ORC_ERR_ARG = 1, ORC_ERR_NONFINITE = 2, ORC_ERR_ALLOC = 3 };
enum { ORC_SCHED_CHUNKED = 0, ORC_SCHED_LAYERED = 1 };

/* Exact widening of one stored element to double. */
static inline double ld(const void *p, int dt, int64_t i)
{
    if (dt == ORC_F64) return ((const double *)p)[i];
    if (dt == ORC_F32) return (double)((const float *)p)[i];
    uint32_t bits = ((uint32_t)((const uint16_t *)p)[i]) << 16;
    float f;
    memcpy(&f, &bits, 4);
    return (double)f;
}

int orc_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/*
 * Round a double to the nearest value representable with `sig` significant
 * bits and a minimum exponent `emin` (value of the least normal = 2^emin),
 * ties to even: sig=8, emin=-126 is bfloat16; sig=24, emin=-126 is binary32.
 * The result is returned as a double.  Overflow gives +-inf.
 */
static double round_to_format(double v, int sig, int emin, int emax)
{
    if (v == 0.0 || !isfinite(v)) return v;
    int e;
    (void)frexp(v, &e);          /* |v| = m * 2^e, m in [0.5, 1) */
    int lsb = e - sig;           /* exponent of the last kept bit */
    if (lsb < emin - (sig - 1)) lsb = emin - (sig - 1);   /* subnormal range */
    double q = nearbyint(ldexp(v, -lsb));                 /* ties to even */
    double r = ldexp(q, lsb);
    if (fabs(r) >= ldexp(1.0, emax + 1)) return v > 0 ? INFINITY : -INFINITY;
    return r;
}

double orc_round_bf16(double v) { return round_to_format(v, 8, -126, 127); }
double orc_round_f32(double v) { return round_to_format(v, 24, -126, 127); }

/* The same, element by element over an array (fmt: ORC_BF16 or ORC_F32; anything else copies). */
void orc_round_array(const double *in, int64_t n, int fmt, double *out)
{
    for (int64_t i = 0; i < n; ++i)
        out[i] = (fmt == ORC_BF16) ? orc_round_bf16(in[i]) : (fmt == ORC_F32) ? orc_round_f32(in[i]) : in[i];
}

/* ------------------------------------------------------------------------
 * Router for one token (Sec. 2.4): logits, top-k selection, mixing weights.
 * z must have room for E doubles.  Returns ORC_ERR_NONFINITE on a NaN/inf
 * logit.  `gap` (optional) receives the smallest difference between
 * neighbouring logits among the k selected ones and the best rejected one:
 * how close this token is to a different routing decision.
 * ---------------------------------------------------------------------- */
static int route_token(const double *xt, int64_t H, const void *Wr, int wdt, const float *bias,
                       int E, int k, int renorm, double *z, int32_t *idx, double *w, double *gap)
{
    for (int e = 0; e < E; ++e) {
        double s = 0.0;
        for (int64_t h = 0; h < H; ++h) s += xt[h] * ld(Wr, wdt, (int64_t)e * H + h);
        if (bias) s += (double)bias[e];
        if (!isfinite(s)) return ORC_ERR_NONFINITE;
        z[e] = s;
    }
    /* k rounds of "largest logit not yet taken"; scanning e upwards with a
     * strict comparison gives ties to the lower index. */
    for (int j = 0; j < k; ++j) {
        int best = -1;
        for (int e = 0; e < E; ++e) {
            int taken = 0;
            for (int i = 0; i < j; ++i) taken |= (idx[i] == e);
            if (taken) continue;
            if (best < 0 || z[e] > z[best]) best = e;
        }
        idx[j] = best;
    }
    double m = z[0];
    for (int e = 1; e < E; ++e) if (z[e] > m) m = z[e];
    double denom = 0.0;
    for (int e = 0; e < E; ++e) denom += exp(z[e] - m);
    double sel = 0.0;
    for (int j = 0; j < k; ++j) { w[j] = exp(z[idx[j]] - m) / denom; sel += w[j]; }
    if (renorm) for (int j = 0; j < k; ++j) w[j] /= sel;
    if (gap) {
        double g = INFINITY;
        for (int j = 0; j + 1 < k; ++j) {
            double d = z[idx[j]] - z[idx[j + 1]];
            if (d < g) g = d;
        }
        if (k < E) {
            int best = -1;
            for (int e = 0; e < E; ++e) {
                int taken = 0;
                for (int i = 0; i < k; ++i) taken |= (idx[i] == e);
                if (taken) continue;
                if (best < 0 || z[e] > z[best]) best = e;
            }
            double d = z[idx[k - 1]] - z[best];
            if (d < g) g = d;
        }
        *gap = g;
    }
    return ORC_OK;
}

/*
 * x [T,H] (xdt), Wr [E,H] (wdt), bias [E] fp32 or NULL ->
 * idx [T,k] int32, w [T,k] f64, logits [T,E] f64 (optional), gap [T] (optional).
 */
int orc_router_topk(const void *x, int xdt, int64_t T, int64_t H, const void *Wr, int wdt,
                    const float *bias, int E, int k, int renorm,
                    int32_t *idx, double *w, double *logits, double *gap)
{
    if (T < 0 || H <= 0 || E <= 0 || k <= 0 || k > E) return ORC_ERR_ARG;
    int status = ORC_OK;
#pragma omp parallel
    {
        double *xt = (double *)malloc(sizeof(double) * (size_t)H);
        double *z = (double *)malloc(sizeof(double) * (size_t)E);
#pragma omp for schedule(static)
        for (int64_t t = 0; t < T; ++t) {
            for (int64_t h = 0; h < H; ++h) xt[h] = ld(x, xdt, t * H + h);
            int rc = route_token(xt, H, Wr, wdt, bias, E, k, renorm, z, idx + t * k, w + t * k,
                                 gap ? gap + t : NULL);
            if (rc != ORC_OK) {
#pragma omp atomic write
                status = rc;
            }
            if (logits) memcpy(logits + t * E, z, sizeof(double) * (size_t)E);
        }
        free(xt);
        free(z);
    }
    return status;
}

/*
 * Token permutation: the assignments (t, j) listed by expert, then token, then
 * slot.  counts [E], offsets [E+1] (exclusive running sum), perm [T*k] with
 * perm[r] = t*k + j, inv [T*k] with inv[perm[r]] = r.  Written as the
 * definition: one pass over all assignments per expert.
 */
int orc_permute(const int32_t *idx, int64_t T, int k, int E,
                int32_t *counts, int32_t *offsets, int32_t *perm, int32_t *inv)
{
    if (T < 0 || k <= 0 || E <= 0) return ORC_ERR_ARG;
    for (int64_t f = 0; f < T * k; ++f)
        if (idx[f] < 0 || idx[f] >= E) return ORC_ERR_ARG;
    int64_t r = 0;
    for (int e = 0; e < E; ++e) {
        offsets[e] = (int32_t)r;
        for (int64_t t = 0; t < T; ++t)
            for (int j = 0; j < k; ++j)
                if (idx[t * k + j] == e) {
                    perm[r] = (int32_t)(t * k + j);
                    inv[t * k + j] = (int32_t)r;
                    ++r;
                }
        counts[e] = (int32_t)r - offsets[e];
    }
    offsets[E] = (int32_t)r;
    return ORC_OK;
}

/*
 * 4-bit expert weights (the paper's broader validation runs a model with fp4 expert weights, Table 7).
 * The format is the published OCP Microscaling MXFP4: elements are FP4 E2M1 (1 sign, 2 exponent, 1
 * mantissa bit: magnitudes 0, 0.5, 1, 1.5, 2, 3, 4, 6), two per byte with the even element in the low
 * nibble; each run of 32 consecutive elements shares one E8M0 scale byte s, worth 2^(s - 127) (s = 255 is
 * not a number and is rejected by the callers' finiteness check downstream).
 * Element i of a tensor: code nibble i, scale byte i / 32 (rows are multiples of 32 long).
 */
double orc_mxfp4_element(const uint8_t *codes, const uint8_t *scales, int64_t i)
{
    static const double mag[8] = {0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0};
    const unsigned c = (codes[i >> 1] >> ((i & 1) * 4)) & 15u;
    const double v = (c & 8u) ? -mag[c & 7u] : mag[c & 7u];
    return ldexp(v, (int)scales[i >> 5] - 127);
}

void orc_mxfp4_dequant(const uint8_t *codes, const uint8_t *scales, int64_t n, double *out)
{
    for (int64_t i = 0; i < n; ++i) out[i] = orc_mxfp4_element(codes, scales, i);
}

/* Expert-weight element i: plain formats through ld(), MXFP4 through its codes and scales. */
static inline double ldw(const void *p, const uint8_t *scales, int dt, int64_t i)
{
    return dt == ORC_MXFP4 ? orc_mxfp4_element((const uint8_t *)p, scales, i) : ld(p, dt, i);
}

/* One expert FFN applied to one token (Sec. 2.1): o = Wd * (silu(Wg x) . Wu x). */
static void expert_token(const double *xt, int64_t H, int64_t I, const void *Wgu, const uint8_t *Sgu,
                         const void *Wd, const uint8_t *Sd, int wdt, int e, double *a, double *o)
{
    const int64_t gu0 = (int64_t)e * 2 * I * H;
    for (int64_t i = 0; i < I; ++i) {
        double g = 0.0, u = 0.0;
        for (int64_t h = 0; h < H; ++h) g += ldw(Wgu, Sgu, wdt, gu0 + i * H + h) * xt[h];
        for (int64_t h = 0; h < H; ++h) u += ldw(Wgu, Sgu, wdt, gu0 + (I + i) * H + h) * xt[h];
        a[i] = g / (1.0 + exp(-g)) * u;
    }
    const int64_t d0 = (int64_t)e * H * I;
    for (int64_t h = 0; h < H; ++h) {
        double s = 0.0;
        for (int64_t i = 0; i < I; ++i) s += ldw(Wd, Sd, wdt, d0 + h * I + i) * a[i];
        o[h] = s;
    }
}

/*
 * One MoE layer over T independent tokens.
 *   x [T,H] (xdt); Wr [E,H], Wgu [E,2I,H], Wd [E,H,I] (all wdt); bias [E] fp32 or NULL
 *   y [T,H] f64 = sum_j w[t,j] * expert_{idx[t,j]}(x_t)  (+ x_t when residual != 0)
 *   idx [T,k], w [T,k] f64 are also returned (either may be NULL).
 *   y_mag [T,H] (optional): sum_j w[t,j] * |expert output| (+ |x_t|), the magnitude of the terms y is
 *   made of; a caller uses it to size the rounding budget of a reduced-precision implementation.
 */
int orc_moe_layer_q(const void *x, int xdt, int64_t T, int64_t H,
                    const void *Wr, int rdt, const float *bias, const void *Wgu, const uint8_t *Sgu,
                    const void *Wd, const uint8_t *Sd, int wdt,
                    int E, int k, int64_t I, int renorm, int residual,
                    double *y, int32_t *idx_out, double *w_out, double *y_mag);

int orc_moe_layer(const void *x, int xdt, int64_t T, int64_t H,
                  const void *Wr, const float *bias, const void *Wgu, const void *Wd, int wdt,
                  int E, int k, int64_t I, int renorm, int residual,
                  double *y, int32_t *idx_out, double *w_out, double *y_mag)
{
    return orc_moe_layer_q(x, xdt, T, H, Wr, wdt, bias, Wgu, NULL, Wd, NULL, wdt, E, k, I, renorm, residual,
                           y, idx_out, w_out, y_mag);
}

/*
 * The same layer with the expert weights in their own format: wdt may be ORC_MXFP4, with Wgu / Wd the
 * packed codes and Sgu / Sd the scale bytes (H and I multiples of 32); the router weights Wr stay in rdt.
 */
int orc_moe_layer_q(const void *x, int xdt, int64_t T, int64_t H,
                    const void *Wr, int rdt, const float *bias, const void *Wgu, const uint8_t *Sgu,
                    const void *Wd, const uint8_t *Sd, int wdt,
                    int E, int k, int64_t I, int renorm, int residual,
                    double *y, int32_t *idx_out, double *w_out, double *y_mag)
{
    if (T < 0 || H <= 0 || I <= 0 || E <= 0 || k <= 0 || k > E) return ORC_ERR_ARG;
    if (rdt == ORC_MXFP4) return ORC_ERR_ARG;
    if (wdt == ORC_MXFP4 && (!Sgu || !Sd || H % 32 || I % 32)) return ORC_ERR_ARG;
    if (wdt == ORC_MXFP4) {      /* scale byte 255 is the format's not-a-number */
        const int64_t n_gu = (int64_t)E * 2 * I * H / 32, n_d = (int64_t)E * H * I / 32;
        for (int64_t i = 0; i < n_gu; ++i) if (Sgu[i] == 255) return ORC_ERR_NONFINITE;
        for (int64_t i = 0; i < n_d; ++i) if (Sd[i] == 255) return ORC_ERR_NONFINITE;
    }
    int status = ORC_OK;
#pragma omp parallel
    {
        double *xt = (double *)malloc(sizeof(double) * (size_t)H);
        double *z = (double *)malloc(sizeof(double) * (size_t)E);
        double *a = (double *)malloc(sizeof(double) * (size_t)I);
        double *o = (double *)malloc(sizeof(double) * (size_t)H);
        double *w = (double *)malloc(sizeof(double) * (size_t)k);
        int32_t *idx = (int32_t *)malloc(sizeof(int32_t) * (size_t)k);
#pragma omp for schedule(dynamic, 1)
        for (int64_t t = 0; t < T; ++t) {
            for (int64_t h = 0; h < H; ++h) xt[h] = ld(x, xdt, t * H + h);
            int rc = route_token(xt, H, Wr, rdt, bias, E, k, renorm, z, idx, w, NULL);
            if (rc != ORC_OK) {
#pragma omp atomic write
                status = rc;
                continue;
            }
            double *yt = y + t * H;
            double *mt = y_mag ? y_mag + t * H : NULL;
            for (int64_t h = 0; h < H; ++h) yt[h] = 0.0;
            if (mt) for (int64_t h = 0; h < H; ++h) mt[h] = 0.0;
            for (int j = 0; j < k; ++j) {
                expert_token(xt, H, I, Wgu, Sgu, Wd, Sd, wdt, idx[j], a, o);
                for (int64_t h = 0; h < H; ++h) yt[h] += w[j] * o[h];
                if (mt) for (int64_t h = 0; h < H; ++h) mt[h] += w[j] * fabs(o[h]);
            }
            if (residual) for (int64_t h = 0; h < H; ++h) yt[h] += xt[h];
            if (residual && mt) for (int64_t h = 0; h < H; ++h) mt[h] += fabs(xt[h]);
            if (idx_out) memcpy(idx_out + t * k, idx, sizeof(int32_t) * (size_t)k);
            if (w_out) memcpy(w_out + t * k, w, sizeof(double) * (size_t)k);
        }
        free(xt); free(z); free(a); free(o); free(w); free(idx);
    }
    return status;
}

/* Counters of the expert-weight traffic model (Sec. 5.4; Fig. 2 caption). */
typedef struct {
    uint64_t expert_bytes;          /* sum over (iteration, layer) of active experts * 3*H*I*sz */
    uint64_t router_bytes;          /* sum over (iteration, layer) of E*H*sz */
    uint64_t active_experts_total;  /* sum over (iteration, layer) of #experts with >= 1 token */
    uint64_t tokens_processed;      /* sum over iterations of the batch size T_it */
    uint32_t iterations;
    uint32_t layer_passes;          /* iterations * n_layers */
} orc_counters;

/*
 * A contiguous layer group driven by one of the two schedules.
 *
 *   layered:    one iteration over the batch [decode rows; all P prefill rows].
 *   chunked(C): ceil(P/C) iterations; iteration c runs the batch
 *               [decode rows; prefill rows c*C .. min((c+1)*C, P)) through all
 *               layers of the group.  The same decode rows accompany every
 *               chunk (their result is the same each time, tokens being
 *               independent).  P = 0 gives exactly one decode-only iteration
 *               under either schedule.
 *
 * Inside an iteration: for each layer, xb <- MoE_l(xb) (+ xb when residual),
 * and between layers xb is rounded to the activation format `act_dt`
 * (ORC_BF16 / ORC_F32; ORC_F64 = no rounding) so that the next layer sees a
 * representable input.  The last layer's output is returned unrounded.
 *
 * Wr/bias/Wgu/Wd are arrays of n_layers pointers (bias entries may be NULL,
 * or bias itself NULL).  y_decode [D,H], y_prefill [P,H] are f64.
 * idx_trace (optional) receives the routing of every (iteration, layer, row):
 * rows are appended in execution order, k entries per row.
 */
int orc_group_forward(const void *const *Wr, const float *const *bias,
                      const void *const *Wgu, const void *const *Wd, int wdt, int n_layers,
                      int64_t H, int E, int k, int64_t I, int renorm, int residual, int act_dt,
                      const void *x_decode, int64_t D, const void *x_prefill, int64_t P, int xdt,
                      int sched, int64_t chunk,
                      double *y_decode, double *y_prefill, orc_counters *ctr, int32_t *idx_trace)
{
    if (n_layers <= 0 || D < 0 || P < 0 || H <= 0 || I <= 0 || E <= 0 || k <= 0 || k > E)
        return ORC_ERR_ARG;
    if (sched != ORC_SCHED_CHUNKED && sched != ORC_SCHED_LAYERED) return ORC_ERR_ARG;
    if (sched == ORC_SCHED_CHUNKED && chunk <= 0) return ORC_ERR_ARG;
    if (D + P == 0) { if (ctr) memset(ctr, 0, sizeof(*ctr)); return ORC_OK; }

    const int64_t step = (sched == ORC_SCHED_LAYERED || P == 0) ? (P > 0 ? P : 1) : chunk;
    const int64_t n_iter = (P == 0) ? 1 : (P + step - 1) / step;
    const int64_t Tmax = D + (P < step ? P : step);
    const int sz = (wdt == ORC_BF16) ? 2 : (wdt == ORC_F32 ? 4 : 8);

    double *xb = (double *)malloc(sizeof(double) * (size_t)(Tmax * H));
    double *yb = (double *)malloc(sizeof(double) * (size_t)(Tmax * H));
    int32_t *idx = (int32_t *)malloc(sizeof(int32_t) * (size_t)(Tmax * k));
    int32_t *seen = (int32_t *)malloc(sizeof(int32_t) * (size_t)E);
    if (!xb || !yb || !idx || !seen) { free(xb); free(yb); free(idx); free(seen); return ORC_ERR_ALLOC; }

    orc_counters c;
    memset(&c, 0, sizeof(c));
    int status = ORC_OK;
    int64_t trace_pos = 0;
    for (int64_t it = 0; it < n_iter && status == ORC_OK; ++it) {
        const int64_t p0 = it * step;
        const int64_t pn = (P == 0) ? 0 : ((p0 + step <= P) ? step : P - p0);
        const int64_t T = D + pn;
        for (int64_t i = 0; i < D * H; ++i) xb[i] = ld(x_decode, xdt, i);
        for (int64_t i = 0; i < pn * H; ++i) xb[D * H + i] = ld(x_prefill, xdt, p0 * H + i);
        for (int l = 0; l < n_layers; ++l) {
            status = orc_moe_layer(xb, ORC_F64, T, H, Wr[l], (bias && bias[l]) ? bias[l] : NULL,
                                   Wgu[l], Wd[l], wdt, E, k, I, renorm, residual, yb, idx, NULL, NULL);
            if (status != ORC_OK) break;
            if (idx_trace) {
                memcpy(idx_trace + trace_pos, idx, sizeof(int32_t) * (size_t)(T * k));
                trace_pos += T * k;
            }
            for (int e = 0; e < E; ++e) seen[e] = 0;
            for (int64_t f = 0; f < T * k; ++f) seen[idx[f]] = 1;
            uint64_t active = 0;
            for (int e = 0; e < E; ++e) active += (uint64_t)seen[e];
            c.active_experts_total += active;
            c.expert_bytes += active * 3ull * (uint64_t)H * (uint64_t)I * (uint64_t)sz;
            c.router_bytes += (uint64_t)E * (uint64_t)H * (uint64_t)sz;
            c.layer_passes += 1;
            if (l + 1 < n_layers) {
                for (int64_t i = 0; i < T * H; ++i)
                    xb[i] = (act_dt == ORC_BF16) ? orc_round_bf16(yb[i])
                          : (act_dt == ORC_F32) ? orc_round_f32(yb[i]) : yb[i];
            }
        }
        if (status != ORC_OK) break;
        c.iterations += 1;
        c.tokens_processed += (uint64_t)T;
        memcpy(y_decode, yb, sizeof(double) * (size_t)(D * H));
        if (pn > 0) memcpy(y_prefill + p0 * H, yb + D * H, sizeof(double) * (size_t)(pn * H));
    }
    if (ctr) *ctr = c;
    free(xb); free(yb); free(idx); free(seen);
    return status;
}


/* ---------------------------------------------------------------------------
 * Whole stack: layer groups, the group-count rule and the one-group-per-
 * iteration schedule.
 * ------------------------------------------------------------------------ */

/*
 * Sec. 4.4: the number of layer groups is chosen so that the prefill work of one
 * iteration matches a chunk of `granule` tokens: N_lg(L) = max(1, ceil(L / granule)).
 * The paper's own worked values, granule 512: L = 8192 -> 16, L = 512 -> 1.
 * (Reading: a group holds at least one layer, so the count is capped at n_layers.)
 */
int orc_num_layer_groups(int64_t L, int n_layers, int64_t granule)
{
    if (L < 0 || n_layers <= 0 || granule <= 0) return 0;
    int64_t n = L / granule + (L % granule != 0);
    if (n < 1) n = 1;
    if (n > n_layers) n = n_layers;
    return (int)n;
}

/*
 * Sec. 4.1: the stack is cut vertically into contiguous layer groups.  The paper does not
 * say how a remainder is spread; reading: sizes differ by at most one, larger groups first.
 * first[g] is the first layer of group g, first[n_groups] = n_layers.
 */
int orc_layer_groups(int n_layers, int n_groups, int32_t *first)
{
    if (!first || n_groups < 1 || n_groups > n_layers) return ORC_ERR_ARG;
    int at = 0;
    for (int g = 0; g < n_groups; ++g) {
        first[g] = at;
        at += n_layers / n_groups + (g < n_layers % n_groups ? 1 : 0);
    }
    first[n_groups] = at;
    return ORC_OK;
}

static double round_act(double v, int act_dt)
{
    return (act_dt == ORC_BF16) ? orc_round_bf16(v) : (act_dt == ORC_F32) ? orc_round_f32(v) : v;
}

/*
 * The stack under the one-group-per-iteration rule (Sec. 4.1-4.2), with the prompt cut into
 * slices of `chunk` tokens (Sec. 4.3; chunk = 0: the whole prompt is one slice).  For a slice
 * the stack has G groups (n_groups, or the rule of Sec. 4.4 applied to the slice length when
 * n_groups = 0) and G iterations run.  In iteration g:
 *   - the decode rows start from x_decode and cross ALL groups in layer order (decode is never
 *     blocked: every iteration includes decode work across all layer groups);
 *   - group g, the designated one, also processes the slice's rows, which it takes in the state
 *     group g-1 left them in the iteration before; the other groups do decode only.
 * After G iterations the slice has crossed every layer exactly once.
 * Between layers activations are rounded to act_dt (what a GPU keeps in memory); the outputs of
 * the stack's last layer are returned unrounded.  Counters as in orc_group_forward: one
 * iteration per (slice, g); every layer pass counts the experts it activates.
 * A call without prompt rows is one decode-only iteration.
 */
int orc_stack_forward(const void *const *Wr, const float *const *bias,
                      const void *const *Wgu, const void *const *Wd, int wdt, int n_layers,
                      int64_t H, int E, int k, int64_t I, int renorm, int residual, int act_dt,
                      const void *x_decode, int64_t D, const void *x_prefill, int64_t P, int xdt,
                      int64_t chunk, int n_groups, int64_t granule,
                      double *y_decode, double *y_prefill, orc_counters *ctr)
{
    if (n_layers <= 0 || D < 0 || P < 0 || H <= 0 || I <= 0 || E <= 0 || k <= 0 || k > E)
        return ORC_ERR_ARG;
    if (chunk < 0 || n_groups < 0 || n_groups > n_layers || (n_groups == 0 && granule <= 0))
        return ORC_ERR_ARG;
    if (ctr) memset(ctr, 0, sizeof(*ctr));
    if (D + P == 0) return ORC_OK;

    const int64_t step = (chunk > 0 && P > 0) ? chunk : (P > 0 ? P : 1);
    const int64_t n_slices = (P == 0) ? 1 : (P + step - 1) / step;
    const int64_t Tmax = D + (P < step ? P : step);
    const int sz = (wdt == ORC_BF16) ? 2 : (wdt == ORC_F32 ? 4 : 8);

    double *dec = (double *)malloc(sizeof(double) * (size_t)(D * H + 1));          /* decode rows' state */
    double *pre = (double *)malloc(sizeof(double) * (size_t)((Tmax - D) * H + 1)); /* slice rows' state */
    double *xb = (double *)malloc(sizeof(double) * (size_t)(Tmax * H));
    double *yb = (double *)malloc(sizeof(double) * (size_t)(Tmax * H));
    int32_t *idx = (int32_t *)malloc(sizeof(int32_t) * (size_t)(Tmax * k));
    int32_t *seen = (int32_t *)malloc(sizeof(int32_t) * (size_t)E);
    int32_t *first = (int32_t *)malloc(sizeof(int32_t) * (size_t)(n_layers + 1));
    if (!dec || !pre || !xb || !yb || !idx || !seen || !first) {
        free(dec); free(pre); free(xb); free(yb); free(idx); free(seen); free(first);
        return ORC_ERR_ALLOC;
    }
    orc_counters c;
    memset(&c, 0, sizeof(c));
    int status = ORC_OK;
    for (int64_t sl = 0; sl < n_slices && status == ORC_OK; ++sl) {
        const int64_t p0 = sl * step;
        const int64_t pn = (P == 0) ? 0 : ((p0 + step <= P) ? step : P - p0);
        const int G = (pn == 0) ? 1 : (n_groups > 0 ? n_groups : orc_num_layer_groups(pn, n_layers, granule));
        status = orc_layer_groups(n_layers, G, first);
        if (status != ORC_OK) break;
        for (int64_t i = 0; i < pn * H; ++i) pre[i] = ld(x_prefill, xdt, p0 * H + i);
        for (int g = 0; g < G && status == ORC_OK; ++g) {
            for (int64_t i = 0; i < D * H; ++i) dec[i] = ld(x_decode, xdt, i);
            for (int j = 0; j < G && status == ORC_OK; ++j) {
                const int with_prompt = (j == g && pn > 0);
                const int64_t T = D + (with_prompt ? pn : 0);
                if (T == 0) continue;
                memcpy(xb, dec, sizeof(double) * (size_t)(D * H));
                if (with_prompt) memcpy(xb + D * H, pre, sizeof(double) * (size_t)(pn * H));
                for (int l = first[j]; l < first[j + 1]; ++l) {
                    status = orc_moe_layer(xb, ORC_F64, T, H, Wr[l], (bias && bias[l]) ? bias[l] : NULL,
                                           Wgu[l], Wd[l], wdt, E, k, I, renorm, residual, yb, idx, NULL, NULL);
                    if (status != ORC_OK) break;
                    for (int e = 0; e < E; ++e) seen[e] = 0;
                    for (int64_t f = 0; f < T * k; ++f) seen[idx[f]] = 1;
                    uint64_t active = 0;
                    for (int e = 0; e < E; ++e) active += (uint64_t)seen[e];
                    c.active_experts_total += active;
                    c.expert_bytes += active * 3ull * (uint64_t)H * (uint64_t)I * (uint64_t)sz;
                    c.router_bytes += (uint64_t)E * (uint64_t)H * (uint64_t)sz;
                    c.layer_passes += 1;
                    const int last_of_stack = (l == n_layers - 1);
                    for (int64_t i = 0; i < T * H; ++i) xb[i] = last_of_stack ? yb[i] : round_act(yb[i], act_dt);
                }
                if (status != ORC_OK) break;
                memcpy(dec, xb, sizeof(double) * (size_t)(D * H));
                if (with_prompt) memcpy(pre, xb + D * H, sizeof(double) * (size_t)(pn * H));
            }
            if (status != ORC_OK) break;
            c.iterations += 1;
            c.tokens_processed += (uint64_t)(D + pn);
            if (D > 0) memcpy(y_decode, dec, sizeof(double) * (size_t)(D * H));
        }
        if (status == ORC_OK && pn > 0) memcpy(y_prefill + p0 * H, pre, sizeof(double) * (size_t)(pn * H));
    }
    if (ctr) *ctr = c;
    free(dec); free(pre); free(xb); free(yb); free(idx); free(seen); free(first);
    return status;
}
