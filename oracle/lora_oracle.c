/*
 * fp64 CPU oracle for the batched heterogeneous-adapter LoRA delta.
 *
 * TEST INFRASTRUCTURE ONLY.  Nothing in the product path may call this; only the tests,
 * the smoke check and the benchmark's cpu_baseline leg do.  It shares no code, header,
 * table or helper with the HIP library.
 *
 * What it computes is the plain definition, one row at a time, never rounding:
 *   - Sec. 2.2 (LoRA update): W' = W + AB with A in R^{h x r}, B in R^{r x d}, so a row
 *     vector x gains  x A B  on top of the base output x W.
 *   - Sec. 2.2 (multi-LoRA batching): every row of a batch computes its own update with
 *     its own adapter, independently of the other rows, and the update is added to the
 *     base output.
 *   - Sec. 2.3 / Sec. 4.1: in MoE layers the adapter holds expert-specific matrices; the
 *     unit that applies to a row is selected by (adapter, layer, expert).
 *   - Sec. 3: the update is applied for the up/gate and for the down projection of an
 *     expert; each call of this oracle handles one projection of one layer.
 * A per-adapter scale multiplies the update once, after the product with B (scale = 1
 * is the paper's formula).  Rows whose adapter id is -1 have no adapter and keep their
 * base output bit for bit.
 *
 * Pins (tests/test_oracle_pins.py): merged-weight form x (A B), B = 0, rank-1 closed
 * form, permutation of rows, id = -1 rows, single-adapter batch against a library
 * matmul, linearity, a hand-worked example, exhaustive tiny integer cases, and the
 * adapter footprint the paper prints for Mixtral-8x7B at rank 64 (Sec. 2.3: 1.69 GB).
 * The segment oracle is pinned against a library stable sort and brute-force properties.
 *
 * Storage: bf16 values are passed as raw uint16 bit patterns; bf16 -> double is exact.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

static double bf16_to_f64(uint16_t h)
{
    uint32_t u = ((uint32_t)h) << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

/* double -> nearest bf16, ties to even, done directly on the double (no fp32 step,
 * so there is no double rounding). bf16: 1 sign, 8 exponent, 7 mantissa bits. */
static uint16_t f64_to_bf16_rne(double v)
{
    if (isnan(v)) return 0x7FC0;
    uint16_t sign = signbit(v) ? 0x8000 : 0;
    double a = fabs(v);
    if (isinf(a)) return sign | 0x7F80;
    if (a == 0.0) return sign;
    int e;
    (void)frexp(a, &e);               /* a = m * 2^e, m in [0.5, 1) */
    int E = e - 1;                    /* a = (2m) * 2^E, 2m in [1, 2) */
    if (E < -126) E = -126;           /* subnormal range: fixed quantum 2^-133 */
    double q = ldexp(1.0, E - 7);     /* spacing of bf16 values in this binade */
    double n = nearbyint(a / q);      /* default rounding mode: ties to even; a/q exact */
    double r = n * q;
    if (r >= ldexp(1.0, 128)) return sign | 0x7F80;
    float f = (float)r;               /* exact: r is a bf16 value */
    uint32_t u;
    memcpy(&u, &f, sizeof u);
    return sign | (uint16_t)(u >> 16);
}

uint16_t lora_oracle_bf16_rne(double v) { return f64_to_bf16_rne(v); }
double lora_oracle_bf16_to_f64(uint16_t h) { return bf16_to_f64(h); }

/*
 * One projection of one layer over P rows.
 *
 *   adapter_id[P]   -1 = no adapter; otherwise 0 .. n_adapters-1
 *   expert_id[P]    NULL for a dense layer (expert 0), else 0 .. n_experts-1
 *   src_row[P]      NULL = row p reads x row p; else x row src_row[p]
 *   x               bf16 bits, row stride ldx elements
 *   A_unit, B_unit  n_adapters*n_experts pointers, index adapter*n_experts + expert, to
 *                   row-major bf16 A[h_in][r] and B[r][h_out] of this layer/projection
 *   scale[n_adapters]
 *   y_in            bf16 bits [P][ldy] base output, or NULL (= all zero)
 * Outputs (each may be NULL):
 *   v      [P][r]      x A               (zero rows for id -1)
 *   delta  [P][h_out]  scale * x A B     (zero rows for id -1)
 *   y_out  [P][h_out]  y_in + delta, unrounded
 *   y_bf16 [P][h_out]  y_out rounded once to bf16 (ties to even); id -1 rows are the
 *                      input bits copied
 * Returns 0, or -1 for an id outside its range (nothing is written for that row).
 */
int lora_oracle_delta(int P, int h_in, int h_out, int r,
                      const uint16_t *x, int64_t ldx, const int32_t *src_row,
                      const int32_t *adapter_id, const int32_t *expert_id,
                      int n_adapters, int n_experts,
                      const uint16_t *const *A_unit, const uint16_t *const *B_unit,
                      const float *scale,
                      const uint16_t *y_in, int64_t ldy,
                      double *v, double *delta, double *y_out, uint16_t *y_bf16)
{
    int bad = 0;
#pragma omp parallel for schedule(dynamic, 1) reduction(| : bad)
    for (int p = 0; p < P; ++p) {
        int a = adapter_id[p];
        int e = expert_id ? expert_id[p] : 0;
        if (a == -1) {
            if (v) for (int j = 0; j < r; ++j) v[(size_t)p * r + j] = 0.0;
            for (int d = 0; d < h_out; ++d) {
                size_t o = (size_t)p * h_out + d;
                uint16_t yb = y_in ? y_in[(size_t)p * ldy + d] : 0;
                if (delta) delta[o] = 0.0;
                if (y_out) y_out[o] = bf16_to_f64(yb);
                if (y_bf16) y_bf16[o] = yb;
            }
            continue;
        }
        if (a < 0 || a >= n_adapters || e < 0 || e >= n_experts) { bad |= 1; continue; }
        const uint16_t *A = A_unit[(size_t)a * n_experts + e];
        const uint16_t *B = B_unit[(size_t)a * n_experts + e];
        const uint16_t *xr = x + (size_t)(src_row ? src_row[p] : p) * ldx;
        double *vv = (double *)malloc(sizeof(double) * (size_t)r);
        /* shrink: v_j = sum over c (ascending) of x_c * A[c][j] */
        for (int j = 0; j < r; ++j) vv[j] = 0.0;
        for (int c = 0; c < h_in; ++c) {
            double xc = bf16_to_f64(xr[c]);
            for (int j = 0; j < r; ++j) vv[j] += xc * bf16_to_f64(A[(size_t)c * r + j]);
        }
        if (v) for (int j = 0; j < r; ++j) v[(size_t)p * r + j] = vv[j];
        /* expand: delta_d = scale * sum over j (ascending) of v_j * B[j][d]; then add */
        double s = (double)scale[a];
        for (int d = 0; d < h_out; ++d) {
            double acc = 0.0;
            for (int j = 0; j < r; ++j) acc += vv[j] * bf16_to_f64(B[(size_t)j * h_out + d]);
            double dl = s * acc;
            size_t o = (size_t)p * h_out + d;
            double yi = y_in ? bf16_to_f64(y_in[(size_t)p * ldy + d]) : 0.0;
            if (delta) delta[o] = dl;
            if (y_out) y_out[o] = yi + dl;
            if (y_bf16) y_bf16[o] = f64_to_bf16_rne(yi + dl);
        }
        free(vv);
    }
    return bad ? -1 : 0;
}

/*
 * Weighted combine of the per-pair updates of the down projection into token rows.
 *
 * Sec. 4.1: a request activates its top-k experts at a layer, so a batch of T tokens is
 * T*k (token, expert) pairs; Sec. 3 / Fig. 7b: the LoRA results come back and are added
 * to the base output.  In a MoE layer the base output of a token is the routing-weighted
 * sum of its experts' outputs, and the update belongs to an expert's weight, so the
 * token's base output gains  sum_j w[t*k+j] * delta[t*k+j]  (the paper does not spell
 * the routing weights out; this is the reading taken).  Pair p = t*k + j.
 *
 *   delta   [T*k][h_out]  per-pair updates as lora_oracle_delta returns them (zero rows
 *                         for pairs without adapter)
 *   w       [T*k]         routing weights
 *   y_in    bf16 bits [T][ldy] token rows of the base output, or NULL (= all zero)
 *   y_out   [T][h_out]    y_in + sum over j = 0 .. k-1 (ascending) of w * delta, unrounded
 *   y_bf16  [T][h_out]    y_out rounded once; a token none of whose pairs has an adapter
 *                         keeps its input bits
 */
void lora_oracle_combine(int T, int k, int h_out, const double *delta, const int32_t *adapter_id,
                         const float *w, const uint16_t *y_in, int64_t ldy,
                         double *y_out, uint16_t *y_bf16)
{
#pragma omp parallel for schedule(static)
    for (int t = 0; t < T; ++t) {
        int any = 0;
        for (int j = 0; j < k; ++j) any |= adapter_id[(size_t)t * k + j] != -1;
        for (int d = 0; d < h_out; ++d) {
            uint16_t yb = y_in ? y_in[(size_t)t * ldy + d] : 0;
            double acc = bf16_to_f64(yb);
            for (int j = 0; j < k; ++j) {
                size_t p = (size_t)t * k + j;
                if (adapter_id[p] != -1) acc += (double)w[p] * delta[p * h_out + d];
            }
            size_t o = (size_t)t * h_out + d;
            if (y_out) y_out[o] = acc;
            if (y_bf16) y_bf16[o] = any ? f64_to_bf16_rne(acc) : yb;
        }
    }
}

/*
 * Canonical segments (App. A.2.2: rows that share an adapter are aggregated into one
 * GEMM; with per-expert matrices, rows that share (adapter, expert)).  Many groupings
 * give the same sums; the contract fixes one:
 *   key = adapter * n_experts + expert; rows with adapter -1 are dropped;
 *   perm lists the remaining rows grouped by ascending key, original order kept inside
 *   a key (a stable counting sort); seg_key[s] is the key of the s-th non-empty group,
 *   seg_start[s] its first position in perm, seg_start[S] = P_act.
 * Ids outside their range are treated as -1 and reported in the return value (count).
 * counts[0] = S, counts[1] = P_act.  perm, seg_key: capacity P; seg_start: P + 1.
 */
int lora_oracle_segments(int P, const int32_t *adapter_id, const int32_t *expert_id,
                         int n_adapters, int n_experts,
                         int32_t *perm, int32_t *seg_start, int32_t *seg_key, int32_t *counts)
{
    int64_t n_keys = (int64_t)n_adapters * n_experts;
    int64_t *hist = (int64_t *)calloc((size_t)n_keys + 1, sizeof(int64_t));
    int64_t *key = (int64_t *)malloc(sizeof(int64_t) * (size_t)(P > 0 ? P : 1));
    int n_bad = 0;
    for (int p = 0; p < P; ++p) {
        int a = adapter_id[p];
        int e = expert_id ? expert_id[p] : 0;
        if (a == -1) { key[p] = -1; continue; }
        if (a < 0 || a >= n_adapters || e < 0 || e >= n_experts) { key[p] = -1; ++n_bad; continue; }
        key[p] = (int64_t)a * n_experts + e;
        hist[key[p]]++;
    }
    /* exclusive prefix over keys -> first position of each key; list non-empty keys */
    int S = 0;
    int64_t run = 0;
    int64_t *first = (int64_t *)malloc(sizeof(int64_t) * ((size_t)n_keys + 1));
    for (int64_t k = 0; k < n_keys; ++k) {
        first[k] = run;
        if (hist[k] > 0) {
            seg_key[S] = (int32_t)k;
            seg_start[S] = (int32_t)run;
            ++S;
        }
        run += hist[k];
    }
    seg_start[S] = (int32_t)run;
    /* place rows in original order: stable */
    for (int p = 0; p < P; ++p)
        if (key[p] >= 0) perm[first[key[p]]++] = p;
    counts[0] = S;
    counts[1] = (int32_t)run;
    free(first);
    free(key);
    free(hist);
    return n_bad;
}

/*
 * Bytes of one adapter held in 16-bit storage: every (layer, expert) unit carries, for
 * each projection, A (h_in x r) and B (r x h_out)  (Sec. 4.1: n x l x e units;
 * Sec. 2.3: size grows with the number of experts).
 */
int64_t lora_oracle_adapter_bytes(int n_layers, int n_experts, int n_proj,
                                  const int32_t *h_in, const int32_t *h_out, int r)
{
    int64_t per_unit = 0;
    for (int i = 0; i < n_proj; ++i) per_unit += ((int64_t)h_in[i] + h_out[i]) * r * 2;
    return (int64_t)n_layers * n_experts * per_unit;
}
