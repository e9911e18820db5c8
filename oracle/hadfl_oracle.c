/*
 * HADFL reference oracle -- TEST INFRASTRUCTURE, NOT THE PRODUCT.
 *
 * A plain, slow, fp64 CPU statement of what one HADFL aggregation cycle
 * computes (Cao et al., "HADFL: Heterogeneity-aware Decentralized Federated
 * Learning Framework", arXiv 2111.08274).  Only the tests, the smoke check and
 * the benchmark's CPU-baseline leg may call it.  It shares no code with the
 * GPU library: no headers, no tables, no helpers.
 *
 * What follows the paper, and where:
 *   step counts      Sec. 2.3 (hyperperiod), Sec. 3.3 (H_E = LCM of epoch
 *                    times), expected-version equation of Sec. 3.2
 *   local training   Sec. 2.1 (forward / backward / update), Algorithm 1
 *                    (local loop), local-update equation of Sec. 2.2
 *   selection        Sec. 3.3, the probability-based selection function
 *   aggregation      Sec. 2.3, the partial-aggregation equation; Algorithm 1
 *                    (partial + global synchronisation)
 *   version forecast Sec. 3.2, the double-exponential-smoothing predictor
 *
 * No blocking, fusion or reordering beyond those definitions.  OpenMP is used
 * across replicas only (replicas are independent; numerics are unchanged).
 *
 * Parity pins live in tests/test_oracle_*.py.  Unpinned: nothing in this file
 * can be checked against the paper's accuracy curves or timing table (they
 * need CIFAR-10 and converged runs) -- "parity unpinned" for those.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* ------------------------------------------------------------------------- */
/* Network description: a list of ops over numbered tensors (tensor 0 = input) */
/* Activations are [B][H][W][C]; conv weights [kh][kw][Cin][Cout]; dense      */
/* weights [in][out] with in = flattened H*W*C of the input tensor.            */
/* ------------------------------------------------------------------------- */
enum { OP_CONV = 0, OP_DENSE = 1, OP_RELU = 2, OP_MAXPOOL = 3, OP_BN = 4, OP_ADD = 5, OP_GAP = 6 };
enum { KIND_WEIGHT = 0, KIND_BIAS = 1, KIND_GAMMA = 2, KIND_BETA = 3, KIND_RMEAN = 4, KIND_RVAR = 5 };
enum { LOSS_SOFTMAX_CE = 0, LOSS_HALF_SQUARED = 1 };

#define OP_FIELDS 9
typedef struct { int type, in0, in1, out, k, stride, pad, cout, bias; } op_t;
typedef struct { int h, w, c; } shape_t;

typedef struct {
    int n_ops, n_tensors;
    op_t *ops;
    shape_t *shp;            /* [n_tensors] */
    int64_t *off_a;          /* weight / gamma offset per op (-1 if none) */
    int64_t *off_b;          /* bias / beta offset per op (-1 if none)   */
    int64_t *off_stat;       /* running mean offset per BN op; running var follows */
    int64_t m_train, m_total;
    int act_rounding;        /* 0: none; 1 (the bf16 workload): every stored
                                activation (input batch and logits included),
                                every stored activation gradient, and the
                                conv / dense weights as used by the forward and
                                backward pass are rounded to bfloat16; biases,
                                BN parameters, sums, weight gradients and the
                                update stay unrounded (fp32 master + fp32
                                accumulation on the GPU side) */
} net_t;

static int64_t numel(shape_t s) { return (int64_t)s.h * s.w * s.c; }

void hadfl_oracle_net_destroy(net_t *n)
{
    if (!n) return;
    free(n->ops); free(n->shp); free(n->off_a); free(n->off_b); free(n->off_stat); free(n);
}

/* ops: [n_ops][OP_FIELDS] int32.  Returns NULL when the description is inconsistent. */
net_t *hadfl_oracle_net_create(const int32_t *ops, int n_ops, int in_h, int in_w, int in_c)
{
    net_t *n = (net_t *)calloc(1, sizeof(net_t));
    n->n_ops = n_ops;
    n->ops = (op_t *)calloc((size_t)n_ops, sizeof(op_t));
    n->off_a = (int64_t *)calloc((size_t)n_ops, sizeof(int64_t));
    n->off_b = (int64_t *)calloc((size_t)n_ops, sizeof(int64_t));
    n->off_stat = (int64_t *)calloc((size_t)n_ops, sizeof(int64_t));
    int max_t = 0;
    for (int i = 0; i < n_ops; ++i) {
        const int32_t *o = ops + (size_t)i * OP_FIELDS;
        op_t p = { o[0], o[1], o[2], o[3], o[4], o[5], o[6], o[7], o[8] };
        n->ops[i] = p;
        if (p.out > max_t) max_t = p.out;
    }
    n->n_tensors = max_t + 1;
    n->shp = (shape_t *)calloc((size_t)n->n_tensors, sizeof(shape_t));
    n->shp[0].h = in_h; n->shp[0].w = in_w; n->shp[0].c = in_c;
    int64_t off = 0;
    for (int i = 0; i < n_ops; ++i) {
        op_t *p = &n->ops[i];
        n->off_a[i] = n->off_b[i] = n->off_stat[i] = -1;
        if (p->in0 < 0 || p->in0 >= p->out || p->out != i + 1) goto bad;   /* op i writes tensor i+1 */
        shape_t a = n->shp[p->in0], r = a;
        switch (p->type) {
        case OP_CONV:
            r.h = (a.h + 2 * p->pad - p->k) / p->stride + 1;
            r.w = (a.w + 2 * p->pad - p->k) / p->stride + 1;
            r.c = p->cout;
            if (r.h < 1 || r.w < 1 || p->k < 1 || p->stride < 1) goto bad;
            n->off_a[i] = off; off += (int64_t)p->k * p->k * a.c * p->cout;
            if (p->bias) { n->off_b[i] = off; off += p->cout; }
            break;
        case OP_DENSE:
            r.h = 1; r.w = 1; r.c = p->cout;
            n->off_a[i] = off; off += numel(a) * p->cout;
            if (p->bias) { n->off_b[i] = off; off += p->cout; }
            break;
        case OP_RELU: break;
        case OP_MAXPOOL:
            if (a.h % 2 || a.w % 2) goto bad;
            r.h = a.h / 2; r.w = a.w / 2; break;
        case OP_BN:
            n->off_a[i] = off; off += a.c;
            n->off_b[i] = off; off += a.c;
            break;
        case OP_ADD: {
            if (p->in1 < 0 || p->in1 >= p->out) goto bad;
            shape_t b = n->shp[p->in1];
            if (a.h != b.h || a.w != b.w || a.c != b.c) goto bad;
            break; }
        case OP_GAP: r.h = 1; r.w = 1; break;
        default: goto bad;
        }
        n->shp[p->out] = r;
    }
    n->m_train = off;
    /* running statistics of every BN op sit after all trainable parameters */
    for (int i = 0; i < n_ops; ++i)
        if (n->ops[i].type == OP_BN) { n->off_stat[i] = off; off += 2 * (int64_t)n->shp[n->ops[i].in0].c; }
    n->m_total = off;
    return n;
bad:
    hadfl_oracle_net_destroy(n);
    return NULL;
}

void hadfl_oracle_net_set_rounding(net_t *n, int mode) { n->act_rounding = mode; }
int64_t hadfl_oracle_net_m_train(const net_t *n) { return n->m_train; }
int64_t hadfl_oracle_net_m_total(const net_t *n) { return n->m_total; }
int hadfl_oracle_net_n_out(const net_t *n) { return (int)numel(n->shp[n->n_tensors - 1]); }

/* Parameter tensors in vector order: rows of (offset, count, kind, fan_in). Returns row count. */
int hadfl_oracle_net_layout(const net_t *n, int64_t *rows, int cap)
{
    int cnt = 0;
#define PUSH(o, c, k, f) do { if (cnt < cap) { rows[4*cnt] = (o); rows[4*cnt+1] = (c); rows[4*cnt+2] = (k); rows[4*cnt+3] = (f); } ++cnt; } while (0)
    for (int i = 0; i < n->n_ops; ++i) {
        const op_t *p = &n->ops[i];
        shape_t a = n->shp[p->in0];
        if (p->type == OP_CONV) {
            int64_t fan = (int64_t)p->k * p->k * a.c;
            PUSH(n->off_a[i], fan * p->cout, KIND_WEIGHT, fan);
            if (p->bias) PUSH(n->off_b[i], p->cout, KIND_BIAS, fan);
        } else if (p->type == OP_DENSE) {
            int64_t fan = numel(a);
            PUSH(n->off_a[i], fan * p->cout, KIND_WEIGHT, fan);
            if (p->bias) PUSH(n->off_b[i], p->cout, KIND_BIAS, fan);
        } else if (p->type == OP_BN) {
            PUSH(n->off_a[i], a.c, KIND_GAMMA, a.c);
            PUSH(n->off_b[i], a.c, KIND_BETA, a.c);
        }
    }
    for (int i = 0; i < n->n_ops; ++i)
        if (n->ops[i].type == OP_BN) {
            int c = n->shp[n->ops[i].in0].c;
            PUSH(n->off_stat[i], c, KIND_RMEAN, c);
            PUSH(n->off_stat[i] + c, c, KIND_RVAR, c);
        }
#undef PUSH
    return cnt;
}

/* ------------------------------------------------------------------------- */
/* bfloat16 rounding (round to nearest even on the top 16 bits of an fp32)    */
/* ------------------------------------------------------------------------- */
static double round_bf16(double v)
{
    float f = (float)v;
    uint32_t u; memcpy(&u, &f, 4);
    if ((u & 0x7f800000u) == 0x7f800000u) return (double)f;      /* inf / nan unchanged */
    u += 0x7fffu + ((u >> 16) & 1u);
    u &= 0xffff0000u;
    memcpy(&f, &u, 4);
    return (double)f;
}
double hadfl_oracle_round_bf16(double v) { return round_bf16(v); }

static void round_buf(const net_t *n, double *p, int64_t cnt)
{
    if (!n->act_rounding) return;
    for (int64_t i = 0; i < cnt; ++i) p[i] = round_bf16(p[i]);
}

/* ------------------------------------------------------------------------- */
/* Forward + loss + backward for one mini-batch (Sec. 2.1 phases 1 and 2;     */
/* Algorithm 1, gradient of the batch-mean loss).                             */
/* params: [m_total] (BN running statistics are updated in place when         */
/* update_stats != 0).  grad: [m_train], overwritten.  Returns the loss.      */
/* x: [B][H][W][C] float; y: int labels (softmax CE) ; target: [B][n_out]     */
/* doubles (half squared error).                                              */
/* ------------------------------------------------------------------------- */
#define BN_EPS 1e-5
#define BN_STAT_MOMENTUM 0.1

double hadfl_oracle_loss_grad(const net_t *n, double *params, const float *x, const int32_t *y,
                              const double *target, int loss_kind, int B, double *grad,
                              int update_stats, double *logits_out)
{
    const int T = n->n_tensors;
    double **act = (double **)calloc((size_t)T, sizeof(double *));
    double **gra = (double **)calloc((size_t)T, sizeof(double *));
    double **bn_mean = (double **)calloc((size_t)n->n_ops, sizeof(double *));
    double **bn_istd = (double **)calloc((size_t)n->n_ops, sizeof(double *));
    /* weights as used by the arithmetic: rounded copy in bf16 mode */
    double *w = params;
    if (n->act_rounding) {
        w = (double *)malloc(sizeof(double) * (size_t)n->m_train);
        memcpy(w, params, sizeof(double) * (size_t)n->m_train);
        for (int i = 0; i < n->n_ops; ++i)
            if (n->ops[i].type == OP_CONV || n->ops[i].type == OP_DENSE) {
                const op_t *p = &n->ops[i];
                int64_t cnt = (p->type == OP_CONV ? (int64_t)p->k * p->k * n->shp[p->in0].c : numel(n->shp[p->in0])) * p->cout;
                for (int64_t j = 0; j < cnt; ++j) w[n->off_a[i] + j] = round_bf16(params[n->off_a[i] + j]);
            }
    }
    for (int t = 0; t < T; ++t) {
        act[t] = (double *)calloc((size_t)(B * numel(n->shp[t])), sizeof(double));
        gra[t] = (double *)calloc((size_t)(B * numel(n->shp[t])), sizeof(double));
    }
    {
        int64_t cnt = B * numel(n->shp[0]);
        for (int64_t i = 0; i < cnt; ++i) act[0][i] = (double)x[i];
        round_buf(n, act[0], cnt);
    }

    /* ---------------- forward ---------------- */
    for (int i = 0; i < n->n_ops; ++i) {
        const op_t *p = &n->ops[i];
        const shape_t a = n->shp[p->in0], r = n->shp[p->out];
        const double *in = act[p->in0];
        double *out = act[p->out];
        switch (p->type) {
        case OP_CONV: {
            const double *wt = w + n->off_a[i];
            for (int b = 0; b < B; ++b)
             for (int ho = 0; ho < r.h; ++ho)
              for (int wo = 0; wo < r.w; ++wo) {
                double *o = out + (((int64_t)b * r.h + ho) * r.w + wo) * r.c;
                for (int co = 0; co < r.c; ++co) o[co] = p->bias ? w[n->off_b[i] + co] : 0.0;
                for (int kh = 0; kh < p->k; ++kh) {
                    int hi = ho * p->stride - p->pad + kh;
                    if (hi < 0 || hi >= a.h) continue;
                    for (int kw = 0; kw < p->k; ++kw) {
                        int wi = wo * p->stride - p->pad + kw;
                        if (wi < 0 || wi >= a.w) continue;
                        const double *xi = in + (((int64_t)b * a.h + hi) * a.w + wi) * a.c;
                        const double *wk = wt + ((int64_t)(kh * p->k + kw) * a.c) * r.c;
                        for (int ci = 0; ci < a.c; ++ci) {
                            double xv = xi[ci];
                            const double *wr = wk + (int64_t)ci * r.c;
                            for (int co = 0; co < r.c; ++co) o[co] += xv * wr[co];
                        }
                    }
                }
              }
            break; }
        case OP_DENSE: {
            const int64_t K = numel(a);
            const double *wt = w + n->off_a[i];
            for (int b = 0; b < B; ++b) {
                double *o = out + (int64_t)b * r.c;
                for (int co = 0; co < r.c; ++co) o[co] = p->bias ? w[n->off_b[i] + co] : 0.0;
                for (int64_t kk = 0; kk < K; ++kk) {
                    double xv = in[(int64_t)b * K + kk];
                    const double *wr = wt + kk * r.c;
                    for (int co = 0; co < r.c; ++co) o[co] += xv * wr[co];
                }
            }
            break; }
        case OP_RELU: {
            int64_t cnt = B * numel(a);
            for (int64_t j = 0; j < cnt; ++j) out[j] = in[j] > 0.0 ? in[j] : 0.0;
            break; }
        case OP_MAXPOOL:
            for (int b = 0; b < B; ++b)
             for (int ho = 0; ho < r.h; ++ho)
              for (int wo = 0; wo < r.w; ++wo)
               for (int c = 0; c < r.c; ++c) {
                   double m = -INFINITY;
                   for (int dh = 0; dh < 2; ++dh)
                    for (int dw = 0; dw < 2; ++dw) {
                        double v = in[(((int64_t)b * a.h + 2 * ho + dh) * a.w + 2 * wo + dw) * a.c + c];
                        if (v > m) m = v;
                    }
                   out[(((int64_t)b * r.h + ho) * r.w + wo) * r.c + c] = m;
               }
            break;
        case OP_BN: {
            /* training-mode batch normalisation: statistics over B*H*W per channel */
            const int64_t rows = (int64_t)B * a.h * a.w;
            const int C = a.c;
            bn_mean[i] = (double *)calloc((size_t)C, sizeof(double));
            bn_istd[i] = (double *)calloc((size_t)C, sizeof(double));
            for (int c = 0; c < C; ++c) {
                double s = 0.0;
                for (int64_t q = 0; q < rows; ++q) s += in[q * C + c];
                double mean = s / (double)rows, v = 0.0;
                for (int64_t q = 0; q < rows; ++q) { double d = in[q * C + c] - mean; v += d * d; }
                double var = v / (double)rows;
                bn_mean[i][c] = mean;
                bn_istd[i][c] = 1.0 / sqrt(var + BN_EPS);
                if (update_stats) {
                    double *rm = params + n->off_stat[i], *rv = rm + C;
                    double unb = rows > 1 ? v / (double)(rows - 1) : var;
                    rm[c] = (1.0 - BN_STAT_MOMENTUM) * rm[c] + BN_STAT_MOMENTUM * mean;
                    rv[c] = (1.0 - BN_STAT_MOMENTUM) * rv[c] + BN_STAT_MOMENTUM * unb;
                }
                double g = w[n->off_a[i] + c], be = w[n->off_b[i] + c];
                for (int64_t q = 0; q < rows; ++q)
                    out[q * C + c] = g * ((in[q * C + c] - mean) * bn_istd[i][c]) + be;
            }
            break; }
        case OP_ADD: {
            const double *in2 = act[p->in1];
            int64_t cnt = B * numel(a);
            for (int64_t j = 0; j < cnt; ++j) out[j] = in[j] + in2[j];
            break; }
        case OP_GAP: {
            const int64_t hw = (int64_t)a.h * a.w;
            for (int b = 0; b < B; ++b)
                for (int c = 0; c < a.c; ++c) {
                    double s = 0.0;
                    for (int64_t q = 0; q < hw; ++q) s += in[((int64_t)b * hw + q) * a.c + c];
                    out[(int64_t)b * a.c + c] = s / (double)hw;
                }
            break; }
        }
        round_buf(n, out, B * numel(r));
    }

    /* ---------------- loss (mean over the batch) and its gradient ---------------- */
    const int NO = (int)numel(n->shp[T - 1]);
    const double *logit = act[T - 1];
    double *dlogit = gra[T - 1];
    double loss = 0.0;
    if (logits_out) memcpy(logits_out, logit, sizeof(double) * (size_t)B * NO);
    for (int b = 0; b < B; ++b) {
        const double *z = logit + (int64_t)b * NO;
        double *dz = dlogit + (int64_t)b * NO;
        if (loss_kind == LOSS_SOFTMAX_CE) {
            double m = z[0], s = 0.0;
            for (int j = 1; j < NO; ++j) if (z[j] > m) m = z[j];
            for (int j = 0; j < NO; ++j) s += exp(z[j] - m);
            loss += (log(s) + m - z[y[b]]) / (double)B;
            for (int j = 0; j < NO; ++j) dz[j] = (exp(z[j] - m) / s - (j == y[b] ? 1.0 : 0.0)) / (double)B;
        } else {
            for (int j = 0; j < NO; ++j) {
                double d = z[j] - target[(int64_t)b * NO + j];
                loss += 0.5 * d * d / (double)B;
                dz[j] = d / (double)B;
            }
        }
    }

    /* ---------------- backward ---------------- */
    memset(grad, 0, sizeof(double) * (size_t)n->m_train);
    for (int i = n->n_ops - 1; i >= 0; --i) {
        const op_t *p = &n->ops[i];
        const shape_t a = n->shp[p->in0], r = n->shp[p->out];
        const double *in = act[p->in0];
        const double *dout = gra[p->out];
        double *din = gra[p->in0];                     /* accumulated: a tensor may feed two ops */
        round_buf(n, gra[p->out], B * numel(r));
        switch (p->type) {
        case OP_CONV: {
            const double *wt = w + n->off_a[i];
            double *dw = grad + n->off_a[i];
            for (int b = 0; b < B; ++b)
             for (int ho = 0; ho < r.h; ++ho)
              for (int wo = 0; wo < r.w; ++wo) {
                const double *d = dout + (((int64_t)b * r.h + ho) * r.w + wo) * r.c;
                if (p->bias) for (int co = 0; co < r.c; ++co) grad[n->off_b[i] + co] += d[co];
                for (int kh = 0; kh < p->k; ++kh) {
                    int hi = ho * p->stride - p->pad + kh;
                    if (hi < 0 || hi >= a.h) continue;
                    for (int kw = 0; kw < p->k; ++kw) {
                        int wi = wo * p->stride - p->pad + kw;
                        if (wi < 0 || wi >= a.w) continue;
                        const int64_t xo = (((int64_t)b * a.h + hi) * a.w + wi) * a.c;
                        const int64_t wo_ = ((int64_t)(kh * p->k + kw) * a.c) * r.c;
                        for (int ci = 0; ci < a.c; ++ci) {
                            double xv = in[xo + ci], acc = 0.0;
                            const double *wr = wt + wo_ + (int64_t)ci * r.c;
                            double *dwr = dw + wo_ + (int64_t)ci * r.c;
                            for (int co = 0; co < r.c; ++co) { dwr[co] += xv * d[co]; acc += wr[co] * d[co]; }
                            if (p->in0 != 0) din[xo + ci] += acc;
                        }
                    }
                }
              }
            break; }
        case OP_DENSE: {
            const int64_t K = numel(a);
            const double *wt = w + n->off_a[i];
            double *dw = grad + n->off_a[i];
            for (int b = 0; b < B; ++b) {
                const double *d = dout + (int64_t)b * r.c;
                if (p->bias) for (int co = 0; co < r.c; ++co) grad[n->off_b[i] + co] += d[co];
                for (int64_t kk = 0; kk < K; ++kk) {
                    double xv = in[(int64_t)b * K + kk], acc = 0.0;
                    for (int co = 0; co < r.c; ++co) { dw[kk * r.c + co] += xv * d[co]; acc += wt[kk * r.c + co] * d[co]; }
                    if (p->in0 != 0) din[(int64_t)b * K + kk] += acc;
                }
            }
            break; }
        case OP_RELU: {
            int64_t cnt = B * numel(a);
            for (int64_t j = 0; j < cnt; ++j) if (in[j] > 0.0) din[j] += dout[j];
            break; }
        case OP_MAXPOOL:
            /* gradient goes to the first maximal element in (dh, dw) scan order */
            for (int b = 0; b < B; ++b)
             for (int ho = 0; ho < r.h; ++ho)
              for (int wo = 0; wo < r.w; ++wo)
               for (int c = 0; c < r.c; ++c) {
                   double m = -INFINITY; int64_t arg = -1;
                   for (int dh = 0; dh < 2; ++dh)
                    for (int dw = 0; dw < 2; ++dw) {
                        int64_t idx = (((int64_t)b * a.h + 2 * ho + dh) * a.w + 2 * wo + dw) * a.c + c;
                        if (in[idx] > m) { m = in[idx]; arg = idx; }
                    }
                   din[arg] += dout[(((int64_t)b * r.h + ho) * r.w + wo) * r.c + c];
               }
            break;
        case OP_BN: {
            const int64_t rows = (int64_t)B * a.h * a.w;
            const int C = a.c;
            for (int c = 0; c < C; ++c) {
                double mean = bn_mean[i][c], istd = bn_istd[i][c], g = w[n->off_a[i] + c];
                double dg = 0.0, db = 0.0;
                for (int64_t q = 0; q < rows; ++q) {
                    double xh = (in[q * C + c] - mean) * istd;
                    dg += dout[q * C + c] * xh; db += dout[q * C + c];
                }
                grad[n->off_a[i] + c] += dg;
                grad[n->off_b[i] + c] += db;
                for (int64_t q = 0; q < rows; ++q) {
                    double xh = (in[q * C + c] - mean) * istd;
                    din[q * C + c] += g * istd * (dout[q * C + c] - db / (double)rows - xh * dg / (double)rows);
                }
            }
            break; }
        case OP_ADD: {
            double *din2 = gra[p->in1];
            int64_t cnt = B * numel(a);
            for (int64_t j = 0; j < cnt; ++j) { din[j] += dout[j]; din2[j] += dout[j]; }
            break; }
        case OP_GAP: {
            const int64_t hw = (int64_t)a.h * a.w;
            for (int b = 0; b < B; ++b)
                for (int64_t q = 0; q < hw; ++q)
                    for (int c = 0; c < a.c; ++c)
                        din[((int64_t)b * hw + q) * a.c + c] += dout[(int64_t)b * a.c + c] / (double)hw;
            break; }
        }
    }

    for (int t = 0; t < T; ++t) { free(act[t]); free(gra[t]); }
    for (int i = 0; i < n->n_ops; ++i) { free(bn_mean[i]); free(bn_istd[i]); }
    free(act); free(gra); free(bn_mean); free(bn_istd);
    if (w != params) free(w);
    return loss;
}

/* ------------------------------------------------------------------------- */
/* Step-count rule (Sec. 2.3, Sec. 3.3; expected-version equation read as     */
/* "unit steps device k completes in one synchronisation period").  With      */
/* integer computing-power ratios r_k (larger = faster, Sec. 4.1) the time    */
/* per unit step is proportional to 1/r_k, the hyperperiod is 1/gcd(r), and   */
/*   E_k = T_sync * steps_per_unit * r_k / gcd(r).                            */
/* Returns 0, or -1 for a non-positive ratio / factor.                        */
/* ------------------------------------------------------------------------- */
int hadfl_oracle_step_counts(const int32_t *ratio, int n, int t_sync, int steps_per_unit, int32_t *steps)
{
    if (n < 1 || t_sync < 1 || steps_per_unit < 1) return -1;
    int64_t g = 0;
    for (int k = 0; k < n; ++k) {
        if (ratio[k] <= 0) return -1;
        int64_t a = ratio[k], b = g;
        while (b) { int64_t t = a % b; a = b; b = t; }
        g = a;
    }
    for (int k = 0; k < n; ++k) steps[k] = (int32_t)((int64_t)t_sync * steps_per_unit * (ratio[k] / g));
    return 0;
}

/* ------------------------------------------------------------------------- */
/* Step counts from warm-up times (Sec. 3.2 mutual negotiation, Sec. 3.3       */
/* hyperperiod).  Device k needed T[k] for e_warmup units, so one unit takes  */
/* T[k]/e_warmup; measured times are not commensurable, so each is expressed  */
/* as the nearest whole number (at least 1) of `quantum`.  The hyperperiod is */
/* the least common multiple of those; within t_sync hyperperiods device k    */
/* finishes t_sync * steps_per_unit * (hyperperiod / its unit time) units.    */
/* Returns 0, or -1 on a non-positive input or a count beyond 2^20.           */
/* ------------------------------------------------------------------------- */
int hadfl_oracle_steps_from_times(const double *T, int n, int e_warmup, double quantum, int t_sync,
                                  int steps_per_unit, int32_t *steps)
{
    if (n < 1 || e_warmup < 1 || t_sync < 1 || steps_per_unit < 1 || !(quantum > 0.0)) return -1;
    int64_t unit[4096];
    if (n > 4096) return -1;
    int64_t hyper = 1;
    for (int k = 0; k < n; ++k) {
        if (!(T[k] > 0.0)) return -1;
        double per_unit = T[k] / (double)e_warmup;
        double whole = rint(per_unit / quantum);
        if (whole >= 1048576.0) return -1;
        unit[k] = whole < 1.0 ? 1 : (int64_t)whole;
        int64_t a = hyper, b = unit[k];
        while (b) { int64_t t = a % b; a = b; b = t; }          /* a = gcd(hyper, unit[k]) */
        hyper = hyper / a * unit[k];
        if (hyper > ((int64_t)1 << 40)) return -1;
    }
    for (int k = 0; k < n; ++k) {
        int64_t e = (int64_t)t_sync * steps_per_unit * (hyper / unit[k]);
        if (e > 1048576) return -1;
        steps[k] = (int32_t)e;
    }
    return 0;
}

/* ------------------------------------------------------------------------- */
/* Local training of every replica for its own number of steps (Algorithm 1,  */
/* inner loop; local-update equation of Sec. 2.2).  Each step: next B rows of */
/* the replica's shard (sequential walk with wrap-around), forward, backward, */
/* buf = momentum*buf + g, w = w - lr*buf (momentum 0 is the paper's update). */
/* params [N][m_total], buf [N][m_train], cursor[N] steps taken so far,       */
/* versions[N] receives the number of steps completed in this call.           */
/* x [N][n_samples][H*W*C] float, y [N][n_samples].  loss_out[N]: last loss.  */
/* ------------------------------------------------------------------------- */
void hadfl_oracle_local_steps(const net_t *n, int N, double *params, double *buf, int64_t *cursor,
                              const int32_t *steps, int32_t *versions, const float *x, const int32_t *y,
                              int n_samples, int B, double lr, double momentum, double *loss_out)
{
    const int64_t in_sz = numel(n->shp[0]);
#pragma omp parallel for schedule(dynamic, 1)
    for (int k = 0; k < N; ++k) {
        double *w = params + (int64_t)k * n->m_total;
        double *bf = buf + (int64_t)k * n->m_train;
        double *g = (double *)malloc(sizeof(double) * (size_t)n->m_train);
        int done = 0;
        for (int e = 0; e < steps[k]; ++e) {
            int64_t first = (cursor[k] * B) % n_samples;
            cursor[k] += 1;
            const float *xb = x + ((int64_t)k * n_samples + first) * in_sz;
            const int32_t *yb = y + (int64_t)k * n_samples + first;
            double loss = hadfl_oracle_loss_grad(n, w, xb, yb, NULL, LOSS_SOFTMAX_CE, B, g, 1, NULL);
            if (loss_out) loss_out[k] = loss;
            for (int64_t j = 0; j < n->m_train; ++j) {
                bf[j] = momentum * bf[j] + g[j];
                w[j] = w[j] - lr * bf[j];
            }
            ++done;
        }
        versions[k] = done;
        free(g);
    }
}

/* ------------------------------------------------------------------------- */
/* Philox4x32-10 (Salmon, Moraes, Dror, Shaw: "Parallel random numbers: as    */
/* easy as 1, 2, 3", SC'11): 10 rounds, multipliers D2511F53 / CD9E8D57, key  */
/* schedule increments 9E3779B9 / BB67AE85.                                   */
/* ------------------------------------------------------------------------- */
void hadfl_oracle_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4])
{
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3], k0 = key[0], k1 = key[1];
    for (int r = 0; r < 10; ++r) {
        uint64_t p0 = (uint64_t)0xD2511F53u * c0, p1 = (uint64_t)0xCD9E8D57u * c2;
        uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0, n1 = (uint32_t)p1;
        uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1, n3 = (uint32_t)p0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += 0x9E3779B9u; k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* Uniform in [0,1) with 53 bits for draw t of cycle `cycle`: counter (cycle_lo, cycle_hi, t, 0), key = seed. */
double hadfl_oracle_uniform(uint64_t seed, uint64_t cycle, uint32_t t)
{
    uint32_t ctr[4] = { (uint32_t)cycle, (uint32_t)(cycle >> 32), t, 0u };
    uint32_t key[2] = { (uint32_t)seed, (uint32_t)(seed >> 32) }, o[4];
    hadfl_oracle_philox4x32_10(ctr, key, o);
    uint64_t bits = ((uint64_t)o[1] << 32) | o[0];
    return (double)(bits >> 11) * 0x1.0p-53;
}

/* ------------------------------------------------------------------------- */
/* exp(x) for x in [-745, 0] from exactly-rounded fp64 operations only, so    */
/* that any IEEE-754 machine returns the same bits: n = rint(x*log2(e));      */
/* r = (x - n*ln2_hi) - n*ln2_lo; Horner evaluation of the degree-13 Taylor   */
/* polynomial of exp(r); scaling by 2^n through the exponent field.           */
/* Built with -ffp-contract=off.                                              */
/* ------------------------------------------------------------------------- */
double hadfl_oracle_exp(double x)
{
    static const double inv_fact[14] = {
        1.0, 1.0, 1.0 / 2.0, 1.0 / 6.0, 1.0 / 24.0, 1.0 / 120.0, 1.0 / 720.0, 1.0 / 5040.0,
        1.0 / 40320.0, 1.0 / 362880.0, 1.0 / 3628800.0, 1.0 / 39916800.0, 1.0 / 479001600.0,
        1.0 / 6227020800.0 };
    const double log2e = 0x1.71547652b82fep+0, ln2_hi = 0x1.62e42feep-1, ln2_lo = 0x1.a39ef35793c76p-33;
    double nn = rint(x * log2e);
    double r = (x - nn * ln2_hi) - nn * ln2_lo;
    double p = inv_fact[13];
    for (int i = 12; i >= 0; --i) p = p * r + inv_fact[i];
    int64_t e = (int64_t)nn + 1023;                     /* >= 1 for x >= -708 */
    if (e < 1) return 0.0;
    uint64_t bits = (uint64_t)e << 52;
    double scale; memcpy(&scale, &bits, 8);
    return p * scale;
}

/* ------------------------------------------------------------------------- */
/* Probability-based selection (Sec. 3.3): mu = third quartile of the         */
/* available replicas' versions (linear interpolation at 0.75*(n-1) of the    */
/* sorted values); f_k = exp(-(v_k-mu)^2/2), exponent clamped at -690 so that */
/* no available replica has probability zero; P_k = f_k / sum f.  n_select    */
/* replicas are drawn one after another without replacement, each draw        */
/* proportional to f over the replicas still remaining (ascending index).     */
/* Outputs: selected[n_select] in draw order, flag[N], f[N] (0 where          */
/* unavailable), *mu_out.  Returns 0, or -1 when fewer than n_select replicas */
/* are available.                                                             */
/* ------------------------------------------------------------------------- */
int hadfl_oracle_select(const double *versions, const uint8_t *avail, int N, int n_select,
                        uint64_t seed, uint64_t cycle, int32_t *selected, uint8_t *flag,
                        double *f, double *mu_out)
{
    double *s = (double *)malloc(sizeof(double) * (size_t)N);
    int na = 0;
    for (int k = 0; k < N; ++k) if (!avail || avail[k]) s[na++] = versions[k];
    if (n_select < 1 || na < n_select) { free(s); return -1; }
    for (int i = 1; i < na; ++i) {                       /* insertion sort, ascending */
        double v = s[i]; int j = i - 1;
        while (j >= 0 && s[j] > v) { s[j + 1] = s[j]; --j; }
        s[j + 1] = v;
    }
    double pos = 0.75 * (double)(na - 1);
    int lo = (int)floor(pos);
    double frac = pos - (double)lo;
    double mu = s[lo];
    if (lo + 1 < na) mu = s[lo] + frac * (s[lo + 1] - s[lo]);
    free(s);
    if (mu_out) *mu_out = mu;

    for (int k = 0; k < N; ++k) {
        flag[k] = 0;
        if (avail && !avail[k]) { f[k] = 0.0; continue; }
        double d = versions[k] - mu;
        double e = -(d * d) * 0.5;
        if (e < -690.0) e = -690.0;
        f[k] = hadfl_oracle_exp(e);
    }
    for (int t = 0; t < n_select; ++t) {
        double S = 0.0;
        int last = -1;
        for (int k = 0; k < N; ++k) if (!flag[k] && f[k] > 0.0) { S += f[k]; last = k; }
        double u = hadfl_oracle_uniform(seed, cycle, (uint32_t)t);
        double thr = u * S, run = 0.0;
        int pick = last;
        for (int k = 0; k < N; ++k) {
            if (flag[k] || !(f[k] > 0.0)) continue;
            run += f[k];
            if (run > thr) { pick = k; break; }
        }
        selected[t] = pick;
        flag[pick] = 1;
    }
    return 0;
}

/* ------------------------------------------------------------------------- */
/* Partial aggregation (Sec. 2.3, partial-aggregation equation, with the      */
/* divisor read as the number of flagged replicas so the weights sum to one): */
/*   w_agg[j] = sum over flagged k, ascending, of a_k * W[k][j].              */
/* a[N] holds the weight of every replica (0 where Flag is 0).                */
/* ------------------------------------------------------------------------- */
void hadfl_oracle_aggregate(const double *params, int N, int64_t M, const double *a, double *agg)
{
#pragma omp parallel for schedule(static)
    for (int64_t j = 0; j < M; ++j) {
        double s = 0.0;
        for (int k = 0; k < N; ++k)
            if (a[k] != 0.0) s += a[k] * params[(int64_t)k * M + j];
        agg[j] = s;
    }
}

/* fp32-stored variant used for the aggregation stress workload (replica rows are given as floats). */
void hadfl_oracle_aggregate_f32(const float *params, int64_t row_stride, int N, int64_t M,
                                const double *a, double *agg)
{
#pragma omp parallel for schedule(static)
    for (int64_t j = 0; j < M; ++j) {
        double s = 0.0;
        for (int k = 0; k < N; ++k)
            if (a[k] != 0.0) s += a[k] * (double)params[(int64_t)k * row_stride + j];
        agg[j] = s;
    }
}

/* Global synchronisation (Algorithm 1): every replica's parameters become the aggregate. */
void hadfl_oracle_resync(double *params, int N, int64_t M, const double *agg)
{
    for (int k = 0; k < N; ++k) memcpy(params + (int64_t)k * M, agg, sizeof(double) * (size_t)M);
}

/* ------------------------------------------------------------------------- */
/* Runtime version predictor (Sec. 3.2): Brown's double exponential smoothing */
/* s1 = a*v + (1-a)*s1; s2 = a*s1 + (1-a)*s2; level = 2*s1 - s2;              */
/* trend = a/(1-a)*(s1-s2); forecast(m) = level + trend*m.                    */
/* s1, s2 are the states (both start at the first observation).               */
/* ------------------------------------------------------------------------- */
double hadfl_oracle_predict(double *s1, double *s2, double v, double alpha, int m, int first)
{
    if (first) { *s1 = v; *s2 = v; }
    else {
        *s1 = alpha * v + (1.0 - alpha) * (*s1);
        *s2 = alpha * (*s1) + (1.0 - alpha) * (*s2);
    }
    double level = 2.0 * (*s1) - (*s2);
    double trend = alpha / (1.0 - alpha) * ((*s1) - (*s2));
    return level + trend * (double)m;
}

int hadfl_oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
