/*
 * Oracle for PASGD + AdaComm.  TEST INFRASTRUCTURE ONLY -- see pasgd_oracle.h.
 * Plain C, fp32 storage, double accumulation, one rounding per stored value.
 */
#include "pasgd_oracle.h"

#include <math.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* Accumulator of the matrix-product reductions (forward products, dW, db, dA).  double is the
 * oracle.  Compiled with -DORC_ACC_FLOAT the same loops add in fp32, in the same order: a second
 * library that exists only so that tests can SHOW how far a result moves, and which ReLU gates
 * change side, when nothing but the summation precision changes.  It is never what the HIP path
 * is compared with. */
#ifdef ORC_ACC_FLOAT
typedef float orc_acc;
#else
typedef double orc_acc;
#endif

int orc_acc_bytes(void) { return (int)sizeof(orc_acc); }

struct orc_state {
    int m;
    int64_t P;
    orc_model md;
    uint64_t seed;
    int64_t k;                 /* local iterations done so far */
    float *X, *V;              /* [m,P] */
    float* last_loss;          /* [m] */
    const float* data;
    const int32_t* labels;
    const float *qa, *qc;      /* QUAD constants [m,P] */
    int block;                 /* block momentum active */
    float beta_glob;
    float *u, *xs;             /* global buffer and last synchronised model [P] */
};

static int g_threads = 1;

/* ---------------------------------------------------------------- pieces -- */

uint64_t orc_mix64(uint64_t z) {
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ULL;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBULL;
    return z ^ (z >> 31);
}

/* Three chained SplitMix64 draws, the state offset in turn by the iteration,
 * the worker and the position in the batch; reduced modulo N. */
int64_t orc_index(uint64_t seed, int i, int64_t k, int b, int64_t N) {
    const uint64_t gamma = 0x9E3779B97F4A7C15ULL;
    uint64_t h = orc_mix64(seed + gamma * ((uint64_t)k + 1));
    h = orc_mix64(h + gamma * ((uint64_t)i + 1));
    h = orc_mix64(h + gamma * ((uint64_t)b + 1));
    return (int64_t)(h % (uint64_t)N);
}

/* Bijection of [0, n): balanced Feistel network on 2w bits (2^(2w) >= n), four rounds whose round
 * function is the SplitMix64 mixer of (round key + right half); values that land outside [0, n) are
 * walked through the network again (the network is a permutation of the 2w-bit domain, so the walk
 * returns below n after finitely many steps). */
static uint64_t feistel_permute(uint64_t x, uint64_t n, uint64_t key) {
    int w = 1;
    while (((uint64_t)1 << (2 * w)) < n) ++w;
    const uint64_t mask = ((uint64_t)1 << w) - 1;
    const uint64_t gamma = 0x9E3779B97F4A7C15ULL;
    do {
        uint64_t l = x >> w, r = x & mask;
        for (int round = 0; round < 4; ++round) {
            const uint64_t f = orc_mix64(key + gamma * (uint64_t)(round + 1) + r) & mask;
            const uint64_t t = l ^ f;
            l = r;
            r = t;
        }
        x = (l << w) | r;
    } while (x >= n);
    return x;
}

int64_t orc_index_partition(uint64_t seed, int i, int64_t k, int b, int64_t N, int m, int B) {
    const int64_t lo = (int64_t)i * N / m, hi = (int64_t)(i + 1) * N / m;
    const int64_t n = hi - lo;
    const int64_t nmin = N / m;                     /* the smallest partition has floor(N / m) samples */
    const int64_t S = nmin / B;
    if (S < 1) return -1;
    const int64_t epoch = k / S, pos = (k % S) * B + b;
    const uint64_t gamma = 0x9E3779B97F4A7C15ULL;
    uint64_t key = orc_mix64(seed + gamma * ((uint64_t)epoch + 1));
    key = orc_mix64(key + gamma * ((uint64_t)i + 1));
    return lo + (int64_t)feistel_permute((uint64_t)pos, (uint64_t)n, key);
}

float orc_bf16_round(float x) {
    uint32_t u;
    memcpy(&u, &x, 4);
    if ((u & 0x7F800000u) == 0x7F800000u) { /* inf / nan: truncate, keep nan a nan */
        u &= 0xFFFF0000u;
        if ((u & 0x007F0000u) == 0 && isnan(x)) u |= 0x00400000u;
    } else {
        u += 0x7FFFu + ((u >> 16) & 1u);
        u &= 0xFFFF0000u;
    }
    memcpy(&x, &u, 4);
    return x;
}

int64_t orc_param_count(const orc_model* md) {
    int64_t p = 0;
    for (int l = 0; l < md->n_layers; ++l)
        p += (int64_t)md->dims[l] * md->dims[l + 1] + md->dims[l + 1];
    return p;
}

/* Forward pass of one sample through layers 1..L.
 *   w_op : parameters whose weight entries are the matrix-product operands
 *   x    : master parameters (biases are read from here)
 *   act  : act[l] points at the sample's d_l activations; act[0] is the input
 * Hidden layers apply ReLU; act[L] receives the logits.  q != 0 rounds every
 * hidden activation to bf16 when it is produced.  zpre (optional) receives the
 * values before the ReLU. */
static void forward_sample(const orc_model* md, const float* w_op, const float* x,
                           float* const* act, orc_acc* acc, int q, float* const* zpre) {
    int64_t off = 0;
    for (int l = 1; l <= md->n_layers; ++l) {
        const int din = md->dims[l - 1], dout = md->dims[l];
        const float* W = w_op + off;
        const float* bias = x + off + (int64_t)din * dout;
        for (int c = 0; c < dout; ++c) acc[c] = 0;
        for (int kk = 0; kk < din; ++kk) {
            const orc_acc a = (orc_acc)act[l - 1][kk];
            const float* wr = W + (int64_t)kk * dout;
            for (int c = 0; c < dout; ++c) acc[c] += a * (orc_acc)wr[c];
        }
        for (int c = 0; c < dout; ++c) {
            float z = (float)(acc[c] + (orc_acc)bias[c]);
            if (zpre && zpre[l]) zpre[l][c] = z;
            if (l < md->n_layers) {
                z = z > 0.0f ? z : 0.0f;
                if (q) z = orc_bf16_round(z);
            }
            act[l][c] = z;
        }
        off += (int64_t)din * dout + dout;
    }
}

/* -log softmax(z)[y] with the maximum subtracted, and optionally p. */
static double softmax_nll(const float* z, int C, int y, double* p) {
    double zmax = (double)z[0];
    for (int c = 1; c < C; ++c)
        if ((double)z[c] > zmax) zmax = (double)z[c];
    double sum = 0.0;
    for (int c = 0; c < C; ++c) {
        const double e = exp((double)z[c] - zmax);
        if (p) p[c] = e;
        sum += e;
    }
    if (p)
        for (int c = 0; c < C; ++c) p[c] /= sum;
    return -((double)z[y] - zmax - log(sum));
}

static int max_dim(const orc_model* md) {
    int d = 0;
    for (int l = 0; l <= md->n_layers; ++l)
        if (md->dims[l] > d) d = md->dims[l];
    return d;
}

float orc_mlp_loss_grad(const orc_model* md, const float* x, const float* data,
                        const int32_t* labels, const int64_t* idx, float* grad) {
    const int L = md->n_layers, B = md->B, q = md->bf16;
    const int C = md->dims[L];
    const int64_t P = orc_param_count(md);
    const int dmax = max_dim(md);

    /* operand copy of the parameters: weights rounded to bf16 in bf16 mode */
    float* w_op = (float*)malloc(sizeof(float) * (size_t)P);
    memcpy(w_op, x, sizeof(float) * (size_t)P);
    if (q) {
        int64_t off = 0;
        for (int l = 1; l <= L; ++l) {
            const int64_t nw = (int64_t)md->dims[l - 1] * md->dims[l];
            for (int64_t j = 0; j < nw; ++j) w_op[off + j] = orc_bf16_round(w_op[off + j]);
            off += nw + md->dims[l];
        }
    }

    /* activations A_l [B,d_l] and deltas dZ_l [B,d_l] */
    float* A[ORC_MAX_LAYERS + 1];
    float* dZ[ORC_MAX_LAYERS + 1];
    for (int l = 0; l <= L; ++l) {
        A[l] = (float*)malloc(sizeof(float) * (size_t)B * md->dims[l]);
        dZ[l] = (l >= 1) ? (float*)malloc(sizeof(float) * (size_t)B * md->dims[l]) : NULL;
    }
    orc_acc* acc = (orc_acc*)malloc(sizeof(orc_acc) * (size_t)(dmax > B ? dmax : B));
    double* p = (double*)malloc(sizeof(double) * (size_t)C);

    double loss_sum = 0.0;
    for (int b = 0; b < B; ++b) {
        const float* row = data + idx[b] * (int64_t)md->dims[0];
        for (int j = 0; j < md->dims[0]; ++j) A[0][(int64_t)b * md->dims[0] + j] = q ? orc_bf16_round(row[j]) : row[j];
        float* act[ORC_MAX_LAYERS + 1];
        for (int l = 0; l <= L; ++l) act[l] = A[l] + (int64_t)b * md->dims[l];
        forward_sample(md, w_op, x, act, acc, q, NULL);
        const int y = labels[idx[b]];
        loss_sum += softmax_nll(act[L], C, y, p);
        /* dZ_L = (p - onehot) / B : gradient of the batch-mean loss */
        for (int c = 0; c < C; ++c) {
            float d = (float)((p[c] - (c == y ? 1.0 : 0.0)) / (double)B);
            dZ[L][(int64_t)b * C + c] = q ? orc_bf16_round(d) : d;
        }
    }
    const float loss = (float)(loss_sum / (double)B);

    if (grad) {
        /* offsets of each layer's block inside the flat vector */
        int64_t offs[ORC_MAX_LAYERS + 1];
        offs[1] = 0;
        for (int l = 1; l < L; ++l) offs[l + 1] = offs[l] + (int64_t)md->dims[l - 1] * md->dims[l] + md->dims[l];
        for (int l = L; l >= 1; --l) {
            const int din = md->dims[l - 1], dout = md->dims[l];
            float* gW = grad + offs[l];
            float* gb = gW + (int64_t)din * dout;
            const float* W = w_op + offs[l];
            /* dW_l = A_{l-1}^T dZ_l */
            for (int kk = 0; kk < din; ++kk) {
                for (int c = 0; c < dout; ++c) acc[c] = 0;
                for (int b = 0; b < B; ++b) {
                    const orc_acc a = (orc_acc)A[l - 1][(int64_t)b * din + kk];
                    const float* dz = dZ[l] + (int64_t)b * dout;
                    for (int c = 0; c < dout; ++c) acc[c] += a * (orc_acc)dz[c];
                }
                for (int c = 0; c < dout; ++c) gW[(int64_t)kk * dout + c] = (float)acc[c];
            }
            /* db_l = sum_b dZ_l */
            for (int c = 0; c < dout; ++c) {
                orc_acc s = 0;
                for (int b = 0; b < B; ++b) s += (orc_acc)dZ[l][(int64_t)b * dout + c];
                gb[c] = (float)s;
            }
            /* dZ_{l-1} = (dZ_l W_l^T) .* [A_{l-1} > 0]   (derivative of ReLU at 0 is 0) */
            if (l > 1) {
                for (int b = 0; b < B; ++b) {
                    const float* dz = dZ[l] + (int64_t)b * dout;
                    for (int kk = 0; kk < din; ++kk) {
                        const float* wr = W + (int64_t)kk * dout;
                        orc_acc s = 0;
                        for (int c = 0; c < dout; ++c) s += (orc_acc)dz[c] * (orc_acc)wr[c];
                        float d = A[l - 1][(int64_t)b * din + kk] > 0.0f ? (float)s : 0.0f;
                        dZ[l - 1][(int64_t)b * din + kk] = q ? orc_bf16_round(d) : d;
                    }
                }
            }
        }
    }

    for (int l = 0; l <= L; ++l) {
        free(A[l]);
        free(dZ[l]);
    }
    free(acc);
    free(p);
    free(w_op);
    return loss;
}

void orc_mlp_preactivations(const orc_model* md, const float* x, const float* data,
                             const int64_t* idx, float* zout) {
    const int L = md->n_layers, B = md->B, q = md->bf16;
    const int64_t P = orc_param_count(md);
    const int dmax = max_dim(md);
    int hidden = 0;
    for (int l = 1; l < L; ++l) hidden += md->dims[l];
    float* w_op = (float*)malloc(sizeof(float) * (size_t)P);
    memcpy(w_op, x, sizeof(float) * (size_t)P);
    if (q) {
        int64_t off = 0;
        for (int l = 1; l <= L; ++l) {
            const int64_t nw = (int64_t)md->dims[l - 1] * md->dims[l];
            for (int64_t j = 0; j < nw; ++j) w_op[off + j] = orc_bf16_round(w_op[off + j]);
            off += nw + md->dims[l];
        }
    }
    orc_acc* acc = (orc_acc*)malloc(sizeof(orc_acc) * (size_t)dmax);
    float* buf[ORC_MAX_LAYERS + 1];
    for (int l = 0; l <= L; ++l) buf[l] = (float*)malloc(sizeof(float) * (size_t)md->dims[l]);
    for (int b = 0; b < B; ++b) {
        const float* row = data + idx[b] * (int64_t)md->dims[0];
        for (int j = 0; j < md->dims[0]; ++j) buf[0][j] = q ? orc_bf16_round(row[j]) : row[j];
        float* zp[ORC_MAX_LAYERS + 1];
        int o = 0;
        for (int l = 0; l <= L; ++l) {
            zp[l] = (l >= 1 && l < L) ? zout + (int64_t)b * hidden + o : NULL;
            if (l >= 1 && l < L) o += md->dims[l];
        }
        forward_sample(md, w_op, x, buf, acc, q, zp);
    }
    for (int l = 0; l <= L; ++l) free(buf[l]);
    free(acc);
    free(w_op);
}

void orc_sgd_update(int64_t P, float* x, float* v, const float* g, float lr, float beta, float wd) {
    for (int64_t j = 0; j < P; ++j) {
        const double gt = (double)g[j] + (double)wd * (double)x[j];
        v[j] = (float)((double)beta * (double)v[j] + gt);
        x[j] = (float)((double)x[j] - (double)lr * (double)v[j]);
    }
}

int orc_next_tau(double F0, double Fl, int tau0) {
    if (!(F0 > 0.0) || !(Fl >= 0.0) || !isfinite(F0) || !isfinite(Fl) || tau0 < 1) return -1;
    const double ratio = Fl / F0;
    const double root = sqrt(ratio);
    const double prod = root * (double)tau0;
    const double up = ceil(prod);
    if (!(up < 2147483647.0)) return -2;
    const int t = (int)up;
    return t < 1 ? 1 : t;
}

int orc_next_tau_ex(double F0, double Fl, int tau0, int tau_prev, double gamma, int slack,
                    double lr0, double lrl, int lr_changed) {
    if (!(F0 > 0.0) || !(Fl >= 0.0) || !isfinite(F0) || !isfinite(Fl) || tau0 < 1 || tau_prev < 1) return -1;
    if (!(gamma > 0.0) || !(gamma < 1.0) || slack < 0) return -1;   /* Sec. 4.3.1: a decay factor below 1 */
    if (!(lr0 > 0.0) || !(lrl > 0.0) || !isfinite(lr0) || !isfinite(lrl)) return -1;
    const double ratio = Fl / F0;
    const double coupling = lr0 / lrl;
    const double scaled = coupling * ratio;
    const double root = sqrt(scaled);
    const double prod = root * (double)tau0;
    const double up = ceil(prod);
    if (!(up < 2147483647.0)) return -2;
    int cand = (int)up;
    if (cand < 1) cand = 1;
    if (lr_changed) return cand;
    if ((int64_t)cand + (int64_t)slack < (int64_t)tau_prev) return cand;
    const double shrunk = ceil(gamma * (double)tau_prev);
    const int t = (int)shrunk;
    return t < 1 ? 1 : t;
}

/* ------------------------------------------------------------------ a run -- */

orc_state* orc_create(int m, const orc_model* md, uint64_t seed, const float* x1,
                      const float* data, const int32_t* labels,
                      const float* qa, const float* qc) {
    orc_state* s = (orc_state*)calloc(1, sizeof(orc_state));
    s->m = m;
    s->md = *md;
    s->P = (md->kind == ORC_KIND_QUAD) ? (int64_t)md->dims[0] : orc_param_count(md);
    s->seed = seed;
    s->k = 0;
    s->X = (float*)malloc(sizeof(float) * (size_t)m * s->P);
    s->V = (float*)calloc((size_t)m * s->P, sizeof(float));
    s->last_loss = (float*)calloc((size_t)m, sizeof(float));
    for (int i = 0; i < m; ++i) memcpy(s->X + (int64_t)i * s->P, x1, sizeof(float) * (size_t)s->P);
    s->data = data;
    s->labels = labels;
    s->qa = qa;
    s->qc = qc;
    return s;
}

void orc_destroy(orc_state* s) {
    if (!s) return;
    free(s->u);
    free(s->xs);
    free(s->X);
    free(s->V);
    free(s->last_loss);
    free(s);
}

int orc_set_threads(int n) {
#ifdef _OPENMP
    if (n >= 1) g_threads = n;
    if (g_threads > omp_get_num_procs()) g_threads = omp_get_num_procs();
#else
    (void)n;
    g_threads = 1;
#endif
    return g_threads;
}

void orc_set_lr(orc_state* s, float lr) { s->md.lr = lr; }
int64_t orc_k(const orc_state* s) { return s->k; }
float* orc_X(orc_state* s) { return s->X; }
float* orc_V(orc_state* s) { return s->V; }
const float* orc_last_losses(const orc_state* s) { return s->last_loss; }

/* one local iteration of worker i at iteration index k */
static void worker_step(orc_state* s, int i, int64_t k) {
    const int64_t P = s->P;
    float* x = s->X + (int64_t)i * P;
    float* v = s->V + (int64_t)i * P;
    float* g = (float*)malloc(sizeof(float) * (size_t)P);
    if (s->md.kind == ORC_KIND_QUAD) {
        /* deterministic gradient of 0.5 sum a (x - c)^2 */
        const float* a = s->qa + (int64_t)i * P;
        const float* c = s->qc + (int64_t)i * P;
        double f = 0.0;
        for (int64_t j = 0; j < P; ++j) {
            const double d = (double)x[j] - (double)c[j];
            f += 0.5 * (double)a[j] * d * d;
            g[j] = (float)((double)a[j] * d);
        }
        s->last_loss[i] = (float)f;
    } else {
        int64_t* idx = (int64_t*)malloc(sizeof(int64_t) * (size_t)s->md.B);
        for (int b = 0; b < s->md.B; ++b)
            idx[b] = s->md.sampler ? orc_index_partition(s->seed, i, k, b, s->md.N, s->m, s->md.B)
                                   : orc_index(s->seed, i, k, b, s->md.N);
        s->last_loss[i] = orc_mlp_loss_grad(&s->md, x, s->data, s->labels, idx, g);
        free(idx);
    }
    orc_sgd_update(P, x, v, g, s->md.lr, s->md.beta, s->md.wd);
    free(g);
}

void orc_local_steps_subset(orc_state* s, int tau, const int* ids, int n) {
    /* workers do not interact between averaging steps, so the loop over workers
     * may run in any order (or in parallel); each worker's steps are sequential */
#ifdef _OPENMP
#pragma omp parallel for schedule(dynamic, 1) num_threads(g_threads)
#endif
    for (int j = 0; j < n; ++j) {
        for (int t = 0; t < tau; ++t) worker_step(s, ids[j], s->k + t);
    }
    s->k += tau;
}

void orc_local_steps(orc_state* s, int tau) {
    int* ids = (int*)malloc(sizeof(int) * (size_t)s->m);
    for (int i = 0; i < s->m; ++i) ids[i] = i;
    orc_local_steps_subset(s, tau, ids, s->m);
    free(ids);
}

void orc_update_from_grad(orc_state* s, const float* G) {
    for (int i = 0; i < s->m; ++i)
        orc_sgd_update(s->P, s->X + (int64_t)i * s->P, s->V + (int64_t)i * s->P, G + (int64_t)i * s->P,
                       s->md.lr, s->md.beta, s->md.wd);
}

static void mean_model(const orc_state* s, float* xbar) {
    for (int64_t j = 0; j < s->P; ++j) {
        double sum = 0.0;
        for (int i = 0; i < s->m; ++i) sum += (double)s->X[(int64_t)i * s->P + j];
        xbar[j] = (float)(sum / (double)s->m);
    }
}

void orc_block_begin(orc_state* s, float beta_glob) {
    if (!s->u) s->u = (float*)malloc(sizeof(float) * (size_t)s->P);
    if (!s->xs) s->xs = (float*)malloc(sizeof(float) * (size_t)s->P);
    memset(s->u, 0, sizeof(float) * (size_t)s->P);
    memcpy(s->xs, s->X, sizeof(float) * (size_t)s->P);
    memset(s->V, 0, sizeof(float) * (size_t)s->m * s->P);
    s->beta_glob = beta_glob;
    s->block = 1;
}

void orc_block_end(orc_state* s) { s->block = 0; }
const float* orc_block_u(const orc_state* s) { return s->block ? s->u : NULL; }

void orc_average(orc_state* s) {
    float* xbar = (float*)malloc(sizeof(float) * (size_t)s->P);
    mean_model(s, xbar);
    if (s->block) {
        const double lr = (double)s->md.lr, bg = (double)s->beta_glob;
        for (int64_t j = 0; j < s->P; ++j) {
            const double G = ((double)s->xs[j] - (double)xbar[j]) / lr;
            s->u[j] = (float)(bg * (double)s->u[j] + G);
            s->xs[j] = (float)((double)s->xs[j] - lr * (double)s->u[j]);
            xbar[j] = s->xs[j];
        }
        memset(s->V, 0, sizeof(float) * (size_t)s->m * s->P);
    }
    for (int i = 0; i < s->m; ++i) memcpy(s->X + (int64_t)i * s->P, xbar, sizeof(float) * (size_t)s->P);
    free(xbar);
}

double orc_loss(orc_state* s) {
    float* xbar = (float*)malloc(sizeof(float) * (size_t)s->P);
    mean_model(s, xbar);
    double F = 0.0;
    if (s->md.kind == ORC_KIND_QUAD) {
        /* F(x) = (1/m) sum_i 0.5 sum_p a_ip (x_p - c_ip)^2 */
        for (int i = 0; i < s->m; ++i) {
            double f = 0.0;
            for (int64_t j = 0; j < s->P; ++j) {
                const double d = (double)xbar[j] - (double)s->qc[(int64_t)i * s->P + j];
                f += 0.5 * (double)s->qa[(int64_t)i * s->P + j] * d * d;
            }
            F += f;
        }
        F /= (double)s->m;
    } else {
        const orc_model* md = &s->md;
        const int L = md->n_layers, E = md->E, C = md->dims[L];
        const int dmax = max_dim(md);
        double* per = (double*)malloc(sizeof(double) * (size_t)E);
#ifdef _OPENMP
#pragma omp parallel num_threads(g_threads)
#endif
        {
            float* buf[ORC_MAX_LAYERS + 1];
            for (int l = 1; l <= L; ++l) buf[l] = (float*)malloc(sizeof(float) * (size_t)md->dims[l]);
            orc_acc* acc = (orc_acc*)malloc(sizeof(orc_acc) * (size_t)dmax);
#ifdef _OPENMP
#pragma omp for schedule(static)
#endif
            for (int e = 0; e < E; ++e) {
                float* act[ORC_MAX_LAYERS + 1];
                act[0] = (float*)(s->data + (int64_t)e * md->dims[0]); /* read only */
                for (int l = 1; l <= L; ++l) act[l] = buf[l];
                forward_sample(md, xbar, xbar, act, acc, 0, NULL);
                per[e] = softmax_nll(act[L], C, s->labels[e], NULL);
            }
            for (int l = 1; l <= L; ++l) free(buf[l]);
            free(acc);
        }
        for (int e = 0; e < E; ++e) F += per[e];
        F /= (double)E;
        free(per);
    }
    free(xbar);
    return F;
}

int orc_run(orc_state* s, int64_t K, int tau0, int adaptive, int64_t interval,
            int64_t* sched_k, int* sched_tau, int cap, int* n_sched, int64_t* rounds) {
    int tau = tau0, ns = 0;
    int64_t r = 0, next_eval = s->k + interval;
    double F0 = 0.0;
    if (adaptive) F0 = orc_loss(s);
    if (ns < cap) { sched_k[ns] = s->k; sched_tau[ns] = tau; }
    ++ns;
    const int64_t k_end = s->k + K;
    while (s->k < k_end) {
        const int64_t left = k_end - s->k;
        const int t = (int64_t)tau < left ? tau : (int)left;
        orc_local_steps(s, t);
        orc_average(s);
        ++r;
        if (adaptive && s->k >= next_eval && s->k < k_end) {
            const double Fl = orc_loss(s);
            const int nt = orc_next_tau(F0, Fl, tau0);
            if (nt < 0) { *n_sched = ns; *rounds = r; return nt; }
            tau = nt;
            if (ns < cap) { sched_k[ns] = s->k; sched_tau[ns] = tau; }
            ++ns;
            while (next_eval <= s->k) next_eval += interval;
        }
    }
    *n_sched = ns;
    *rounds = r;
    return 0;
}

int orc_run_ex(orc_state* s, int64_t K, int tau0, int64_t interval, int refine, double gamma, int slack,
               int n_lr, const int64_t* lr_at, const float* lr_val, int postpone_lr,
               int64_t* sched_k, int* sched_tau, float* sched_lr, int cap, int* n_sched, int64_t* rounds) {
    int tau = tau0, ns = 0, next_lr = 0, lr_changed = 0;
    int64_t r = 0, next_eval = s->k + interval;
    const double lr0 = (double)s->md.lr;
    const double F0 = orc_loss(s);
    if (ns < cap) { sched_k[ns] = s->k; sched_tau[ns] = tau; sched_lr[ns] = s->md.lr; }
    ++ns;
    const int64_t k_end = s->k + K;
    while (s->k < k_end) {
        const int64_t left = k_end - s->k;
        const int t = (int64_t)tau < left ? tau : (int)left;
        orc_local_steps(s, t);
        orc_average(s);
        ++r;
        /* scheduled learning-rate changes, applied at synchronisation points */
        while (next_lr < n_lr && s->k >= lr_at[next_lr] && (!postpone_lr || tau == 1)) {
            s->md.lr = lr_val[next_lr];
            ++next_lr;
            lr_changed = 1;
        }
        if (s->k >= next_eval && s->k < k_end) {
            const double Fl = orc_loss(s);
            const int nt = refine ? orc_next_tau_ex(F0, Fl, tau0, tau, gamma, slack, lr0, (double)s->md.lr, lr_changed)
                                  : orc_next_tau(F0, Fl, tau0);
            if (nt < 0) { *n_sched = ns; *rounds = r; return nt; }
            tau = nt;
            lr_changed = 0;
            if (ns < cap) { sched_k[ns] = s->k; sched_tau[ns] = tau; sched_lr[ns] = s->md.lr; }
            ++ns;
            while (next_eval <= s->k) next_eval += interval;
        }
    }
    *n_sched = ns;
    *rounds = r;
    return 0;
}
