/*
 * Oracle for periodic-averaging SGD (PASGD) with the AdaComm controller.
 *
 * THIS IS TEST INFRASTRUCTURE.  It is a plain, slow CPU statement of what the
 * method computes (Wang & Joshi, "Adaptive Communication Strategies to Achieve
 * the Best Error-Runtime Trade-off in Local-Update SGD"), used only by the
 * tests, the smoke check and the benchmark's CPU-baseline leg.  It shares no
 * code with the HIP library and the HIP library never calls it.
 *
 * Arithmetic: every stored value is fp32; every reduction (dot products, batch
 * means, the mean over workers) is accumulated in double and rounded to fp32
 * once.  In bf16 mode activations, deltas and the weight operand of every
 * matrix product are rounded to bfloat16 (nearest, ties to even) before the
 * multiply; master weights and momentum buffers stay fp32.
 *
 * Parity pins (tests/test_oracle_*.py): tau=1 equals synchronous SGD on the
 * mean gradient; m=1 equals serial SGD bit for bit; rows identical after
 * averaging; mean preserved; spread identity inside a period; closed forms on
 * a diagonal quadratic (with and without momentum); the MLP step against
 * PyTorch CPU autograd + torch.optim.SGD in fp64 and against central finite
 * differences; the controller against exact rational arithmetic; the index
 * stream's mixer against the published SplitMix64 output sequence; bf16
 * rounding against torch's conversion; the refined controller against exact
 * rational arithmetic and its driver against the quadratic closed form; block
 * momentum against synchronous momentum SGD (tau=1), plain averaging
 * (beta_glob=0) and a quadratic recurrence; the pre-activation observer against an
 * fp64 numpy forward pass (values and layout); the index stream against a Python
 * restatement of its chaining.  No function here is "parity unpinned".
 */
#ifndef PASGD_ORACLE_H
#define PASGD_ORACLE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define ORC_MAX_LAYERS 8
#define ORC_KIND_QUAD 0
#define ORC_KIND_MLP 1

typedef struct {
    int kind;                      /* ORC_KIND_QUAD or ORC_KIND_MLP (softmax regression = 1 layer) */
    int n_layers;                  /* L: number of weight layers */
    int dims[ORC_MAX_LAYERS + 1];  /* d_0 .. d_L */
    int B;                         /* mini-batch size per worker */
    int64_t N;                     /* dataset size */
    int E;                         /* evaluation subset: first E samples */
    float lr, beta, wd;            /* eta, momentum factor, weight decay */
    int bf16;                      /* 1: bf16 operands in the training GEMMs */
    int sampler;                   /* 0: with replacement from the whole set; 1: per-worker partition, reshuffled every epoch */
} orc_model;

typedef struct orc_state orc_state;

/* --- pieces ---------------------------------------------------------------- */

/* sizeof the accumulator of the matrix-product reductions: 8 in the oracle.  The same source
 * compiled with -DORC_ACC_FLOAT (libpasgd_oracle_f32acc.so) reports 4: a sensitivity probe that
 * adds in fp32 in the same order, used by tests only to show which results and ReLU gates move
 * with the summation precision -- never as the reference of a comparison with the HIP path. */
int orc_acc_bytes(void);

/* SplitMix64 output function (Steele, Lea & Flood 2014; Vigna's reference). */
uint64_t orc_mix64(uint64_t z);

/* Mini-batch index stream: sample b of worker i at local iteration k (k counts
 * from 0) is drawn with replacement from the whole dataset (Sec. 2: a random
 * mini-batch per step, one stream per worker as in the tau=1 special case). */
int64_t orc_index(uint64_t seed, int i, int64_t k, int b, int64_t N);

/* Partition sampler (Sec. 5.1, dataset paragraph: every worker owns one partition of the data and
 * reshuffles it after each epoch).  Worker i of m owns samples [floor(i N / m), floor((i+1) N / m));
 * an epoch is S = floor(min_i n_i / B) iterations; in epoch e = k / S the worker walks a pseudo-random
 * permutation of its partition (4-round Feistel network keyed by seed, worker and epoch, with cycle
 * walking), B positions per iteration.  Returns the dataset index, or -1 if a partition is smaller
 * than one batch. */
int64_t orc_index_partition(uint64_t seed, int i, int64_t k, int b, int64_t N, int m, int B);

/* fp32 -> nearest bfloat16 value (ties to even), returned as fp32. */
float orc_bf16_round(float x);

/* P for the model (biases included). */
int64_t orc_param_count(const orc_model* md);

/* Mini-batch loss and stochastic gradient g(x; xi) = (1/|xi|) sum grad f
 * (Sec. 2, mini-batch SGD) of an MLP at parameters x on the samples idx[0..B).
 * grad may be NULL.  Returns the mean cross-entropy of the batch. */
float orc_mlp_loss_grad(const orc_model* md, const float* x, const float* data,
                        const int32_t* labels, const int64_t* idx, float* grad);

/* Values Z_l before the ReLU of every hidden layer l = 1..L-1 for the samples
 * idx[0..B): zout is [B][d_1 + ... + d_{L-1}].  Lets a test see which ReLU gates
 * sit so close to zero that accumulation order decides them. */
void orc_mlp_preactivations(const orc_model* md, const float* x, const float* data,
                             const int64_t* idx, float* zout);

/* One (momentum-)SGD update  g += wd x;  v = beta v + g;  x = x - lr v
 * (mini-batch SGD update rule of Sec. 2; per-worker buffer of Sec. 5.3). */
void orc_sgd_update(int64_t P, float* x, float* v, const float* g, float lr, float beta, float wd);

/* AdaComm basic update rule: tau_l = ceil( sqrt(F_l / F_0) * tau_0 ), at least 1.
 * Negative on invalid input (F0 <= 0, Fl < 0, non-finite, tau0 < 1). */
int orc_next_tau(double F0, double Fl, int tau0);

/* AdaComm refinements (Sec. 4.3): candidate c = ceil( sqrt( (lr0/lrl) * Fl/F0 ) * tau0 ), the
 * practical learning-rate coupling of Sec. 4.3.2 (lr0 = lrl gives the basic rule).  Saturation
 * refinement (Sec. 4.3.1): c is taken only if c + slack < tau_prev,
 * otherwise the period becomes ceil(gamma * tau_prev).  At the first decision after a
 * learning-rate change (lr_changed != 0) c is taken as it is, since the coupling exists to let
 * the period grow there.  Result at least 1; negative on invalid input. */
int orc_next_tau_ex(double F0, double Fl, int tau0, int tau_prev, double gamma, int slack,
                    double lr0, double lrl, int lr_changed);

/* --- a run ------------------------------------------------------------------ */

/* m workers all starting at x1[P].  data [N,d_0] fp32, labels [N]; for QUAD
 * pass qa, qc as [m,P] (worker i minimises 0.5 sum_p qa (x - qc)^2).  The arrays
 * are borrowed, not copied, except x1. */
orc_state* orc_create(int m, const orc_model* md, uint64_t seed, const float* x1,
                      const float* data, const int32_t* labels,
                      const float* qa, const float* qc);
void orc_destroy(orc_state* s);

int orc_set_threads(int n);              /* OpenMP threads over workers; returns count in use */
void orc_set_lr(orc_state* s, float lr);
int64_t orc_k(const orc_state* s);
float* orc_X(orc_state* s);              /* [m,P] */
float* orc_V(orc_state* s);              /* [m,P] */
const float* orc_last_losses(const orc_state* s);  /* [m] mini-batch loss of the last step */

/* tau local iterations on every worker (no communication); k += tau. */
void orc_local_steps(orc_state* s, int tau);
/* Same, but only workers ids[0..n) are advanced (k still += tau).  For sampled
 * full-size parity checks: workers are independent between averaging steps. */
void orc_local_steps_subset(orc_state* s, int tau, const int* ids, int n);
/* One update from explicit gradients G[m,P] on every worker (k unchanged). */
void orc_update_from_grad(orc_state* s, const float* G);
/* Replace every worker's model by the mean of all models; buffers untouched. */
void orc_average(orc_state* s);
/* Block momentum (Sec. 5.3.1).  orc_block_begin() records the current (synchronised) model of
 * worker 0 as x_sync, sets the global buffer u = 0 and clears the local buffers; from then on
 * orc_average() is the block-momentum step
 *     G = (x_sync - x_bar) / lr        the accumulated step of the period, in gradient units
 *     u <- beta_glob u + G ;  x_sync <- x_sync - lr u ;  every worker <- x_sync
 * and clears every worker's local momentum buffer (momentum SGD restarts after each averaging
 * step).  orc_block_end() returns to plain averaging. */
void orc_block_begin(orc_state* s, float beta_glob);
void orc_block_end(orc_state* s);
const float* orc_block_u(const orc_state* s);   /* [P] or NULL */

/* Training loss of the averaged model on the first E samples, fp32 operands. */
double orc_loss(orc_state* s);

/* Driver: K iterations; periods of tau local steps each followed by averaging,
 * the last one truncated.  adaptive: every `interval` iterations (at the first
 * averaging boundary at or after the multiple) evaluate the loss and set tau by
 * orc_next_tau.  sched_k/sched_tau receive the (iteration, tau) decisions,
 * starting with (0, tau0); *n_sched their count (capacity cap); *rounds the
 * number of averaging steps.  Returns 0, or a negative orc_next_tau error. */
int orc_run(orc_state* s, int64_t K, int tau0, int adaptive, int64_t interval,
            int64_t* sched_k, int* sched_tau, int cap, int* n_sched, int64_t* rounds);

/* Driver with the refinements.  The learning-rate schedule is n_lr pairs (lr_at[j], lr_val[j]):
 * from iteration lr_at[j] on the rate should be lr_val[j].  Changes take effect at averaging
 * steps only; with postpone_lr != 0 a due change waits until tau has reached 1 (Sec. 4.3.2,
 * last paragraph).  refine = 0 uses orc_next_tau with the coupling factor ignored.
 * sched_lr receives the learning rate in force after each decision. */
int orc_run_ex(orc_state* s, int64_t K, int tau0, int64_t interval, int refine, double gamma, int slack,
               int n_lr, const int64_t* lr_at, const float* lr_val, int postpone_lr,
               int64_t* sched_k, int* sched_tau, float* sched_lr, int cap, int* n_sched, int64_t* rounds);

#ifdef __cplusplus
}
#endif
#endif
