/*
 * localcomm -- local-update SGD (periodic-averaging SGD, PASGD) with the
 * AdaComm communication-period controller, for one AMD MI355X (gfx950).
 *
 * Method: Wang & Joshi, "Adaptive Communication Strategies to Achieve the Best
 * Error-Runtime Trade-off in Local-Update SGD".  The m workers of the paper are
 * m model replicas held on one GPU as the rows of X[m, P]; a local SGD step is a
 * set of per-replica matrix products followed by a fused update; the averaging
 * step is a reduce over the m rows written back to every row.
 *
 * Conventions
 *   - Every function is extern "C", takes plain pointers and sizes, never throws
 *     and never aborts.  Unless stated otherwise it returns LC_OK (0) or a
 *     negative lc_status; lc_strerror() names it.
 *   - "device" pointers are HIP device memory owned by the caller (for example
 *     torch tensors); the library never frees or reallocates them.  "host"
 *     pointers are ordinary host memory.  The handle owns only host metadata.
 *   - All device work is enqueued on the stream given to lc_attach() and is
 *     asynchronous unless the function says it synchronises.
 *   - Parameter layout inside one replica row (P floats, fp32): for each layer
 *     l = 1..L the weight matrix W_l stored row-major as [d_{l-1}, d_l] followed
 *     by the bias b_l [d_l].  Rows of X and V are separated by
 *     lc_row_stride(P) floats (P rounded up to a multiple of 64, so that every
 *     row starts on a 256-byte boundary); the padding must be zero and stays zero.
 */
#ifndef LOCALCOMM_H
#define LOCALCOMM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define LC_MAX_LAYERS 8

typedef enum {
    LC_OK = 0,
    LC_ERR_ARG = -1,        /* invalid argument (null pointer, size, range) */
    LC_ERR_MODEL = -2,      /* inconsistent model description or P != P(model) */
    LC_ERR_STATE = -3,      /* call out of order (e.g. not attached) */
    LC_ERR_ALIGN = -4,      /* a device pointer is not 256-byte aligned */
    LC_ERR_WORKSPACE = -5,  /* scratch buffer too small */
    LC_ERR_HIP = -6,        /* a HIP call failed; lc_last_hip_error() has the code */
    LC_ERR_NONFINITE = -7,  /* the evaluated loss is not finite */
    LC_ERR_UNSUPPORTED = -8, /* shape outside what the kernels handle */
    LC_ERR_SYNC = -9,        /* a replica-wide barrier of the resident step kernel timed out */
    LC_ERR_PLACEMENT = -10,  /* a workgroup of the resident step kernel ran on another XCD than the probe predicted */
    LC_ERR_TOO_LARGE = -11   /* more parameters than the library's static scratch holds (LC_STATIC_MAX_PARAMS) */
} lc_status;

typedef enum { LC_KIND_QUAD = 0, LC_KIND_MLP = 1 } lc_kind;
typedef enum { LC_GEMM_FP32 = 0, LC_GEMM_BF16 = 1 } lc_gemm_dtype;
typedef enum { LC_SAMPLE_REPLACEMENT = 0, LC_SAMPLE_PARTITION = 1 } lc_sampler;

/* Model and optimiser description.
 *   LC_KIND_MLP : ReLU multi-layer perceptron with softmax cross-entropy loss;
 *                 n_layers = L weight layers, dims[0..L]; n_layers = 1 is
 *                 softmax regression.
 *   LC_KIND_QUAD: test objective; worker i minimises 0.5 sum_p a[i,p] (x_p -
 *                 c[i,p])^2 with the exact gradient (no sampling); dims[0] = P.
 *   gemm        : LC_GEMM_BF16 rounds activations, deltas and the weight operand
 *                 of every matrix product to bfloat16 (accumulation fp32, master
 *                 weights and momentum fp32); the dataset is then bf16 too.
 *   sampler     : LC_SAMPLE_REPLACEMENT draws every sample with replacement from the
 *                 whole set (the index stream documented at lc_init).
 *                 LC_SAMPLE_PARTITION follows the data handling of Sec. 5.1 (every worker owns a
 *                 fixed share of the training set and reshuffles that share once per epoch):
 *                 worker i of m owns samples [floor(i N / m), floor((i+1) N / m)); an epoch
 *                 is S = floor(floor(N / m) / B) iterations; in epoch e = k / S the worker
 *                 walks a pseudo-random permutation of its partition, B positions per
 *                 iteration: position p = (k mod S) B + b maps to lo_i + pi(p), pi being a
 *                 4-round balanced Feistel network on 2w bits (2^(2w) >= n_i) with round
 *                 function mix(key + G (round+1) + right half) and cycle walking, key =
 *                 mix(mix(seed + G (e+1)) + G (i+1)).  Needs floor(N / m) >= B. */
typedef struct {
    int32_t kind;                     /* lc_kind */
    int32_t n_layers;
    int32_t dims[LC_MAX_LAYERS + 1];
    int32_t B;                        /* mini-batch size per worker, 1..128 */
    int64_t N;                        /* dataset size */
    int32_t E;                        /* lc_loss() uses the first E samples, E <= N */
    float lr;                         /* learning rate eta */
    float beta;                       /* momentum factor, 0 = plain SGD */
    float wd;                         /* weight decay added to the gradient */
    int32_t gemm;                     /* lc_gemm_dtype */
    int32_t sampler;                  /* lc_sampler */
} lc_model;

typedef struct lc_handle lc_handle;

/* Human-readable name of a status code (static string). */
const char* lc_strerror(int status);
/* Raw hipError_t of the last failing HIP call on this handle (0 if none). */
int lc_last_hip_error(const lc_handle* h);

/* P(model): parameters of one replica, biases included (Sec. 2: x in R^d).
 * Negative lc_status if the description is invalid. */
int64_t lc_param_count(const lc_model* model);
/* Distance in floats between consecutive rows of X and of V. */
int64_t lc_row_stride(int64_t P);

/* Create a run of m workers with P parameters each (Sec. 2, PASGD: the m workers
 * begin from one common model x_1).  seed keys the
 * mini-batch index stream: sample b of worker i at local iteration k is
 *   idx = mix(mix(mix(seed + G (k+1)) + G (i+1)) + G (b+1)) mod N,
 * mix = SplitMix64 output function, G = 0x9E3779B97F4A7C15 (sampling with
 * replacement from the whole set, an independent stream per worker).
 * The iteration counter starts at k = 0.  No device memory is touched.
 * Four environment variables are read here, for measurement runs only (results are bit-identical
 * whatever they say): LC_AVG_CHUNK_MB (1..1024, column chunk of the two-kernel averaging step),
 * LC_AVG_TWO_PHASE (0: one averaging kernel at every size), LC_SHARED_W_ORDER (0: replica-major
 * block order everywhere; n: sets of n replicas, see lc_set_lazy_broadcast), LC_SYNC_FIRST_LAYER
 * (0: no tile-owner kernels at tau = 1, 1: for the first layer only; see lc_set_deferred_update).
 * Errors: LC_ERR_ARG (m < 1, null), LC_ERR_MODEL (P != lc_param_count, bad dims,
 * B outside 1..128, E > N). */
int lc_init(int m, int64_t P, const lc_model* model, uint64_t seed, lc_handle** out);
void lc_destroy(lc_handle* h);

/* Bytes of device scratch lc_attach() needs for this run. */
size_t lc_workspace_bytes(const lc_handle* h);

/* Bind caller-owned device memory and the stream.
 *   X, V     : device, fp32 [m, lc_row_stride(P)], 256-byte aligned.  X holds the
 *              models, V the per-worker momentum buffers (Sec. 5.3: each worker
 *              keeps its own buffer).  Contents are taken as they are.
 *   scratch  : device, >= lc_workspace_bytes(), 256-byte aligned; zeroed here.
 *   data     : device, the dataset [N, d_0] row-major; fp32 for LC_GEMM_FP32,
 *              bfloat16 for LC_GEMM_BF16.  NULL for LC_KIND_QUAD.
 *   labels   : device, int32 [N], values in [0, d_L).  NULL for LC_KIND_QUAD.
 *   stream   : a hipStream_t (NULL = the default stream).
 * Synchronises the stream once.  Errors: LC_ERR_ARG, LC_ERR_ALIGN,
 * LC_ERR_WORKSPACE, LC_ERR_HIP. */
int lc_attach(lc_handle* h, void* X, void* V, void* scratch, size_t scratch_bytes,
              const void* data, const int32_t* labels, void* stream);

/* LC_KIND_QUAD only: curvatures a and centres c, device fp32 [m, lc_row_stride(P)]. */
int lc_attach_quad(lc_handle* h, const float* a, const float* c);

/* tau local iterations on every worker, no communication (Sec. 2, the
 * "otherwise" branch of the PASGD update rule): sample a mini-batch, forward,
 * softmax cross-entropy, backward, x <- x - lr v with v <- beta v + g.
 * The iteration counter advances by tau.  Asynchronous.
 * Errors: LC_ERR_ARG (tau < 1), LC_ERR_STATE, LC_ERR_HIP. */
int lc_local_steps(lc_handle* h, int tau);

/* The averaging step (Sec. 2: the branch of the update rule taken when k is a multiple of tau): every row of X is
 * replaced by the mean of all rows, X <- X J with J = 11^T/m (Appendix).  V is
 * not touched.  Afterwards all rows are bit-identical; calling it twice changes
 * nothing more.  Asynchronous. */
int lc_average(lc_handle* h);

/* n_periods times { tau local iterations; averaging step } (Sec. 2: the PASGD update rule run
 * over n_periods communication periods of length tau).  The result is that of calling
 * lc_local_steps(h, tau); lc_average(h) n_periods times, and that is what happens for most
 * shapes.  Where the resident step kernel applies (see lc_set_resident), tau is at most the
 * number of steps it takes per launch, and the model is small (one layer; or two layers with
 * m * ceil64(d0) * 64 bytes <= 200 KB, the amount a workgroup then reads from the other replicas),
 * several whole periods are ONE launch: at an averaging step every workgroup hands over its part
 * of the model, all workgroups of all replicas meet at a barrier in device memory (bounded wait,
 * LC_ERR_SYNC as described at lc_set_resident), and each forms the mean of its own part -- same
 * arithmetic as lc_average(), so the results are bit-identical to the call-by-call form with the
 * resident kernel.  lc_set_resident(h, 2) lifts the size condition.  Not used while block
 * momentum is on.  Afterwards every row of X holds the averaged model.  Asynchronous.
 * Errors: LC_ERR_ARG (tau < 1 or n_periods < 1), LC_ERR_STATE, LC_ERR_HIP. */
int lc_local_periods(lc_handle* h, int tau, int n_periods);

/* Deferred broadcast.  With on != 0 (LC_KIND_MLP only) lc_average() only computes the averaged
 * model (reads m rows, writes one vector in scratch): the next local step reads that one model for
 * every replica -- it is served from cache m-1 times out of m -- and writes every row of X, as it
 * does anyway.  This removes the m row writes of the averaging step and most weight reads of the
 * step after it; at tau = 1 the traffic per iteration falls from about 28 to 16 bytes per
 * parameter.  Results are bit-identical to the eager form.  While a broadcast is pending the rows
 * of X in device memory are STALE; every entry point of this library accounts for that, but a
 * caller who reads X directly must call lc_materialize() first.  Turning the mode off materialises.
 * In a step that reads the one model for all replicas, layers of 8 MB and more (in a state above
 * 256 MB) are worked through tile by tile for sets of 8 replicas at a time instead of replica by
 * replica, so that a weight tile is fetched once per set. */
int lc_set_lazy_broadcast(lc_handle* h, int on);
int lc_materialize(lc_handle* h);

/* Resident local steps (Sec. 2: a worker's tau local updates touch only its own model).  For
 * two-layer LC_KIND_MLP models with at most 16 classes, B <= 64, padded widths d0 <= 1024 and
 * d1 <= 256, m <= 64 and m * ceil64(d1) / 16 <= 256, lc_local_steps() runs up to 32 consecutive
 * steps (8 when the gathered inputs of a step exceed 4 MB) as ONE kernel: each workgroup keeps a 16-unit slice of the first layer, the matching
 * rows of the second layer and their momentum on chip (LDS and registers) for all of them, and the
 * workgroups of a replica meet once per step at a barrier in device memory to exchange their shares
 * of the logits.  One-layer models (softmax
 * regression) with at most 16 classes, B <= 64 and padded d0 <= 256 take the same route with one
 * workgroup per replica and no barrier.  Same arithmetic as the
 * launch-per-layer path up to the summation order (results agree to rounding, not bit for bit).
 * on = 0 selects the launch-per-layer path for every shape; the default is on (1); on = 2
 * additionally makes lc_local_periods() take the averaging steps inside the launch at every
 * shape the kernel handles, also where ending the launch is the faster way.  Shapes outside
 * the limits always take the launch-per-layer path.  The barrier wait is bounded: if it ever
 * times out the kernel still terminates, and the next synchronising call (lc_loss,
 * lc_get_state, lc_get_local_losses) returns LC_ERR_SYNC; the state is then undefined.  The
 * barrier needs all workgroups of the launch on the chip together: that holds when the kernel
 * has the GPU to itself (at most 256 workgroups, one per compute unit), not necessarily when
 * other streams keep compute units busy at the same time -- turn the mode off for such use. */
int lc_set_resident(lc_handle* h, int on);
/* Exchange inside one XCD.  The resident step kernel's workgroups of one replica exchange their
 * shares of the logits once per step.  Blocks are numbered so that a replica's workgroups run on one XCD
 * (one L2 cache) whenever m * ceil64(d1) / 16 / 8 is a multiple of ceil64(d1) / 16; counter and
 * exchanged values then stay in that L2 (workgroup-scope atomics, which the hardware performs in the
 * L2, and an invalidate of the compute unit's L1 only) instead of travelling to the memory side
 * and back.  The placement rule (hardware block id mod 8 selects the XCD) is observed by a probe
 * kernel at lc_attach(), and every workgroup compares its own XCD id with it when it starts: a
 * mismatch is reported as LC_ERR_PLACEMENT by the next synchronising call (the state is then
 * undefined).  Where the rule does not hold, or with on = 0, the agent-scope exchange is used.
 * Identical results either way.  Default on. */
int lc_set_xcd_local_exchange(lc_handle* h, int on);

/* First-layer fusion across steps (Sec. 2: between two averaging steps a worker's updates touch
 * only its own model, so the first layer's weights after step k are what step k+1 multiplies its
 * mini-batch with).  Inside one lc_local_steps() call, for LC_KIND_MLP models with at least two
 * layers, first-layer rows that are a multiple of 64 columns long and m * d1 / 64 >= 192, the
 * first layer's backward kernel of a step also computes the first hidden activations of the
 * next step from the weight tile it has just updated, and that step's first-layer forward launch
 * is dropped: W_1 then moves 16 instead of 20 bytes per parameter and step.  The first step of a
 * call and steps whose inputs are gathered by a later launch run the forward pass on its own.
 * Same arithmetic up to the summation order of the first-layer products.  Default on;
 * on = 0 keeps the separate forward launch and the row-owner backward kernel everywhere. */
int lc_set_first_layer_fusion(lc_handle* h, int on);

/* Deferred update at tau = 1 (Sec. 2, the k mod tau = 0 branch taken at every iteration: all
 * workers start each iteration from the same averaged model).  Under the deferred broadcast, in
 * lc_local_periods(h, 1, n) and the schedule drivers while tau is 1, replica i's model after its
 * step is x_bar - lr * v_i with v_i the momentum row the step has just written.  The backward
 * kernels then leave the rows of X unwritten, and the averaging step reads the rows of V and
 * forms each replica's weights on the fly (same expression, same rounding) before it adds them
 * up in double: 12 instead of 16 bytes per parameter, replica and iteration, bit-identical
 * results.  Layers of 8 MB or more with rows of a multiple of 64 columns (the last layer excepted)
 * go further: one kernel owns such a layer's weights by tile, walks over the replicas, updates
 * their momentum tiles and writes the layer's new average itself (8 bytes per parameter and
 * replica); above the first layer a pass over the old weights forms the deltas of the layer below
 * beforehand.  Applies to LC_KIND_MLP models on the launch-per-layer path whose last layer has more
 * than 128 inputs, not while block momentum is on, and not to lc_local_steps() + lc_average()
 * called one by one (the library cannot know that an averaging step follows).  Default on. */
int lc_set_deferred_update(lc_handle* h, int on);

/* Implicit momentum inside a period (Sec. 2: tau local updates between two averaging steps; Sec. 5.3:
 * one momentum buffer per worker).  The update x_{k+1} = x_k - lr v_{k+1} lets v_k be read off two
 * consecutive models, v_k = (x_{k-1} - x_k) / lr.  For the layers this applies to, the steps of a
 * period except the last keep x_k and x_{k-1} in the two row buffers (the caller's X and V) instead
 * of x_k and v_k, read both and write x_{k+1} over x_{k-1}: 12 instead of 16 bytes per parameter,
 * replica and step.  The last step of every period -- and of every lc_local_steps() call -- writes
 * x to X and v to V again, so every entry point of this library finds and leaves the documented
 * state; only a caller who reads X or V while an asynchronous call is still running sees the
 * intermediate form.  The recovered momentum differs from the stored one by the rounding of x_k,
 * ulp(x) / (2 lr): relative to v about 6e-8 divided by the relative size of one step (1e-4 .. 1e-3
 * in training).  That is far below the rounding of bf16 operands and above that of fp32 operands.
 *   mode 1 (default): layers of at least 1 MB, the last layer excepted, of LC_KIND_MLP runs with
 *           LC_GEMM_BF16 whose state exceeds the caches (X and V above 256 MB), on the
 *           launch-per-layer path, while block momentum is off and lr >= 1e-4 (the absolute
 *           error of the recovered momentum grows as 1 / lr);
 *   mode 2: every layer but the last, with either operand type and at any size;
 *   mode 0: off -- x in X and v in V after every step. */
int lc_set_implicit_momentum(lc_handle* h, int mode);

/* The averaging step of large layers folded into the last local step of a period (Sec. 2: the
 * k mod tau = 0 branch follows that step at once).  Inside lc_local_periods() and the schedule
 * drivers, with tau > 1, the deferred broadcast on and block momentum off, the last step of a
 * period does not write the rows of X for such a layer: one kernel owns the layer's weights by
 * tile, walks over the workers, updates each worker's momentum tile from that worker's own weights
 * and adds the worker's new weights to a sum kept in double; after the last worker the tile of the
 * averaged model is written, and the averaging kernels skip the layer's weights (its biases are
 * written to X and averaged as before).  Bit-identical to the step followed by the averaging
 * step; 12 instead of 20-24 bytes per parameter and replica for the two together.  Layers as for
 * the tile-owner kernel of tau = 1 (lc_set_deferred_update): 8 MB or more, rows of a multiple of
 * 64 columns, not the last layer.
 *   mode 1: the first layer (it needs no deltas for a layer below);
 *   mode 2 (default): the hidden layers too (after a pass over the old weights that forms the
 *           deltas of the layer below);
 *   mode 0: off. */
int lc_set_fused_averaging(lc_handle* h, int mode);

/* Number of layers of this (attached) handle whose steps inside a period take the implicit form
 * under the current mode, operand type, sizes, learning rate and block-momentum setting (0 where
 * the resident step kernel runs the steps); negative on error. */
int lc_implicit_momentum_layers(const lc_handle* h);

/* 1 if lc_local_steps() of this (attached) handle takes the resident step kernel, else 0. */
int lc_resident_active(const lc_handle* h);

/* How many times a workgroup of the resident step kernel re-reads a replica's arrival counter
 * before it gives up waiting (default 400000, several hundred milliseconds).  0 makes every
 * wait give up at once: the kernel then runs to its end on incomplete data and the next
 * synchronising call reports LC_ERR_SYNC -- the way to exercise that error path.  polls >= 0. */
int lc_set_barrier_polls(lc_handle* h, int polls);

/* Training loss of the averaged model F(x_bar) on the first E samples (the
 * quantity the basic update rule of Sec. 4.2 reads).  Always evaluated with
 * fp32 operands.  Does not modify X or V.  Synchronises the stream; *out is a
 * host double.  Errors: LC_ERR_NONFINITE (and *out is still written). */
int lc_loss(lc_handle* h, double* out);

/* AdaComm basic update rule (Sec. 4.2): tau_l = ceil( sqrt(F_l / F_0) * tau_0 ),
 * not below 1.  Pure host function, evaluated in IEEE double in exactly this
 * order: ratio = Fl / F0; root = sqrt(ratio); prod = root * tau0; ceil(prod).
 * Returns tau_l >= 1, or LC_ERR_ARG for F0 <= 0, Fl < 0, a non-finite input,
 * tau0 < 1, or a result that does not fit an int. */
int adacomm_next_tau(double F0, double Fl, int tau0);

/* AdaComm with the refinements of Sec. 4.3.  Candidate
 *   c = ceil( sqrt( (lr0 / lrl) * Fl / F0 ) * tau0 )      (Sec. 4.3.2, practical coupling; lr0 = lrl
 *                                                           gives the basic rule)
 * Saturation refinement (Sec. 4.3.1): c is taken only if c + slack < tau_prev,
 * otherwise the period becomes ceil(gamma * tau_prev), 0 < gamma < 1 (the paper uses 1/2).  At the
 * first decision after a learning-rate change (lr_changed != 0) c is taken as it is: the coupling
 * exists to let the period grow there.  Evaluated in IEEE double in this order: Fl/F0, lr0/lrl,
 * their product, sqrt, times tau0, ceil; gamma * tau_prev, ceil.  Returns the period >= 1 or
 * LC_ERR_ARG. */
int adacomm_next_tau_ex(double F0, double Fl, int tau0, int tau_prev, double gamma, int slack,
                        double lr0, double lrl, int lr_changed);

/* Whole schedule on the host side of the library: K iterations as periods of
 * tau local steps each followed by lc_average(), the last period truncated.
 * adaptive != 0: F_0 = lc_loss() at entry; at the first averaging step at or
 * after every multiple of `interval` iterations (the paper's wall-clock interval
 * T_0 of Sec. 4, counted in iterations) F_l = lc_loss() and tau for the
 * following periods is adacomm_next_tau(F_0, F_l, tau0).
 *   sched_k, sched_tau : host arrays of capacity cap receiving the decisions
 *                        (iteration, tau), the first being (k at entry, tau0)
 *   n_sched            : host, number of decisions made (may exceed cap)
 *   rounds             : host, number of averaging steps performed
 * Synchronises before returning. */
int lc_run(lc_handle* h, int64_t K, int tau0, int adaptive, int64_t interval,
           int64_t* sched_k, int32_t* sched_tau, int cap, int32_t* n_sched, int64_t* rounds);

/* Choosing tau_0 (Sec. 4.2, last sentences: a heuristic estimate from a grid search over several
 * communication periods, each run for a short while).  For every candidate taus[i], from the
 * model as it is now: K iterations with that fixed period (lc_run without adaptation), then the
 * training loss of the averaged model into loss_out[i] and the wall-clock seconds of the run into
 * seconds_out[i]; the state (X, V, k) is put back after each candidate and at the end.  *best is
 * the index with the largest loss decrease per second, (F_now - loss_out[i]) / seconds_out[i] --
 * the error-runtime trade-off of the paper read on this machine, where a long period saves
 * averaging steps and kernel launches instead of network time.  The paper does not state its
 * criterion; callers who want another one have the two arrays.  The state travels through host
 * memory (2 m P floats).  Not for use while block momentum is on (LC_ERR_STATE).
 * Errors: LC_ERR_ARG, LC_ERR_STATE, LC_ERR_HIP, LC_ERR_NONFINITE, LC_ERR_SYNC. */
int lc_grid_search_tau0(lc_handle* h, const int32_t* taus, int n, int64_t K, double* loss_out,
                        double* seconds_out, int32_t* best);

/* lc_run() with the refinements.  refine != 0 decides with adacomm_next_tau_ex (lr0 = the rate
 * in force at entry).  The learning-rate schedule is n_lr pairs: from iteration lr_at[j] on
 * (counted from 0 at lc_init, increasing) the rate is lr_val[j].  Changes take effect at
 * averaging steps only; with postpone_lr != 0 a due change waits until the period has reached 1
 * (Sec. 4.3.2: the period is brought down to 1 first, the rate is lowered only then).  sched_lr (host, capacity cap) receives the rate in force after each decision.
 * F_0 is always evaluated, so interval >= 1 is required.  The call begins a schedule: F_0 and
 * lr0 are taken at entry and the period starts at tau0.  It is not a resume point (a caller that
 * continues an earlier schedule keeps F_0, lr0 and the period itself and decides with
 * adacomm_next_tau_ex, which takes all of them as arguments). */
int lc_run_ex(lc_handle* h, int64_t K, int tau0, int64_t interval, int refine, double gamma, int slack,
              int n_lr, const int64_t* lr_at, const float* lr_val, int postpone_lr,
              int64_t* sched_k, int32_t* sched_tau, float* sched_lr, int cap, int32_t* n_sched,
              int64_t* rounds);

/* Block momentum (Sec. 5.3.1): treat the local updates of one period as one big step between two
 * synchronised models and give that step a global momentum.  lc_block_momentum_begin() records
 * the current model of worker 0 as x_sync (call it when the workers are synchronised: right after
 * lc_set_state with equal rows, or after lc_average), sets the global buffer u = 0 and clears the
 * local buffers.  While the mode is on, lc_average() (also inside lc_run / lc_run_ex) computes
 *     G = (x_sync - x_bar) / lr ;  u <- beta_glob u + G ;  x_sync <- x_sync - lr u
 * writes x_sync to every row and clears every worker's local momentum buffer (Sec. 5.3.1: local
 * momentum SGD begins afresh after each averaging step; the paper uses beta_glob = 0.3 with
 * local momentum 0.9).  G is read as the averaged model change per unit learning rate, which for
 * plain local SGD is the paper's accumulated mean gradient.  u and x_sync live in the scratch
 * buffer.  lc_block_momentum_end() returns to plain averaging.  lc_get_block_momentum() copies
 * u and x_sync to host arrays of P floats (either may be NULL); it synchronises. */
int lc_block_momentum_begin(lc_handle* h, float beta_glob);
int lc_block_momentum_end(lc_handle* h);
int lc_get_block_momentum(lc_handle* h, float* u_host, float* x_sync_host);

/* The block-momentum averaging step for callers that cannot allocate device memory: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arithmetic and same
 * kernel as lc_average() while block momentum is on, but no handle, no workspace and no allocation
 * of any kind (no hipMalloc / hipFree, no host allocation, no memset node: clearing is done by small
 * fill kernels): the global buffer u and the last synchronised model x_sync live in an array of
 * 2 * LC_STATIC_MAX_PARAMS floats inside the library's device image, which every GPU the library
 * runs on holds until the process ends.
 *   X          : device fp32 [m, row_stride], 256-byte aligned; row_stride a multiple of 4 floats,
 *                >= P; entries of a row beyond P must be zero and stay zero.
 *   V          : device fp32 [m, row_stride], 256-byte aligned, or NULL: the workers' local momentum
 *                buffers, cleared by both forms of the call (Sec. 5.3.1: local momentum restarts).
 *   begin != 0 : the rows of X are synchronised; record row 0 as x_sync, set u = 0.  X is not changed.
 *                (What lc_block_momentum_begin() does.)
 *   begin == 0 : x_bar = mean of the rows; G = (x_sync - x_bar) / lr; u <- beta_glob u + G;
 *                x_sync <- x_sync - lr u; every row of X <- x_sync.
 * Asynchronous on `stream`.  All calls on one GPU share the one array, which keeps what the last
 * call left there: one block-momentum run per GPU at a time, a new run starts with begin != 0, and
 * calls that overlap on one GPU (other streams, other threads) race.  The array's address is looked
 * up once per device, at the first call on that device.
 * Errors: LC_ERR_ARG (null X, m < 1, P < 1, bad stride, lr <= 0, beta_glob outside [0, 1)),
 * LC_ERR_ALIGN, LC_ERR_TOO_LARGE (P > LC_STATIC_MAX_PARAMS), LC_ERR_HIP. */
#define LC_STATIC_MAX_PARAMS 4456448
int lc_average_block_momentum_static(float* X, float* V, int m, int64_t P, int64_t row_stride, float lr,
                                     float beta_glob, int begin, void* stream);

/* One (momentum-)SGD update of every worker from explicit gradients G (device,
 * fp32 [m, lc_row_stride(P)], 256-byte aligned): g <- G + wd x; v <- beta v + g;
 * x <- x - lr v (mini-batch SGD update of Sec. 2).  The iteration counter is
 * unchanged.  Asynchronous. */
int lc_set_grad(lc_handle* h, const void* G);
int lc_update_from_grad(lc_handle* h);

/* Fused form of lc_update_from_grad() followed by lc_average() for the fully
 * synchronous case tau = 1 (Sec. 2, special case): one pass over X, V and G. */
int lc_update_from_grad_and_average(lc_handle* h);

/* State access for tests and checkpoints.  X_host / V_host are host fp32 [m, P]
 * (dense, no row padding); either may be NULL.  Both calls synchronise. */
int lc_get_state(lc_handle* h, float* X_host, float* V_host, int64_t* k);
int lc_set_state(lc_handle* h, const float* X_host, const float* V_host, int64_t k);

int lc_set_lr(lc_handle* h, float lr);

/* Mini-batch loss of every worker at its last local step: host float [m].
 * Synchronises. */
int lc_get_local_losses(lc_handle* h, float* losses_host);
/* Dataset indices drawn at the last local step: host int32 [m, B].  Synchronises. */
int lc_get_last_indices(lc_handle* h, int32_t* idx_host);

/* Per-kernel timing for measurement: while enabled, every launch of the named
 * kernel class is bracketed by HIP events on the run's stream.
 * lc_timing_read() synchronises and returns the number of launches and their
 * summed duration since lc_timing_begin().  which: 0 = backward+update kernel,
 * 1 = forward kernel, 2 = averaging kernel, 3 = update-from-gradient kernel,
 * 4 = fused update+average kernel.  If an event could not be created or recorded since
 * lc_timing_begin(), lc_timing_read() returns LC_ERR_HIP instead of incomplete figures. */
int lc_timing_begin(lc_handle* h, int which);
int lc_timing_read(lc_handle* h, int64_t* launches, double* total_ms);
/* Narrows class 0 to the launches that work on layer `layer` (1..L; 0 = every layer) and to one
 * kernel (0 = any, 1 = row-owner backward kernel, 2 = first-layer kernel that also runs the next
 * forward pass, 3 = tile-owner kernel of tau = 1, 4 = fused last-layer kernel, 5 = resident step
 * kernel, which counts as layer 0).  Call after lc_timing_begin(), which resets both to 0. */
int lc_timing_select(lc_handle* h, int layer, int kernel);

#ifdef __cplusplus
}
#endif
#endif
