// Internal declarations shared by the translation units of liblocalcomm.
// Nothing here is part of the C ABI (see include/localcomm.h for that).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <vector>

#include "localcomm.h"

namespace lc {

typedef __bf16 bf16_t;
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kWave = 64;
constexpr int kColChunk = 64;   // columns of W handled per wave and per loop trip
constexpr int kRowsPerWave = 16;
constexpr int kXcds = 8;
constexpr int kGatherSlots = 8;  // local steps whose mini-batches one gather launch prepares (at least; see carve())
constexpr int kLossParts = 8;    // partial loss sums per group (one per block that shares a group's batch)

inline int64_t round_up(int64_t a, int64_t b) { return (a + b - 1) / b * b; }

// Kernel classes for lc_timing_begin().
enum TimedKernel { kTimeBwd = 0, kTimeFwd = 1, kTimeAvg = 2, kTimeUpd = 3, kTimeUpdAvg = 4, kTimeNone = -1 };
// Kernels of the backward class, for lc_timing_select().
enum BwdKernel { kBwdAny = 0, kBwdRowOwner = 1, kBwdFirstLayer = 2, kBwdTileOwner = 3, kBwdHead = 4, kBwdResident = 5 };

// Implicit momentum: where a layer's parameters of the current and of the previous step are.
enum ImpBuf { kBufX = 0, kBufV = 1, kBufXbar = 2 };
struct ImpState {
    bool active;   // false: parameters in X (or the averaged model while a broadcast is pending), momentum in V
    int cur, prev; // active: x_k in `cur` (X or V rows), x_{k-1} in `prev` (the other rows, or the averaged model)
};
// Buffers of one backward-class launch of a layer, and the layer's form after it.
struct StepBufs {
    const float* xr;      // parameters are read here
    int64_t xr_stride;
    const float* aux;     // momentum rows, or (imp_in) the parameters of one step earlier
    int64_t aux_stride;
    int imp_in;
    float* ox;            // new parameters
    float* ov;            // new momentum, or null (implicit)
    ImpState next;
};

// One layer of the per-replica MLP as the kernels see it.
struct LayerGeom {
    int d_in, d_out;      // logical sizes
    int dp_in, dp_out;    // padded to a multiple of 64
    int64_t w_off, b_off; // offsets inside a replica row (floats)
};

// Device buffers of one "activation set": either the training set (operand type
// of the run) or the evaluation set (always fp32).
struct ActSet {
    int G;                 // groups (replicas, or evaluation chunks)
    int B, Bp;             // valid rows and rows padded to a multiple of 32
    void* a_bm[LC_MAX_LAYERS + 1];  // A_l batch-major   [G][Bp][dp_l]   (l = L: logits, fp32)
    void* a_fm[LC_MAX_LAYERS + 1];  // A_l feature-major [G][dp_l][Bp]   (training only, l < L)
    void* dz_bm[LC_MAX_LAYERS + 1]; // dZ_l batch-major  (training only, l >= 1)
    void* dz_fm[LC_MAX_LAYERS + 1]; // dZ_l feature-major
    int32_t* labels;       // [slots][G][Bp]
    int32_t* idx;          // [slots][G][Bp]
    int slots, cur_slot;   // training keeps the inputs of several consecutive steps (A_0, labels, indices)
    float* loss;           // [.. G][kLossParts] partial sums: training batch means, evaluation sums over valid rows
};

}  // namespace lc

struct lc_handle {
    int m;
    int64_t P, Ps;
    lc_model md;
    uint64_t seed;
    int64_t k;
    int L;
    lc::LayerGeom layer[LC_MAX_LAYERS + 1];  // index 1..L
    bool attached;
    bool stream_weights;    // X and V together exceed the on-chip caches by far
    bool avg_two_phase;        // averaging: two-kernel form for states larger than the caches
    int64_t avg_chunk_floats;  // its column chunk (x_bar chunk stays cached between the kernels)
    float *X, *V;
    const float* G;
    const float *qa, *qc;
    const void* data;
    const int32_t* labels;
    char* scratch;
    size_t scratch_bytes;
    hipStream_t stream;
    lc::ActSet train, eval;
    float* xbar;            // [Ps]
    // block momentum: global buffer, last synchronised model, and the deferred clearing of V
    float *bm_u, *bm_xs;    // [Ps]
    bool bm_on;
    float bm_beta;
    bool v_cleared;         // V counts as zero: the next update uses beta = 0 and overwrites it
    // lazy broadcast: after an averaging step the rows of X are stale and every replica's model is
    // the single vector xbar, until the next local step (which writes every row) or a materialise
    bool lazy_enabled, lazy_rows;
    int loss_parts_train, loss_parts_eval;   // how many of the kLossParts slots the last launch wrote
    bool lazy_enabled_step;   // set only while lc_average runs its reduce-only form
    // deferred update (tau = 1 under the deferred broadcast): every replica starts the iteration
    // from xbar, so its new weights are xbar - lr V_i; the backward kernels write V only and the
    // averaging step forms the weights from V on the fly.  defer_x is set only while run_periods
    // queues such an iteration and its averaging step.
    bool defer_x_on, defer_x;
    // tau = 1, first layer: backward pass, update of V and the layer's averaging in one kernel; sync1_done
    // is set while the averaging step of the iteration still has to skip the layer
    bool sync1_on, sync_all_on;   // layer 1 / the layers above it as well
    unsigned sync_done;           // bit l: the iteration in progress has averaged layer l's weights already
    // Last step of a period of tau > 1 whose averaging step follows with the broadcast deferred: the
    // large layers' tile-owner kernel forms the step and the layer's average together (the rows of X
    // stay unwritten).  fuse_avg is set only while run_periods takes such a step and its averaging step.
    int fuse_avg_on;              // 0 off, 1 the first layer, 2 the large hidden layers as well
    bool fuse_avg;
    bool share_w_on;          // block order of the steps that read one model for all replicas (see FwdArgs)
    bool group_shared_on;     // ... and several replicas' batches per block in them (see FwdArgs::fm_Bp)
    int share_w_set;          // ... replicas per set
    // resident local steps (small two-layer models): exchange buffer, barrier counters, switches
    float* res_a1x;         // [2 parities][m][dp1/16][Bp][16] exchange buffer of the resident kernel, null when the shape does not qualify
    unsigned* res_ctr;      // [0..63] arrival counters per replica, [64] error flag, [65] all-replica counter, [128..383] placement probe
    unsigned res_arrivals;  // value of every counter once the queued launches have run (zeroed with the scratch at attach)
    float* res_avx;         // [2 parities][m][Ps] models handed over at averaging steps inside a launch
    unsigned res_garrivals; // the same for the all-replica counter of those averaging steps (res_ctr[65])
    bool res_on;            // lc_set_resident
    bool res_local_on;      // lc_set_xcd_local_exchange
    bool res_xcc_known;     // the probe found blocks dealt to the XCDs by id mod 8
    unsigned res_xcc_of;    // 4 bits per residue: the XCD it runs on
    int imp_mode;           // lc_set_implicit_momentum: 0 off, 1 where it pays, 2 wherever the kernels allow
    bool imp_out;           // the step being queued may leave its layers in implicit form (not the last of a period or call)
    lc::ImpState imp[LC_MAX_LAYERS + 1];   // index 1..L
    bool fl_on;             // lc_set_first_layer_fusion
    bool a1_ready;          // A_1 of the step about to run was produced by the previous step's backward pass
    bool res_fuse_always;   // lc_set_resident(2): averaging steps inside the launch at every eligible shape
    bool res_used;          // a resident launch has run since the error flag was last read
    int res_spin_limit;     // polls a barrier wait may take
    double* partial;        // reduction partials
    int n_partial;
    int last_hip;
    // timing
    int timing_which;
    std::vector<hipEvent_t> ev_pool;
    size_t ev_used;
    int timing_layer, timing_kernel;   // lc_timing_select(): backward-class launches of this layer / kernel only (0 = all)
    int timing_err;         // hipError_t of an event that could not be created or recorded since lc_timing_begin
};

namespace lc {

// ---- launchers (each returns a hipError_t from hipGetLastError) --------------
hipError_t launch_average(lc_handle* h, const float* X, float* out_rows, float* out_single);
inline float effective_beta(const lc_handle* h) { return h->v_cleared ? 0.f : h->md.beta; }
hipError_t launch_broadcast_xbar(lc_handle* h);   // xbar -> every row of X
hipError_t launch_update_from_grad(lc_handle* h);
hipError_t launch_update_and_average(lc_handle* h);
hipError_t launch_quad_step(lc_handle* h);
hipError_t launch_quad_loss(lc_handle* h, int* n_partial);

hipError_t launch_gather(lc_handle* h, bool eval, int64_t k_or_base, int n_steps);
hipError_t launch_forward(lc_handle* h, bool eval, int l, int loss_offset);
bool forward_fuses_softmax(const lc_handle* h);  // last layer's kernel also does a3
hipError_t launch_softmax(lc_handle* h, bool eval, int loss_offset);
hipError_t launch_backward(lc_handle* h, int l, bool da_only = false);   // da_only: dZ_{l-1} only, no update
bool first_layer_kernel_ok(const lc_handle* h);   // layer 1: backward kernel that also runs the next step's forward
hipError_t launch_first_layer(lc_handle* h);
bool implicit_layer_ok(const lc_handle* h, int l);   // layer l may keep its momentum implicitly inside a period
void layer_weights(const lc_handle* h, int l, const float** base, int64_t* stride);   // where layer l's current parameters are read
StepBufs plan_step_buffers(const lc_handle* h, int l);
bool sync_layer_ok(const lc_handle* h, int l);    // layer l at tau = 1: dW, update of V and averaging of the layer by tile
hipError_t launch_sync_layer(lc_handle* h, int l);
bool shared_weight_order(const lc_handle* h, const LayerGeom& g);   // tile-major block order on steps that read one model
int shared_set(const lc_handle* h, int G);                          // ... replicas per set
bool head_is_fused(const lc_handle* h);   // last layer: forward + softmax + backward in one kernel
hipError_t launch_head(lc_handle* h);

// resident path (weights stay in LDS over a run of local steps)
bool resident_shape_ok(const lc_handle* h);
size_t resident_exchange_floats(const lc_handle* h);
hipError_t probe_block_placement(lc_handle* h);   // synchronises the stream once
hipError_t launch_resident(lc_handle* h, int slot0, int n_steps, int period);  // the steps gathered into slots slot0 .. slot0+n_steps-1

// timing helpers used by the launchers
// (layer, kernel: what a backward-class launch works on, for lc_timing_select(); 0 elsewhere)
void timing_start(lc_handle* h, int which, int layer = 0, int kernel = 0);
void timing_stop(lc_handle* h, int which, int layer = 0, int kernel = 0);

}  // namespace lc
