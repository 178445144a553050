// Host side of liblocalcomm: the C ABI declared in include/localcomm.h.
// Argument checking, workspace carving, kernel sequencing, the AdaComm
// controller and the schedule driver live here; all arithmetic of the method
// on parameters runs in the kernels.
#include <math.h>
#include <stdlib.h>
#include <string.h>
#include <time.h>

#include <new>

#include "lc_internal.h"

using namespace lc;

#define LC_HIP(h, call)                             \
    do {                                            \
        hipError_t e__ = (call);                    \
        if (e__ != hipSuccess) {                    \
            (h)->last_hip = static_cast<int>(e__);  \
            return LC_ERR_HIP;                      \
        }                                           \
    } while (0)

namespace lc {

// does this launch belong to what lc_timing_begin() / lc_timing_select() asked for?
static bool timing_wanted(const lc_handle* h, int which, int layer, int kernel) {
    if (h->timing_which != which) return false;
    if (h->timing_layer != 0 && layer != h->timing_layer) return false;
    return h->timing_kernel == 0 || kernel == h->timing_kernel;
}

void timing_start(lc_handle* h, int which, int layer, int kernel) {
    if (!timing_wanted(h, which, layer, kernel)) return;
    if (h->ev_used + 2 > h->ev_pool.size()) {
        for (int i = 0; i < 256; ++i) {
            hipEvent_t e;
            const hipError_t rc = hipEventCreate(&e);
            if (rc != hipSuccess) {   // reported by lc_timing_read(): a count that silently stops would be wrong
                h->timing_err = static_cast<int>(rc);
                return;
            }
            h->ev_pool.push_back(e);
        }
    }
    const hipError_t rc = hipEventRecord(h->ev_pool[h->ev_used], h->stream);
    if (rc != hipSuccess) h->timing_err = static_cast<int>(rc);
}

void timing_stop(lc_handle* h, int which, int layer, int kernel) {
    if (!timing_wanted(h, which, layer, kernel)) return;
    if (h->ev_used + 2 > h->ev_pool.size()) return;
    const hipError_t rc = hipEventRecord(h->ev_pool[h->ev_used + 1], h->stream);
    if (rc != hipSuccess) h->timing_err = static_cast<int>(rc);
    h->ev_used += 2;
}

}  // namespace lc

namespace {

bool aligned256(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 255u) == 0; }

int padded_batch(int B) { return B <= 32 ? 32 : (B <= 64 ? 64 : 128); }

int model_ok(const lc_model* md) {
    if (!md) return LC_ERR_ARG;
    if (md->kind == LC_KIND_QUAD) return md->dims[0] >= 1 ? LC_OK : LC_ERR_MODEL;
    if (md->kind != LC_KIND_MLP) return LC_ERR_MODEL;
    if (md->n_layers < 1 || md->n_layers > LC_MAX_LAYERS) return LC_ERR_MODEL;
    for (int l = 0; l <= md->n_layers; ++l)
        if (md->dims[l] < 1) return LC_ERR_MODEL;
    if (md->dims[md->n_layers] > 1024) return LC_ERR_UNSUPPORTED;  // classes per sample handled by one thread
    if (md->B < 1 || md->B > 128) return LC_ERR_MODEL;
    if (md->N < 1 || md->N > 2147483647LL) return LC_ERR_MODEL;
    if (md->E < 1 || md->E > md->N) return LC_ERR_MODEL;
    if (md->gemm != LC_GEMM_FP32 && md->gemm != LC_GEMM_BF16) return LC_ERR_MODEL;
    if (md->sampler != LC_SAMPLE_REPLACEMENT && md->sampler != LC_SAMPLE_PARTITION) return LC_ERR_MODEL;
    return LC_OK;
}

// Carves the scratch buffer.  With base == nullptr only the size is computed.
struct Carver {
    char* base;
    size_t off;
    void* take(size_t bytes) {
        off = static_cast<size_t>(round_up(static_cast<int64_t>(off), 256));
        void* p = base ? base + off : nullptr;
        off += bytes;
        return p;
    }
};

size_t carve(lc_handle* h, char* base) {
    Carver c{base, 0};
    h->xbar = static_cast<float*>(c.take(sizeof(float) * static_cast<size_t>(h->Ps)));
    h->bm_u = static_cast<float*>(c.take(sizeof(float) * static_cast<size_t>(h->Ps)));
    h->bm_xs = static_cast<float*>(c.take(sizeof(float) * static_cast<size_t>(h->Ps)));
    if (h->md.kind == LC_KIND_QUAD) {
        h->n_partial = static_cast<int>((h->P + 255) / 256);
        h->partial = static_cast<double*>(c.take(sizeof(double) * static_cast<size_t>(h->n_partial)));
        return static_cast<size_t>(round_up(static_cast<int64_t>(c.off), 256));
    }
    const int L = h->L;
    const size_t ot = h->md.gemm == LC_GEMM_BF16 ? 2 : 4;
    for (int pass = 0; pass < 2; ++pass) {
        ActSet& S = pass == 0 ? h->train : h->eval;
        const bool eval = pass == 1;
        const size_t es = eval ? 4 : ot;
        if (eval) {  // evaluation: chunks of 128 samples, at most 64 chunks per pass
            S.B = S.Bp = 128;
            const int chunks = (h->md.E + 127) / 128;
            S.G = chunks < 64 ? chunks : 64;
        } else {
            S.G = h->m;
            S.B = h->md.B;
            S.Bp = padded_batch(h->md.B);
        }
        S.slots = 1;
        if (!eval) {
            // 8 steps' inputs per gather launch; up to 32 where they are small (the resident step
            // kernel then also takes that many steps per launch), within about 128 MB
            const size_t slot_bytes = 2 * static_cast<size_t>(S.G) * S.Bp * h->layer[1].dp_in * ot;
            size_t n = (static_cast<size_t>(128) << 20) / slot_bytes;
            S.slots = n < kGatherSlots ? kGatherSlots : (n > 4 * kGatherSlots ? 4 * kGatherSlots : static_cast<int>(n));
            // the first-layer kernel folds a step's first forward pass into the step before it, which
            // needs that step's inputs gathered by the same launch: fewer, longer runs -- 32 steps
            // where that stays within 1 GB (800 MB at the two large configurations: a period of 20
            // is then gathered whole), else 16
            if (first_layer_kernel_ok(h) && S.slots < 4 * kGatherSlots)
                S.slots = 4 * kGatherSlots * slot_bytes <= (static_cast<size_t>(1) << 30) ? 4 * kGatherSlots
                          : (S.slots < 2 * kGatherSlots ? 2 * kGatherSlots : S.slots);
        }
        S.cur_slot = 0;
        for (int l = 0; l <= L; ++l) {
            const size_t dp = static_cast<size_t>(l == 0 ? h->layer[1].dp_in : h->layer[l].dp_out);
            const size_t n = static_cast<size_t>(S.G) * S.Bp * dp;
            const size_t copies = l == 0 ? static_cast<size_t>(S.slots) : 1;
            S.a_bm[l] = c.take(n * (l == L ? 4 : es) * copies);
            S.a_fm[l] = (!eval && l < L) ? c.take(n * es * copies) : nullptr;
            S.dz_bm[l] = (!eval && l >= 1) ? c.take(n * es) : nullptr;
            S.dz_fm[l] = (!eval && l >= 1) ? c.take(n * es) : nullptr;
        }
        S.labels = static_cast<int32_t*>(c.take(sizeof(int32_t) * static_cast<size_t>(S.G) * S.Bp * S.slots));
        S.idx = static_cast<int32_t*>(c.take(sizeof(int32_t) * static_cast<size_t>(S.G) * S.Bp * S.slots));
        const int per_pass = S.G * S.B;
        const int passes = eval ? (h->md.E + per_pass - 1) / per_pass : 1;
        S.loss = static_cast<float*>(c.take(sizeof(float) * static_cast<size_t>(S.G) * passes * kLossParts));
    }
    if (resident_shape_ok(h)) {
        h->res_a1x = static_cast<float*>(c.take(sizeof(float) * resident_exchange_floats(h)));
        h->res_ctr = static_cast<unsigned*>(c.take(sizeof(unsigned) * 384));
        h->res_avx = static_cast<float*>(c.take(sizeof(float) * 2 * static_cast<size_t>(h->m) * h->Ps));
    } else {
        h->res_a1x = nullptr;
        h->res_ctr = nullptr;
        h->res_avx = nullptr;
    }
    h->n_partial = 0;
    h->partial = nullptr;
    return static_cast<size_t>(round_up(static_cast<int64_t>(c.off), 256));
}

int require_attached(const lc_handle* h) {
    if (!h) return LC_ERR_ARG;
    if (!h->attached) return LC_ERR_STATE;
    return LC_OK;
}

// the quadratic objective also needs its constants before it can step or be evaluated
int require_objective(const lc_handle* h) {
    const int rc = require_attached(h);
    if (rc != LC_OK) return rc;
    if (h->md.kind == LC_KIND_QUAD && (!h->qa || !h->qc)) return LC_ERR_STATE;
    return LC_OK;
}

// Make the rows of X real again after a deferred broadcast.
int materialise(lc_handle* h) {
    if (!h->lazy_rows) return LC_OK;
    LC_HIP(h, launch_broadcast_xbar(h));
    h->lazy_rows = false;
    return LC_OK;
}

// next_gathered: the step after this one belongs to the same call and its mini-batch is already
// in the next input slot, so the first layer's backward kernel may run that step's first-layer
// forward pass on the weights it has just updated.
// implicit_out: the step may leave the large layers with their momentum in implicit form (it is
// not the last step of its period or of the call).
int one_local_step(lc_handle* h, bool next_gathered, bool implicit_out = false) {
    h->imp_out = implicit_out;
    if (h->md.kind == LC_KIND_QUAD) {
        const int rc = materialise(h);
        if (rc != LC_OK) return rc;
        LC_HIP(h, launch_quad_step(h));
    } else {
        // (the mini-batch of this step was gathered into slot train.cur_slot by lc_local_steps)
        // layer L first in the backward sweep: dZ_{l-1} is produced from W_l before W_l
        // is overwritten inside the same kernel, and kernels run in stream order
        // (as a plain backward pass the column-owner kernel is a few per cent slower than the
        // row-owner one: it is taken only when it also saves the next forward launch)
        const bool first_fused = h->fl_on && next_gathered && first_layer_kernel_ok(h);
        const int l_lo = h->a1_ready ? 2 : 1;   // A_1 of this step came out of the previous step's backward pass
        if (head_is_fused(h)) {
            for (int l = l_lo; l < h->L; ++l) LC_HIP(h, launch_forward(h, false, l, 0));
            LC_HIP(h, launch_head(h));
        } else {
            for (int l = l_lo; l <= h->L; ++l) LC_HIP(h, launch_forward(h, false, l, 0));
            if (!forward_fuses_softmax(h)) LC_HIP(h, launch_softmax(h, false, 0));
        }
        for (int l = head_is_fused(h) ? h->L - 1 : h->L; l >= 1; --l) {
            if (l == 1 && first_fused) {
                LC_HIP(h, launch_first_layer(h));
            } else if ((h->defer_x || (h->fuse_avg && (l == 1 || h->fuse_avg_on > 1))) && sync_layer_ok(h, l)) {
                if (l > 1) LC_HIP(h, launch_backward(h, l, true));   // dZ_{l-1} from the weights of before the update
                LC_HIP(h, launch_sync_layer(h, l));   // dW_l, V, and the layer's part of the averaging step
                h->sync_done |= 1u << l;
            } else {
                LC_HIP(h, launch_backward(h, l));
            }
        }
        h->a1_ready = first_fused;
    }
    h->k += 1;
    h->v_cleared = false;   // the step just queued wrote V = g
    h->lazy_rows = false;   // ... and every row of X
    return LC_OK;
}

// Reads and clears the error flag of the resident step kernel.  Call after a stream synchronise.
int check_resident(lc_handle* h) {
    if (!h->res_used || !h->res_ctr) return LC_OK;
    unsigned flag = 0;
    LC_HIP(h, hipMemcpyAsync(&flag, h->res_ctr + 64, sizeof(unsigned), hipMemcpyDeviceToHost, h->stream));
    LC_HIP(h, hipStreamSynchronize(h->stream));
    h->res_used = false;
    if (flag == 0) return LC_OK;
    LC_HIP(h, hipMemsetAsync(h->res_ctr + 64, 0, sizeof(unsigned), h->stream));
    return (flag & 2u) ? LC_ERR_PLACEMENT : LC_ERR_SYNC;
}

// Whole periods of tau iterations that can be taken from iteration k on without looking at the
// schedule in between: it is looked at again at the first averaging step at or after `lim` (the
// next loss evaluation, learning-rate change, or the end).  0 when less than one period is left.
int whole_periods(int64_t k, int tau, int64_t lim, int64_t k_end) {
    const int64_t fit = (k_end - k) / tau;
    if (fit < 1) return 0;
    int64_t np = lim > k ? (lim - k + tau - 1) / tau : 1;
    if (np > fit) np = fit;
    if (np > 65536) np = 65536;
    return static_cast<int>(np);
}

// tau local iterations, n_periods times, with the averaging step after each period where asked.
// Mini-batch selection does not depend on the weights, so one gather launch prepares the inputs
// of a whole chunk of steps: as many whole periods as it has slots for, or a piece of a period
// that is longer than that.  Inside a chunk a period's steps are one resident launch (small
// models), or one launch sequence per step in which the first layer's backward kernel may run
// the next step's first forward pass as long as that step belongs to the same period and chunk.
int run_periods(lc_handle* h, int tau, int n_periods, bool average) {
    const bool mlp = h->md.kind == LC_KIND_MLP;
    const int slots = mlp ? h->train.slots : kGatherSlots;
    const bool resident = mlp && h->res_on && h->res_a1x;
    const bool defer_ok = mlp && !resident && average && tau == 1 && h->defer_x_on && h->lazy_enabled &&
                          !h->bm_on && !head_is_fused(h);
    const bool fuse_ok = mlp && !resident && average && tau > 1 && h->fuse_avg_on && h->lazy_enabled && !h->bm_on &&
                         h->m >= 2 && !head_is_fused(h);
    int64_t left = static_cast<int64_t>(tau) * n_periods;
    int pos = 0;   // steps of the current period already taken
    while (left > 0) {
        int64_t n = (pos == 0 && tau <= slots) ? static_cast<int64_t>(slots / tau) * tau : (tau - pos < slots ? tau - pos : slots);
        if (n > left) n = left;
        if (mlp) LC_HIP(h, launch_gather(h, false, h->k, static_cast<int>(n)));
        h->a1_ready = false;
        for (int t = 0; t < n;) {
            const int in_period = tau - pos < n - t ? tau - pos : static_cast<int>(n - t);
            if (resident) {
                LC_HIP(h, launch_resident(h, t, in_period, 0));
                t += in_period;
                h->train.cur_slot = t - 1;
                h->k += in_period;
                h->v_cleared = false;
                h->lazy_rows = false;
                h->res_used = true;
            } else {
                // tau = 1 while a broadcast is pending: every replica starts from xbar, so the
                // iteration writes V only and the averaging step forms xbar - lr V_i itself
                const bool defer = defer_ok && h->lazy_rows;
                h->defer_x = defer;
                for (int u = 0; u < in_period; ++u, ++t) {
                    h->train.cur_slot = t;
                    // the last step of a longer period, the averaging step next: the large layers take
                    // the step and their average together
                    h->fuse_avg = fuse_ok && pos + u + 1 == tau;
                    // (the last step of a period -- of a call -- leaves x in X and v in V; a period
                    // longer than one gather launch stays implicit across the launches)
                    const int r = one_local_step(h, u + 1 < in_period, !defer && pos + u + 1 < tau);
                    if (r != LC_OK) {
                        h->defer_x = h->fuse_avg = false;
                        h->sync_done = 0;
                        return r;
                    }
                }
            }
            pos += in_period;
            if (pos == tau) {
                pos = 0;
                if (average) {
                    const int r = lc_average(h);   // (reads V instead of X while defer_x is set)
                    h->defer_x = h->fuse_avg = false;
                    h->sync_done = 0;
                    if (r != LC_OK) return r;
                }
            }
        }
        left -= n;
    }
    return LC_OK;
}

}  // namespace

extern "C" {

const char* lc_strerror(int status) {
    switch (status) {
        case LC_OK: return "ok";
        case LC_ERR_ARG: return "invalid argument";
        case LC_ERR_MODEL: return "inconsistent model description";
        case LC_ERR_STATE: return "call out of order (not attached?)";
        case LC_ERR_ALIGN: return "device pointer not 256-byte aligned";
        case LC_ERR_WORKSPACE: return "scratch buffer too small";
        case LC_ERR_HIP: return "HIP call failed";
        case LC_ERR_NONFINITE: return "loss is not finite";
        case LC_ERR_UNSUPPORTED: return "shape not supported";
        case LC_ERR_SYNC: return "replica barrier timed out in the resident step kernel";
        case LC_ERR_PLACEMENT: return "resident step kernel: a workgroup ran on another XCD than the placement probe predicted";
        case LC_ERR_TOO_LARGE: return "more parameters than the library's static scratch holds";
        default: return "unknown status";
    }
}

int lc_last_hip_error(const lc_handle* h) { return h ? h->last_hip : 0; }

int64_t lc_param_count(const lc_model* md) {
    const int rc = model_ok(md);
    if (rc != LC_OK) return rc;
    if (md->kind == LC_KIND_QUAD) return md->dims[0];
    int64_t p = 0;
    for (int l = 0; l < md->n_layers; ++l) p += static_cast<int64_t>(md->dims[l]) * md->dims[l + 1] + md->dims[l + 1];
    return p;
}

int64_t lc_row_stride(int64_t P) { return P < 1 ? LC_ERR_ARG : round_up(P, 64); }

int lc_init(int m, int64_t P, const lc_model* md, uint64_t seed, lc_handle** out) {
    if (!out) return LC_ERR_ARG;
    *out = nullptr;
    if (m < 1 || m > 65535 || !md) return LC_ERR_ARG;
    const int64_t want = lc_param_count(md);
    if (want < 0) return static_cast<int>(want);
    if (P != want) return LC_ERR_MODEL;
    if (md->kind == LC_KIND_MLP && md->sampler == LC_SAMPLE_PARTITION && md->N / m < md->B) return LC_ERR_MODEL;
    lc_handle* h = new (std::nothrow) lc_handle();
    if (!h) return LC_ERR_ARG;
    h->m = m;
    h->P = P;
    h->Ps = round_up(P, 64);
    h->md = *md;
    h->seed = seed;
    h->k = 0;
    h->L = md->kind == LC_KIND_MLP ? md->n_layers : 0;
    int64_t off = 0;
    for (int l = 1; l <= h->L; ++l) {
        LayerGeom& g = h->layer[l];
        g.d_in = md->dims[l - 1];
        g.d_out = md->dims[l];
        g.dp_in = static_cast<int>(round_up(g.d_in, 64));
        g.dp_out = static_cast<int>(round_up(g.d_out, 64));
        g.w_off = off;
        g.b_off = off + static_cast<int64_t>(g.d_in) * g.d_out;
        off = g.b_off + g.d_out;
    }
    h->attached = false;
    // 256 MB: the size of the memory-side cache; below it weights are worth keeping cached
    h->stream_weights = 8.0 * static_cast<double>(m) * static_cast<double>(h->Ps) > 256.0 * 1024 * 1024;
    h->avg_two_phase = true;
    // chunk of one row that the broadcast re-reads from cache (measured optima: 24 MB for few
    // rows, 22 MB from a dozen rows on, 8 MB when very many rows follow each reduce; above 24 MB
    // the rate falls off sharply)
    h->avg_chunk_floats = (m >= 48 ? 8 : m >= 12 ? 22 : 24) * 256 * 1024;
    if (const char* e = getenv("LC_AVG_CHUNK_MB")) {   // tuning knobs for measurement runs
        const int mb = atoi(e);
        if (mb >= 1 && mb <= 1024) h->avg_chunk_floats = static_cast<int64_t>(mb) * 256 * 1024;
    }
    if (const char* e = getenv("LC_AVG_TWO_PHASE")) h->avg_two_phase = atoi(e) != 0;
    h->share_w_on = true;
    h->group_shared_on = true;
    if (const char* e = getenv("LC_GROUP_SHARED")) h->group_shared_on = atoi(e) != 0;   // tuning knob for measurement runs
    h->share_w_set = 8;
    if (const char* e = getenv("LC_SHARED_W_ORDER")) {   // 0: replica-major everywhere; n: sets of n replicas
        h->share_w_on = atoi(e) != 0;
        if (atoi(e) > 0) h->share_w_set = atoi(e);
    }
    h->X = h->V = nullptr;
    h->G = h->qa = h->qc = nullptr;
    h->data = nullptr;
    h->labels = nullptr;
    h->scratch = nullptr;
    h->scratch_bytes = 0;
    h->stream = nullptr;
    h->last_hip = 0;
    h->res_a1x = nullptr;
    h->res_ctr = nullptr;
    h->res_on = true;
    h->res_fuse_always = false;
    h->fl_on = true;
    h->imp_mode = 1;
    h->imp_out = false;
    for (int l = 0; l <= LC_MAX_LAYERS; ++l) h->imp[l] = ImpState{false, kBufX, kBufV};
    h->a1_ready = false;
    h->res_local_on = true;
    h->res_xcc_known = false;
    h->res_xcc_of = 0;
    h->res_used = false;
    h->res_arrivals = 0;
    h->res_garrivals = 0;
    h->res_spin_limit = 400000;   // several hundred milliseconds of polling
    h->timing_which = kTimeNone;
    h->ev_used = 0;
    h->timing_err = 0;
    h->timing_layer = h->timing_kernel = 0;
    h->bm_on = false;
    h->bm_beta = 0.f;
    h->v_cleared = false;
    h->lazy_enabled = h->lazy_rows = h->lazy_enabled_step = false;
    h->defer_x_on = true;
    h->defer_x = false;
    h->sync1_on = h->sync_all_on = true;
    h->fuse_avg_on = 2;
    h->fuse_avg = false;
    if (const char* e = getenv("LC_SYNC_FIRST_LAYER")) {   // tuning knob for measurement runs: 0 off, 1 layer 1 only
        h->sync1_on = atoi(e) != 0;
        h->sync_all_on = atoi(e) > 1;
    }
    h->sync_done = 0;
    h->loss_parts_train = h->loss_parts_eval = 1;
    (void)carve(h, nullptr);
    *out = h;
    return LC_OK;
}

void lc_destroy(lc_handle* h) {
    if (!h) return;
    for (hipEvent_t e : h->ev_pool) (void)hipEventDestroy(e);
    delete h;
}

size_t lc_workspace_bytes(const lc_handle* h) {
    if (!h) return 0;
    lc_handle tmp = *h;  // carve() only writes pointers; keep the caller's handle const
    tmp.ev_pool.clear();
    return carve(&tmp, nullptr);
}

int lc_attach(lc_handle* h, void* X, void* V, void* scratch, size_t scratch_bytes, const void* data,
              const int32_t* labels, void* stream) {
    if (!h || !X || !V || !scratch) return LC_ERR_ARG;
    if (h->md.kind == LC_KIND_MLP && (!data || !labels)) return LC_ERR_ARG;
    if (!aligned256(X) || !aligned256(V) || !aligned256(scratch) || (data && !aligned256(data))) return LC_ERR_ALIGN;
    const size_t need = lc_workspace_bytes(h);
    if (scratch_bytes < need) return LC_ERR_WORKSPACE;
    h->X = static_cast<float*>(X);
    h->V = static_cast<float*>(V);
    h->data = data;
    h->labels = labels;
    h->scratch = static_cast<char*>(scratch);
    h->scratch_bytes = scratch_bytes;
    h->stream = static_cast<hipStream_t>(stream);
    (void)carve(h, h->scratch);
    LC_HIP(h, hipMemsetAsync(scratch, 0, need, h->stream));
    h->res_arrivals = 0;
    h->res_garrivals = 0;
    LC_HIP(h, hipStreamSynchronize(h->stream));
    LC_HIP(h, probe_block_placement(h));   // (only where the resident kernel applies)
    h->attached = true;
    return LC_OK;
}

int lc_attach_quad(lc_handle* h, const float* a, const float* c) {
    if (!h || !a || !c) return LC_ERR_ARG;
    if (h->md.kind != LC_KIND_QUAD) return LC_ERR_MODEL;
    if (!aligned256(a) || !aligned256(c)) return LC_ERR_ALIGN;
    h->qa = a;
    h->qc = c;
    return LC_OK;
}

int lc_local_steps(lc_handle* h, int tau) {
    const int rc = require_objective(h);
    if (rc != LC_OK) return rc;
    if (tau < 1) return LC_ERR_ARG;
    return run_periods(h, tau, 1, false);
}

int lc_local_periods(lc_handle* h, int tau, int n_periods) {
    const int rc = require_objective(h);
    if (rc != LC_OK) return rc;
    if (tau < 1 || n_periods < 1) return LC_ERR_ARG;
    // In-kernel averaging pays while the m copies a workgroup has to read from the other replicas
    // (other XCDs) are small: measured on the 784-256-10 model at m = 8, 400 KB per workgroup take
    // 15 us, more than ending the launch and running the averaging kernel costs.
    const bool small = h->L == 1 || static_cast<int64_t>(h->m) * h->layer[1].dp_in * 64 <= 200 * 1024;
    const bool fused = h->md.kind == LC_KIND_MLP && h->res_on && h->res_a1x && h->res_avx && !h->bm_on &&
                       tau <= h->train.slots && (small || h->res_fuse_always);
    if (!fused) return run_periods(h, tau, n_periods, true);
    // weights resident on chip: as many whole periods per launch as one gather launch has inputs
    // for, the averaging steps taken inside the kernel
    const int per_launch = h->train.slots / tau;
    for (int done = 0; done < n_periods; done += per_launch) {
        const int p = n_periods - done < per_launch ? n_periods - done : per_launch;
        LC_HIP(h, launch_gather(h, false, h->k, p * tau));
        LC_HIP(h, launch_resident(h, 0, p * tau, tau));
        h->train.cur_slot = p * tau - 1;
        h->k += static_cast<int64_t>(p) * tau;
        h->v_cleared = false;
        h->lazy_rows = false;   // every row of X holds the mean
        h->res_used = true;
    }
    return LC_OK;
}

int lc_average(lc_handle* h) {
    const int rc = require_attached(h);
    if (rc != LC_OK) return rc;
    for (int l = 1; l <= h->L; ++l)
        if (h->imp[l].active) return LC_ERR_STATE;   // (cannot happen: every call ends with x in X and v in V)
    if (h->lazy_rows) {
        if (!h->bm_on) return LC_OK;   // already synchronised: averaging again changes nothing
        const int mrc = materialise(h);   // block momentum moves even a synchronised model (u decays)
        if (mrc != LC_OK) return mrc;
    }
    if (h->lazy_enabled && h->md.kind == LC_KIND_MLP) {
        // reduce only: the next local step reads the one averaged model and writes every row
        h->lazy_enabled_step = true;
        const hipError_t e = launch_average(h, h->X, nullptr, h->xbar);
        h->lazy_enabled_step = false;
        LC_HIP(h, e);
        h->lazy_rows = true;
    } else {
        LC_HIP(h, launch_average(h, h->X, h->X, nullptr));
    }
    if (h->bm_on) h->v_cleared = true;   // local momentum restarts after every block-momentum step
    return LC_OK;
}

int lc_set_lazy_broadcast(lc_handle* h, int on) {
    if (!h) return LC_ERR_ARG;
    if (!on && h->attached) {
        const int rc = materialise(h);
        if (rc != LC_OK) return rc;
    }
    h->lazy_enabled = on != 0;
    return LC_OK;
}

int lc_set_resident(lc_handle* h, int on) {
    if (!h) return LC_ERR_ARG;
    h->res_on = on != 0;
    h->res_fuse_always = on == 2;
    return LC_OK;
}

int lc_set_xcd_local_exchange(lc_handle* h, int on) {
    if (!h) return LC_ERR_ARG;
    h->res_local_on = on != 0;
    return LC_OK;
}

int lc_set_first_layer_fusion(lc_handle* h, int on) {
    if (!h) return LC_ERR_ARG;
    h->fl_on = on != 0;
    return LC_OK;
}

int lc_set_implicit_momentum(lc_handle* h, int mode) {
    if (!h || mode < 0 || mode > 2) return LC_ERR_ARG;
    h->imp_mode = mode;
    return LC_OK;
}

int lc_set_fused_averaging(lc_handle* h, int mode) {
    if (!h || mode < 0 || mode > 2) return LC_ERR_ARG;
    h->fuse_avg_on = mode;
    return LC_OK;
}

int lc_implicit_momentum_layers(const lc_handle* h) {
    if (!h) return LC_ERR_ARG;
    if (!h->attached) return LC_ERR_STATE;
    if (h->res_on && h->res_a1x) return 0;
    int n = 0;
    for (int l = 1; l <= h->L; ++l) n += implicit_layer_ok(h, l) ? 1 : 0;
    return n;
}

int lc_set_deferred_update(lc_handle* h, int on) {
    if (!h) return LC_ERR_ARG;
    h->defer_x_on = on != 0;
    return LC_OK;
}

int lc_resident_active(const lc_handle* h) {
    if (!h) return LC_ERR_ARG;
    if (!h->attached) return LC_ERR_STATE;
    return (h->res_on && h->res_a1x) ? 1 : 0;
}

int lc_set_barrier_polls(lc_handle* h, int polls) {
    if (!h || polls < 0) return LC_ERR_ARG;
    h->res_spin_limit = polls;
    return LC_OK;
}

int lc_materialize(lc_handle* h) {
    const int rc = require_attached(h);
    if (rc != LC_OK) return rc;
    return materialise(h);
}

int lc_block_momentum_begin(lc_handle* h, float beta_glob) {
    const int rc = require_attached(h);
    if (rc != LC_OK) return rc;
    if (!(beta_glob >= 0.f) || !(beta_glob < 1.f) || !(h->md.lr > 0.f)) return LC_ERR_ARG;
    const int mrc = materialise(h);
    if (mrc != LC_OK) return mrc;
    const size_t bytes = sizeof(float) * static_cast<size_t>(h->Ps);
    LC_HIP(h, hipMemsetAsync(h->bm_u, 0, bytes, h->stream));
    LC_HIP(h, hipMemcpyAsync(h->bm_xs, h->X, bytes, hipMemcpyDeviceToDevice, h->stream));
    h->bm_on = true;
    h->bm_beta = beta_glob;
    h->v_cleared = true;
    return LC_OK;
}

int lc_block_momentum_end(lc_handle* h) {
    if (!h) return LC_ERR_ARG;
    h->bm_on = false;
    return LC_OK;
}

int lc_get_block_momentum(lc_handle* h, float* u_host, float* x_sync_host) {
    const int rc = require_attached(h);
    if (rc != LC_OK) return rc;
    if (!h->bm_on) return LC_ERR_STATE;
    const size_t bytes = sizeof(float) * static_cast<size_t>(h->P);
    if (u_host) LC_HIP(h, hipMemcpyAsync(u_host, h->bm_u, bytes, hipMemcpyDeviceToHost, h->stream));
    if (x_sync_host) LC_HIP(h, hipMemcpyAsync(x_sync_host, h->bm_xs, bytes, hipMemcpyDeviceToHost, h->stream));
    LC_HIP(h, hipStreamSynchronize(h->stream));
    return LC_OK;
}

int lc_loss(lc_handle* h, double* out) {
    const int rc = require_objective(h);
    if (rc != LC_OK) return rc;
    if (!out) return LC_ERR_ARG;
    if (!h->lazy_rows) LC_HIP(h, launch_average(h, h->X, nullptr, h->xbar));   // else xbar is the model already
    double F = 0.0;
    if (h->md.kind == LC_KIND_QUAD) {
        int np = 0;
        LC_HIP(h, launch_quad_loss(h, &np));
        double* host = static_cast<double*>(malloc(sizeof(double) * static_cast<size_t>(np)));
        if (!host) return LC_ERR_ARG;
        hipError_t e = hipMemcpyAsync(host, h->partial, sizeof(double) * static_cast<size_t>(np), hipMemcpyDeviceToHost, h->stream);
        if (e == hipSuccess) e = hipStreamSynchronize(h->stream);
        if (e != hipSuccess) {
            free(host);
            h->last_hip = static_cast<int>(e);
            return LC_ERR_HIP;
        }
        for (int i = 0; i < np; ++i) F += host[i];
        free(host);
        F /= static_cast<double>(h->m);
    } else {
        const int per_pass = h->eval.G * h->eval.B;
        const int E = h->md.E;
        const int passes = (E + per_pass - 1) / per_pass;
        const size_t n = static_cast<size_t>(h->eval.G) * passes * kLossParts;
        float* host = static_cast<float*>(malloc(sizeof(float) * n));
        if (!host) return LC_ERR_ARG;
        hipError_t e = hipSuccess;
        for (int p = 0; p < passes && e == hipSuccess; ++p) {
            e = launch_gather(h, true, static_cast<int64_t>(p) * per_pass, 1);
            for (int l = 1; l <= h->L && e == hipSuccess; ++l) e = launch_forward(h, true, l, p * h->eval.G);
            if (e == hipSuccess && !forward_fuses_softmax(h)) e = launch_softmax(h, true, p * h->eval.G);
        }
        if (e == hipSuccess) e = hipMemcpyAsync(host, h->eval.loss, sizeof(float) * n, hipMemcpyDeviceToHost, h->stream);
        if (e == hipSuccess) e = hipStreamSynchronize(h->stream);
        if (e != hipSuccess) {
            free(host);
            h->last_hip = static_cast<int>(e);
            return LC_ERR_HIP;
        }
        for (size_t g = 0; g < n; g += kLossParts)
            for (int q = 0; q < h->loss_parts_eval; ++q) F += static_cast<double>(host[g + q]);
        free(host);
        F /= static_cast<double>(E);
    }
    *out = F;
    const int src = check_resident(h);
    if (src != LC_OK) return src;
    return isfinite(F) ? LC_OK : LC_ERR_NONFINITE;
}

int adacomm_next_tau(double F0, double Fl, int tau0) {
    if (!(F0 > 0.0) || !(Fl >= 0.0) || !isfinite(F0) || !isfinite(Fl) || tau0 < 1) return LC_ERR_ARG;
    volatile double ratio = Fl / F0;        // volatile: each operation rounded to double, nothing fused
    volatile double root = sqrt(ratio);
    volatile double prod = root * static_cast<double>(tau0);
    const double up = ceil(prod);
    if (!(up < 2147483647.0)) return LC_ERR_ARG;
    const int t = static_cast<int>(up);
    return t < 1 ? 1 : t;
}

int adacomm_next_tau_ex(double F0, double Fl, int tau0, int tau_prev, double gamma, int slack, double lr0,
                        double lrl, int lr_changed) {
    if (!(F0 > 0.0) || !(Fl >= 0.0) || !isfinite(F0) || !isfinite(Fl) || tau0 < 1 || tau_prev < 1) return LC_ERR_ARG;
    if (!(gamma > 0.0) || !(gamma < 1.0) || slack < 0) return LC_ERR_ARG;   // Sec. 4.3.1: a decay factor below 1
    if (!(lr0 > 0.0) || !(lrl > 0.0) || !isfinite(lr0) || !isfinite(lrl)) return LC_ERR_ARG;
    volatile double ratio = Fl / F0;
    volatile double coupling = lr0 / lrl;
    volatile double scaled = coupling * ratio;
    volatile double root = sqrt(scaled);
    volatile double prod = root * static_cast<double>(tau0);
    const double up = ceil(prod);
    if (!(up < 2147483647.0)) return LC_ERR_ARG;
    int cand = static_cast<int>(up);
    if (cand < 1) cand = 1;
    if (lr_changed) return cand;
    if (static_cast<int64_t>(cand) + slack < static_cast<int64_t>(tau_prev)) return cand;
    volatile double shrunk = gamma * static_cast<double>(tau_prev);
    const int t = static_cast<int>(ceil(shrunk));
    return t < 1 ? 1 : t;
}

int lc_run_ex(lc_handle* h, int64_t K, int tau0, int64_t interval, int refine, double gamma, int slack, int n_lr,
              const int64_t* lr_at, const float* lr_val, int postpone_lr, int64_t* sched_k, int32_t* sched_tau,
              float* sched_lr, int cap, int32_t* n_sched, int64_t* rounds) {
    const int rc = require_attached(h);
    if (rc != LC_OK) return rc;
    if (K < 0 || tau0 < 1 || interval < 1 || cap < 0 || n_lr < 0 || !n_sched || !rounds) return LC_ERR_ARG;
    if (cap > 0 && (!sched_k || !sched_tau || !sched_lr)) return LC_ERR_ARG;
    if (n_lr > 0 && (!lr_at || !lr_val)) return LC_ERR_ARG;
    for (int j = 0; j < n_lr; ++j)
        if (!(lr_val[j] > 0.f) || (j > 0 && lr_at[j] < lr_at[j - 1])) return LC_ERR_ARG;
    int tau = tau0, ns = 0, next_lr = 0, lr_changed = 0;
    int64_t r = 0, next_eval = h->k + interval;
    const double lr0 = static_cast<double>(h->md.lr);
    double F0 = 0.0;
    *n_sched = 0;
    *rounds = 0;
    int e = lc_loss(h, &F0);
    if (e != LC_OK) return e;
    if (ns < cap) {
        sched_k[ns] = h->k;
        sched_tau[ns] = tau;
        sched_lr[ns] = h->md.lr;
    }
    ++ns;
    const int64_t k_end = h->k + K;
    while (h->k < k_end) {
        const int64_t left = k_end - h->k;
        int64_t lim = next_eval < k_end ? next_eval : k_end;
        if (next_lr < n_lr && lr_at[next_lr] < lim) lim = lr_at[next_lr];
        const int np = whole_periods(h->k, tau, lim, k_end);
        if (np > 0) {
            e = lc_local_periods(h, tau, np);
        } else {
            e = lc_local_steps(h, static_cast<int>(left));   // the last, shortened period
            if (e == LC_OK) e = lc_average(h);
        }
        if (e != LC_OK) return e;
        r += np > 0 ? np : 1;
        while (next_lr < n_lr && h->k >= lr_at[next_lr] && (!postpone_lr || tau == 1)) {
            h->md.lr = lr_val[next_lr];
            ++next_lr;
            lr_changed = 1;
        }
        if (h->k >= next_eval && h->k < k_end) {
            double Fl = 0.0;
            e = lc_loss(h, &Fl);
            if (e != LC_OK) return e;
            const int nt = refine ? adacomm_next_tau_ex(F0, Fl, tau0, tau, gamma, slack, lr0,
                                                        static_cast<double>(h->md.lr), lr_changed)
                                  : adacomm_next_tau(F0, Fl, tau0);
            if (nt < 0) return nt;
            tau = nt;
            lr_changed = 0;
            if (ns < cap) {
                sched_k[ns] = h->k;
                sched_tau[ns] = tau;
                sched_lr[ns] = h->md.lr;
            }
            ++ns;
            while (next_eval <= h->k) next_eval += interval;
        }
        *n_sched = ns;
        *rounds = r;
    }
    *n_sched = ns;
    *rounds = r;
    LC_HIP(h, hipStreamSynchronize(h->stream));
    return LC_OK;
}

int lc_run(lc_handle* h, int64_t K, int tau0, int adaptive, int64_t interval, int64_t* sched_k,
           int32_t* sched_tau, int cap, int32_t* n_sched, int64_t* rounds) {
    const int rc = require_attached(h);
    if (rc != LC_OK) return rc;
    if (K < 0 || tau0 < 1 || cap < 0 || (cap > 0 && (!sched_k || !sched_tau)) || !n_sched || !rounds) return LC_ERR_ARG;
    if (adaptive && interval < 1) return LC_ERR_ARG;
    int tau = tau0, ns = 0;
    int64_t r = 0, next_eval = h->k + interval;
    double F0 = 0.0;
    *n_sched = 0;
    *rounds = 0;
    if (adaptive) {
        const int e = lc_loss(h, &F0);
        if (e != LC_OK) return e;
    }
    if (ns < cap) {
        sched_k[ns] = h->k;
        sched_tau[ns] = tau;
    }
    ++ns;
    const int64_t k_end = h->k + K;
    while (h->k < k_end) {
        const int64_t left = k_end - h->k;
        const int np = whole_periods(h->k, tau, adaptive && next_eval < k_end ? next_eval : k_end, k_end);
        int e;
        if (np > 0) {
            e = lc_local_periods(h, tau, np);
        } else {
            e = lc_local_steps(h, static_cast<int>(left));   // the last, shortened period
            if (e == LC_OK) e = lc_average(h);
        }
        if (e != LC_OK) return e;
        r += np > 0 ? np : 1;
        if (adaptive && h->k >= next_eval && h->k < k_end) {
            double Fl = 0.0;
            e = lc_loss(h, &Fl);
            if (e != LC_OK) return e;
            const int nt = adacomm_next_tau(F0, Fl, tau0);
            if (nt < 0) return nt;
            tau = nt;
            if (ns < cap) {
                sched_k[ns] = h->k;
                sched_tau[ns] = tau;
            }
            ++ns;
            while (next_eval <= h->k) next_eval += interval;
        }
        *n_sched = ns;
        *rounds = r;
    }
    *n_sched = ns;
    *rounds = r;
    LC_HIP(h, hipStreamSynchronize(h->stream));
    return LC_OK;
}

int lc_grid_search_tau0(lc_handle* h, const int32_t* taus, int n, int64_t K, double* loss_out, double* seconds_out,
                        int32_t* best) {
    const int rc = require_objective(h);
    if (rc != LC_OK) return rc;
    if (!taus || n < 1 || K < 1 || !loss_out || !seconds_out || !best) return LC_ERR_ARG;
    for (int i = 0; i < n; ++i)
        if (taus[i] < 1) return LC_ERR_ARG;
    if (h->bm_on) return LC_ERR_STATE;   // a block-momentum run has state this helper does not save
    // every candidate starts from the model as it is now: kept on the host meanwhile
    const size_t count = static_cast<size_t>(h->m) * static_cast<size_t>(h->P);
    float* X0 = static_cast<float*>(malloc(sizeof(float) * count));
    float* V0 = static_cast<float*>(malloc(sizeof(float) * count));
    int64_t k0 = 0;
    int e = (X0 && V0) ? lc_get_state(h, X0, V0, &k0) : LC_ERR_ARG;
    double F0 = 0.0;
    if (e == LC_OK) e = lc_loss(h, &F0);
    double best_rate = 0.0;
    *best = -1;
    for (int i = 0; i < n && e == LC_OK; ++i) {
        int64_t sk = 0, rounds = 0;
        int32_t st = 0, ns = 0;
        timespec t0, t1;
        clock_gettime(CLOCK_MONOTONIC, &t0);
        e = lc_run(h, K, taus[i], 0, 0, &sk, &st, 1, &ns, &rounds);   // synchronises the stream at its end
        clock_gettime(CLOCK_MONOTONIC, &t1);
        if (e == LC_OK) e = lc_loss(h, &loss_out[i]);
        if (e != LC_OK) break;
        seconds_out[i] = static_cast<double>(t1.tv_sec - t0.tv_sec) + 1e-9 * static_cast<double>(t1.tv_nsec - t0.tv_nsec);
        // the error-runtime trade-off: loss gained per second of this machine's time
        const double rate = (F0 - loss_out[i]) / (seconds_out[i] > 0.0 ? seconds_out[i] : 1e-9);
        if (*best < 0 || rate > best_rate) {
            *best = i;
            best_rate = rate;
        }
        e = lc_set_state(h, X0, V0, k0);
    }
    if (e != LC_OK && X0 && V0) (void)lc_set_state(h, X0, V0, k0);
    free(X0);
    free(V0);
    return e;
}

int lc_set_grad(lc_handle* h, const void* G) {
    if (!h || !G) return LC_ERR_ARG;
    if (!aligned256(G)) return LC_ERR_ALIGN;
    h->G = static_cast<const float*>(G);
    return LC_OK;
}

int lc_update_from_grad(lc_handle* h) {
    if (!h) return LC_ERR_ARG;
    if (!h->attached || !h->G) return LC_ERR_STATE;
    const int mrc = materialise(h);
    if (mrc != LC_OK) return mrc;
    LC_HIP(h, launch_update_from_grad(h));
    h->v_cleared = false;
    return LC_OK;
}

int lc_update_from_grad_and_average(lc_handle* h) {
    if (!h) return LC_ERR_ARG;
    if (!h->attached || !h->G) return LC_ERR_STATE;
    const int mrc = materialise(h);
    if (mrc != LC_OK) return mrc;
    LC_HIP(h, launch_update_and_average(h));
    h->v_cleared = false;
    return LC_OK;
}

int lc_get_state(lc_handle* h, float* X_host, float* V_host, int64_t* k) {
    if (!h) return LC_ERR_ARG;
    if (!h->attached) return LC_ERR_STATE;
    const size_t row = sizeof(float) * static_cast<size_t>(h->P), pitch = sizeof(float) * static_cast<size_t>(h->Ps);
    if (X_host) {
        const int mrc = materialise(h);
        if (mrc != LC_OK) return mrc;
        LC_HIP(h, hipMemcpy2DAsync(X_host, row, h->X, pitch, row, h->m, hipMemcpyDeviceToHost, h->stream));
    }
    if (V_host && !h->v_cleared)
        LC_HIP(h, hipMemcpy2DAsync(V_host, row, h->V, pitch, row, h->m, hipMemcpyDeviceToHost, h->stream));
    LC_HIP(h, hipStreamSynchronize(h->stream));
    if (V_host && h->v_cleared) memset(V_host, 0, row * static_cast<size_t>(h->m));   // cleared, not yet rewritten
    if (k) *k = h->k;
    return check_resident(h);
}

int lc_set_state(lc_handle* h, const float* X_host, const float* V_host, int64_t k) {
    if (!h || k < 0) return LC_ERR_ARG;
    if (!h->attached) return LC_ERR_STATE;
    const size_t row = sizeof(float) * static_cast<size_t>(h->P), pitch = sizeof(float) * static_cast<size_t>(h->Ps);
    if (X_host) {
        LC_HIP(h, hipMemcpy2DAsync(h->X, pitch, X_host, row, row, h->m, hipMemcpyHostToDevice, h->stream));
        h->lazy_rows = false;
    }
    if (V_host) {
        LC_HIP(h, hipMemcpy2DAsync(h->V, pitch, V_host, row, row, h->m, hipMemcpyHostToDevice, h->stream));
        h->v_cleared = false;
    }
    LC_HIP(h, hipStreamSynchronize(h->stream));
    h->k = k;
    return LC_OK;
}

int lc_set_lr(lc_handle* h, float lr) {
    if (!h || !(lr >= 0.f)) return LC_ERR_ARG;
    h->md.lr = lr;
    return LC_OK;
}

int lc_get_local_losses(lc_handle* h, float* losses_host) {
    if (!h || !losses_host) return LC_ERR_ARG;
    if (!h->attached) return LC_ERR_STATE;
    if (h->md.kind != LC_KIND_MLP) return LC_ERR_UNSUPPORTED;
    float* parts = static_cast<float*>(malloc(sizeof(float) * static_cast<size_t>(h->m) * kLossParts));
    if (!parts) return LC_ERR_ARG;
    hipError_t e = hipMemcpyAsync(parts, h->train.loss, sizeof(float) * static_cast<size_t>(h->m) * kLossParts,
                                  hipMemcpyDeviceToHost, h->stream);
    if (e == hipSuccess) e = hipStreamSynchronize(h->stream);
    if (e != hipSuccess) {
        free(parts);
        h->last_hip = static_cast<int>(e);
        return LC_ERR_HIP;
    }
    for (int i = 0; i < h->m; ++i) {
        float sum = 0.f;
        for (int q = 0; q < h->loss_parts_train; ++q) sum += parts[static_cast<size_t>(i) * kLossParts + q];
        losses_host[i] = sum;
    }
    free(parts);
    return check_resident(h);
}

int lc_get_last_indices(lc_handle* h, int32_t* idx_host) {
    if (!h || !idx_host) return LC_ERR_ARG;
    if (!h->attached) return LC_ERR_STATE;
    if (h->md.kind != LC_KIND_MLP) return LC_ERR_UNSUPPORTED;
    const size_t row = sizeof(int32_t) * static_cast<size_t>(h->train.B), pitch = sizeof(int32_t) * static_cast<size_t>(h->train.Bp);
    const int32_t* src = h->train.idx + static_cast<size_t>(h->train.cur_slot) * h->train.G * h->train.Bp;
    LC_HIP(h, hipMemcpy2DAsync(idx_host, row, src, pitch, row, h->m, hipMemcpyDeviceToHost, h->stream));
    LC_HIP(h, hipStreamSynchronize(h->stream));
    return LC_OK;
}

int lc_timing_begin(lc_handle* h, int which) {
    if (!h || which < kTimeNone || which > kTimeUpdAvg) return LC_ERR_ARG;
    h->timing_which = which;
    h->timing_layer = h->timing_kernel = 0;
    h->ev_used = 0;
    h->timing_err = 0;
    return LC_OK;
}

int lc_timing_select(lc_handle* h, int layer, int kernel) {
    if (!h || layer < 0 || layer > LC_MAX_LAYERS || kernel < kBwdAny || kernel > kBwdResident) return LC_ERR_ARG;
    h->timing_layer = layer;
    h->timing_kernel = kernel;
    h->ev_used = 0;
    return LC_OK;
}

int lc_timing_read(lc_handle* h, int64_t* launches, double* total_ms) {
    if (!h || !launches || !total_ms) return LC_ERR_ARG;
    if (!h->attached) return LC_ERR_STATE;
    LC_HIP(h, hipStreamSynchronize(h->stream));
    if (h->timing_err) {   // an event could not be created or recorded: the figures would be incomplete
        h->last_hip = h->timing_err;
        h->timing_err = 0;
        h->ev_used = 0;
        return LC_ERR_HIP;
    }
    double sum = 0.0;
    for (size_t i = 0; i + 1 < h->ev_used; i += 2) {
        float ms = 0.f;
        LC_HIP(h, hipEventElapsedTime(&ms, h->ev_pool[i], h->ev_pool[i + 1]));
        sum += static_cast<double>(ms);
    }
    *launches = static_cast<int64_t>(h->ev_used / 2);
    *total_ms = sum;
    h->ev_used = 0;
    return LC_OK;
}

}  // extern "C"
