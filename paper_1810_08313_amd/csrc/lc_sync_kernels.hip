// First layer at tau = 1: backward pass, momentum update and the averaging of the layer in one kernel.
//
// With tau = 1 the k mod tau = 0 branch of the update rule (Sec. 2) is taken at every iteration:
// all workers start an iteration from the same averaged model x_bar, worker i's model after its
// step is x_bar - lr v_i, and the next model is the mean of those.  The first layer needs no dA,
// so its weights can be shared out by TILE instead of by replica: a workgroup owns a 64 x 64 tile
// of W_1 and walks over the replicas.  Per replica it forms the replica's dW tile from that
// replica's A_0^T rows and dZ_1 slice (matrix cores, the summation order of backward_kernel),
// updates the replica's momentum tile v_i in place, and adds x_bar - lr v_i to a sum kept in
// double (exact for m floats, so the order does not matter and the result is the correctly
// rounded mean, as in the averaging kernels).  After the last replica the mean goes straight
// into x_bar.  The tile of x_bar is read once and written once, the replicas' weights never
// exist in memory, and the averaging kernels skip the layer: 8 bytes per parameter and replica
// (v_i in, v_i out) is all that moves.
//
// The same decomposition serves the LAST step of a longer period (OWN instances): there every
// worker has weights of its own, so the walk reads worker i's tile of weights and of momentum (or,
// where the momentum is implicit, of the model one step earlier), writes v_i, and adds the worker's
// new weights to the sum -- the rows of X are not written, since the averaging step that follows
// would only read them once and overwrite them: 8 bytes read and 4 written per parameter and
// replica for the step and the layer's averaging together, instead of 16 + 4.
#include "lc_internal.h"
#include "lc_mma.h"

namespace lc {

namespace {

struct SyncArgs {
    float* V;             // momentum rows [G][x_stride]
    int64_t x_stride;
    float* xbar;          // the shared model: the tile is read before the walk and overwritten after it
    // OWN instances: every worker's own weights, and the second operand of its update (see BwdArgs::Aux)
    const float* Xr;
    int64_t xr_stride;
    const float* Aux;
    int64_t aux_stride;
    int imp_in;
    float inv_lr;
    float* X;             // rows of X: only the bias entries are written there (they are averaged by the averaging kernels)
    int64_t w_off, b_off;
    int d_in, d_out, dp_in, dp_out;
    int B, G;
    const void* a_fm;     // A_0^T of this iteration [G][dp_in][Bp]
    const void* dz_fm;    // dZ_1^T of this iteration [G][dp_out][Bp]
    float lr, beta, wd;
    int n_row_blocks, n_cc;
    int64_t total_blocks;
};

// Workgroup (row block rb, column chunk cc), 4 wavefronts of 16 rows each.  The loads of replica
// g + 1 (momentum tile, A_0^T rows, dZ_1 slice) are in flight while replica g is worked on; the
// slice is staged in LDS in two buffers, one barrier per replica.
template <typename OT, int NT, bool OWN = false>
__global__ __launch_bounds__(256) void sync_first_layer_kernel(SyncArgs a) {
    constexpr int kPad = sizeof(OT) == 2 ? 8 : 4;
    constexpr int Bp = 16 * NT;
    constexpr int NS = NT / 2;
    // row (c % 4) * 16 + c / 4 holds column c0 + c (the layout backward_kernel uses)
    __shared__ __attribute__((aligned(16))) OT dzt_lds[2][kColChunk][Bp + kPad];

    const int64_t logical = xcd_logical_block(a.total_blocks);
    if (logical < 0) return;
    const int rb = static_cast<int>(logical / a.n_cc), cc = static_cast<int>(logical % a.n_cc);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int j = lane & 15, q = lane >> 4;
    const int k0 = (rb * 4 + wave) * kRowsPerWave;
    const int c0 = cc * kColChunk;

    // the tile of the shared model, rows k0 + 4 q + r, columns c0 + 4 j .. + 3 (rows past d_in read
    // the last row; they are never stored)
    float4 w[4], wn[4];
    int at[4];   // (offsets inside one model: below 2^31 for any layer this kernel takes)
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int row = k0 + 4 * q + r;
        const int rr = row < a.d_in ? row : a.d_in - 1;
        at[r] = static_cast<int>(a.w_off + static_cast<int64_t>(rr) * a.d_out + c0 + 4 * j);
        if constexpr (!OWN) w[r] = *reinterpret_cast<const float4*>(a.xbar + at[r]);
    }
    const bool bias_job = rb == cc % a.n_row_blocks && tid < kColChunk && c0 + tid < a.d_out;
    const float xb_bias = (!OWN && bias_job) ? a.xbar[a.b_off + c0 + tid] : 0.f;

    double sum[4][4];
#pragma unroll
    for (int r = 0; r < 4; ++r) sum[r][0] = sum[r][1] = sum[r][2] = sum[r][3] = 0.0;

    float4 v[4], vn[4];
    Frag<OT> af[NS], st_t[NS];
    auto load_rows = [&](int g) {   // this lane's A_0^T operands of replica g
        const OT* AT = static_cast<const OT*>(a.a_fm) + static_cast<int64_t>(g) * a.dp_in * Bp;
#pragma unroll
        for (int s = 0; s < NS; ++s) af[s] = load8(AT + static_cast<int64_t>(k0 + j) * Bp + 32 * s + 8 * q);
    };
    auto issue_loads = [&](int g, float4 (&vv)[4], float4 (&ww)[4]) {
        if constexpr (OWN) {
            const float* Wg = a.Xr + static_cast<int64_t>(g) * a.xr_stride;
            const float* Ag = a.Aux + static_cast<int64_t>(g) * a.aux_stride;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                ww[r] = load_wm<kWVectorStream>(Wg + at[r], 0, a.d_out, true);
                vv[r] = load_wm<kWVectorStream>(Ag + at[r], 0, a.d_out, true);
            }
        } else {
            const float* Vg = a.V + static_cast<int64_t>(g) * a.x_stride;
#pragma unroll
            for (int r = 0; r < 4; ++r) vv[r] = load_wm<kWVectorStream>(Vg + at[r], 0, a.d_out, true);
        }
        // the dZ^T slice is one contiguous run of 64 * Bp elements
        const OT* src_t = static_cast<const OT*>(a.dz_fm) + (static_cast<int64_t>(g) * a.dp_out + c0) * Bp;
#pragma unroll
        for (int s = 0; s < NS; ++s) st_t[s] = load8(src_t + static_cast<int64_t>(tid + 256 * s) * 8);
    };
    auto stage_to_lds = [&](int buf) {
#pragma unroll
        for (int s = 0; s < NS; ++s) {
            const int p = tid + 256 * s;
            const int c = p / (Bp / 8), seg = p % (Bp / 8);
            *reinterpret_cast<Frag<OT>*>(&dzt_lds[buf][(c & 3) * 16 + (c >> 2)][seg * 8]) = st_t[s];
        }
    };

    issue_loads(0, v, w);
    load_rows(0);
    stage_to_lds(0);
    __syncthreads();

    for (int g = 0; g < a.G; ++g) {
        const int buf = g & 1;
        const bool has_next = g + 1 < a.G;
        if (has_next) issue_loads(g + 1, vn, wn);

        // bias of these 64 columns for replica g (one thread per column): the momentum entry is
        // updated here, the averaging kernels form x_bar - lr v from it like for every other layer
        if (bias_job) {
            float* bv = a.V + static_cast<int64_t>(g) * a.x_stride + a.b_off + c0 + tid;
            float xb = xb_bias, v0;
            if constexpr (OWN) {   // the worker's own bias; its new value goes to its row of X
                xb = a.Xr[static_cast<int64_t>(g) * a.xr_stride + a.b_off + c0 + tid];
                v0 = a.Aux[static_cast<int64_t>(g) * a.aux_stride + a.b_off + c0 + tid];
                if (a.imp_in) v0 = (v0 - xb) * a.inv_lr;
            } else {
                v0 = *bv;
            }
            const OT* zr = dzt_lds[buf][(tid & 3) * 16 + (tid >> 2)];
            float sb = 0.f;
#pragma unroll
            for (int b8 = 0; b8 < Bp; b8 += 8) {
                const Frag<OT> f = *reinterpret_cast<const Frag<OT>*>(zr + b8);
#pragma unroll
                for (int e = 0; e < 8; ++e) sb += to_f32(f.v[e]);
            }
            const float vb = momentum_update(a.beta, v0, sb, a.wd, xb);
            *bv = vb;
            if constexpr (OWN) a.X[static_cast<int64_t>(g) * a.x_stride + a.b_off + c0 + tid] = weight_update(xb, a.lr, vb);
        }
        // dW tile: sum over the batch of A^T[k][b] dZ^T[c][b]
        f32x4 acc[4];
#pragma unroll
        for (int t = 0; t < 4; ++t) acc[t] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int s = 0; s < NS; ++s) {
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const Frag<OT> bf = *reinterpret_cast<const Frag<OT>*>(&dzt_lds[buf][t * 16 + j][32 * s + 8 * q]);
                acc[t] = mma8(af[s], bf, acc[t]);
            }
        }
        if (has_next) load_rows(g + 1);   // (the operand registers are free again; no second set)
        // momentum update, the replica's weights, their contribution to the mean
        float* Vg = a.V + static_cast<int64_t>(g) * a.x_stride;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int row = k0 + 4 * q + r;
            const float4 gr = make_float4(acc[0][r], acc[1][r], acc[2][r], acc[3][r]);
            if (OWN && a.imp_in) {   // the tile holds the parameters of one step earlier: v = (x_prev - x) / lr
                v[r].x = (v[r].x - w[r].x) * a.inv_lr;
                v[r].y = (v[r].y - w[r].y) * a.inv_lr;
                v[r].z = (v[r].z - w[r].z) * a.inv_lr;
                v[r].w = (v[r].w - w[r].w) * a.inv_lr;
            }
            v[r].x = momentum_update(a.beta, v[r].x, gr.x, a.wd, w[r].x);
            v[r].y = momentum_update(a.beta, v[r].y, gr.y, a.wd, w[r].y);
            v[r].z = momentum_update(a.beta, v[r].z, gr.z, a.wd, w[r].z);
            v[r].w = momentum_update(a.beta, v[r].w, gr.w, a.wd, w[r].w);
            const float4 x = make_float4(weight_update(w[r].x, a.lr, v[r].x), weight_update(w[r].y, a.lr, v[r].y),
                                         weight_update(w[r].z, a.lr, v[r].z), weight_update(w[r].w, a.lr, v[r].w));
            if (row < a.d_in) store_wm<kWVectorStream>(Vg + at[r], 0, a.d_out, true, v[r]);
            sum[r][0] += static_cast<double>(x.x);
            sum[r][1] += static_cast<double>(x.y);
            sum[r][2] += static_cast<double>(x.z);
            sum[r][3] += static_cast<double>(x.w);
        }
        if (has_next) {
            stage_to_lds(buf ^ 1);   // (its last readers passed the barrier of the previous replica)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                v[r] = vn[r];
                if constexpr (OWN) w[r] = wn[r];
            }
        }
        __syncthreads();
    }
    const double dm = static_cast<double>(a.G);
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int row = k0 + 4 * q + r;
        if (row < a.d_in)
            *reinterpret_cast<float4*>(a.xbar + at[r]) =
                make_float4(static_cast<float>(sum[r][0] / dm), static_cast<float>(sum[r][1] / dm),
                            static_cast<float>(sum[r][2] / dm), static_cast<float>(sum[r][3] / dm));
    }
}

template <typename OT, bool OWN>
hipError_t launch_sync1(const SyncArgs& a, int nt, unsigned grid, hipStream_t st) {
    if (nt == 2) hipLaunchKernelGGL((sync_first_layer_kernel<OT, 2, OWN>), dim3(grid), dim3(256), 0, st, a);
    else if (nt == 4) hipLaunchKernelGGL((sync_first_layer_kernel<OT, 4, OWN>), dim3(grid), dim3(256), 0, st, a);
    else hipLaunchKernelGGL((sync_first_layer_kernel<OT, 8, OWN>), dim3(grid), dim3(256), 0, st, a);
    return hipGetLastError();
}

}  // namespace

// Layers of models with at least two layers whose rows are 16-byte aligned and a multiple of 64
// columns long; large layers only (the ones the shared-model block order is for): small ones are
// cache-resident and gain nothing.  The last layer keeps its own kernels (its forward pass forms
// the loss and dZ_L).
bool sync_layer_ok(const lc_handle* h, int l) {
    if (h->md.kind != LC_KIND_MLP || h->L < 2 || !h->sync1_on || l < 1 || l >= h->L) return false;
    const LayerGeom& g = h->layer[l];
    const ActSet& S = h->train;
    if (g.w_off % 4 != 0 || g.d_out % kColChunk != 0 || h->Ps % 4 != 0) return false;
    if (S.Bp != 32 && S.Bp != 64 && S.Bp != 128) return false;
    if (g.dp_in % 64 != 0 || g.d_in < 1) return false;
    if (l > 1 && !h->sync_all_on) return false;
    return shared_weight_order(h, g);
}

// dW_l of every replica from A_{l-1}^T and dZ_l, the update of V, and the new averaged weights of
// the layer written over the old ones in xbar.  Inside a tau = 1 iteration whose replicas all
// start from xbar (lc_handle::defer_x), or as the last step of a longer period whose averaging step
// follows with the broadcast deferred (lc_handle::fuse_avg: every worker's own weights); for l > 1
// after dZ_{l-1} has been formed from the old weights (launch_backward(h, l, true)).
hipError_t launch_sync_layer(lc_handle* h, int l) {
    const ActSet& S = h->train;
    if (!sync_layer_ok(h, l)) return hipErrorInvalidValue;
    const bool own = !h->defer_x;
    if (own ? !h->fuse_avg : !h->lazy_rows) return hipErrorInvalidValue;
    const LayerGeom& g = h->layer[l];
    const bool bf16 = h->md.gemm == LC_GEMM_BF16;
    SyncArgs a;
    a.V = h->V;
    a.x_stride = h->Ps;
    a.xbar = h->xbar;
    const StepBufs sb = plan_step_buffers(h, l);
    if (own && (!sb.ov || !(h->md.lr > 0.f || !sb.imp_in))) return hipErrorInvalidValue;   // (the step leaves v in V)
    a.Xr = sb.xr;
    a.xr_stride = sb.xr_stride;
    a.Aux = sb.aux;
    a.aux_stride = sb.aux_stride;
    a.imp_in = sb.imp_in;
    a.inv_lr = h->md.lr > 0.f ? 1.f / h->md.lr : 0.f;
    a.X = h->X;
    a.w_off = g.w_off;
    a.b_off = g.b_off;
    a.d_in = g.d_in;
    a.d_out = g.d_out;
    a.dp_in = g.dp_in;
    a.dp_out = g.dp_out;
    a.B = S.B;
    a.G = S.G;
    if (l == 1) {
        const size_t slot_bytes = static_cast<size_t>(S.G) * S.Bp * g.dp_in * (bf16 ? 2 : 4);
        a.a_fm = static_cast<const char*>(S.a_fm[0]) + static_cast<size_t>(S.cur_slot) * slot_bytes;
    } else {
        a.a_fm = S.a_fm[l - 1];
    }
    a.dz_fm = S.dz_fm[l];
    a.lr = h->md.lr;
    a.beta = effective_beta(h);
    a.wd = h->md.wd;
    a.n_row_blocks = g.dp_in / 64;
    a.n_cc = g.d_out / kColChunk;
    a.total_blocks = static_cast<int64_t>(a.n_row_blocks) * a.n_cc;
    const unsigned grid = static_cast<unsigned>((a.total_blocks + kXcds - 1) / kXcds * kXcds);
    timing_start(h, kTimeBwd, l, kBwdTileOwner);
    hipError_t e;
    if (own) e = bf16 ? launch_sync1<bf16_t, true>(a, S.Bp / 16, grid, h->stream) : launch_sync1<float, true>(a, S.Bp / 16, grid, h->stream);
    else e = bf16 ? launch_sync1<bf16_t, false>(a, S.Bp / 16, grid, h->stream) : launch_sync1<float, false>(a, S.Bp / 16, grid, h->stream);
    timing_stop(h, kTimeBwd, l, kBwdTileOwner);
    if (e == hipSuccess && own) h->imp[l] = sb.next;   // (explicit again: v is in V; the rows of X wait for the broadcast)
    return e;
}

}  // namespace lc
