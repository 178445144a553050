// Bandwidth-bound kernels over the stacked models X[m, Ps]: replica averaging
// (the communication step of PASGD, Sec. 2), the momentum-SGD update from
// explicit gradients, their fusion for tau = 1, and the quadratic test
// objective.  Every thread owns one 16-byte column of the [m, Ps] matrix, so
// the reduction over the m axis happens in registers and each row is read and
// written in fully coalesced 1 KiB wavefront segments.
#include <mutex>

#include "lc_internal.h"

// Scratch of lc_average_block_momentum_static(): u in the first half, x_sync in the second.  In
// host code this name is only a handle for hipGetSymbolAddress(); the device address is looked up
// once per device (static_scratch() below) and that pointer is what kernels and copies get.
static __device__ __align__(256) float scratch[2 * LC_STATIC_MAX_PARAMS];

namespace lc {

namespace {

constexpr int kThreads = 256;
constexpr int kRowBatch = 8;  // rows whose loads are issued before any is consumed

__device__ __forceinline__ float4 ld_stream(const float* p) {
    const f32x4 v = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(p));
    return make_float4(v[0], v[1], v[2], v[3]);
}
__device__ __forceinline__ void st_stream(float* p, float4 v) {
    __builtin_nontemporal_store(f32x4{v.x, v.y, v.z, v.w}, reinterpret_cast<f32x4*>(p));
}

// Block momentum (Sec. 5.3.1) applied to one float4 of the mean: G = (x_sync - x_bar) / lr,
// u <- beta_glob u + G, x_sync <- x_sync - lr u; returns the new synchronised values.
struct BlockMomentum {
    float* u;      // null: plain averaging
    float* xs;
    float beta_glob, lr, inv_lr;
};

__device__ __forceinline__ float4 apply_block_momentum(const BlockMomentum& bm, int64_t col, float4 mean) {
    if (!bm.u) return mean;
    float4 u = *reinterpret_cast<const float4*>(bm.u + col);
    float4 xs = *reinterpret_cast<const float4*>(bm.xs + col);
    u.x = bm.beta_glob * u.x + (xs.x - mean.x) * bm.inv_lr;
    u.y = bm.beta_glob * u.y + (xs.y - mean.y) * bm.inv_lr;
    u.z = bm.beta_glob * u.z + (xs.z - mean.z) * bm.inv_lr;
    u.w = bm.beta_glob * u.w + (xs.w - mean.w) * bm.inv_lr;
    xs.x -= bm.lr * u.x;
    xs.y -= bm.lr * u.y;
    xs.z -= bm.lr * u.z;
    xs.w -= bm.lr * u.w;
    *reinterpret_cast<float4*>(bm.u + col) = u;
    *reinterpret_cast<float4*>(bm.xs + col) = xs;
    return xs;
}

// Deferred update (tau = 1 right after an averaging step): all replicas started the iteration from
// the same model xb, the backward kernels wrote only the momentum rows V, and the rows handed to
// the averaging kernels are those V: replica i's weights are formed here, with the expression and
// the rounding of the update in the backward kernels (one fused multiply-add), and never stored.
struct DeferredUpdate {
    const float* xb;   // null: the rows are the weights themselves
    float lr;
};

__device__ __forceinline__ float4 weights_from_momentum(const float4& xb, const float4& v, float lr) {
    return make_float4(__builtin_fmaf(-lr, v.x, xb.x), __builtin_fmaf(-lr, v.y, xb.y),
                       __builtin_fmaf(-lr, v.z, xb.z), __builtin_fmaf(-lr, v.w, xb.w));
}

// x_bar = (1/m) sum_i x^(i), written to every row of out_rows (in place when
// out_rows == X) and/or to the single vector out_single.  The sum is carried in
// double: adding m floats in double is exact for any realistic spread of
// magnitudes, so the result is the correctly rounded mean whatever the order.
__global__ __launch_bounds__(kThreads) void average_kernel(const float* X, float* out_rows, float* out_single,
                                                           int m, int64_t Ps, BlockMomentum bm, DeferredUpdate du,
                                                           int64_t c_lo, int64_t c_hi) {
    const int64_t col = c_lo + (static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x) * 4;
    if (col >= c_hi) return;
    float4 xb = make_float4(0.f, 0.f, 0.f, 0.f);
    if (du.xb) xb = *reinterpret_cast<const float4*>(du.xb + col);
    double s0 = 0, s1 = 0, s2 = 0, s3 = 0;
    for (int i0 = 0; i0 < m; i0 += kRowBatch) {
        float4 r[kRowBatch];
#pragma unroll
        for (int u = 0; u < kRowBatch; ++u)
            if (i0 + u < m) r[u] = ld_stream(X + static_cast<int64_t>(i0 + u) * Ps + col);
#pragma unroll
        for (int u = 0; u < kRowBatch; ++u)
            if (i0 + u < m) {
                if (du.xb) r[u] = weights_from_momentum(xb, r[u], du.lr);
                s0 += static_cast<double>(r[u].x);
                s1 += static_cast<double>(r[u].y);
                s2 += static_cast<double>(r[u].z);
                s3 += static_cast<double>(r[u].w);
            }
    }
    const double dm = static_cast<double>(m);
    float4 mean = make_float4(static_cast<float>(s0 / dm), static_cast<float>(s1 / dm),
                              static_cast<float>(s2 / dm), static_cast<float>(s3 / dm));
    mean = apply_block_momentum(bm, col, mean);
    if (out_single) *reinterpret_cast<float4*>(out_single + col) = mean;
    if (out_rows)
        for (int i = 0; i < m; ++i) st_stream(out_rows + static_cast<int64_t>(i) * Ps + col, mean);
}

// Two-kernel form of the averaging step for states larger than the caches.
// Writing m row streams from one kernel while it is still reading them costs
// this memory system about a fifth of its bandwidth; separating the phases does
// not.  The columns are processed in chunks small enough for one row's chunk to
// stay in the L2 / memory-side cache between the two kernels:
//   reduce_chunk    reads the m rows of the chunk and writes the mean over row 0
//                   (one stream out, and no bytes beyond the algorithmic ones)
//   broadcast_chunk copies the cached row-0 chunk to rows 1..m-1, one row after
//                   the other; consecutive blocks write consecutive addresses
constexpr int kReduceCols = 8;   // float4 columns per thread in reduce_chunk

template <bool DU>
__global__ __launch_bounds__(kThreads) void reduce_chunk_kernel(const float* X, float* dst, int m, int64_t Ps,
                                                                int64_t c_lo, int64_t c_hi, BlockMomentum bm,
                                                                DeferredUpdate du) {
    const int64_t base = c_lo / 4 + static_cast<int64_t>(blockIdx.x) * kThreads * kReduceCols;
    double s[kReduceCols][4];
    float4 xb[DU ? kReduceCols : 1];
#pragma unroll
    for (int u = 0; u < kReduceCols; ++u) {
        s[u][0] = s[u][1] = s[u][2] = s[u][3] = 0.0;
        if constexpr (DU) {
            const int64_t c = (base + u * kThreads + threadIdx.x) * 4;
            xb[u] = c < c_hi ? *reinterpret_cast<const float4*>(du.xb + c) : make_float4(0.f, 0.f, 0.f, 0.f);
        }
    }
    for (int i = 0; i < m; ++i) {
        float4 r[kReduceCols];
#pragma unroll
        for (int u = 0; u < kReduceCols; ++u) {
            const int64_t c = (base + u * kThreads + threadIdx.x) * 4;
            r[u] = c < c_hi ? ld_stream(X + static_cast<int64_t>(i) * Ps + c) : make_float4(0.f, 0.f, 0.f, 0.f);
        }
#pragma unroll
        for (int u = 0; u < kReduceCols; ++u) {
            if constexpr (DU) r[u] = weights_from_momentum(xb[u], r[u], du.lr);
            s[u][0] += static_cast<double>(r[u].x);
            s[u][1] += static_cast<double>(r[u].y);
            s[u][2] += static_cast<double>(r[u].z);
            s[u][3] += static_cast<double>(r[u].w);
        }
    }
    const double dm = static_cast<double>(m);
#pragma unroll
    for (int u = 0; u < kReduceCols; ++u) {
        const int64_t c = (base + u * kThreads + threadIdx.x) * 4;
        if (c < c_hi)
            *reinterpret_cast<float4*>(dst + c) = apply_block_momentum(
                bm, c,
                make_float4(static_cast<float>(s[u][0] / dm), static_cast<float>(s[u][1] / dm),
                            static_cast<float>(s[u][2] / dm), static_cast<float>(s[u][3] / dm)));
    }
}

__global__ __launch_bounds__(kThreads) void broadcast_chunk_kernel(const float* src, float* X, int first_row,
                                                                   int64_t Ps, int64_t c_lo, int64_t c_hi,
                                                                   int64_t blocks_per_row) {
    const int64_t row = first_row + blockIdx.x / blocks_per_row, b = blockIdx.x % blocks_per_row;
    const int64_t col = c_lo + (b * kThreads + threadIdx.x) * 4;
    if (col >= c_hi) return;
    st_stream(X + row * Ps + col, *reinterpret_cast<const float4*>(src + col));
}

// (the roundings of lc_mma.h's momentum_update / weight_update: two fused multiply-adds each)
__device__ __forceinline__ void sgd_update4(float4& x, float4& v, const float4& g, float lr, float beta, float wd) {
    v.x = __builtin_fmaf(beta, v.x, __builtin_fmaf(wd, x.x, g.x));
    v.y = __builtin_fmaf(beta, v.y, __builtin_fmaf(wd, x.y, g.y));
    v.z = __builtin_fmaf(beta, v.z, __builtin_fmaf(wd, x.z, g.z));
    v.w = __builtin_fmaf(beta, v.w, __builtin_fmaf(wd, x.w, g.w));
    x.x = __builtin_fmaf(-lr, v.x, x.x);
    x.y = __builtin_fmaf(-lr, v.y, x.y);
    x.z = __builtin_fmaf(-lr, v.z, x.z);
    x.w = __builtin_fmaf(-lr, v.w, x.w);
}

// g <- G + wd x; v <- beta v + g; x <- x - lr v over the whole [m, Ps] block.
__global__ __launch_bounds__(kThreads) void update_kernel(float* X, float* V, const float* __restrict__ G,
                                                          int64_t n4, float lr, float beta, float wd) {
    const int64_t j = static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x;
    if (j >= n4) return;
    float4 x = ld_stream(X + j * 4), v = ld_stream(V + j * 4);
    const float4 g = ld_stream(G + j * 4);
    sgd_update4(x, v, g, lr, beta, wd);
    st_stream(V + j * 4, v);
    st_stream(X + j * 4, x);
}

// tau = 1: the update of every worker and the averaging in one pass.
__global__ __launch_bounds__(kThreads) void update_average_kernel(float* X, float* V, const float* __restrict__ G,
                                                                  int m, int64_t Ps, float lr, float beta, float wd) {
    const int64_t col = (static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x) * 4;
    if (col >= Ps) return;
    double s0 = 0, s1 = 0, s2 = 0, s3 = 0;
    for (int i0 = 0; i0 < m; i0 += 4) {
        float4 x[4], v[4], g[4];
#pragma unroll
        for (int u = 0; u < 4; ++u)
            if (i0 + u < m) {
                const int64_t o = static_cast<int64_t>(i0 + u) * Ps + col;
                x[u] = ld_stream(X + o);
                v[u] = ld_stream(V + o);
                g[u] = ld_stream(G + o);
            }
#pragma unroll
        for (int u = 0; u < 4; ++u)
            if (i0 + u < m) {
                sgd_update4(x[u], v[u], g[u], lr, beta, wd);
                st_stream(V + static_cast<int64_t>(i0 + u) * Ps + col, v[u]);
                s0 += static_cast<double>(x[u].x);
                s1 += static_cast<double>(x[u].y);
                s2 += static_cast<double>(x[u].z);
                s3 += static_cast<double>(x[u].w);
            }
    }
    const double dm = static_cast<double>(m);
    const float4 mean = make_float4(static_cast<float>(s0 / dm), static_cast<float>(s1 / dm),
                                    static_cast<float>(s2 / dm), static_cast<float>(s3 / dm));
    for (int i = 0; i < m; ++i) st_stream(X + static_cast<int64_t>(i) * Ps + col, mean);
}

// Quadratic test objective: exact gradient g = a (x - c), then the same update.
__global__ __launch_bounds__(kThreads) void quad_step_kernel(float* X, float* V, const float* __restrict__ A,
                                                             const float* __restrict__ C, int64_t n4, float lr,
                                                             float beta, float wd) {
    const int64_t j = static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x;
    if (j >= n4) return;
    float4 x = *reinterpret_cast<const float4*>(X + j * 4), v = *reinterpret_cast<const float4*>(V + j * 4);
    const float4 a = *reinterpret_cast<const float4*>(A + j * 4), c = *reinterpret_cast<const float4*>(C + j * 4);
    const float4 g = make_float4(a.x * (x.x - c.x), a.y * (x.y - c.y), a.z * (x.z - c.z), a.w * (x.w - c.w));
    sgd_update4(x, v, g, lr, beta, wd);
    *reinterpret_cast<float4*>(V + j * 4) = v;
    *reinterpret_cast<float4*>(X + j * 4) = x;
}

// partial[block] = sum over the block's columns and all workers of
// 0.5 a (xbar - c)^2, in double, in a fixed order.
__global__ __launch_bounds__(kThreads) void quad_loss_kernel(const float* __restrict__ xbar,
                                                             const float* __restrict__ A,
                                                             const float* __restrict__ C, int m, int64_t P,
                                                             int64_t Ps, double* partial) {
    __shared__ double red[kThreads];
    const int64_t p = static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x;
    double s = 0.0;
    if (p < P) {
        const double xb = static_cast<double>(xbar[p]);
        for (int i = 0; i < m; ++i) {
            const double d = xb - static_cast<double>(C[static_cast<int64_t>(i) * Ps + p]);
            s += 0.5 * static_cast<double>(A[static_cast<int64_t>(i) * Ps + p]) * d * d;
        }
    }
    red[threadIdx.x] = s;
    __syncthreads();
    for (int w = kThreads / 2; w > 0; w >>= 1) {
        if (threadIdx.x < w) red[threadIdx.x] += red[threadIdx.x + w];
        __syncthreads();
    }
    if (threadIdx.x == 0) partial[blockIdx.x] = red[0];
}

inline unsigned blocks_for(int64_t threads) { return static_cast<unsigned>((threads + kThreads - 1) / kThreads); }

}  // namespace

hipError_t launch_average(lc_handle* h, const float* X, float* out_rows, float* out_single) {
    // block momentum belongs to the averaging step proper (some destination for the new model),
    // not to the mean that lc_loss takes of unsynchronised workers
    const bool step = out_rows != nullptr || h->lazy_enabled_step;
    BlockMomentum bm{nullptr, nullptr, 0.f, 0.f, 0.f};
    if (h->bm_on && step) bm = BlockMomentum{h->bm_u, h->bm_xs, h->bm_beta, h->md.lr, 1.f / h->md.lr};
    // a state larger than the caches: chunked reduce (into row 0, or into xbar when the broadcast
    // is deferred), then row-by-row broadcast
    const bool big = static_cast<double>(h->m) * static_cast<double>(h->Ps) * 4.0 > 512.0 * 1024 * 1024;
    // deferred update: the rows are the momentum rows, the common starting model is xbar (which
    // each thread reads before it writes the new mean of the same columns there)
    const DeferredUpdate du{h->defer_x ? h->xbar : nullptr, h->md.lr};
    if (h->defer_x) X = h->V;
    const bool own_rows = X == h->X || h->defer_x;
    // column ranges still to be averaged: everything, minus the weights of the layers that a
    // tile-owner kernel of this tau = 1 iteration has averaged already (multiples of 4 columns)
    int64_t r_lo[LC_MAX_LAYERS + 2], r_hi[LC_MAX_LAYERS + 2];
    int n_r = 0;
    {
        int64_t lo = 0;
        for (int l = 1; l <= h->L && (h->defer_x || h->fuse_avg); ++l) {
            if (!(h->sync_done >> l & 1u)) continue;
            const int64_t w_lo = h->layer[l].w_off, w_hi = h->layer[l].b_off;
            if (w_lo > lo) { r_lo[n_r] = lo; r_hi[n_r] = w_lo; ++n_r; }
            lo = w_hi;
        }
        if (lo < h->Ps) { r_lo[n_r] = lo; r_hi[n_r] = h->Ps; ++n_r; }
    }
    if (step && own_rows && h->m >= 2 && h->avg_two_phase && big) {
        timing_start(h, kTimeAvg);
        const int64_t chunk = h->avg_chunk_floats;
        float* dst = out_rows ? h->X : out_single;
        for (int r = 0; r < n_r; ++r) {
            if (r_hi[r] - r_lo[r] <= 256 * 1024) {
                // a short range (biases, a small last layer): one thread per 16-byte column walks the
                // rows with several loads in flight; the chunked kernel would put it all on one workgroup
                hipLaunchKernelGGL(average_kernel, dim3(blocks_for((r_hi[r] - r_lo[r]) / 4)), dim3(kThreads), 0,
                                   h->stream, X, out_rows, out_single, h->m, h->Ps, bm, du, r_lo[r], r_hi[r]);
                continue;
            }
            for (int64_t lo = r_lo[r]; lo < r_hi[r]; lo += chunk) {
                const int64_t hi = lo + chunk < r_hi[r] ? lo + chunk : r_hi[r];
                const int64_t nblk = ((hi - lo) / 4 + kThreads - 1) / kThreads;
                const int64_t nred = (nblk + kReduceCols - 1) / kReduceCols;
                if (du.xb)
                    hipLaunchKernelGGL(reduce_chunk_kernel<true>, dim3(static_cast<unsigned>(nred)), dim3(kThreads), 0,
                                       h->stream, X, dst, h->m, h->Ps, lo, hi, bm, du);
                else
                    hipLaunchKernelGGL(reduce_chunk_kernel<false>, dim3(static_cast<unsigned>(nred)), dim3(kThreads),
                                       0, h->stream, X, dst, h->m, h->Ps, lo, hi, bm, du);
                if (out_rows)
                    hipLaunchKernelGGL(broadcast_chunk_kernel, dim3(static_cast<unsigned>(nblk * (h->m - 1))),
                                       dim3(kThreads), 0, h->stream, h->X, h->X, 1, h->Ps, lo, hi, nblk);
            }
        }
        timing_stop(h, kTimeAvg);
        return hipGetLastError();
    }
    if (step) timing_start(h, kTimeAvg);
    for (int r = 0; r < n_r; ++r)
        hipLaunchKernelGGL(average_kernel, dim3(blocks_for((r_hi[r] - r_lo[r]) / 4)), dim3(kThreads), 0, h->stream, X,
                           out_rows, out_single, h->m, h->Ps, bm, du, r_lo[r], r_hi[r]);
    if (step) timing_stop(h, kTimeAvg);
    return hipGetLastError();
}

namespace {

// Start of a block-momentum run in the static scratch: u = 0, x_sync = row 0 of X, V = 0.
__global__ __launch_bounds__(kThreads) void static_begin_kernel(const float* X, float* V, float* u, float* xs, int m,
                                                                int64_t Ps, int64_t cols) {
    const int64_t col = (static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x) * 4;
    if (col >= cols) return;
    const float4 zero = make_float4(0.f, 0.f, 0.f, 0.f);
    *reinterpret_cast<float4*>(u + col) = zero;
    *reinterpret_cast<float4*>(xs + col) = *reinterpret_cast<const float4*>(X + col);
    if (V)
        for (int i = 0; i < m; ++i) *reinterpret_cast<float4*>(V + static_cast<int64_t>(i) * Ps + col) = zero;
}

__global__ __launch_bounds__(kThreads) void zero_rows_kernel(float* V, int m, int64_t Ps, int64_t cols) {
    const int64_t col = (static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x) * 4;
    if (col >= cols) return;
    for (int i = 0; i < m; ++i)
        *reinterpret_cast<float4*>(V + static_cast<int64_t>(i) * Ps + col) = make_float4(0.f, 0.f, 0.f, 0.f);
}

constexpr int kMaxDevices = 64;
std::mutex g_static_mu;
float* g_static_ptr[kMaxDevices];   // device address of `scratch` on each device, once looked up

// Device address of the static scratch on the current device (each GPU holds its own copy).
int static_scratch(float** out) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return LC_ERR_HIP;
    std::lock_guard<std::mutex> lock(g_static_mu);
    if (!g_static_ptr[dev]) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return LC_ERR_HIP;
        g_static_ptr[dev] = static_cast<float*>(p);
    }
    *out = g_static_ptr[dev];
    return LC_OK;
}

}  // namespace

hipError_t launch_broadcast_xbar(lc_handle* h) {
    const int64_t chunk = h->avg_chunk_floats;
    for (int64_t lo = 0; lo < h->Ps; lo += chunk) {
        const int64_t hi = lo + chunk < h->Ps ? lo + chunk : h->Ps;
        const int64_t nblk = ((hi - lo) / 4 + kThreads - 1) / kThreads;
        hipLaunchKernelGGL(broadcast_chunk_kernel, dim3(static_cast<unsigned>(nblk * h->m)), dim3(kThreads), 0,
                           h->stream, h->xbar, h->X, 0, h->Ps, lo, hi, nblk);
    }
    return hipGetLastError();
}

hipError_t launch_update_from_grad(lc_handle* h) {
    const int64_t n4 = static_cast<int64_t>(h->m) * h->Ps / 4;
    timing_start(h, kTimeUpd);
    hipLaunchKernelGGL(update_kernel, dim3(blocks_for(n4)), dim3(kThreads), 0, h->stream, h->X, h->V, h->G, n4,
                       h->md.lr, effective_beta(h), h->md.wd);
    timing_stop(h, kTimeUpd);
    return hipGetLastError();
}

hipError_t launch_update_and_average(lc_handle* h) {
    timing_start(h, kTimeUpdAvg);
    hipLaunchKernelGGL(update_average_kernel, dim3(blocks_for(h->Ps / 4)), dim3(kThreads), 0, h->stream, h->X, h->V,
                       h->G, h->m, h->Ps, h->md.lr, effective_beta(h), h->md.wd);
    timing_stop(h, kTimeUpdAvg);
    return hipGetLastError();
}

hipError_t launch_quad_step(lc_handle* h) {
    const int64_t n4 = static_cast<int64_t>(h->m) * h->Ps / 4;
    hipLaunchKernelGGL(quad_step_kernel, dim3(blocks_for(n4)), dim3(kThreads), 0, h->stream, h->X, h->V, h->qa,
                       h->qc, n4, h->md.lr, effective_beta(h), h->md.wd);
    return hipGetLastError();
}

hipError_t launch_quad_loss(lc_handle* h, int* n_partial) {
    const unsigned nb = blocks_for(h->P);
    *n_partial = static_cast<int>(nb);
    hipLaunchKernelGGL(quad_loss_kernel, dim3(nb), dim3(kThreads), 0, h->stream, h->xbar, h->qa, h->qc, h->m, h->P,
                       h->Ps, h->partial);
    return hipGetLastError();
}

}  // namespace lc

extern "C" int lc_average_block_momentum_static(float* X, float* V, int m, int64_t P, int64_t row_stride, float lr,
                                                float beta_glob, int begin, void* stream) {
    using namespace lc;
    if (!X || m < 1 || m > 65535 || P < 1 || row_stride < P || row_stride % 4 != 0) return LC_ERR_ARG;
    if (!(lr > 0.f) || !(beta_glob >= 0.f) || !(beta_glob < 1.f)) return LC_ERR_ARG;
    if (P > LC_STATIC_MAX_PARAMS) return LC_ERR_TOO_LARGE;
    if ((reinterpret_cast<uintptr_t>(X) & 255u) != 0 || (reinterpret_cast<uintptr_t>(V) & 255u) != 0) return LC_ERR_ALIGN;
    float* base = nullptr;
    const int rc = static_scratch(&base);
    if (rc != LC_OK) return rc;
    float* u = base;
    float* xs = base + LC_STATIC_MAX_PARAMS;
    const int64_t cols = round_up(P, 4);   // (<= row_stride, and <= LC_STATIC_MAX_PARAMS, a multiple of 4)
    hipStream_t st = static_cast<hipStream_t>(stream);
    const dim3 grid(blocks_for(cols / 4)), block(kThreads);
    if (begin) {
        hipLaunchKernelGGL(static_begin_kernel, grid, block, 0, st, X, V, u, xs, m, row_stride, cols);
    } else {
        const BlockMomentum bm{u, xs, beta_glob, lr, 1.f / lr};
        const DeferredUpdate du{nullptr, lr};
        hipLaunchKernelGGL(average_kernel, grid, block, 0, st, X, X, static_cast<float*>(nullptr), m, row_stride, bm,
                           du, static_cast<int64_t>(0), cols);
        if (V) hipLaunchKernelGGL(zero_rows_kernel, grid, block, 0, st, V, m, row_stride, cols);
    }
    return hipGetLastError() == hipSuccess ? LC_OK : LC_ERR_HIP;
}
