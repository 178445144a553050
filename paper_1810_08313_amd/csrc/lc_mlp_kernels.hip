// The local SGD step of every replica (Sec. 2, mini-batch SGD inside PASGD) as
// grouped per-replica matrix products on the gfx950 matrix cores:
//
//   gather   : mini-batch selection by the integer index stream + row gather
//   forward  : Z_l = A_{l-1} W_l + b_l, A_l = ReLU(Z_l)
//   softmax  : cross-entropy loss and dZ_L = (p - onehot) / B
//   backward : dW_l = A_{l-1}^T dZ_l, db_l, dZ_{l-1} = (dZ_l W_l^T) .* [A_{l-1} > 0]
//              with the momentum-SGD update applied to the dW tile while it is
//              still in registers (the gradient never reaches memory)
//
// Weights are private to a replica and reused only B times per product, so the
// step is bound by streaming W and V through HBM, not by the matrix cores.  The
// kernels are therefore organised around the weight stream: each wavefront owns
// a slab of W, reads it exactly once per kernel with 16-byte loads straight into
// the MFMA operand/accumulator register layout, and activations (small, shared
// by all wavefronts of a replica) are kept in memory in BOTH batch-major and
// feature-major form, zero padded, so that every MFMA operand is one aligned
// 16-byte load with no bounds checks.
//
// MFMA shapes: v_mfma_f32_16x16x32_bf16 (bf16 operands) and v_mfma_f32_16x16x4_f32
// (fp32 operands).  With l = lane, an A operand lane holds row (l & 15) and a B
// operand lane holds column (l & 15); both hold the reduction indices
// 8 (l >> 4) .. 8 (l >> 4) + 7 of a 32-wide step (one bf16 instruction, or eight
// fp32 instructions taking one element each; the order inside the step does not
// matter because both operands use the same one).  The 16x16 result has row
// 4 (l >> 4) + r in register r and column (l & 15).
//
// Column trick: a wavefront covers 64 columns of W as four 16-column MFMA tiles,
// but tile t, lane column j stands for memory column c0 + 4 j + t.  A lane's four
// tiles are then four consecutive floats of one row of W: one float4.
#include "lc_internal.h"
#include "lc_mma.h"

namespace lc {

namespace {

// ----------------------------------------------------------------- index hash

__device__ __forceinline__ uint64_t mix64(uint64_t z) {
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ULL;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBULL;
    return z ^ (z >> 31);
}
__device__ __forceinline__ int64_t batch_index(uint64_t seed, int i, int64_t k, int b, int64_t N) {
    const uint64_t gamma = 0x9E3779B97F4A7C15ULL;
    uint64_t hsh = mix64(seed + gamma * (static_cast<uint64_t>(k) + 1));
    hsh = mix64(hsh + gamma * (static_cast<uint64_t>(i) + 1));
    hsh = mix64(hsh + gamma * (static_cast<uint64_t>(b) + 1));
    return static_cast<int64_t>(hsh % static_cast<uint64_t>(N));
}

// Partition sampler: bijection of [0, n) by a 4-round balanced Feistel network on 2w bits with
// cycle walking.  The network permutes its 2w-bit domain, so a walk that starts below n returns
// below n after finitely many rounds (fewer than four on average, as the domain is < 4 n).
__device__ __forceinline__ uint64_t feistel_permute(uint64_t x, uint64_t n, uint64_t key) {
    int w = 1;
    while ((1ULL << (2 * w)) < n) ++w;
    const uint64_t mask = (1ULL << w) - 1;
    const uint64_t gamma = 0x9E3779B97F4A7C15ULL;
    do {
        uint64_t l = x >> w, r = x & mask;
#pragma unroll
        for (int round = 0; round < 4; ++round) {
            const uint64_t f = mix64(key + gamma * static_cast<uint64_t>(round + 1) + r) & mask;
            const uint64_t t = l ^ f;
            l = r;
            r = t;
        }
        x = (l << w) | r;
    } while (x >= n);
    return x;
}
__device__ __forceinline__ int64_t partition_index(uint64_t seed, int i, int64_t k, int b, int64_t N, int m, int B) {
    const int64_t lo = static_cast<int64_t>(i) * N / m, hi = static_cast<int64_t>(i + 1) * N / m;
    const int64_t S = (N / m) / B;   // >= 1, checked by lc_init
    const int64_t epoch = k / S, pos = (k % S) * B + b;
    const uint64_t gamma = 0x9E3779B97F4A7C15ULL;
    uint64_t key = mix64(seed + gamma * (static_cast<uint64_t>(epoch) + 1));
    key = mix64(key + gamma * (static_cast<uint64_t>(i) + 1));
    return lo + static_cast<int64_t>(feistel_permute(static_cast<uint64_t>(pos), static_cast<uint64_t>(hi - lo), key));
}

// --------------------------------------------------------------------- gather

struct GatherArgs {
    const void* data;       // [N][d0] of DT
    const int32_t* labels;  // [N]
    void* a_bm;             // [G][Bp][dp0] of OT
    void* a_fm;             // [G][dp0][Bp] of OT or null
    int32_t* lab_out;       // [G][Bp]
    int32_t* idx_out;       // [G][Bp]
    int d0, dp0, B, Bp;
    int64_t N;
    uint64_t seed;
    int64_t k;              // training: local iteration; evaluation: first sample of the pass
    int64_t limit;          // evaluation: samples >= limit are invalid
    int eval;
    int sampler, m;         // training: lc_sampler and the number of workers
    int G;                  // groups per step; blockIdx.z = step * G + group
    int64_t a_slot, lab_slot;  // elements between the buffers of consecutive steps
};

// One block copies a 32-sample x 64-feature tile through LDS and writes it in
// both layouts.  grid = (dp0/64, Bp/32, G * steps): one launch prepares the
// mini-batches of several consecutive local iterations.
template <typename DT, typename OT>
__global__ __launch_bounds__(256) void gather_kernel(GatherArgs a) {
    __shared__ float tile[32][65];
    __shared__ int64_t rows[32];
    const int g = blockIdx.z % a.G, step = blockIdx.z / a.G;
    const int b0 = blockIdx.y * 32, k0 = blockIdx.x * 64;
    const int t = threadIdx.x;
    if (t < 32) {
        const int b = b0 + t;
        int64_t idx = -1;
        if (b < a.B) {
            if (a.eval) {
                idx = a.k + static_cast<int64_t>(g) * a.B + b;
                if (idx >= a.limit) idx = -1;
            } else {
                idx = a.sampler ? partition_index(a.seed, g, a.k + step, b, a.N, a.m, a.B)
                                : batch_index(a.seed, g, a.k + step, b, a.N);
            }
        }
        rows[t] = idx;
        if (blockIdx.x == 0) {
            const int64_t o = step * a.lab_slot + static_cast<int64_t>(g) * a.Bp + b;
            a.idx_out[o] = static_cast<int32_t>(idx);
            a.lab_out[o] = idx >= 0 ? a.labels[idx] : -1;
        }
    }
    __syncthreads();
    const DT* data = static_cast<const DT*>(a.data);
    // every thread moves 8 consecutive values: one vector load where the row piece is whole and
    // aligned (d0 a multiple of 8), one vector store per layout (the padded widths are multiples
    // of 64 and 32; padding positions receive the zeros they must hold anyway)
    {
        const int r = t >> 3, seg = (t & 7) * 8;
        const int64_t idx = rows[r];
        const int kk0 = k0 + seg;
        float x[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        if (idx >= 0) {
            if (a.d0 % 8 == 0 && kk0 + 8 <= a.d0) {
                const Frag<DT> f = load8(data + idx * a.d0 + kk0);
#pragma unroll
                for (int e = 0; e < 8; ++e) x[e] = to_f32(f.v[e]);
            } else {
#pragma unroll
                for (int e = 0; e < 8; ++e)
                    if (kk0 + e < a.d0) x[e] = to_f32(data[idx * a.d0 + kk0 + e]);
            }
        }
#pragma unroll
        for (int e = 0; e < 8; ++e) tile[r][seg + e] = x[e];
        OT* bm = static_cast<OT*>(a.a_bm) + step * a.a_slot + static_cast<int64_t>(g) * a.Bp * a.dp0;
        store8(bm + static_cast<int64_t>(b0 + r) * a.dp0 + kk0, x);
    }
    __syncthreads();
    if (a.a_fm) {
        OT* fm = static_cast<OT*>(a.a_fm) + step * a.a_slot + static_cast<int64_t>(g) * a.dp0 * a.Bp;
        const int kk = t >> 2, seg = (t & 3) * 8;
        float y[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) y[e] = tile[seg + e][kk];
        store8(fm + static_cast<int64_t>(k0 + kk) * a.Bp + b0 + seg, y);
    }
}

// -------------------------------------------------------------------- forward

struct FwdArgs {
    const float* X;       // parameters; replica g at X + g * x_stride
    int64_t x_stride;     // 0: every group uses the same parameters (evaluation)
    int64_t w_off, b_off;
    int d_in, d_out, dp_in, dp_out;
    int B, Bp;
    const void* a_in;     // [G][Bp][dp_in] of OT
    void* out_bm;         // [G][Bp][dp_out] of OT, or fp32 logits when last
    void* out_fm;         // [G][dp_out][Bp] of OT or null
    int last;             // 1: no ReLU, fp32 output
    int vec;              // weight rows may be read with 16-byte loads
    int stream;           // non-temporal weight loads
    int n_chunks;         // column chunks per group
    int m_split;          // workgroups sharing one column chunk, each taking MT batch tiles
    int64_t total_blocks;
    // last layer with all classes in one chunk: softmax cross-entropy in the epilogue
    int fuse_softmax;
    const int32_t* labels;  // [G][Bp], -1 = no sample
    void* dz_bm;            // [G][Bp][dp_out] of OT or null (evaluation)
    void* dz_fm;            // [G][dp_out][Bp] of OT or null
    float* loss;            // [G]
    int eval;               // 1: loss[g] = sum over valid samples; 0: mean over B
    const void* a_in_fm;    // [G][dp_in][Bp] of OT: the same activations feature-major (AFM instances)
    // Steps in which all replicas read one model may hand several replicas' batches to one block as
    // one batch of Bp rows (their batch-major activations lie one after the other): the weight tile
    // then crosses the L2 once per set of replicas instead of once per replica.  Bp is the batch of
    // such a set, fm_Bp the padded batch of ONE replica, by which the feature-major copies are laid
    // out (equal when nothing is grouped).
    int fm_Bp;
    int shared_w;           // > 0: every group reads the same weights from memory (x_stride 0, training step
                            // right after an averaging step) and neighbouring blocks take the same tile of W
                            // for different replicas, in sets of this many replicas (see shared_order), so
                            // that the tile crosses HBM once per set instead of once per replica
};

// One block = one replica x 64 output columns x MT batch tiles of 16 rows; its
// NW wavefronts split the reduction over d_in and combine their partial tiles
// in LDS.  Large models use MT = all batch tiles (every weight is read from
// memory once); small ones split the batch over several blocks to fill the chip.
//
// AFM instances (the block holds the whole padded batch, Bp = 16 MT) read the activations from
// the feature-major copy.  The batch-major read hands each lane of an MFMA operand its 8
// consecutive k of one batch row, so 16 lanes touch 16 different rows and every load
// instruction costs the L1 sixteen cache-line lookups per 16 lanes; at B = 128 that takes about
// as long as streaming the weights and does not overlap with it.  Feature-major, a lane reads 16
// contiguous bytes of row k (VW = 8 bf16 or 4 fp32 batch entries), 16 lanes cover 256
// contiguous bytes, and component t of the 8 vectors (k = 8q .. 8q+7) is the operand of tile t:
// the same trick as for the weight columns.  Tile VW h + t then holds batch rows
// 16 VW h + VW i + t (i = 0..15) instead of 16 mt + i; only the epilogue needs to know.
template <typename OT, int MT, int NW, int PF, int WM, bool AFM>
__global__ __launch_bounds__(NW * 64) void forward_kernel(FwdArgs a) {
    constexpr int VW = 16 / sizeof(OT);
    static_assert(!AFM || MT % VW == 0, "AFM needs whole groups of VW tiles");
    // batch row (within the block) of accumulator row i of tile mt, and the inverse as the
    // row of the LDS tile that holds batch row b
    auto batch_row = [](int mt, int i) { return AFM ? 16 * VW * (mt / VW) + VW * i + mt % VW : 16 * mt + i; };
    auto tile_row = [](int b) {
        return AFM ? 16 * (VW * (b / (16 * VW)) + b % VW) + (b % (16 * VW)) / VW : b;
    };
    static_assert(NW * MT <= 32, "the partial tiles must fit in LDS (139 KB at 32 tiles)");
    __shared__ __attribute__((aligned(16))) float part[NW][MT * 16][kColChunk + 4];   // one partial tile per wavefront
    const int64_t logical = xcd_logical_block(a.total_blocks);
    if (logical < 0) return;
    const int per_group = a.n_chunks * a.m_split;
    int g, rem;
    shared_order(logical, per_group, a.shared_w, g, rem);
    const int c0 = (rem / a.m_split) * kColChunk;
    const int row0 = (rem % a.m_split) * MT * 16;   // first batch row of this block
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int j = lane & 15, q = lane >> 4;

    const float* W = a.X + g * a.x_stride + a.w_off;
    const OT* A = static_cast<const OT*>(a.a_in) + (static_cast<int64_t>(g) * a.Bp + row0) * a.dp_in;
    const bool vec = a.vec != 0;
    const bool narrow = WM == kWGeneric && a.d_out <= 16;   // see load_w_step

    // everything the epilogue needs from memory is requested now, so that it does not add
    // dependent round trips after the reduction (these kernels are latency-bound when small)
    __shared__ float bias_s[kColChunk];
    if (threadIdx.x < kColChunk) {
        const int c = c0 + threadIdx.x;
        bias_s[threadIdx.x] = c < a.d_out ? a.X[g * a.x_stride + a.b_off + c] : 0.f;
    }
    int my_label = -1;
    if (a.fuse_softmax && threadIdx.x < MT * 16) {
        const int b = row0 + batch_row(threadIdx.x / 16, threadIdx.x % 16);
        if (b < a.B) my_label = a.labels[static_cast<int64_t>(g) * a.Bp + b];
    }

    f32x4 acc[MT][4];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int t = 0; t < 4; ++t) acc[mt][t] = f32x4{0.f, 0.f, 0.f, 0.f};

    // The weight rows of the next PF steps are always in flight: the achieved bandwidth of this
    // kernel is (bytes in flight) / (memory latency), and registers are the only place to hold them.
    const int n_steps = a.dp_in / 32;
    auto load_w_step = [&](int s, float4 (&w)[8]) {
        if constexpr (WM == kWGeneric) {
            // (steps past the end are never used: any valid step is read for them)
            const int k0 = (s < n_steps ? s : n_steps - 1) * 32 + 8 * q;
            if (narrow) {
                // at most 16 columns (a classifier's last layer): lane column j stands for column
                // j itself and only the first of the four tiles is used, so a step costs a lane
                // 8 loads instead of 32 of which most lanes would sit out
                float x[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
                if (j < a.d_out) {
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        const int rr = k0 + e < a.d_in ? k0 + e : a.d_in - 1;
                        x[e] = W[static_cast<int64_t>(rr) * a.d_out + j];
                    }
                }
#pragma unroll
                for (int e = 0; e < 8; ++e) w[e] = make_float4(k0 + e < a.d_in ? x[e] : 0.f, 0.f, 0.f, 0.f);
            } else {
#pragma unroll
                for (int e = 0; e < 8; ++e) w[e] = load_w4_rows(W, k0 + e, a.d_in, c0 + 4 * j, a.d_out, vec, false);
            }
        } else {
            // Rows past d_in meet activation columns that are zero, and steps past the end are
            // never used: both are redirected to valid rows instead of being branched around.
            const int k0 = (s < n_steps ? s : n_steps - 1) * 32 + 8 * q;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int row = k0 + e < a.d_in ? k0 + e : a.d_in - 1;
                w[e] = load_wm<WM>(W + static_cast<int64_t>(row) * a.d_out, c0 + 4 * j, a.d_out, vec);
            }
        }
    };
    // Loads retire in issue order, so the activation fragments of step s are requested before the
    // weight rows of the later steps: waiting for them then leaves those rows in flight.
    const OT* AF = static_cast<const OT*>(a.a_in_fm) + static_cast<int64_t>(g) * a.dp_in * a.Bp;
    auto load_a_step = [&](int s, Frag<OT> (&f)[MT]) {
        const int k0 = (s < n_steps ? s : n_steps - 1) * 32 + 8 * q;   // past the end: any valid step, never used
        if constexpr (!AFM) {
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) f[mt] = load8(A + static_cast<int64_t>(16 * mt + j) * a.dp_in + k0);
        } else if constexpr (sizeof(OT) == 4) {
#pragma unroll
            for (int h = 0; h < MT / 4; ++h)
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const float4 x = *reinterpret_cast<const float4*>(AF + static_cast<int64_t>(k0 + e) * a.Bp + 64 * h + 4 * j);
                    f[4 * h + 0].v[e] = x.x; f[4 * h + 1].v[e] = x.y; f[4 * h + 2].v[e] = x.z; f[4 * h + 3].v[e] = x.w;
                }
        } else {
            // the fragments hold the raw vectors until transpose_a_step() runs at the point of use
#pragma unroll
            for (int e = 0; e < 8; ++e) f[e] = load8(AF + static_cast<int64_t>(k0 + e) * a.Bp + 8 * j);
        }
    };
    // bf16 AFM: f[e] holds k = 8q + e for batch entries 8j .. 8j+7; the operand of tile t wants
    // batch entry 8j + t for e = 0..7, an 8 x 8 transpose of 16-bit values inside the lane
    auto transpose_a_step = [&](Frag<OT> (&f)[MT]) {
        if constexpr (AFM && sizeof(OT) == 2) {
            u32x4 x[8], y[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) x[e] = __builtin_bit_cast(u32x4, f[e].v);
#pragma unroll
            for (int t = 0; t < 8; ++t)
#pragma unroll
                for (int d = 0; d < 4; ++d)   // dword d of tile t: (k = 2d, k = 2d + 1)
                    y[t][d] = __builtin_amdgcn_perm(x[2 * d + 1][t / 2], x[2 * d][t / 2],
                                                    (t & 1) ? 0x07060302u : 0x05040100u);
#pragma unroll
            for (int t = 0; t < 8; ++t) f[t].v = __builtin_bit_cast(bf16x8, y[t]);
        }
    };
    // The queue is addressed with compile-time indices (the loop body covers PF + 1 steps), so a
    // register that a load is still filling is never copied.
    static_assert((PF + 1) % 2 == 0, "the activation double buffer needs an even trip count");
    float4 wq[PF + 1][8];
    Frag<OT> af[2][MT];
    auto multiply_step = [&](Frag<OT> (&f)[MT], float4 (&w)[8]) {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) consume_here(f[mt]);
#pragma unroll
        for (int e = 0; e < 8; ++e) consume_here(w[e]);
        transpose_a_step(f);
        Frag<OT> bf;
        float x[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) x[e] = w[e].x;
        pack8(bf, x);
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) acc[mt][0] = mma8(f[mt], bf, acc[mt][0]);
#pragma unroll
        for (int e = 0; e < 8; ++e) x[e] = w[e].y;
        pack8(bf, x);
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) acc[mt][1] = mma8(f[mt], bf, acc[mt][1]);
#pragma unroll
        for (int e = 0; e < 8; ++e) x[e] = w[e].z;
        pack8(bf, x);
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) acc[mt][2] = mma8(f[mt], bf, acc[mt][2]);
#pragma unroll
        for (int e = 0; e < 8; ++e) x[e] = w[e].w;
        pack8(bf, x);
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) acc[mt][3] = mma8(f[mt], bf, acc[mt][3]);
    };
    load_a_step(wave, af[0]);
#pragma unroll
    for (int p = 0; p < PF; ++p) load_w_step(wave + p * NW, wq[p]);
    // Full groups of PF + 1 steps run without control flow (a branch inside would make the
    // compiler drain all outstanding loads where the paths meet); the last few steps, whose
    // weight rows are already in the queue, follow separately.
    int s0 = wave;
    for (; s0 + PF * NW < n_steps; s0 += NW * (PF + 1)) {
#pragma unroll
        for (int u = 0; u <= PF; ++u) {
            const int s = s0 + u * NW;
            load_a_step(s + NW, af[(u + 1) & 1]);
            load_w_step(s + PF * NW, wq[(u + PF) % (PF + 1)]);
            multiply_step(af[u & 1], wq[u]);
            __builtin_amdgcn_sched_barrier(0);   // keep the next step's loads below this step's products
        }
    }
#pragma unroll
    for (int u = 0; u < PF; ++u) {
        const int s = s0 + u * NW;
        if (s < n_steps) {   // uniform over the wavefront
            load_a_step(s + NW, af[(u + 1) & 1]);
            multiply_step(af[u & 1], wq[u]);
        }
    }

    // combine the wavefronts' partial tiles: every wavefront parks its own, then all threads add
    // them up in wavefront order (the order fixes the rounding) into the first one
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            if (narrow) {   // column j in place j; places 16.. of the tile are not used in this mode
                part[wave][16 * mt + 4 * q + r][j] = acc[mt][0][r];
            } else {
                *reinterpret_cast<float4*>(&part[wave][16 * mt + 4 * q + r][4 * j]) =
                    make_float4(acc[mt][0][r], acc[mt][1][r], acc[mt][2][r], acc[mt][3][r]);
            }
        }
    __syncthreads();
    for (int f = threadIdx.x; f < MT * 16 * (kColChunk / 4); f += NW * 64) {
        const int row = f / (kColChunk / 4), c4 = (f % (kColChunk / 4)) * 4;
        float4 v = *reinterpret_cast<const float4*>(&part[0][row][c4]);
#pragma unroll
        for (int w = 1; w < NW; ++w) {
            const float4 o = *reinterpret_cast<const float4*>(&part[w][row][c4]);
            v.x = o.x + v.x; v.y = o.y + v.y; v.z = o.z + v.z; v.w = o.w + v.w;
        }
        *reinterpret_cast<float4*>(&part[0][row][c4]) = v;
    }
    __syncthreads();
    float (&red)[MT * 16][kColChunk + 4] = part[0];

    // epilogue: bias, ReLU, both layouts; only valid (b, c) are written so the
    // zero padding of the activation buffers is preserved
    const int nthr = NW * 64;
    if (a.last) {
        float* out = static_cast<float*>(a.out_bm) + static_cast<int64_t>(g) * a.Bp * a.dp_out;
        for (int e = threadIdx.x; e < MT * 16 * kColChunk; e += nthr) {
            const int bl = e / kColChunk, b = row0 + batch_row(bl / 16, bl % 16), c = c0 + e % kColChunk;
            if (b < a.B && c < a.d_out) {
                const float z = red[bl][e % kColChunk] + bias_s[e % kColChunk];
                out[static_cast<int64_t>(b) * a.dp_out + c] = z;
                red[bl][e % kColChunk] = z;
            }
        }
        if (a.fuse_softmax) {
            // all classes of a sample sit in this block's tile: loss and dZ_L here, for the
            // block's own samples; the loss is left as one partial sum per block
            __shared__ float lred[128];
            __syncthreads();
            const int t = threadIdx.x;
            float nll = 0.f;
            if (t < 128) {
                const int b = row0 + batch_row(t / 16, t % 16);
                if (t < MT * 16 && b < a.B && my_label >= 0) {
                    const int y = my_label;
                    const float* z = red[t];
                    float zmax = z[0];
                    for (int c = 1; c < a.d_out; ++c) zmax = fmaxf(zmax, z[c]);
                    float s_other = 0.f;
                    for (int c = 0; c < a.d_out; ++c) s_other += c == y ? 0.f : expf(z[c] - zmax);
                    const float e_y = expf(z[y] - zmax);
                    nll = xent_loss(s_other, e_y, z[y] - zmax);
                    if (a.dz_bm) {
                        OT* dbm = static_cast<OT*>(a.dz_bm) + (static_cast<int64_t>(g) * a.Bp + b) * a.dp_out;
                        OT* dfm = static_cast<OT*>(a.dz_fm) + static_cast<int64_t>(g) * a.dp_out * a.Bp + b;
                        const float inv = 1.f / (s_other + e_y), invB = 1.f / static_cast<float>(a.B);
                        for (int c = 0; c < a.d_out; ++c) {
                            const OT d = static_cast<OT>(xent_delta(expf(z[c] - zmax), c == y, s_other, inv) * invB);
                            dbm[c] = d;
                            dfm[static_cast<int64_t>(c) * a.Bp] = d;
                        }
                    }
                }
                lred[t] = nll;
            }
            __syncthreads();
            for (int w = 64; w > 0; w >>= 1) {
                if (t < w) lred[t] += lred[t + w];
                __syncthreads();
            }
            if (t == 0)
                a.loss[static_cast<int64_t>(g) * kLossParts + rem % a.m_split] =
                    a.eval ? lred[0] : lred[0] / static_cast<float>(a.B);
        }
    } else {
        // 8 outputs per thread and pass, stored as one vector where all 8 are valid: along the
        // columns for the batch-major copy, along the batch for the feature-major one
        OT* obm = static_cast<OT*>(a.out_bm) + static_cast<int64_t>(g) * a.Bp * a.dp_out;
        for (int e = threadIdx.x; e < MT * 16 * (kColChunk / 8); e += nthr) {
            const int bl = e / (kColChunk / 8), cl = (e % (kColChunk / 8)) * 8;
            const int b = row0 + batch_row(bl / 16, bl % 16), c = c0 + cl;
            if (b >= a.B || c >= a.d_out) continue;
            const float4 z0 = *reinterpret_cast<const float4*>(&red[bl][cl]);
            const float4 z1 = *reinterpret_cast<const float4*>(&red[bl][cl + 4]);
            float y[8] = {z0.x, z0.y, z0.z, z0.w, z1.x, z1.y, z1.z, z1.w};
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                y[i] += bias_s[cl + i];
                y[i] = y[i] > 0.f ? y[i] : 0.f;
            }
            OT* dst = obm + static_cast<int64_t>(b) * a.dp_out + c;
            if (c + 8 <= a.d_out) {
                store8(dst, y);
            } else {
                for (int i = 0; c + i < a.d_out; ++i) dst[i] = static_cast<OT>(y[i]);
            }
        }
        if (a.out_fm) {
            OT* ofm = static_cast<OT*>(a.out_fm) + static_cast<int64_t>(g) * a.dp_out * a.Bp;
            for (int e = threadIdx.x; e < MT * 16 * (kColChunk / 8); e += nthr) {
                const int cl = e / (MT * 2), bl = (e % (MT * 2)) * 8;
                const int b = row0 + bl, c = c0 + cl;
                if (b >= a.B || c >= a.d_out) continue;
                if (a.fm_Bp != a.Bp) {
                    // several replicas' batches in this block (all rows valid, see launch_forward): the
                    // 8 entries belong to replica b / fm_Bp of the set, whose copy has rows of fm_Bp
                    float y[8];
#pragma unroll
                    for (int i = 0; i < 8; ++i) {
                        const float z = red[tile_row(bl + i)][cl] + bias_s[cl];
                        y[i] = z > 0.f ? z : 0.f;
                    }
                    store8(ofm + (static_cast<int64_t>(b / a.fm_Bp) * a.dp_out + c) * a.fm_Bp + b % a.fm_Bp, y);
                    continue;
                }
                float y[8];
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    const float z = red[tile_row(bl + i)][cl] + bias_s[cl];
                    y[i] = z > 0.f ? z : 0.f;
                }
                OT* dst = ofm + static_cast<int64_t>(c) * a.Bp + b;
                if (b + 8 <= a.B) {
                    store8(dst, y);
                } else {
                    for (int i = 0; b + i < a.B; ++i) dst[i] = static_cast<OT>(y[i]);
                }
            }
        }
    }
}

// -------------------------------------------------------------------- softmax

struct SoftmaxArgs {
    const float* logits;    // [G][Bp][dpL]
    const int32_t* labels;  // [G][Bp], -1 = no sample
    void* dz_bm;            // [G][Bp][dpL] of OT or null (evaluation)
    void* dz_fm;            // [G][dpL][Bp] of OT or null
    float* loss;            // [G]
    int C, dpL, B, Bp;
    int eval;               // 1: loss[g] = sum over valid samples; 0: mean over B
};

// One block per group, one thread per sample.
template <typename OT>
__global__ __launch_bounds__(128) void softmax_kernel(SoftmaxArgs a) {
    __shared__ float red[128];
    const int g = blockIdx.x, b = threadIdx.x;
    float nll = 0.f;
    if (b < a.B) {
        const int y = a.labels[static_cast<int64_t>(g) * a.Bp + b];
        if (y >= 0) {
            const float* z = a.logits + (static_cast<int64_t>(g) * a.Bp + b) * a.dpL;
            float zmax = z[0];
            for (int c = 1; c < a.C; ++c) zmax = fmaxf(zmax, z[c]);
            float s_other = 0.f;
            for (int c = 0; c < a.C; ++c) s_other += c == y ? 0.f : expf(z[c] - zmax);
            const float e_y = expf(z[y] - zmax);
            nll = xent_loss(s_other, e_y, z[y] - zmax);
            if (a.dz_bm) {
                OT* dbm = static_cast<OT*>(a.dz_bm) + (static_cast<int64_t>(g) * a.Bp + b) * a.dpL;
                OT* dfm = static_cast<OT*>(a.dz_fm) + static_cast<int64_t>(g) * a.dpL * a.Bp + b;
                const float inv = 1.f / (s_other + e_y), invB = 1.f / static_cast<float>(a.B);
                for (int c = 0; c < a.C; ++c) {
                    const OT d = static_cast<OT>(xent_delta(expf(z[c] - zmax), c == y, s_other, inv) * invB);
                    dbm[c] = d;
                    dfm[static_cast<int64_t>(c) * a.Bp] = d;
                }
            }
        }
    }
    red[b] = nll;
    __syncthreads();
    for (int w = 64; w > 0; w >>= 1) {
        if (b < w) red[b] += red[b + w];
        __syncthreads();
    }
    if (b == 0) a.loss[static_cast<int64_t>(g) * kLossParts] = a.eval ? red[0] : red[0] / static_cast<float>(a.B);
}

// ------------------------------------------------------------------- backward

struct BwdArgs {
    float* X;            // where the new parameters are written (rows of stride x_stride)
    float* V;            // where the new momentum is written, or null: implicit momentum (see Aux)
    int64_t x_stride;
    const float* Xr;     // where the weights are READ: X itself, or the single averaged model that all
    int64_t xr_stride;   // replicas share right after a lazy averaging step (stride 0), or the other row buffer
    // Second operand of the update.  imp_in == 0: the momentum rows v.  imp_in != 0: the parameters of
    // ONE STEP EARLIER, x_prev, from which the momentum is recovered as (x_prev - x) / lr -- the update
    // x = x_prev - lr v read backwards.  Inside a period the buffer that held v then holds the newer of
    // two consecutive models instead, and a step reads 8 and writes 4 bytes per parameter.
    const float* Aux;
    int64_t aux_stride;
    int imp_in;
    float inv_lr;
    int64_t w_off, b_off;
    int d_in, d_out, dp_in, dp_out;
    int B, Bp;
    const void* a_bm;    // A_{l-1} batch-major   [G][Bp][dp_in]  (unused here)
    const void* a_fm;    // A_{l-1} feature-major [G][dp_in][Bp]
    const void* dz_bm;   // dZ_l batch-major      [G][Bp][dp_out]
    const void* dz_fm;   // dZ_l feature-major    [G][dp_out][Bp]
    void* dzp_bm;        // dZ_{l-1} batch-major  [G][Bp][dp_in]  or null (layer 1)
    void* dzp_fm;        // dZ_{l-1} feature-major[G][dp_in][Bp]
    float lr, beta, wd;
    int vec;
    int stream;          // non-temporal weight loads and stores
    int n_row_blocks;    // row blocks per group (64 rows each)
    int col_split;       // workgroups sharing one row block's columns (1 when dA is needed)
    int shared_w;        // > 0: all replicas read the same weights (xr_stride 0) and neighbouring blocks take
                         // the same rows of W for different replicas, in sets of this many (see FwdArgs)
    int fm_Bp;           // DAO instances: padded batch of ONE replica when a block takes the batches of several
                         // (see FwdArgs::fm_Bp); the feature-major buffers are laid out by it.  Else = Bp
    int skip_x;          // V is updated, X is left unwritten: the averaging step that follows forms
                         // every replica's new weights from Xr and V itself (tau = 1, deferred update)
    int64_t total_blocks;
};

// One workgroup (4 wavefronts) owns 64 rows of W_l and V_l of one replica, 16
// rows per wavefront, and walks along them 64 columns per trip.  Per trip
//   (0) the 64-column slice of dZ_l is staged once per workgroup in LDS, in
//       both layouts, from loads that were issued one trip ahead;
//   (1) each wavefront holds its W and V tiles (also loaded one trip ahead,
//       float4 per lane, straight into the MFMA accumulator layout);
//   (2) the dW tile is formed with MFMA over the batch;
//   (3) the *old* W tile is parked in LDS, re-read in operand layout and its
//       contribution to dA_{l-1} accumulated (the chain rule needs the weights
//       of before the update);
//   (4) v <- beta v + dW + wd w, w <- w - lr v, both tiles stored.
// W and V cross HBM exactly once in each direction; the gradient never exists
// in memory; dA is complete when the wavefront has walked its rows, so nothing
// is reduced across workgroups.  When dA is not needed (first layer) the
// columns may additionally be split over several workgroups.
// DAO instances (tau = 1, layers whose update and averaging a tile-owner kernel does afterwards)
// form dZ_{l-1} only: the same walk over W_l without V, dW, the update or any store to X and V.
template <typename OT, int NT, int WM, bool DAO = false>
__global__ __launch_bounds__(256) void backward_kernel(BwdArgs a) {
    constexpr int kPad = sizeof(OT) == 2 ? 8 : 4;
    constexpr int Bp = 16 * NT;
    constexpr int NS = NT / 2;                 // 32-wide steps over the batch; also staging pieces per thread
    // dZ^T slice: row (c % 4) * 16 + c / 4 holds column c0 + c, so that the 16 lanes
    // of a B-operand read (columns 4 j + t) hit 16 consecutive LDS rows
    __shared__ __attribute__((aligned(16))) OT dzt_lds[kColChunk][Bp + kPad];
    __shared__ __attribute__((aligned(16))) OT dz_lds[Bp][kColChunk + kPad];
    __shared__ __attribute__((aligned(16))) OT wlds[4][kRowsPerWave][kColChunk + kPad];

    const int64_t logical = xcd_logical_block(a.total_blocks);
    if (logical < 0) return;
    const int per_group = a.n_row_blocks * a.col_split;
    int g, rem;
    shared_order(logical, per_group, a.shared_w, g, rem);
    const int rb = rem / a.col_split, cs = rem % a.col_split;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int j = lane & 15, q = lane >> 4;
    const int k0 = (rb * 4 + wave) * kRowsPerWave;   // < dp_in: the grid covers dp_in / 64 row blocks exactly
    const bool vec = a.vec != 0;
    const bool need_da = a.dzp_bm != nullptr;

    float* W = a.X + g * a.x_stride + a.w_off;
    const float* Wr = a.Xr + g * a.xr_stride + a.w_off;
    float* Vw = a.V ? a.V + g * a.x_stride + a.w_off : nullptr;
    const float* Va = DAO ? nullptr : a.Aux + g * a.aux_stride + a.w_off;
    const OT* AT = static_cast<const OT*>(a.a_fm) + static_cast<int64_t>(g) * a.dp_in * Bp;
    const OT* dZ = static_cast<const OT*>(a.dz_bm) + static_cast<int64_t>(g) * Bp * a.dp_out;
    const OT* dZT = static_cast<const OT*>(a.dz_fm) + static_cast<int64_t>(g) * a.dp_out * Bp;

    // column chunks of this workgroup
    const int n_cc = (a.d_out + kColChunk - 1) / kColChunk;
    const int cc_per = (n_cc + a.col_split - 1) / a.col_split;
    const int cc_lo = cs * cc_per;
    const int cc_hi = cc_lo + cc_per < n_cc ? cc_lo + cc_per : n_cc;
    if (cc_lo >= cc_hi) return;   // uniform over the workgroup
    // Workgroups advance through their columns at about the same pace; if all of
    // them started at column 0 the rows they touch at any moment would differ by
    // multiples of 16 * d_out * 4 bytes and pile onto the same memory channels.
    // Each workgroup therefore starts its walk at a different chunk and wraps.
    const int cc_n = cc_hi - cc_lo;
    const int cc_shift = static_cast<int>((logical * 7) % cc_n);
    auto chunk_at = [&](int i) {   // i-th chunk of this workgroup's walk
        int c = i + cc_shift;
        if (c >= cc_n) c -= cc_n;
        return cc_lo + c;
    };

    f32x4 dacc[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) dacc[nt] = f32x4{0.f, 0.f, 0.f, 0.f};

    // this lane's A operands for the dW product: row k0 + j of A_{l-1}^T, all batch steps
    Frag<OT> af[NS];
    if constexpr (!DAO) {
#pragma unroll
        for (int s = 0; s < NS; ++s) af[s] = load8(AT + static_cast<int64_t>(k0 + j) * Bp + 32 * s + 8 * q);
    }

    // ReLU gates of this lane's dA entries, fetched now (one bit each) instead of after the walk
    // (DAO instances may hold several replicas' batches: entry b of the block is entry b % fm_Bp of
    // replica b / fm_Bp of the set, and every replica's feature-major copy has rows of fm_Bp)
    auto fm_at = [&](int row, int b, int dp) {
        if constexpr (DAO) return (static_cast<int64_t>(b / a.fm_Bp) * dp + row) * a.fm_Bp + b % a.fm_Bp;
        else return static_cast<int64_t>(row) * Bp + b;
    };
    uint32_t gate = 0;
    if (need_da) {
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
#pragma unroll
            for (int r = 0; r < 4; ++r)
                if (to_f32(AT[fm_at(k0 + 4 * q + r, 16 * nt + j, a.dp_in)]) > 0.f) gate |= 1u << (nt * 4 + r);
    }

    float4 w[4], v[4], wn[4], vn[4];
    Frag<OT> st_t[NS], st_b[NS];   // staging registers for the dZ^T and dZ slices

    auto issue_loads = [&](int cc, float4 (&ww)[4], float4 (&vv)[4]) {
        const int c0 = cc * kColChunk;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int row = k0 + 4 * q + r;
            if constexpr (WM == kWGeneric) {
                ww[r] = load_w4_rows(Wr, row, a.d_in, c0 + 4 * j, a.d_out, vec, false);
                vv[r] = load_w4_rows(Va, row, a.d_in, c0 + 4 * j, a.d_out, vec, false);
            } else {
                // rows past d_in read the last row instead (no branch between the loads); their
                // weights are zeroed when used and they are never stored
                const int rr = row < a.d_in ? row : a.d_in - 1;
                // (weights that all replicas share are wanted in the L2 by the neighbouring blocks)
                if (WM == kWVectorStream && a.shared_w)
                    ww[r] = load_wm<kWVector>(Wr + static_cast<int64_t>(rr) * a.d_out, c0 + 4 * j, a.d_out, vec);
                else
                    ww[r] = load_wm<WM>(Wr + static_cast<int64_t>(rr) * a.d_out, c0 + 4 * j, a.d_out, vec);
                if constexpr (!DAO) vv[r] = load_wm<WM>(Va + static_cast<int64_t>(rr) * a.d_out, c0 + 4 * j, a.d_out, vec);
            }
        }
        if constexpr (!DAO) {
            // the dZ^T slice is one contiguous run of 64 * Bp elements
            const OT* src_t = dZT + static_cast<int64_t>(c0) * Bp;
#pragma unroll
            for (int s = 0; s < NS; ++s) st_t[s] = load8(src_t + static_cast<int64_t>(tid + 256 * s) * 8);
        }
        if (need_da) {
#pragma unroll
            for (int s = 0; s < NS; ++s) {
                const int p = tid + 256 * s;
                st_b[s] = load8(dZ + static_cast<int64_t>(p >> 3) * a.dp_out + c0 + (p & 7) * 8);
            }
        }
    };
    auto stage_to_lds = [&]() {
        if constexpr (!DAO) {
#pragma unroll
            for (int s = 0; s < NS; ++s) {
                const int p = tid + 256 * s;
                const int c = p / (Bp / 8), seg = p % (Bp / 8);
                *reinterpret_cast<Frag<OT>*>(&dzt_lds[(c & 3) * 16 + (c >> 2)][seg * 8]) = st_t[s];
            }
        }
        if (need_da) {
#pragma unroll
            for (int s = 0; s < NS; ++s) {
                const int p = tid + 256 * s;
                *reinterpret_cast<Frag<OT>*>(&dz_lds[p >> 3][(p & 7) * 8]) = st_b[s];
            }
        }
    };

    issue_loads(chunk_at(0), w, v);
    stage_to_lds();
    __syncthreads();

    for (int i = 0; i < cc_n; ++i) {
        const int c0 = chunk_at(i) * kColChunk;
        const bool has_next = i + 1 < cc_n;
        if (has_next) issue_loads(chunk_at(i + 1), wn, vn);

        // bias of these 64 columns: db_l = sum_b dZ_l from the staged slice, then the same update
        // (one thread per column).  Every row block of the replica walks this chunk; the job goes
        // to them in turn, so that no workgroup carries it on all of its trips and finishes late.
        if (!DAO && rb == chunk_at(i) % a.n_row_blocks && tid < kColChunk && c0 + tid < a.d_out) {
            float* bx = a.X + g * a.x_stride + a.b_off + c0 + tid;
            const float x = a.Xr[g * a.xr_stride + a.b_off + c0 + tid];   // requested before the sum below
            float v0 = a.Aux[g * a.aux_stride + a.b_off + c0 + tid];
            if (a.imp_in) v0 = (v0 - x) * a.inv_lr;
            const OT* zr = dzt_lds[(tid & 3) * 16 + (tid >> 2)];
            float sb = 0.f;   // (batch entries beyond B are zeros; the order of the sum is the batch order)
#pragma unroll
            for (int b8 = 0; b8 < Bp; b8 += 8) {
                const Frag<OT> f = *reinterpret_cast<const Frag<OT>*>(zr + b8);
#pragma unroll
                for (int e = 0; e < 8; ++e) sb += to_f32(f.v[e]);
            }
            const float vb = momentum_update(a.beta, v0, sb, a.wd, x);
            if (a.V) a.V[g * a.x_stride + a.b_off + c0 + tid] = vb;
            if (!a.skip_x) *bx = weight_update(x, a.lr, vb);
        }
        // dW tile: sum over the batch of A^T[k][b] dZ^T[c][b]
        f32x4 acc[4];
        if constexpr (!DAO) {
#pragma unroll
            for (int t = 0; t < 4; ++t) acc[t] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int s = 0; s < NS; ++s) {
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    const Frag<OT> bf = *reinterpret_cast<const Frag<OT>*>(&dzt_lds[t * 16 + j][32 * s + 8 * q]);
                    acc[t] = mma8(af[s], bf, acc[t]);
                }
            }
        }
        if (need_da) {
            // old weights, in operand precision, to LDS in natural column order
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const bool in = WM == kWGeneric || k0 + 4 * q + r < a.d_in;
                store4<OT>(&wlds[wave][4 * q + r][4 * j], in ? w[r].x : 0.f, in ? w[r].y : 0.f, in ? w[r].z : 0.f,
                           in ? w[r].w : 0.f);
            }
        }
        // update and store
#pragma unroll
        for (int r = 0; r < 4 && !DAO; ++r) {
            const int row = k0 + 4 * q + r;
            const float4 gr = make_float4(acc[0][r], acc[1][r], acc[2][r], acc[3][r]);
            if (a.imp_in) {   // the tile holds the parameters of one step earlier: v = (x_prev - x) / lr
                v[r].x = (v[r].x - w[r].x) * a.inv_lr;
                v[r].y = (v[r].y - w[r].y) * a.inv_lr;
                v[r].z = (v[r].z - w[r].z) * a.inv_lr;
                v[r].w = (v[r].w - w[r].w) * a.inv_lr;
            }
            v[r].x = momentum_update(a.beta, v[r].x, gr.x, a.wd, w[r].x);
            v[r].y = momentum_update(a.beta, v[r].y, gr.y, a.wd, w[r].y);
            v[r].z = momentum_update(a.beta, v[r].z, gr.z, a.wd, w[r].z);
            v[r].w = momentum_update(a.beta, v[r].w, gr.w, a.wd, w[r].w);
            w[r].x = weight_update(w[r].x, a.lr, v[r].x);
            w[r].y = weight_update(w[r].y, a.lr, v[r].y);
            w[r].z = weight_update(w[r].z, a.lr, v[r].z);
            w[r].w = weight_update(w[r].w, a.lr, v[r].w);
            if (row < a.d_in) {
                if (Vw) store_wm<WM>(Vw + static_cast<int64_t>(row) * a.d_out, c0 + 4 * j, a.d_out, vec, v[r]);
                if (!a.skip_x) store_wm<WM>(W + static_cast<int64_t>(row) * a.d_out, c0 + 4 * j, a.d_out, vec, w[r]);
            }
        }
        if (need_da) {
            wave_sync_lds();
            // dA^T[k][b] += sum_c W[k][c] dZ[b][c] over this chunk's 64 columns
#pragma unroll
            for (int s = 0; s < 2; ++s) {
                const Frag<OT> wf = *reinterpret_cast<const Frag<OT>*>(&wlds[wave][j][32 * s + 8 * q]);
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) {
                    const Frag<OT> zf = *reinterpret_cast<const Frag<OT>*>(&dz_lds[16 * nt + j][32 * s + 8 * q]);
                    dacc[nt] = mma8(wf, zf, dacc[nt]);
                }
            }
        }
        if (has_next) {
            __syncthreads();   // every wavefront is done with this chunk's LDS tiles
            stage_to_lds();
            __syncthreads();
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                w[r] = wn[r];
                if constexpr (!DAO) v[r] = vn[r];
            }
        }
    }

    if (need_da) {
        // dZ_{l-1} = dA .* [A_{l-1} > 0], both layouts.  Rows beyond d_in and batch
        // entries beyond B come out as exact zeros (zero operands), which is what
        // the padding must hold.
        OT* pbm = static_cast<OT*>(a.dzp_bm) + static_cast<int64_t>(g) * Bp * a.dp_in;
        OT* pfm = static_cast<OT*>(a.dzp_fm) + static_cast<int64_t>(g) * a.dp_in * Bp;
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            const int b = 16 * nt + j;
            float d[4];
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int row = k0 + 4 * q + r;
                d[r] = ((gate >> (nt * 4 + r)) & 1u) ? dacc[nt][r] : 0.f;
                pfm[fm_at(row, b, a.dp_in)] = static_cast<OT>(d[r]);
            }
            store4<OT>(pbm + static_cast<int64_t>(b) * a.dp_in + k0 + 4 * q, d[0], d[1], d[2], d[3]);
        }
    }
}

// ----------------------------------------------------------------------- head
//
// Last layer with all classes inside one 64-column tile (d_L <= 64): forward,
// softmax cross-entropy and the layer's whole backward pass (dW_L, db_L, update,
// dZ_{L-1}) in ONE kernel, one workgroup of 8 wavefronts per replica.  The deltas
// dZ_L never leave LDS.  For very small layers this replaces three launches whose
// cost is dominated by dependent memory round trips, not by work.

struct HeadArgs {
    float* X;
    float* V;
    int64_t x_stride;
    const float* Xr;         // read source of the weights (see BwdArgs)
    int64_t xr_stride;
    int64_t w_off, b_off;
    int d_in, d_out, dp_in, dp_out;
    int B;
    const void* a_bm;        // A_{L-1} batch-major   [G][Bp][dp_in]
    const void* a_fm;        // A_{L-1} feature-major [G][dp_in][Bp]
    const int32_t* labels;   // [G][Bp]
    float* logits;           // [G][Bp][dp_out] fp32
    void* dzp_bm;            // dZ_{L-1} batch-major  or null (single-layer model)
    void* dzp_fm;
    float* loss;             // [G]
    float lr, beta, wd;
    int vec, stream;
};

template <typename OT, int NT>
__global__ __launch_bounds__(512) void head_kernel(HeadArgs a) {
    constexpr int kPad = sizeof(OT) == 2 ? 8 : 4;
    constexpr int Bp = 16 * NT, NS = NT / 2, NW = 8;
    __shared__ float red[Bp][kColChunk + 4];
    __shared__ __attribute__((aligned(16))) OT dzt_lds[kColChunk][Bp + kPad];
    __shared__ __attribute__((aligned(16))) OT dz_lds[Bp][kColChunk + kPad];
    __shared__ __attribute__((aligned(16))) OT wlds[NW][kRowsPerWave][kColChunk + kPad];
    __shared__ float lred[128];

    const int g = blockIdx.x;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int j = lane & 15, q = lane >> 4;
    const bool vec = a.vec != 0, stream = a.stream != 0;
    const bool need_da = a.dzp_bm != nullptr;
    float* W = a.X + g * a.x_stride + a.w_off;
    const float* Wr = a.Xr + g * a.xr_stride + a.w_off;
    float* Vw = a.V + g * a.x_stride + a.w_off;
    const OT* A = static_cast<const OT*>(a.a_bm) + static_cast<int64_t>(g) * Bp * a.dp_in;
    const OT* AT = static_cast<const OT*>(a.a_fm) + static_cast<int64_t>(g) * a.dp_in * Bp;

    // ---- phase 1: logits = A_{L-1} W_L + b_L (reduction over d_in split over the wavefronts)
    {
        f32x4 acc[NT][4];
#pragma unroll
        for (int mt = 0; mt < NT; ++mt)
#pragma unroll
            for (int t = 0; t < 4; ++t) acc[mt][t] = f32x4{0.f, 0.f, 0.f, 0.f};
        const int n_steps = a.dp_in / 32;
        for (int s = wave; s < n_steps; s += NW) {
            const int k0 = s * 32 + 8 * q;
            float4 w[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                w[e] = load_w4_rows(Wr, k0 + e, a.d_in, 4 * j, a.d_out, vec, stream);
            }
            Frag<OT> af[NT];
#pragma unroll
            for (int mt = 0; mt < NT; ++mt) af[mt] = load8(A + static_cast<int64_t>(16 * mt + j) * a.dp_in + k0);
            Frag<OT> bf;
            float x[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) x[e] = w[e].x;
            pack8(bf, x);
#pragma unroll
            for (int mt = 0; mt < NT; ++mt) acc[mt][0] = mma8(af[mt], bf, acc[mt][0]);
#pragma unroll
            for (int e = 0; e < 8; ++e) x[e] = w[e].y;
            pack8(bf, x);
#pragma unroll
            for (int mt = 0; mt < NT; ++mt) acc[mt][1] = mma8(af[mt], bf, acc[mt][1]);
#pragma unroll
            for (int e = 0; e < 8; ++e) x[e] = w[e].z;
            pack8(bf, x);
#pragma unroll
            for (int mt = 0; mt < NT; ++mt) acc[mt][2] = mma8(af[mt], bf, acc[mt][2]);
#pragma unroll
            for (int e = 0; e < 8; ++e) x[e] = w[e].w;
            pack8(bf, x);
#pragma unroll
            for (int mt = 0; mt < NT; ++mt) acc[mt][3] = mma8(af[mt], bf, acc[mt][3]);
        }
        for (int w = 0; w < NW; ++w) {
            if (wave == w) {
#pragma unroll
                for (int mt = 0; mt < NT; ++mt)
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        float4* p = reinterpret_cast<float4*>(&red[16 * mt + 4 * q + r][4 * j]);
                        float4 v = make_float4(acc[mt][0][r], acc[mt][1][r], acc[mt][2][r], acc[mt][3][r]);
                        if (w > 0) {
                            const float4 o = *p;
                            v.x += o.x; v.y += o.y; v.z += o.z; v.w += o.w;
                        }
                        *p = v;
                    }
            }
            __syncthreads();
        }
    }
    // bias; logits to memory; clear the delta tiles (entries beyond B and d_out must be zero)
    {
        const float* bias = a.Xr + g * a.xr_stride + a.b_off;
        float* out = a.logits + static_cast<int64_t>(g) * Bp * a.dp_out;
        for (int e = tid; e < Bp * kColChunk; e += NW * 64) {
            const int b = e / kColChunk, c = e % kColChunk;
            if (b < a.B && c < a.d_out) {
                const float z = red[b][c] + bias[c];
                out[static_cast<int64_t>(b) * a.dp_out + c] = z;
                red[b][c] = z;
            }
        }
        for (int e = tid; e < kColChunk * (Bp + kPad); e += NW * 64) (&dzt_lds[0][0])[e] = static_cast<OT>(0.f);
        for (int e = tid; e < Bp * (kColChunk + kPad); e += NW * 64) (&dz_lds[0][0])[e] = static_cast<OT>(0.f);
    }
    __syncthreads();

    // ---- phase 2: softmax cross-entropy; dZ_L = (p - onehot) / B goes to the LDS tiles
    {
        const int b = tid;
        float nll = 0.f;
        if (b < 128) {
            if (b < a.B) {
                const int y = a.labels[static_cast<int64_t>(g) * Bp + b];
                if (y >= 0) {
                    const float* z = red[b];
                    float zmax = z[0];
                    for (int c = 1; c < a.d_out; ++c) zmax = fmaxf(zmax, z[c]);
                    float s_other = 0.f;
                    for (int c = 0; c < a.d_out; ++c) s_other += c == y ? 0.f : expf(z[c] - zmax);
                    const float e_y = expf(z[y] - zmax);
                    nll = xent_loss(s_other, e_y, z[y] - zmax);
                    const float inv = 1.f / (s_other + e_y), invB = 1.f / static_cast<float>(a.B);
                    for (int c = 0; c < a.d_out; ++c) {
                        const OT d = static_cast<OT>(xent_delta(expf(z[c] - zmax), c == y, s_other, inv) * invB);
                        dz_lds[b][c] = d;
                        dzt_lds[(c & 3) * 16 + (c >> 2)][b] = d;
                    }
                }
            }
            lred[b] = nll;
        }
        __syncthreads();
        for (int w = 64; w > 0; w >>= 1) {
            if (b < w) lred[b] += lred[b + w];
            __syncthreads();
        }
        if (b == 0) a.loss[static_cast<int64_t>(g) * kLossParts] = lred[0] / static_cast<float>(a.B);
    }

    // ---- phase 3: backward of the layer.  Bias first (one thread per class) ...
    if (tid < a.d_out) {
        const OT* zr = dzt_lds[(tid & 3) * 16 + (tid >> 2)];
        float sb = 0.f;
        for (int b = 0; b < a.B; ++b) sb += to_f32(zr[b]);
        float* bx = a.X + g * a.x_stride + a.b_off + tid;
        float* bv = a.V + g * a.x_stride + a.b_off + tid;
        const float x = a.Xr[g * a.xr_stride + a.b_off + tid];
        const float vb = momentum_update(a.beta, *bv, sb, a.wd, x);
        *bv = vb;
        *bx = weight_update(x, a.lr, vb);
    }
    // ... then the weight rows, 16 per wavefront and trip
    OT* pbm = need_da ? static_cast<OT*>(a.dzp_bm) + static_cast<int64_t>(g) * Bp * a.dp_in : nullptr;
    OT* pfm = need_da ? static_cast<OT*>(a.dzp_fm) + static_cast<int64_t>(g) * a.dp_in * Bp : nullptr;
    const int n_rg = a.dp_in / kRowsPerWave;
    for (int rg = wave; rg < n_rg; rg += NW) {
        const int k0 = rg * kRowsPerWave;
        float4 w[4], v[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int row = k0 + 4 * q + r;
            w[r] = load_w4_rows(Wr, row, a.d_in, 4 * j, a.d_out, vec, stream);
            v[r] = load_w4_rows(Vw, row, a.d_in, 4 * j, a.d_out, vec, stream);
        }
        f32x4 acc[4];
#pragma unroll
        for (int t = 0; t < 4; ++t) acc[t] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int s = 0; s < NS; ++s) {
            const Frag<OT> af = load8(AT + static_cast<int64_t>(k0 + j) * Bp + 32 * s + 8 * q);
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const Frag<OT> bf = *reinterpret_cast<const Frag<OT>*>(&dzt_lds[t * 16 + j][32 * s + 8 * q]);
                acc[t] = mma8(af, bf, acc[t]);
            }
        }
        if (need_da) {
#pragma unroll
            for (int r = 0; r < 4; ++r) store4<OT>(&wlds[wave][4 * q + r][4 * j], w[r].x, w[r].y, w[r].z, w[r].w);
        }
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int row = k0 + 4 * q + r;
            const float4 gr = make_float4(acc[0][r], acc[1][r], acc[2][r], acc[3][r]);
            v[r].x = momentum_update(a.beta, v[r].x, gr.x, a.wd, w[r].x);
            v[r].y = momentum_update(a.beta, v[r].y, gr.y, a.wd, w[r].y);
            v[r].z = momentum_update(a.beta, v[r].z, gr.z, a.wd, w[r].z);
            v[r].w = momentum_update(a.beta, v[r].w, gr.w, a.wd, w[r].w);
            w[r].x = weight_update(w[r].x, a.lr, v[r].x);
            w[r].y = weight_update(w[r].y, a.lr, v[r].y);
            w[r].z = weight_update(w[r].z, a.lr, v[r].z);
            w[r].w = weight_update(w[r].w, a.lr, v[r].w);
            if (row < a.d_in) {
                store_w4(Vw + static_cast<int64_t>(row) * a.d_out, 4 * j, a.d_out, vec, stream, v[r]);
                store_w4(W + static_cast<int64_t>(row) * a.d_out, 4 * j, a.d_out, vec, stream, w[r]);
            }
        }
        if (need_da) {
            wave_sync_lds();
            f32x4 dacc[NT];
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) dacc[nt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int s = 0; s < 2; ++s) {
                const Frag<OT> wf = *reinterpret_cast<const Frag<OT>*>(&wlds[wave][j][32 * s + 8 * q]);
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) {
                    const Frag<OT> zf = *reinterpret_cast<const Frag<OT>*>(&dz_lds[16 * nt + j][32 * s + 8 * q]);
                    dacc[nt] = mma8(wf, zf, dacc[nt]);
                }
            }
            wave_sync_lds();
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
                const int b = 16 * nt + j;
                float d[4];
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int row = k0 + 4 * q + r;
                    const float act = to_f32(AT[static_cast<int64_t>(row) * Bp + b]);
                    d[r] = act > 0.f ? dacc[nt][r] : 0.f;
                    pfm[static_cast<int64_t>(row) * Bp + b] = static_cast<OT>(d[r]);
                }
                store4<OT>(pbm + static_cast<int64_t>(b) * a.dp_in + k0 + 4 * q, d[0], d[1], d[2], d[3]);
            }
        }
    }
}

// ------------------------------------------------------------------ dispatch

// Rows that are 16-byte aligned and a whole number of 64-column chunks long need no per-element checks.
int weight_mode(bool vec, bool stream, int d_out) {
    if (!vec || d_out % kColChunk != 0) return kWGeneric;
    return stream ? kWVectorStream : kWVector;
}

// Batch tiles per block (MT), wavefronts per block (NW) and weight steps kept in flight (PF).
// The accumulators of a full 128-row batch leave no registers for prefetching at two
// wavefronts per SIMD, so that case runs four wavefronts per block with a deeper queue.
template <typename OT, int WM>
hipError_t launch_fwd_cfg(const FwdArgs& a, int mt, bool wide, bool afm, unsigned grid, hipStream_t s) {
#define LC_FWD(MT_, NW_, PF_, AFM_) \
    hipLaunchKernelGGL((forward_kernel<OT, MT_, NW_, PF_, WM, AFM_>), dim3(grid), dim3(NW_ * 64), 0, s, a)
    switch (mt) {
        case 1: if (wide) LC_FWD(1, 8, 3, false); else LC_FWD(1, 4, 3, false); break;
        case 2: if (wide) LC_FWD(2, 8, 3, false); else LC_FWD(2, 4, 1, false); break;   // many blocks: occupancy 3 beats a deeper queue
        case 4: if (wide) LC_FWD(4, 8, 1, false); else LC_FWD(4, 4, 3, false); break;
        case 8: if (afm) LC_FWD(8, 4, 1, true); else LC_FWD(8, 4, 1, false); break;
        default: return hipErrorInvalidValue;
    }
#undef LC_FWD
    return hipGetLastError();
}
template <typename OT>
hipError_t launch_fwd_wm(const FwdArgs& a, int mt, bool wide, bool afm, unsigned grid, hipStream_t s) {
    switch (weight_mode(a.vec != 0, a.stream != 0, a.d_out)) {
        case kWVector: return launch_fwd_cfg<OT, kWVector>(a, mt, wide, afm, grid, s);
        case kWVectorStream: return launch_fwd_cfg<OT, kWVectorStream>(a, mt, wide, afm, grid, s);
        default: return launch_fwd_cfg<OT, kWGeneric>(a, mt, wide, afm, grid, s);
    }
}

template <typename OT, int WM>
hipError_t launch_bwd_nt(const BwdArgs& a, int nt, unsigned grid, hipStream_t s) {
    switch (nt) {
        case 2: hipLaunchKernelGGL((backward_kernel<OT, 2, WM>), dim3(grid), dim3(256), 0, s, a); break;
        case 4: hipLaunchKernelGGL((backward_kernel<OT, 4, WM>), dim3(grid), dim3(256), 0, s, a); break;
        case 8: hipLaunchKernelGGL((backward_kernel<OT, 8, WM>), dim3(grid), dim3(256), 0, s, a); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}
// dZ_{l-1} only (see backward_kernel); for layers with 16-byte aligned rows of a multiple of 64 columns
template <typename OT>
hipError_t launch_bwd_da_only(const BwdArgs& a, int nt, unsigned grid, hipStream_t s) {
    switch (nt) {
        case 2: hipLaunchKernelGGL((backward_kernel<OT, 2, kWVectorStream, true>), dim3(grid), dim3(256), 0, s, a); break;
        case 4: hipLaunchKernelGGL((backward_kernel<OT, 4, kWVectorStream, true>), dim3(grid), dim3(256), 0, s, a); break;
        case 8: hipLaunchKernelGGL((backward_kernel<OT, 8, kWVectorStream, true>), dim3(grid), dim3(256), 0, s, a); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}
template <typename OT>
hipError_t launch_bwd_wm(const BwdArgs& a, int nt, unsigned grid, hipStream_t s) {
    switch (weight_mode(a.vec != 0, a.stream != 0, a.d_out)) {
        case kWVector: return launch_bwd_nt<OT, kWVector>(a, nt, grid, s);
        case kWVectorStream: return launch_bwd_nt<OT, kWVectorStream>(a, nt, grid, s);
        default: return launch_bwd_nt<OT, kWGeneric>(a, nt, grid, s);
    }
}

inline int mt_for(int Bp) { return Bp / 16; }  // Bp is 32, 64 or 128

inline unsigned xcd_grid(int64_t total) { return static_cast<unsigned>((total + kXcds - 1) / kXcds * kXcds); }

}  // namespace

// Input buffers of the training step in progress (slot train.cur_slot).
inline size_t a0_slot_elems(const lc_handle* h, const ActSet& S) {
    return static_cast<size_t>(S.G) * S.Bp * h->layer[1].dp_in;
}
inline const void* a0_ptr(const lc_handle* h, const ActSet& S, const void* base, bool eval) {
    const size_t es = (!eval && h->md.gemm == LC_GEMM_BF16) ? 2 : 4;
    return static_cast<const char*>(base) + static_cast<size_t>(S.cur_slot) * a0_slot_elems(h, S) * es;
}
inline const int32_t* labels_ptr(const ActSet& S) {
    return S.labels + static_cast<size_t>(S.cur_slot) * S.G * S.Bp;
}

hipError_t launch_gather(lc_handle* h, bool eval, int64_t k_or_base, int n_steps) {
    const ActSet& S = eval ? h->eval : h->train;
    const bool bf16 = h->md.gemm == LC_GEMM_BF16;
    GatherArgs a;
    a.data = h->data;
    a.labels = h->labels;
    a.a_bm = S.a_bm[0];
    a.a_fm = S.a_fm[0];
    a.lab_out = S.labels;
    a.idx_out = S.idx;
    a.d0 = h->layer[1].d_in;
    a.dp0 = h->layer[1].dp_in;
    a.B = S.B;
    a.Bp = S.Bp;
    a.N = h->md.N;
    a.seed = h->seed;
    a.k = k_or_base;
    a.limit = h->md.E;
    a.eval = eval ? 1 : 0;
    a.sampler = h->md.sampler;
    a.m = h->m;
    a.G = S.G;
    a.a_slot = static_cast<int64_t>(a0_slot_elems(h, S));
    a.lab_slot = static_cast<int64_t>(S.G) * S.Bp;
    const dim3 grid(a.dp0 / 64, a.Bp / 32, S.G * n_steps);
    if (eval) {
        if (bf16) hipLaunchKernelGGL((gather_kernel<bf16_t, float>), grid, dim3(256), 0, h->stream, a);
        else hipLaunchKernelGGL((gather_kernel<float, float>), grid, dim3(256), 0, h->stream, a);
    } else {
        if (bf16) hipLaunchKernelGGL((gather_kernel<bf16_t, bf16_t>), grid, dim3(256), 0, h->stream, a);
        else hipLaunchKernelGGL((gather_kernel<float, float>), grid, dim3(256), 0, h->stream, a);
    }
    return hipGetLastError();
}

// ---- implicit momentum: which buffer holds what ---------------------------------------------------
//
// Inside a period (Sec. 2: tau local updates between two averaging steps) the update
// x_{k+1} = x_k - lr v_{k+1} lets the momentum be read off two consecutive models,
// v_k = (x_{k-1} - x_k) / lr.  A layer in implicit form keeps x_k in one of the two row buffers (X, V)
// and x_{k-1} in the other (or in the one averaged model, right after an averaging step); a step
// then reads both and writes x_{k+1} over x_{k-1}: 12 instead of 16 bytes per parameter.  The last
// step of a period (of a call) writes x to X and v to V again.  The recovered momentum differs from
// the stored one by the rounding of x_k, ulp(x) / (2 lr): relative to v that is 6e-8 divided by the
// relative size of a step, 1e-4 .. 1e-3 in training -- invisible beside bf16 operands (bar 2e-2), not
// beside fp32 operands (bar 1e-4), so it is taken for bf16 runs whose state streams from memory.
bool implicit_layer_ok(const lc_handle* h, int l) {
    if (h->imp_mode == 0 || h->md.kind != LC_KIND_MLP || l < 1 || l >= h->L) return false;   // the last layer is small: explicit
    if (h->bm_on || !(h->md.lr > 0.f)) return false;
    if (h->imp_mode == 2) return true;
    const LayerGeom& g = h->layer[l];
    // (the recovered momentum is off by up to ulp(x) / (2 lr) per element: not with very small rates)
    return h->md.gemm == LC_GEMM_BF16 && h->stream_weights && h->md.lr >= 1e-4f && 4.0 * g.d_in * g.d_out >= 1024.0 * 1024;
}

namespace {
const float* buffer_of(const lc_handle* h, int b, int64_t* stride) {
    *stride = b == kBufXbar ? 0 : h->Ps;
    return b == kBufX ? h->X : (b == kBufV ? h->V : h->xbar);
}
}  // namespace

void layer_weights(const lc_handle* h, int l, const float** base, int64_t* stride) {
    const ImpState& s = h->imp[l];
    *base = buffer_of(h, s.active ? s.cur : (h->lazy_rows ? kBufXbar : kBufX), stride);
}

StepBufs plan_step_buffers(const lc_handle* h, int l) {
    StepBufs b;
    const ImpState& s = h->imp[l];
    const int cur = s.active ? s.cur : (h->lazy_rows ? kBufXbar : kBufX);
    b.xr = buffer_of(h, cur, &b.xr_stride);
    if (s.active) {
        b.aux = buffer_of(h, s.prev, &b.aux_stride);
        b.imp_in = 1;
    } else {
        b.aux = h->V;
        b.aux_stride = h->Ps;
        b.imp_in = 0;
    }
    if (h->imp_out && implicit_layer_ok(h, l)) {
        // the new parameters go to the row buffer that does not hold the current ones: over the
        // momentum or the older model, which the same thread has read by then
        const int dst = cur == kBufV ? kBufX : kBufV;
        b.ox = dst == kBufX ? h->X : h->V;
        b.ov = nullptr;
        b.next = ImpState{true, dst, cur};
    } else {
        b.ox = h->X;
        b.ov = h->V;
        b.next = ImpState{false, kBufX, kBufV};
    }
    return b;
}

// Replicas that read one model take the same weight tile in neighbouring blocks when the layer is
// too large for an XCD's L2 to hold until the next replica comes by (measured: +14 % at m = 64 with
// 16-25 MB layers; a few per cent slower for models that are cache-resident anyway, whose blocks
// then no longer share their replica's activations).
bool shared_weight_order(const lc_handle* h, const LayerGeom& g) {
    return h->share_w_on && h->stream_weights && 4.0 * g.d_in * g.d_out >= 8.0 * 1024 * 1024;
}

// Replicas per set: 8 (one set per XCD at m = 64; sets of 4 to 32 measure the same, all replicas in
// one set 3 % less: a set's activations and deltas then no longer fit the L2 beside the tiles).
int shared_set(const lc_handle* h, int G) {
    const int set = h->share_w_set;
    return (set >= 1 && set < G && G % set == 0) ? set : G;
}

hipError_t launch_forward(lc_handle* h, bool eval, int l, int loss_offset) {
    const ActSet& S = eval ? h->eval : h->train;
    const LayerGeom& g = h->layer[l];
    const bool bf16 = !eval && h->md.gemm == LC_GEMM_BF16;
    FwdArgs a;
    // one model for all groups (the averaged one), or every replica's own rows -- which inside a
    // period with implicit momentum may be the rows of the other buffer
    const float* src = h->xbar;
    int64_t src_stride = 0;
    if (!eval) layer_weights(h, l, &src, &src_stride);
    const bool shared = src_stride == 0;
    a.X = src;
    a.x_stride = src_stride;
    a.w_off = g.w_off;
    a.b_off = g.b_off;
    a.d_in = g.d_in;
    a.d_out = g.d_out;
    a.dp_in = g.dp_in;
    a.dp_out = g.dp_out;
    a.B = S.B;
    a.Bp = S.Bp;
    a.fm_Bp = S.Bp;
    // one model for all replicas, every batch row valid, not the last layer (whose epilogue works
    // per replica): sets of replicas as one batch of up to 128 rows
    int n_groups = S.G;
    if (!eval && shared && h->group_shared_on && l < h->L && S.B == S.Bp && S.Bp < 128) {
        int gr = 128 / S.Bp;
        while (gr > 1 && S.G % gr != 0) gr /= 2;
        // (not when that leaves most of the chip idle)
        while (gr > 1 && static_cast<int64_t>(S.G / gr) * (g.dp_out / kColChunk) < 256) gr /= 2;
        if (gr > 1) {
            a.B = a.Bp = S.Bp * gr;
            n_groups = S.G / gr;
        }
    }
    const bool grouped = n_groups != S.G;
    a.a_in = l == 1 ? a0_ptr(h, S, S.a_bm[0], eval) : S.a_bm[l - 1];
    a.out_bm = S.a_bm[l];
    a.out_fm = S.a_fm[l];
    a.last = l == h->L ? 1 : 0;
    a.vec = (g.d_out % 4 == 0 && g.w_off % 4 == 0) ? 1 : 0;
    a.stream = (!shared && h->stream_weights) ? 1 : 0;
    a.n_chunks = g.dp_out / kColChunk;
    // softmax cross-entropy rides in the epilogue when one block sees all classes of all samples
    a.fuse_softmax = (a.last && g.d_out <= kColChunk) ? 1 : 0;
    a.labels = labels_ptr(S);
    a.dz_bm = eval ? nullptr : S.dz_bm[h->L];
    a.dz_fm = eval ? nullptr : S.dz_fm[h->L];
    a.loss = S.loss + static_cast<int64_t>(loss_offset) * kLossParts;
    a.eval = eval ? 1 : 0;
    a.shared_w = (!eval && shared && shared_weight_order(h, g)) ? shared_set(h, n_groups) : 0;
    // batch tiles per block: all of them, unless that leaves most of the chip idle
    int mt = mt_for(a.Bp);
    a.m_split = 1;
    while (!grouped && mt > 1 && static_cast<int64_t>(S.G) * a.n_chunks * a.m_split < 256) {
        mt /= 2;
        a.m_split *= 2;
    }
    if (a.fuse_softmax) (eval ? h->loss_parts_eval : h->loss_parts_train) = a.m_split;
    a.total_blocks = static_cast<int64_t>(n_groups) * a.n_chunks * a.m_split;
    const unsigned grid = xcd_grid(a.total_blocks);
    // few blocks: split the reduction over more wavefronts per block
    const bool wide = a.total_blocks * 4 < 2048 && g.dp_in >= 512;
    if (!eval) timing_start(h, kTimeFwd);
    hipError_t e;
    // whole padded batch in one block and a feature-major copy of the input at hand
    const void* in_fm = eval ? nullptr : (l == 1 ? a0_ptr(h, S, S.a_fm[0], false) : S.a_fm[l - 1]);
    const bool afm = in_fm != nullptr && !grouped && a.m_split == 1 && mt * 16 == S.Bp && mt == 8;
    a.a_in_fm = in_fm;
    if (bf16) e = launch_fwd_wm<bf16_t>(a, mt, wide, afm, grid, h->stream);
    else e = launch_fwd_wm<float>(a, mt, wide, afm, grid, h->stream);
    if (!eval) timing_stop(h, kTimeFwd);
    return e;
}

bool forward_fuses_softmax(const lc_handle* h) { return h->layer[h->L].d_out <= kColChunk; }

// One workgroup per replica is only faster than three spread-out launches while the
// layer is tiny (measured: wins at 64 input rows, loses from 256 on).
bool head_is_fused(const lc_handle* h) {
    return h->layer[h->L].d_out <= kColChunk && h->layer[h->L].dp_in <= 128;
}

hipError_t launch_head(lc_handle* h) {
    const ActSet& S = h->train;
    const int L = h->L;
    const LayerGeom& g = h->layer[L];
    const bool bf16 = h->md.gemm == LC_GEMM_BF16;
    HeadArgs a;
    a.X = h->X;
    a.V = h->V;
    a.x_stride = h->Ps;
    a.Xr = h->lazy_rows ? h->xbar : h->X;
    a.xr_stride = h->lazy_rows ? 0 : h->Ps;
    a.w_off = g.w_off;
    a.b_off = g.b_off;
    a.d_in = g.d_in;
    a.d_out = g.d_out;
    a.dp_in = g.dp_in;
    a.dp_out = g.dp_out;
    a.B = S.B;
    a.a_bm = L == 1 ? a0_ptr(h, S, S.a_bm[0], false) : S.a_bm[L - 1];
    a.a_fm = L == 1 ? a0_ptr(h, S, S.a_fm[0], false) : S.a_fm[L - 1];
    a.labels = labels_ptr(S);
    a.logits = static_cast<float*>(S.a_bm[L]);
    a.dzp_bm = L > 1 ? S.dz_bm[L - 1] : nullptr;
    a.dzp_fm = L > 1 ? S.dz_fm[L - 1] : nullptr;
    a.loss = S.loss;
    h->loss_parts_train = 1;
    a.lr = h->md.lr;
    a.beta = effective_beta(h);
    a.wd = h->md.wd;
    a.vec = (g.d_out % 4 == 0 && g.w_off % 4 == 0) ? 1 : 0;
    a.stream = 0;   // the last layer is small: keep it cached
    const dim3 grid(S.G), block(512);
    timing_start(h, kTimeBwd, L, kBwdHead);
    const int nt = S.Bp / 16;
    if (bf16) {
        if (nt == 2) hipLaunchKernelGGL((head_kernel<bf16_t, 2>), grid, block, 0, h->stream, a);
        else if (nt == 4) hipLaunchKernelGGL((head_kernel<bf16_t, 4>), grid, block, 0, h->stream, a);
        else hipLaunchKernelGGL((head_kernel<bf16_t, 8>), grid, block, 0, h->stream, a);
    } else {
        if (nt == 2) hipLaunchKernelGGL((head_kernel<float, 2>), grid, block, 0, h->stream, a);
        else if (nt == 4) hipLaunchKernelGGL((head_kernel<float, 4>), grid, block, 0, h->stream, a);
        else hipLaunchKernelGGL((head_kernel<float, 8>), grid, block, 0, h->stream, a);
    }
    timing_stop(h, kTimeBwd, L, kBwdHead);
    return hipGetLastError();
}

hipError_t launch_softmax(lc_handle* h, bool eval, int loss_offset) {
    const ActSet& S = eval ? h->eval : h->train;
    const bool bf16 = !eval && h->md.gemm == LC_GEMM_BF16;
    SoftmaxArgs a;
    a.logits = static_cast<const float*>(S.a_bm[h->L]);
    a.labels = labels_ptr(S);
    a.dz_bm = eval ? nullptr : S.dz_bm[h->L];
    a.dz_fm = eval ? nullptr : S.dz_fm[h->L];
    a.loss = S.loss + static_cast<int64_t>(loss_offset) * kLossParts;
    (eval ? h->loss_parts_eval : h->loss_parts_train) = 1;
    a.C = h->layer[h->L].d_out;
    a.dpL = h->layer[h->L].dp_out;
    a.B = S.B;
    a.Bp = S.Bp;
    a.eval = eval ? 1 : 0;
    if (bf16) hipLaunchKernelGGL((softmax_kernel<bf16_t>), dim3(S.G), dim3(128), 0, h->stream, a);
    else hipLaunchKernelGGL((softmax_kernel<float>), dim3(S.G), dim3(128), 0, h->stream, a);
    return hipGetLastError();
}

hipError_t launch_backward(lc_handle* h, int l, bool da_only) {
    const ActSet& S = h->train;
    const LayerGeom& g = h->layer[l];
    const bool bf16 = h->md.gemm == LC_GEMM_BF16;
    BwdArgs a;
    const StepBufs sb = plan_step_buffers(h, l);
    if (da_only && !sb.ov) return hipErrorInvalidValue;   // (only before a step that leaves v in V; the pass reads the weights alone)
    a.X = sb.ox;
    a.V = sb.ov;
    a.x_stride = h->Ps;
    a.Xr = sb.xr;
    a.xr_stride = sb.xr_stride;
    a.Aux = sb.aux;
    a.aux_stride = sb.aux_stride;
    a.imp_in = sb.imp_in;
    a.inv_lr = h->md.lr > 0.f ? 1.f / h->md.lr : 0.f;
    a.w_off = g.w_off;
    a.b_off = g.b_off;
    a.d_in = g.d_in;
    a.d_out = g.d_out;
    a.dp_in = g.dp_in;
    a.dp_out = g.dp_out;
    a.B = S.B;
    a.Bp = S.Bp;
    a.a_bm = l == 1 ? a0_ptr(h, S, S.a_bm[0], false) : S.a_bm[l - 1];
    a.a_fm = l == 1 ? a0_ptr(h, S, S.a_fm[0], false) : S.a_fm[l - 1];
    a.dz_bm = S.dz_bm[l];
    a.dz_fm = S.dz_fm[l];
    a.dzp_bm = l > 1 ? S.dz_bm[l - 1] : nullptr;
    a.dzp_fm = l > 1 ? S.dz_fm[l - 1] : nullptr;
    a.lr = h->md.lr;
    a.beta = effective_beta(h);
    a.wd = h->md.wd;
    a.vec = (g.d_out % 4 == 0 && g.w_off % 4 == 0) ? 1 : 0;
    a.stream = h->stream_weights ? 1 : 0;
    a.n_row_blocks = g.dp_in / 64;
    a.col_split = 1;
    a.skip_x = h->defer_x ? 1 : 0;
    a.fm_Bp = S.Bp;
    // the dA-only pass over one model that all replicas share: sets of replicas as one batch of up
    // to 128 rows (see launch_forward)
    int n_groups = S.G;
    if (da_only && sb.xr_stride == 0 && h->group_shared_on && S.B == S.Bp && S.Bp < 128) {
        int gr = 128 / S.Bp;
        while (gr > 1 && S.G % gr != 0) gr /= 2;
        while (gr > 1 && static_cast<int64_t>(S.G / gr) * (g.dp_in / 64) < 256) gr /= 2;
        if (gr > 1) {
            a.B = a.Bp = S.Bp * gr;
            n_groups = S.G / gr;
        }
    }
    a.shared_w = (sb.xr_stride == 0 && shared_weight_order(h, g)) ? shared_set(h, n_groups) : 0;
    if (l == 1) {
        // no dA: the columns can be shared out, to fill the chip and to keep the walk of a
        // workgroup short (measured: walks of 2-4 trips stream faster than long ones, a single
        // trip loses the load-ahead)
        const int n_cc = (g.d_out + kColChunk - 1) / kColChunk;
        const int64_t base = static_cast<int64_t>(S.G) * a.n_row_blocks;
        int want = static_cast<int>((1024 + base - 1) / base);
        if (want < n_cc / 4) want = n_cc / 4;
        a.col_split = want < 1 ? 1 : (want > n_cc ? n_cc : want);
        // a state that streams from memory: as few trips per workgroup as the per-workgroup set-up
        // (staging the dZ slice, the A operands: proportional to the batch tile) allows -- one at
        // 32 samples, four at 128.  Many short-lived workgroups sweep memory in dispatch order and
        // stream faster than few long walks (3072x2048 layer, 64 replicas, B = 32: 5.24 TB/s with 1
        // workgroup per row block, 5.55 with 8, 5.9 with 32; 3072x1024, 16 replicas, B = 128:
        // 155 us with 4 or 8 per row block, 191 us with 16)
        if (h->stream_weights && a.col_split < n_cc * 32 / S.Bp) a.col_split = n_cc * 32 / S.Bp;
    }
    a.total_blocks = static_cast<int64_t>(n_groups) * a.n_row_blocks * a.col_split;
    const unsigned grid = xcd_grid(a.total_blocks);
    // (same conditions as the tile-owner kernel that follows; the columns are not shared out here)
    if (da_only && (l < 2 || !a.vec || g.d_out % kColChunk != 0 || !a.stream)) return hipErrorInvalidValue;
    timing_start(h, kTimeBwd, l, kBwdRowOwner);
    hipError_t e;
    if (da_only) {
        e = bf16 ? launch_bwd_da_only<bf16_t>(a, a.Bp / 16, grid, h->stream)
                 : launch_bwd_da_only<float>(a, a.Bp / 16, grid, h->stream);
    } else {
        e = bf16 ? launch_bwd_wm<bf16_t>(a, S.Bp / 16, grid, h->stream)
                 : launch_bwd_wm<float>(a, S.Bp / 16, grid, h->stream);
    }
    timing_stop(h, kTimeBwd, l, kBwdRowOwner);
    if (e == hipSuccess && !da_only) h->imp[l] = sb.next;
    return e;
}

}  // namespace lc
