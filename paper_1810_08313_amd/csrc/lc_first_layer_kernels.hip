// Backward pass of the first layer, with the forward pass of the NEXT local step folded in.
//
// Between two averaging steps a worker's local updates touch only its own model (Sec. 2), so the
// first layer's weights after the update of step k are exactly the weights the forward pass of
// step k+1 multiplies its mini-batch with -- and that mini-batch does not depend on the model.
// The first layer needs no dA, so its rows can be shared out any way: here a workgroup owns 64
// COLUMNS of W_1 over all rows (the forward pass's decomposition).  While a tile of W_1, V_1 is
// in registers for
//     dW_1 = A_0^T dZ_1,   v <- beta v + dW_1 + wd w,   w <- w - lr v        (step k)
// the updated tile is used at once as the operand of
//     Z_1' = A_0' W_1 + b_1                                                  (step k+1)
// and W_1 crosses the memory system 16 instead of 20 bytes per parameter and step (12 instead of
// 16 where the momentum is implicit, see FirstArgs::Aux).
//
// This needs no exchange between lanes: the dW tile comes out of the matrix cores in accumulator
// layout (lane (j, q) holds rows 4q..4q+3 of a 16-row block, column j), and a matrix instruction
// with a reduction length of 16 takes its weight operand in exactly that shape (4 consecutive
// reduction indices per lane).  A step of the walk is therefore one 16-row block: the updated
// rows go from the update straight into the forward product, the activation operand is 4
// consecutive entries per lane.
#include "lc_internal.h"
#include "lc_mma.h"

#include <type_traits>

namespace lc {

namespace {

constexpr int kFlWaves = 4;

struct FirstArgs {
    float* X;             // where the new parameters are written
    float* V;             // where the new momentum is written, or null (implicit momentum, see BwdArgs::Aux)
    int64_t x_stride;
    const float* Xr;      // where the weights are read: X, the one averaged model (stride 0), or the other row buffer
    int64_t xr_stride;
    const float* Aux;     // the momentum rows, or (imp_in) the parameters of one step earlier
    int64_t aux_stride;
    int imp_in;
    float inv_lr;
    int shared_w;         // > 0: block order of steps in which all replicas read one model (see shared_order)
    int64_t w_off, b_off;
    int d_in, d_out, dp_in, dp_out;
    int B;
    const void* a_fm;     // A_0 of this step, feature-major [G][dp_in][Bp]
    const void* dz_fm;    // dZ_1 of this step, feature-major [G][dp_out][Bp]
    float lr, beta, wd;
    const void* an_bm;    // A_0 of the next step, batch-major [G][Bp][dp_in]
    void* out_bm;         // A_1 of the next step [G][Bp][dp_out]
    void* out_fm;         //                      [G][dp_out][Bp]
    int n_chunks;         // 64-column chunks per replica
    int64_t total_blocks;
};

// operand fragments of the 16-deep product: 4 consecutive reduction indices per lane
template <typename OT>
struct Frag4;
template <>
struct Frag4<float> {
    float v[4];
};
template <>
struct Frag4<bf16_t> {
    bf16x4 v;
};
__device__ __forceinline__ Frag4<float> load4(const float* p) {
    const float4 a = *reinterpret_cast<const float4*>(p);
    return Frag4<float>{{a.x, a.y, a.z, a.w}};
}
__device__ __forceinline__ Frag4<bf16_t> load4(const bf16_t* p) {
    Frag4<bf16_t> f;
    f.v = *reinterpret_cast<const bf16x4*>(p);
    return f;
}
__device__ __forceinline__ void pack4(Frag4<float>& f, float a, float b, float c, float d) {
    f.v[0] = a; f.v[1] = b; f.v[2] = c; f.v[3] = d;
}
__device__ __forceinline__ void pack4(Frag4<bf16_t>& f, float a, float b, float c, float d) {
    f.v[0] = static_cast<bf16_t>(a); f.v[1] = static_cast<bf16_t>(b);
    f.v[2] = static_cast<bf16_t>(c); f.v[3] = static_cast<bf16_t>(d);
}
__device__ __forceinline__ f32x4 mma4(const Frag4<float>& a, const Frag4<float>& b, f32x4 c) {
#pragma unroll
    for (int e = 0; e < 4; ++e) c = __builtin_amdgcn_mfma_f32_16x16x4f32(a.v[e], b.v[e], c, 0, 0, 0);
    return c;
}
__device__ __forceinline__ f32x4 mma4(const Frag4<bf16_t>& a, const Frag4<bf16_t>& b, f32x4 c) {
    typedef short s16x4 __attribute__((ext_vector_type(4)));
    return __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(__builtin_bit_cast(s16x4, a.v), __builtin_bit_cast(s16x4, b.v), c,
                                                     0, 0, 0);
}

// Steps a wavefront requests ahead of the one it works on, and wavefronts per SIMD the register
// budget is set for.  Up to 64 samples two workgroups share a CU (256 registers per lane) with one
// step ahead: what the walk responds to is the number of wavefronts that can issue, not the depth
// of a wavefront's queue (two steps ahead at one workgroup per CU: 1072 us on the 3072x2048 layer
// of 64 replicas, one or two steps ahead at two per CU: 900 us, none ahead at three or four per
// CU: 920 us -- measured while the weight-read mode was still a per-load choice, see WMR below;
// 887 us since).  At 128 samples the 32 accumulator tiles of the forward product leave room for one
// workgroup per CU only.  (fp32 operands at 64 samples spill at 256 registers with a step ahead.)
template <typename OT, int NT>
struct FlBudget {
    static constexpr int kWavesPerSimd = NT >= 8 ? 1 : 2;
    static constexpr int kAhead = (NT == 4 && sizeof(OT) == 4) ? 0 : 1;
};

// One workgroup = one replica x 64 columns of W_1; its 4 wavefronts take the 16-row steps
// wave, wave + 4, ... and never synchronise inside the walk: the dZ_1 slice is staged once, the
// A_0 tiles go from memory straight into operand registers.  The loads of a wavefront's next PD
// steps are in flight while it works on the current one (PD + 1 register sets, addressed
// statically); a step is small enough (about 20 memory instructions with its stores) that the
// steps in flight stay below the 64 outstanding memory instructions a wavefront can have.
// Rows are 16-byte aligned and a multiple of 64 columns long and d_in is a multiple of 16 (the
// launcher checks), so every weight access is one unconditional 16-byte instruction.
// WM is the access mode of the state that streams (momentum or older model, all stores), WMR that of
// the weights read: cached where all replicas read one model, which the neighbouring blocks want in
// the L2.  (A template parameter, not a run-time flag: with the choice made per load the compiler
// waited for each load before it issued the next.)
template <typename OT, int NT, int WM, int WMR>
__global__ __launch_bounds__(256, (FlBudget<OT, NT>::kWavesPerSimd)) void first_layer_kernel(FirstArgs a) {
    constexpr int kPad = sizeof(OT) == 2 ? 8 : 4;
    constexpr int Bp = 16 * NT;
    constexpr int NS = Bp / 32;
    constexpr int PD = FlBudget<OT, NT>::kAhead;
    // the dZ^T slice during the walk; the wavefronts' partial Z_1' tiles after it
    constexpr size_t kSliceBytes = sizeof(OT) * kColChunk * (Bp + kPad);
    constexpr size_t kPartBytes = sizeof(float) * kFlWaves * Bp * (kColChunk + 4);
    __shared__ __attribute__((aligned(16))) char smem[kSliceBytes > kPartBytes ? kSliceBytes : kPartBytes];
    __shared__ float bias_s[kColChunk];
    // row (c % 4) * 16 + c / 4 holds column c0 + c: the 16 lanes of an operand read (columns
    // 4 j + t) then hit 16 consecutive LDS rows
    OT (*dzt)[Bp + kPad] = reinterpret_cast<OT (*)[Bp + kPad]>(smem);

    const int64_t logical = xcd_logical_block(a.total_blocks);
    if (logical < 0) return;
    int g, chunk;
    shared_order(logical, a.n_chunks, a.shared_w, g, chunk);
    const int c0 = chunk * kColChunk;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // uniform: step bases live in scalar registers
    const int j = lane & 15, q = lane >> 4;

    float* W = a.X + g * a.x_stride + a.w_off;
    const float* Wr = a.Xr + g * a.xr_stride + a.w_off;
    float* Vw = a.V ? a.V + g * a.x_stride + a.w_off : nullptr;
    const float* Va = a.Aux + g * a.aux_stride + a.w_off;
    const OT* AT = static_cast<const OT*>(a.a_fm) + static_cast<int64_t>(g) * a.dp_in * Bp;
    const OT* AN = static_cast<const OT*>(a.an_bm) + static_cast<int64_t>(g) * Bp * a.dp_in;
    const int n_steps = a.d_in / 16;

    struct Set {
        float4 w[4], v[4];      // rows k0 + 4 q + r, columns c0 + 4 j ..
        Frag<OT> af[NS];        // A_0^T tile of the 16 rows
        Frag4<OT> an[NT];       // next step's A_0, 4 entries of each batch row
    };
    Set set[PD + 1];

    // A step's addresses are a base that is the same for the whole wavefront (scalar registers)
    // plus byte offsets that a lane keeps for the whole walk: 4 registers serve the loads and the
    // stores of W and V alike.
    unsigned woff[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) woff[r] = 4u * static_cast<unsigned>((4 * q + r) * a.d_out + c0 + 4 * j);
    const unsigned atoff = static_cast<unsigned>(sizeof(OT)) * static_cast<unsigned>(j * Bp + 8 * q);
    const unsigned anoff = static_cast<unsigned>(sizeof(OT)) * static_cast<unsigned>(j * a.dp_in + 4 * q);
    auto at_byte = [](auto* base, unsigned off) {
        using T = std::remove_pointer_t<decltype(base)>;
        using C = std::conditional_t<std::is_const_v<T>, const char, char>;
        return reinterpret_cast<T*>(reinterpret_cast<C*>(base) + off);
    };

    auto load_step = [&](int s, Set& x) {
        // steps past the end are never used: a valid step is read for them, so that no branch
        // sits between the loads
        const int k0 = 16 * (s < n_steps ? s : n_steps - 1);
        const float* wb = Wr + static_cast<int64_t>(k0) * a.d_out;
        const float* vb = Va + static_cast<int64_t>(k0) * a.d_out;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            x.w[r] = load_wm<WMR>(at_byte(wb, woff[r]), 0, a.d_out, true);
            x.v[r] = load_wm<WM>(at_byte(vb, woff[r]), 0, a.d_out, true);
        }
        const OT* ab = AT + static_cast<int64_t>(k0) * Bp;
#pragma unroll
        for (int st = 0; st < NS; ++st) x.af[st] = load8(at_byte(ab + 32 * st, atoff));
        const OT* nb = AN + k0;
#pragma unroll
        for (int mt = 0; mt < NT; ++mt) x.an[mt] = load4(at_byte(nb + static_cast<int64_t>(16 * mt) * a.dp_in, anoff));
    };

    // first loads, then the staging of the slice (its own round trip overlaps with them)
#pragma unroll
    for (int p = 0; p < PD; ++p) load_step(wave + p * kFlWaves, set[p]);
    {
        const OT* ZT = static_cast<const OT*>(a.dz_fm) + (static_cast<int64_t>(g) * a.dp_out + c0) * Bp;
        for (int p = tid; p < kColChunk * (Bp / 8); p += 256) {
            const int c = p / (Bp / 8), seg = p % (Bp / 8);
            *reinterpret_cast<Frag<OT>*>(&dzt[(c & 3) * 16 + (c >> 2)][seg * 8]) = load8(ZT + static_cast<int64_t>(p) * 8);
        }
    }
    __syncthreads();
    // bias of these columns: db_1 = sum_b dZ_1, the same update; kept for the forward epilogue
    if (tid < kColChunk) {
        float* bx = a.X + g * a.x_stride + a.b_off + c0 + tid;
        const float x = a.Xr[g * a.xr_stride + a.b_off + c0 + tid];
        float vb0 = a.Aux[g * a.aux_stride + a.b_off + c0 + tid];
        if (a.imp_in) vb0 = (vb0 - x) * a.inv_lr;
        const OT* zr = dzt[(tid & 3) * 16 + (tid >> 2)];
        float sb = 0.f;
        for (int b = 0; b < a.B; ++b) sb += to_f32(zr[b]);
        const float vb = a.beta * vb0 + (sb + a.wd * x);
        if (a.V) a.V[g * a.x_stride + a.b_off + c0 + tid] = vb;
        *bx = x - a.lr * vb;
        bias_s[tid] = x - a.lr * vb;
    }

    f32x4 facc[NT][4];
#pragma unroll
    for (int mt = 0; mt < NT; ++mt)
#pragma unroll
        for (int t = 0; t < 4; ++t) facc[mt][t] = f32x4{0.f, 0.f, 0.f, 0.f};

    auto process = [&](int s, Set& x) {
        float* ws = W + static_cast<int64_t>(16 * s) * a.d_out;
        float* vs = Vw ? Vw + static_cast<int64_t>(16 * s) * a.d_out : nullptr;
        // dW tile: sum over the batch of A_0^T[k][b] dZ_1^T[c][b]
        f32x4 acc[4];
#pragma unroll
        for (int t = 0; t < 4; ++t) acc[t] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int st = 0; st < NS; ++st)
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const Frag<OT> zf = *reinterpret_cast<const Frag<OT>*>(&dzt[t * 16 + j][32 * st + 8 * q]);
                acc[t] = mma8(x.af[st], zf, acc[t]);
            }
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            consume_here(x.w[r]);
            consume_here(x.v[r]);
            if (a.imp_in) {   // the tile holds the parameters of one step earlier: v = (x_prev - x) / lr
                x.v[r].x = (x.v[r].x - x.w[r].x) * a.inv_lr;
                x.v[r].y = (x.v[r].y - x.w[r].y) * a.inv_lr;
                x.v[r].z = (x.v[r].z - x.w[r].z) * a.inv_lr;
                x.v[r].w = (x.v[r].w - x.w[r].w) * a.inv_lr;
            }
            x.v[r].x = a.beta * x.v[r].x + (acc[0][r] + a.wd * x.w[r].x);
            x.v[r].y = a.beta * x.v[r].y + (acc[1][r] + a.wd * x.w[r].y);
            x.v[r].z = a.beta * x.v[r].z + (acc[2][r] + a.wd * x.w[r].z);
            x.v[r].w = a.beta * x.v[r].w + (acc[3][r] + a.wd * x.w[r].w);
            x.w[r].x -= a.lr * x.v[r].x;
            x.w[r].y -= a.lr * x.v[r].y;
            x.w[r].z -= a.lr * x.v[r].z;
            x.w[r].w -= a.lr * x.v[r].w;
            if (vs) store_wm<WM>(at_byte(vs, woff[r]), 0, a.d_out, true, x.v[r]);
            store_wm<WM>(at_byte(ws, woff[r]), 0, a.d_out, true, x.w[r]);
        }
        // Z_1' += A_0'[:, k0 .. k0+15] W_1[k0 .. k0+15, :] with the tile just updated
        Frag4<OT> bf;
        pack4(bf, x.w[0].x, x.w[1].x, x.w[2].x, x.w[3].x);
#pragma unroll
        for (int mt = 0; mt < NT; ++mt) facc[mt][0] = mma4(x.an[mt], bf, facc[mt][0]);
        pack4(bf, x.w[0].y, x.w[1].y, x.w[2].y, x.w[3].y);
#pragma unroll
        for (int mt = 0; mt < NT; ++mt) facc[mt][1] = mma4(x.an[mt], bf, facc[mt][1]);
        pack4(bf, x.w[0].z, x.w[1].z, x.w[2].z, x.w[3].z);
#pragma unroll
        for (int mt = 0; mt < NT; ++mt) facc[mt][2] = mma4(x.an[mt], bf, facc[mt][2]);
        pack4(bf, x.w[0].w, x.w[1].w, x.w[2].w, x.w[3].w);
#pragma unroll
        for (int mt = 0; mt < NT; ++mt) facc[mt][3] = mma4(x.an[mt], bf, facc[mt][3]);
    };

    // groups of PD + 1 steps without control flow in between (a branch would make the compiler
    // drain the loads in flight where the paths meet), then the steps whose loads are under way
    int s0 = wave;
    for (; s0 + PD * kFlWaves < n_steps; s0 += kFlWaves * (PD + 1)) {
#pragma unroll
        for (int u = 0; u <= PD; ++u) {
            const int s = s0 + u * kFlWaves;
            load_step(s + PD * kFlWaves, set[(u + PD) % (PD + 1)]);
            process(s, set[u]);
            __builtin_amdgcn_sched_barrier(0);
        }
    }
#pragma unroll
    for (int u = 0; u < PD; ++u) {
        const int s = s0 + u * kFlWaves;
        if (s < n_steps) process(s, set[u]);   // uniform over the wavefront
    }

    // A_1' = ReLU(Z_1' + b_1): the wavefronts' partial tiles are added in wavefront order
    __syncthreads();   // every wavefront is done with the slice that shares this memory
    float (*part)[Bp][kColChunk + 4] = reinterpret_cast<float (*)[Bp][kColChunk + 4]>(smem);
#pragma unroll
    for (int mt = 0; mt < NT; ++mt)
#pragma unroll
        for (int r = 0; r < 4; ++r)
            *reinterpret_cast<float4*>(&part[wave][16 * mt + 4 * q + r][4 * j]) =
                make_float4(facc[mt][0][r], facc[mt][1][r], facc[mt][2][r], facc[mt][3][r]);
    __syncthreads();
    for (int f = tid; f < Bp * (kColChunk / 4); f += 256) {
        const int b = f / (kColChunk / 4), c4 = (f % (kColChunk / 4)) * 4;
        float4 z = *reinterpret_cast<const float4*>(&part[0][b][c4]);
#pragma unroll
        for (int wv = 1; wv < kFlWaves; ++wv) {
            const float4 o = *reinterpret_cast<const float4*>(&part[wv][b][c4]);
            z.x += o.x; z.y += o.y; z.z += o.z; z.w += o.w;
        }
        z.x += bias_s[c4]; z.y += bias_s[c4 + 1]; z.z += bias_s[c4 + 2]; z.w += bias_s[c4 + 3];
        *reinterpret_cast<float4*>(&part[0][b][c4]) =
            make_float4(z.x > 0.f ? z.x : 0.f, z.y > 0.f ? z.y : 0.f, z.z > 0.f ? z.z : 0.f, z.w > 0.f ? z.w : 0.f);
    }
    __syncthreads();
    OT* obm = static_cast<OT*>(a.out_bm) + static_cast<int64_t>(g) * Bp * a.dp_out;
    OT* ofm = static_cast<OT*>(a.out_fm) + static_cast<int64_t>(g) * a.dp_out * Bp;
    auto value = [&](int b, int c) { return part[0][b][c]; };
    // 8 outputs per thread and pass, one vector store each: along the columns for the
    // batch-major copy, along the batch for the feature-major one; only batch rows below B
    // are written, so the zero padding of the buffers is preserved
    for (int e = tid; e < Bp * (kColChunk / 8); e += 256) {
        const int b = e / (kColChunk / 8), cl = (e % (kColChunk / 8)) * 8;
        if (b >= a.B) continue;
        float y[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) y[i] = value(b, cl + i);
        store8(obm + static_cast<int64_t>(b) * a.dp_out + c0 + cl, y);
    }
    for (int e = tid; e < kColChunk * (Bp / 8); e += 256) {
        const int c = e / (Bp / 8), bl = (e % (Bp / 8)) * 8;
        if (bl >= a.B) continue;
        float y[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) y[i] = bl + i < a.B ? value(bl + i, c) : 0.f;
        if (bl + 8 <= a.B) {
            store8(ofm + static_cast<int64_t>(c0 + c) * Bp + bl, y);
        } else {
            for (int i = 0; bl + i < a.B; ++i) ofm[static_cast<int64_t>(c0 + c) * Bp + bl + i] = static_cast<OT>(y[i]);
        }
    }
}


// The same step at 128 samples.  Sharing out the rows alone leaves each wavefront with the whole
// 128 x 64 tile of Z_1' (128 accumulator registers per lane), so four wavefronts fill a CU's register
// file with two steps in flight each, and the walk waits for memory.  Here a workgroup has 8
// wavefronts that share out BOTH: wavefront w updates the 16-row steps 8 r + w (r = 0, 1, ... :
// "rounds") as above, publishes each updated tile in LDS in operand precision, and after one
// barrier per round multiplies all 8 tiles of the round with ITS 16 samples of A_0' -- 4
// accumulator tiles per wavefront, complete at the end of the walk, nothing to add up across
// wavefronts.  Two sets of loads per wavefront, twice the wavefronts (3072x1024, 16 replicas: 161 ->
// 148 us; a third set changes nothing, nor does leaving out either product: what remains is the
// memory system's rate for 256 column walks).
// The tiles are double-buffered: a wavefront can only write round r + 1's buffer (that of round
// r - 1) after the barrier of round r, which every reader of round r - 1 has passed.
constexpr int kWideWaves = 8;

template <typename OT, int WM, int WMR, int PD = 1>
__global__ __launch_bounds__(64 * kWideWaves) void first_layer_wide_kernel(FirstArgs a) {
    static_assert(sizeof(OT) == 2, "operand fragments of fp32 do not fit the register budget here");
    constexpr int kPad = 8;
    constexpr int Bp = 128, NS = Bp / 32, NTH = 64 * kWideWaves;
    constexpr size_t kSliceBytes = sizeof(OT) * kColChunk * (Bp + kPad);
    constexpr size_t kTileBytes = 2 * kWideWaves * 2 * 64 * sizeof(bf16x8);
    constexpr size_t kPartBytes = sizeof(float) * Bp * (kColChunk + 4);
    constexpr size_t kWalkBytes = kSliceBytes + kTileBytes;
    __shared__ __attribute__((aligned(16))) char smem[kWalkBytes > kPartBytes ? kWalkBytes : kPartBytes];
    __shared__ float bias_s[kColChunk];
    OT (*dzt)[Bp + kPad] = reinterpret_cast<OT (*)[Bp + kPad]>(smem);
    // [buffer][wavefront][half][lane]: a lane's 4 x 4 block of the tile as 4 operand fragments
    // (columns 4 j + t, rows 4 q ..), 16 bytes per lane and half: consecutive lanes, no bank conflicts
    bf16x8 (*wt)[kWideWaves][2][64] = reinterpret_cast<bf16x8 (*)[kWideWaves][2][64]>(smem + kSliceBytes);

    const int64_t logical = xcd_logical_block(a.total_blocks);
    if (logical < 0) return;
    int g, chunk;
    shared_order(logical, a.n_chunks, a.shared_w, g, chunk);
    const int c0 = chunk * kColChunk;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int j = lane & 15, q = lane >> 4;

    float* W = a.X + g * a.x_stride + a.w_off;
    const float* Wr = a.Xr + g * a.xr_stride + a.w_off;
    float* Vw = a.V ? a.V + g * a.x_stride + a.w_off : nullptr;
    const float* Va = a.Aux + g * a.aux_stride + a.w_off;
    const OT* AT = static_cast<const OT*>(a.a_fm) + static_cast<int64_t>(g) * a.dp_in * Bp;
    // this wavefront's 16 samples of the next step's input
    const OT* AN = static_cast<const OT*>(a.an_bm) + (static_cast<int64_t>(g) * Bp + 16 * wave) * a.dp_in;
    const int n_rounds = a.d_in / (16 * kWideWaves);   // the launcher checks that this divides

    struct Set {
        float4 w[4], v[4];            // rows k0 + 4 q + r, columns c0 + 4 j ..
        Frag<OT> af[NS];              // A_0^T tile of this wavefront's 16 rows
        Frag4<OT> an[kWideWaves];     // A_0' of this wavefront's samples, 4 entries for each tile of the round
    };
    Set set[PD + 1];

    unsigned woff[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) woff[r] = 4u * static_cast<unsigned>((4 * q + r) * a.d_out + c0 + 4 * j);
    const unsigned atoff = static_cast<unsigned>(sizeof(OT)) * static_cast<unsigned>(j * Bp + 8 * q);
    const unsigned anoff = static_cast<unsigned>(sizeof(OT)) * static_cast<unsigned>(j * a.dp_in + 4 * q);
    auto at_byte = [](auto* base, unsigned off) {
        using T = std::remove_pointer_t<decltype(base)>;
        using C = std::conditional_t<std::is_const_v<T>, const char, char>;
        return reinterpret_cast<T*>(reinterpret_cast<C*>(base) + off);
    };

    auto load_round = [&](int r, Set& x) {
        // rounds past the end are never used: the last one is read for them (no branch between the loads)
        const int rr = r < n_rounds ? r : n_rounds - 1;
        const int k0 = 16 * (kWideWaves * rr + wave);
        const float* wb = Wr + static_cast<int64_t>(k0) * a.d_out;
        const float* vb = Va + static_cast<int64_t>(k0) * a.d_out;
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4) {
            x.w[r4] = load_wm<WMR>(at_byte(wb, woff[r4]), 0, a.d_out, true);
            x.v[r4] = load_wm<WM>(at_byte(vb, woff[r4]), 0, a.d_out, true);
        }
        const OT* ab = AT + static_cast<int64_t>(k0) * Bp;
#pragma unroll
        for (int st = 0; st < NS; ++st) x.af[st] = load8(at_byte(ab + 32 * st, atoff));
        const OT* nb = AN + 16 * kWideWaves * rr;
#pragma unroll
        for (int u = 0; u < kWideWaves; ++u) x.an[u] = load4(at_byte(nb + 16 * u, anoff));
    };

#pragma unroll
    for (int p = 0; p < PD; ++p) load_round(p, set[p]);
    {
        const OT* ZT = static_cast<const OT*>(a.dz_fm) + (static_cast<int64_t>(g) * a.dp_out + c0) * Bp;
        for (int p = tid; p < kColChunk * (Bp / 8); p += NTH) {
            const int c = p / (Bp / 8), seg = p % (Bp / 8);
            *reinterpret_cast<Frag<OT>*>(&dzt[(c & 3) * 16 + (c >> 2)][seg * 8]) = load8(ZT + static_cast<int64_t>(p) * 8);
        }
    }
    __syncthreads();
    if (tid < kColChunk) {
        float* bx = a.X + g * a.x_stride + a.b_off + c0 + tid;
        const float x = a.Xr[g * a.xr_stride + a.b_off + c0 + tid];
        float vb0 = a.Aux[g * a.aux_stride + a.b_off + c0 + tid];
        if (a.imp_in) vb0 = (vb0 - x) * a.inv_lr;
        const OT* zr = dzt[(tid & 3) * 16 + (tid >> 2)];
        float sb = 0.f;
        for (int b = 0; b < a.B; ++b) sb += to_f32(zr[b]);
        const float vb = a.beta * vb0 + (sb + a.wd * x);
        if (a.V) a.V[g * a.x_stride + a.b_off + c0 + tid] = vb;
        *bx = x - a.lr * vb;
        bias_s[tid] = x - a.lr * vb;
    }

    f32x4 facc[4];
#pragma unroll
    for (int t = 0; t < 4; ++t) facc[t] = f32x4{0.f, 0.f, 0.f, 0.f};

    auto process = [&](int r, Set& x) {
        const int64_t row0 = static_cast<int64_t>(16 * (kWideWaves * r + wave)) * a.d_out;
        float* ws = W + row0;
        float* vs = Vw ? Vw + row0 : nullptr;
        f32x4 acc[4];
#pragma unroll
        for (int t = 0; t < 4; ++t) acc[t] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int st = 0; st < NS; ++st)
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const Frag<OT> zf = *reinterpret_cast<const Frag<OT>*>(&dzt[t * 16 + j][32 * st + 8 * q]);
                acc[t] = mma8(x.af[st], zf, acc[t]);
            }
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4) {
            consume_here(x.w[r4]);
            consume_here(x.v[r4]);
            if (a.imp_in) {   // the tile holds the parameters of one step earlier: v = (x_prev - x) / lr
                x.v[r4].x = (x.v[r4].x - x.w[r4].x) * a.inv_lr;
                x.v[r4].y = (x.v[r4].y - x.w[r4].y) * a.inv_lr;
                x.v[r4].z = (x.v[r4].z - x.w[r4].z) * a.inv_lr;
                x.v[r4].w = (x.v[r4].w - x.w[r4].w) * a.inv_lr;
            }
            x.v[r4].x = a.beta * x.v[r4].x + (acc[0][r4] + a.wd * x.w[r4].x);
            x.v[r4].y = a.beta * x.v[r4].y + (acc[1][r4] + a.wd * x.w[r4].y);
            x.v[r4].z = a.beta * x.v[r4].z + (acc[2][r4] + a.wd * x.w[r4].z);
            x.v[r4].w = a.beta * x.v[r4].w + (acc[3][r4] + a.wd * x.w[r4].w);
            x.w[r4].x -= a.lr * x.v[r4].x;
            x.w[r4].y -= a.lr * x.v[r4].y;
            x.w[r4].z -= a.lr * x.v[r4].z;
            x.w[r4].w -= a.lr * x.v[r4].w;
            if (vs) store_wm<WM>(at_byte(vs, woff[r4]), 0, a.d_out, true, x.v[r4]);
            store_wm<WM>(at_byte(ws, woff[r4]), 0, a.d_out, true, x.w[r4]);
        }
        // the updated tile, as the 4 operand fragments of this lane
        Frag4<OT> b0, b1, b2, b3;
        pack4(b0, x.w[0].x, x.w[1].x, x.w[2].x, x.w[3].x);
        pack4(b1, x.w[0].y, x.w[1].y, x.w[2].y, x.w[3].y);
        pack4(b2, x.w[0].z, x.w[1].z, x.w[2].z, x.w[3].z);
        pack4(b3, x.w[0].w, x.w[1].w, x.w[2].w, x.w[3].w);
        bf16x8 lo, hi;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            lo[e] = b0.v[e]; lo[4 + e] = b1.v[e];
            hi[e] = b2.v[e]; hi[4 + e] = b3.v[e];
        }
        wt[r & 1][wave][0][lane] = lo;
        wt[r & 1][wave][1][lane] = hi;
        __syncthreads();
        // Z_1'[these 16 samples] += A_0'[.., the round's 128 rows] W_1[the round's 128 rows, :]
#pragma unroll
        for (int u = 0; u < kWideWaves; ++u) {
            const bf16x8 l2 = wt[r & 1][u][0][lane], h2 = wt[r & 1][u][1][lane];
            Frag4<OT> f0, f1, f2, f3;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                f0.v[e] = l2[e]; f1.v[e] = l2[4 + e];
                f2.v[e] = h2[e]; f3.v[e] = h2[4 + e];
            }
            facc[0] = mma4(x.an[u], f0, facc[0]);
            facc[1] = mma4(x.an[u], f1, facc[1]);
            facc[2] = mma4(x.an[u], f2, facc[2]);
            facc[3] = mma4(x.an[u], f3, facc[3]);
        }
    };

    // groups of PD + 1 rounds without control flow in between, then the rounds whose loads are under way
    int r0 = 0;
    for (; r0 + PD < n_rounds; r0 += PD + 1) {
#pragma unroll
        for (int u = 0; u <= PD; ++u) {
            load_round(r0 + u + PD, set[(u + PD) % (PD + 1)]);
            process(r0 + u, set[u]);
            __builtin_amdgcn_sched_barrier(0);
        }
    }
#pragma unroll
    for (int u = 0; u < PD; ++u)
        if (r0 + u < n_rounds) process(r0 + u, set[u]);   // uniform over the workgroup

    // A_1' = ReLU(Z_1' + b_1), through LDS for the two layouts of the stores
    __syncthreads();   // every wavefront is done with the slice and the tiles that share this memory
    float (*part)[kColChunk + 4] = reinterpret_cast<float (*)[kColChunk + 4]>(smem);
#pragma unroll
    for (int r4 = 0; r4 < 4; ++r4) {
        float4 z = make_float4(facc[0][r4] + bias_s[4 * j], facc[1][r4] + bias_s[4 * j + 1], facc[2][r4] + bias_s[4 * j + 2],
                               facc[3][r4] + bias_s[4 * j + 3]);
        z = make_float4(z.x > 0.f ? z.x : 0.f, z.y > 0.f ? z.y : 0.f, z.z > 0.f ? z.z : 0.f, z.w > 0.f ? z.w : 0.f);
        *reinterpret_cast<float4*>(&part[16 * wave + 4 * q + r4][4 * j]) = z;
    }
    __syncthreads();
    OT* obm = static_cast<OT*>(a.out_bm) + static_cast<int64_t>(g) * Bp * a.dp_out;
    OT* ofm = static_cast<OT*>(a.out_fm) + static_cast<int64_t>(g) * a.dp_out * Bp;
    for (int e = tid; e < Bp * (kColChunk / 8); e += NTH) {
        const int b = e / (kColChunk / 8), cl = (e % (kColChunk / 8)) * 8;
        if (b >= a.B) continue;
        float y[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) y[i] = part[b][cl + i];
        store8(obm + static_cast<int64_t>(b) * a.dp_out + c0 + cl, y);
    }
    for (int e = tid; e < kColChunk * (Bp / 8); e += NTH) {
        const int c = e / (Bp / 8), bl = (e % (Bp / 8)) * 8;
        if (bl >= a.B) continue;
        float y[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) y[i] = bl + i < a.B ? part[bl + i][c] : 0.f;
        if (bl + 8 <= a.B) {
            store8(ofm + static_cast<int64_t>(c0 + c) * Bp + bl, y);
        } else {
            for (int i = 0; bl + i < a.B; ++i) ofm[static_cast<int64_t>(c0 + c) * Bp + bl + i] = static_cast<OT>(y[i]);
        }
    }
}

template <typename OT, int NT>
void launch_fl_wm(const FirstArgs& a, bool stream_w, unsigned grid, hipStream_t st) {
    if (stream_w && !a.shared_w)
        hipLaunchKernelGGL((first_layer_kernel<OT, NT, kWVectorStream, kWVectorStream>), dim3(grid), dim3(256), 0, st, a);
    else if (stream_w) hipLaunchKernelGGL((first_layer_kernel<OT, NT, kWVectorStream, kWVector>), dim3(grid), dim3(256), 0, st, a);
    else hipLaunchKernelGGL((first_layer_kernel<OT, NT, kWVector, kWVector>), dim3(grid), dim3(256), 0, st, a);
}

template <typename OT>
hipError_t launch_fl(const FirstArgs& a, int nt, bool stream_w, unsigned grid, hipStream_t st) {
    if constexpr (sizeof(OT) == 2) {
        if (nt == 8 && a.d_in % (16 * kWideWaves) == 0) {
            const dim3 block(64 * kWideWaves);
            if (stream_w && !a.shared_w)
                hipLaunchKernelGGL((first_layer_wide_kernel<OT, kWVectorStream, kWVectorStream>), dim3(grid), block, 0, st, a);
            else if (stream_w) hipLaunchKernelGGL((first_layer_wide_kernel<OT, kWVectorStream, kWVector>), dim3(grid), block, 0, st, a);
            else hipLaunchKernelGGL((first_layer_wide_kernel<OT, kWVector, kWVector>), dim3(grid), block, 0, st, a);
            return hipGetLastError();
        }
    }
    if (nt == 2) launch_fl_wm<OT, 2>(a, stream_w, grid, st);
    else if (nt == 4) launch_fl_wm<OT, 4>(a, stream_w, grid, st);
    else launch_fl_wm<OT, 8>(a, stream_w, grid, st);
    return hipGetLastError();
}

}  // namespace

// The kernel serves layer 1 of models with at least two layers whose first-layer rows are 16-byte
// aligned and a multiple of 64 columns long and whose input width is a multiple of 16, when there
// are enough (replica, column chunk) pairs to fill the chip; everything else keeps the row-owner
// backward kernel and the separate forward launch.
bool first_layer_kernel_ok(const lc_handle* h) {
    if (h->md.kind != LC_KIND_MLP || h->L < 2) return false;
    const LayerGeom& g = h->layer[1];
    const ActSet& S = h->train;
    if (g.d_out % kColChunk != 0 || g.w_off % 4 != 0 || h->Ps % 4 != 0) return false;
    if (S.Bp != 32 && S.Bp != 64 && S.Bp != 128) return false;
    if (g.d_in % 16 != 0 || g.d_in < 16 * kFlWaves) return false;
    // fp32 operands at 128 samples: the operand fragments of two steps and the 32 accumulator tiles
    // do not fit the register file
    if (h->md.gemm != LC_GEMM_BF16 && S.Bp == 128) return false;
    return static_cast<int64_t>(S.G) * (g.d_out / kColChunk) >= 192;
}

// Backward pass and update of layer 1 for the step in slot train.cur_slot, and A_1 of the step in
// the next slot (which must have been gathered already).
hipError_t launch_first_layer(lc_handle* h) {
    const ActSet& S = h->train;
    const LayerGeom& g = h->layer[1];
    const bool bf16 = h->md.gemm == LC_GEMM_BF16;
    const size_t es = bf16 ? 2 : 4;
    const size_t slot_bytes = static_cast<size_t>(S.G) * S.Bp * g.dp_in * es;
    if (!first_layer_kernel_ok(h)) return hipErrorInvalidValue;
    if (S.cur_slot + 1 >= S.slots) return hipErrorInvalidValue;
    FirstArgs a;
    const StepBufs sb = plan_step_buffers(h, 1);
    a.X = sb.ox;
    a.V = sb.ov;
    a.x_stride = h->Ps;
    a.Xr = sb.xr;
    a.xr_stride = sb.xr_stride;
    a.Aux = sb.aux;
    a.aux_stride = sb.aux_stride;
    a.imp_in = sb.imp_in;
    a.inv_lr = 1.f / h->md.lr;
    a.shared_w = (sb.xr_stride == 0 && shared_weight_order(h, g)) ? shared_set(h, S.G) : 0;
    a.w_off = g.w_off;
    a.b_off = g.b_off;
    a.d_in = g.d_in;
    a.d_out = g.d_out;
    a.dp_in = g.dp_in;
    a.dp_out = g.dp_out;
    a.B = S.B;
    a.a_fm = static_cast<const char*>(S.a_fm[0]) + static_cast<size_t>(S.cur_slot) * slot_bytes;
    a.dz_fm = S.dz_fm[1];
    a.lr = h->md.lr;
    a.beta = effective_beta(h);
    a.wd = h->md.wd;
    a.an_bm = static_cast<const char*>(S.a_bm[0]) + static_cast<size_t>(S.cur_slot + 1) * slot_bytes;
    a.out_bm = S.a_bm[1];
    a.out_fm = S.a_fm[1];
    a.n_chunks = g.d_out / kColChunk;
    a.total_blocks = static_cast<int64_t>(S.G) * a.n_chunks;
    const unsigned grid = static_cast<unsigned>((a.total_blocks + kXcds - 1) / kXcds * kXcds);
    timing_start(h, kTimeBwd, 1, kBwdFirstLayer);
    const hipError_t e = bf16 ? launch_fl<bf16_t>(a, S.Bp / 16, h->stream_weights, grid, h->stream)
                              : launch_fl<float>(a, S.Bp / 16, h->stream_weights, grid, h->stream);
    timing_stop(h, kTimeBwd, 1, kBwdFirstLayer);
    if (e == hipSuccess) h->imp[1] = sb.next;
    return e;
}

}  // namespace lc
