// Local steps of small two-layer models with the weights resident on chip.
//
// Between two averaging steps a PASGD worker touches nothing but its own model (Sec. 2:
// tau local mini-batch SGD updates, then one averaging step).  When a replica's first layer,
// cut into slices of 16 hidden units, fits the LDS of the compute units, a whole run of local
// steps is one kernel launch: every workgroup loads its slice of W_1 (into LDS) and of the
// momentum V_1 (into registers) once, takes all the steps on them, and writes them back once.
// The streaming kernels need four launches per step and move W and V through the memory
// system in every one of them; at this size those launches, not the arithmetic, are the cost.
//
// Work split for a model d0 -> d1 -> d2 (d2 <= 16), replica g, workgroup cb of NB = dp1 / 16:
//   owns   hidden units C = [16 cb, 16 cb + 16): columns C of W_1, V_1, entries C of b_1, and the
//          matching ROWS C of W_2, V_2 -- every weight of the model has exactly one owner;
//   keeps  a private copy of b_2 (d2 values), updated identically by every workgroup.
// One step:
//   (1) A_1[:, C] = ReLU(A_0 W_1[:, C] + b_1[C])          MFMA; the 16 wavefronts split batch tiles and K
//   (2) this slice's share of the logits, A_1[:, C] W_2[C, :] (Bp x 16 values), handed to the
//       replica; replica-wide barrier
//   (3) Z_2 = sum of the NB shares in slice order + b_2, softmax cross-entropy, dZ_2
//       (redundantly in every workgroup: a few hundred values)
//   (4) dZ_1[:, C] = (dZ_2 W_2[C, :]^T) .* [A_1[:, C] > 0]  with the weights of before the update
//   (5) dW_2[C, :] = A_1[:, C]^T dZ_2, db_2 and their momentum updates
//   (6) dW_1[:, C] = A_0^T dZ_1[:, C], db_1[C] and the momentum update of the slice
// The only communication is the share of the logits (Bp x 16 values per workgroup and step),
// double buffered by step parity so that a fast workgroup never overwrites what a slow one still
// reads.  (Exchanging the logit shares instead of the activations is what lets W_2 be
// partitioned: with the activations exchanged every workgroup had to keep and update a full
// copy of W_2, and the second layer's products, done 16 times over, were a quarter of the step.)
//
// The barrier is a counter per replica in device memory: arrive with an agent-scope release,
// poll with relaxed loads, then an agent-scope acquire.  The shares are published with
// agent-scope (write-through) stores, so the release has no dirty cache lines to write back;
// the counters are never reset, each launch is told their value at its start.  All workgroups of a launch are
// co-resident (the launcher refuses grids above one workgroup per compute unit), and the
// poll loop is bounded: a workgroup that runs out of polls raises the error flag, stops
// waiting for good and finishes its steps, so the grid always drains.  (A cooperative launch
// would have the runtime vouch for the co-residency, but costs 18 us more per launch here, a
// tenth of the throughput at five steps per launch; the bounded wait covers the same case.)
// Where the block numbering puts all workgroups of a replica on one XCD, slices and counter stay
// in that XCD's L2 (arrive_and_wait_same_xcd).
//
// A launch may also hold several whole communication periods: after every `period` steps the
// averaging step of Sec. 2 is taken inside the kernel (average_resident), with one barrier over
// all workgroups of all replicas, always at agent scope.
#include "lc_internal.h"
#include "lc_mma.h"

namespace lc {

namespace {

constexpr int kResMaxD0 = 1024;   // padded input width the LDS slice is sized for
constexpr int kResMaxD1 = 256;    // padded hidden width (private W_2^T copy)
constexpr int kResK1P = kResMaxD0 + 4;
constexpr int kResK2P = kResMaxD1 + 4;
constexpr int kResWaves = 16;                    // wavefronts per workgroup: four per SIMD hide each other's waits
constexpr int kResThreads = kResWaves * 64;
constexpr int kResTiles = kResMaxD0 / 16 / kResWaves;   // 16-row tiles of W_1 per wavefront

struct ResArgs {
    float* X;
    float* V;
    int64_t x_stride;
    const float* Xr;      // where the weights are read at the start: X, or the one averaged model
    int64_t xr_stride;
    int64_t w1_off, b1_off, w2_off, b2_off;
    int d0, d1, d2, dp0, dp1;
    int B, G, NB;
    const void* a0_bm;    // [slots][G][Bp][dp0] of OT
    const void* a0_fm;    // [slots][G][dp0][Bp] of OT
    int64_t a0_slot;      // elements per slot
    const int32_t* labels;  // [slots][G][Bp]
    int slot0, n_steps;
    float lr, beta_first, beta, wd;
    int vec;              // rows of W_1 may be accessed 16 bytes at a time
    float* zx;            // [2][G][NB][Bp][16] exchange buffer: the slices' shares of the logits, by step parity
    unsigned* ctr;        // [G] arrivals since attach (every workgroup arrives once per step, whatever happens)
    unsigned ctr_base;    // their value when this launch starts
    unsigned* err;        // set to 1 when a barrier wait ran out of polls
    int spin_limit;       // polls one barrier wait may take
    float* loss;          // [G][kLossParts], slot 0 written
    int local_xcd;        // every replica's workgroups share one XCD (one L2): exchange through that L2
    unsigned xcc_of;      // 4 bits per residue of the hardware block id mod 8: the XCD such blocks run on
    int period;           // averaging step after every `period` steps inside the launch; 0: none
    float* avx;           // [2][G][x_stride] models handed over at an averaging step, by parity of the period
    unsigned* gctr;       // arrivals of all workgroups at averaging steps since attach
    unsigned gctr_base;   // its value when this launch starts
};

// Barrier among the workgroups that add to *ctr, called by one thread per workgroup after a
// workgroup barrier: what the workgroup wrote before is visible to every workgroup that leaves
// the wait.  The wait is bounded; a workgroup that runs out of polls raises the error flag and
// never waits again (it still arrives, so the counts stay right), so the grid always drains.
__device__ __forceinline__ void arrive_and_wait(unsigned* ctr, unsigned target, int spin_limit, unsigned* err,
                                                bool& gave_up) {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
    __hip_atomic_fetch_add(ctr, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    int polls = 0;
    while (!gave_up) {
        if (polls++ >= spin_limit) {   // a limit of 0 gives up without looking: the host's way to force this path
            gave_up = true;
            atomicOr(err, 1u);
            break;
        }
        const unsigned seen = __hip_atomic_load(ctr, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (static_cast<int>(seen - target) >= 0) break;
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
}

// The same barrier for workgroups that all run on one XCD, i.e. behind one L2: counter and data
// need not leave that L2.  Read-modify-write atomics without the device-scope bit are performed
// in the L2, so the counter is added to and polled there (the poll is a compare-and-swap that
// never matches: a workgroup-scope LOAD may be served by the compute unit's L1 and then never sees
// the count move -- measured).  The slices were written through to the L2 and stay there as
// dirty lines; after the L1 has been invalidated (the agent-scope acquire does that) loads find
// them in the L2, where the agent-scope form sends data and counter to the memory side and
// back.  Valid only while the participants really share an L2: the launcher checks the placement
// rule once with a probe kernel, and every workgroup checks its own XCD id against it.
__device__ __forceinline__ void arrive_and_wait_same_xcd(unsigned* ctr, unsigned target, int spin_limit, unsigned* err,
                                                         bool& gave_up) {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __hip_atomic_fetch_add(ctr, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    int polls = 0;
    while (!gave_up) {
        if (polls++ >= spin_limit) {
            gave_up = true;
            atomicOr(err, 1u);
            break;
        }
        unsigned seen = 0xFFFFFFFFu;   // (were the count ever this, the swap would write the same value back)
        __hip_atomic_compare_exchange_strong(ctr, &seen, 0xFFFFFFFFu, __ATOMIC_RELAXED, __ATOMIC_RELAXED,
                                             __HIP_MEMORY_SCOPE_WORKGROUP);
        if (static_cast<int>(seen - target) >= 0) break;
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
}

// The XCD this wavefront runs on: hardware register XCC_ID (number 20), bits 3:0.  The operand
// of s_getreg is (size - 1) << 11 | offset << 6 | register.
__device__ __forceinline__ unsigned this_xcd() { return __builtin_amdgcn_s_getreg(((4 - 1) << 11) | (0 << 6) | 20); }

__global__ void xcd_probe_kernel(unsigned* out) {
    if (threadIdx.x == 0) out[blockIdx.x] = this_xcd();
}

// x_bar = (1/m) sum_i x^(i) of one entry (Sec. 2, the averaging step), summed in double in
// replica order and rounded once: the same arithmetic, bit for bit, as the averaging kernels.
__device__ __forceinline__ float mean_of_replicas(const float* p, int64_t stride, int G) {
    double s = 0.0;
    for (int i0 = 0; i0 < G; i0 += 4) {   // four loads in flight, added in replica order
        float r[4];
#pragma unroll
        for (int u = 0; u < 4; ++u)
            if (i0 + u < G) r[u] = p[(i0 + u) * stride];
#pragma unroll
        for (int u = 0; u < 4; ++u)
            if (i0 + u < G) s += static_cast<double>(r[u]);
    }
    return static_cast<float>(s / static_cast<double>(G));
}

__device__ __forceinline__ float round_operand(float x, bf16_t) { return static_cast<float>(static_cast<bf16_t>(x)); }
__device__ __forceinline__ float round_operand(float x, float) { return x; }

// The averaging step inside a resident launch (Sec. 2: after tau local updates the models are
// replaced by their mean; the momentum buffers stay local).  Every workgroup hands over its part
// of the model, waits for all workgroups of all replicas, and forms the mean of its own part from
// the m copies.  Two buffers, by parity of the period: a workgroup overwrites a buffer only after
// the barrier of the period in between, which every reader of the older contents has reached by
// then.
__device__ __forceinline__ void average_resident(const ResArgs& a, int tid, int pi, int g, int cb,
                                                 float (*w1s)[kResK1P], float (*w2s)[17], float* b1s,
                                                 float* b2s, bool& gave_up) {
    const int wave = tid >> 6, j = tid & 15, q = (tid >> 4) & 3;
    const int c_base = 16 * cb, n_kt = a.dp0 / 16;
    const bool vec = a.vec != 0;
    float* all = a.avx + static_cast<int64_t>(pi & 1) * a.G * a.x_stride;
    float* mine = all + g * a.x_stride;
    for (int kt = wave; kt < n_kt; kt += kResWaves) {
        const int k = 16 * kt + j, c = c_base + 4 * q;
        if (k < a.d0) {
            const float4 w = make_float4(w1s[4 * q + 0][k], w1s[4 * q + 1][k], w1s[4 * q + 2][k], w1s[4 * q + 3][k]);
            store_w4(mine + a.w1_off + static_cast<int64_t>(k) * a.d1, c, a.d1, vec, false, w);
        }
    }
    if (tid < 16 && c_base + tid < a.d1) mine[a.b1_off + c_base + tid] = b1s[tid];
    if (tid >= 64 && tid < 320) {   // own rows of the second layer
        const int kk = (tid - 64) >> 4, c2 = tid & 15;
        if (c_base + kk < a.d1 && c2 < a.d2) mine[a.w2_off + static_cast<int64_t>(c_base + kk) * a.d2 + c2] = w2s[c2][kk];
    }
    if (cb == 0 && tid < a.d2) mine[a.b2_off + tid] = b2s[tid];
    __builtin_amdgcn_s_waitcnt(0);   // this wavefront's stores have left before the workgroup arrives
    __syncthreads();
    if (tid == 0)
        arrive_and_wait(a.gctr, a.gctr_base + static_cast<unsigned>(pi + 1) * static_cast<unsigned>(a.G * a.NB),
                        a.spin_limit, a.err, gave_up);
    __syncthreads();
    for (int kt = wave; kt < n_kt; kt += kResWaves) {
        const int k = 16 * kt + j, c = c_base + 4 * q;
        if (k < a.d0) {
            const float* src = all + a.w1_off + static_cast<int64_t>(k) * a.d1;
            double s0 = 0, s1 = 0, s2 = 0, s3 = 0;
            for (int g0 = 0; g0 < a.G; g0 += 8) {
                float4 r[8];
#pragma unroll
                for (int u = 0; u < 8; ++u)
                    if (g0 + u < a.G) r[u] = load_w4(src + (g0 + u) * a.x_stride, c, a.d1, vec, false);
#pragma unroll
                for (int u = 0; u < 8; ++u)
                    if (g0 + u < a.G) {
                        s0 += static_cast<double>(r[u].x);
                        s1 += static_cast<double>(r[u].y);
                        s2 += static_cast<double>(r[u].z);
                        s3 += static_cast<double>(r[u].w);
                    }
            }
            const double dm = static_cast<double>(a.G);
            w1s[4 * q + 0][k] = static_cast<float>(s0 / dm);
            w1s[4 * q + 1][k] = static_cast<float>(s1 / dm);
            w1s[4 * q + 2][k] = static_cast<float>(s2 / dm);
            w1s[4 * q + 3][k] = static_cast<float>(s3 / dm);
        }
    }
    // the second layer and the biases, an entry at a time (its m loads together): this phase must
    // stay light in registers, the step loop around it has none to spare
    if (tid >= 128 && tid < 384) {
        const int kk = (tid - 128) >> 4, c2 = tid & 15;
        if (c_base + kk < a.d1 && c2 < a.d2)
            w2s[c2][kk] = mean_of_replicas(all + a.w2_off + static_cast<int64_t>(c_base + kk) * a.d2 + c2, a.x_stride, a.G);
    }
    if (tid < 16 && c_base + tid < a.d1) b1s[tid] = mean_of_replicas(all + a.b1_off + c_base + tid, a.x_stride, a.G);
    if (tid >= 64 && tid < 64 + a.d2) b2s[tid - 64] = mean_of_replicas(all + a.b2_off + tid - 64, a.x_stride, a.G);
    __syncthreads();
}

template <typename OT, int MT>
__global__ __launch_bounds__(kResThreads) void resident_kernel(ResArgs a) {
    constexpr int Bp = 16 * MT;
    constexpr int NS = Bp / 32;   // 32-wide steps over the batch
    constexpr int KP = kResWaves / MT;   // wavefronts that share one batch tile and split the reduction
    __shared__ __attribute__((aligned(16))) float w1s[16][kResK1P];    // W_1[:, C]^T
    __shared__ float w2s[16][17], v2s[16][17];                          // W_2[C, :]^T, V_2[C, :]^T: [class][own hidden unit]
    __shared__ __attribute__((aligned(16))) float part[KP][Bp][17];
    __shared__ float a1s[Bp][17];                                       // own slice of A_1
    __shared__ float z2s[Bp][17];                                       // logits, then dZ_2
    __shared__ __attribute__((aligned(16))) OT dz1t[16][Bp + 8];        // dZ_1[:, C]^T
    __shared__ float b1s[16], vb1s[16], b2s[16], vb2s[16];
    __shared__ float lred[Bp];
    __shared__ float colsum1[kResWaves][16], colsum2[kResWaves][16];

    const int64_t logical = xcd_logical_block(static_cast<int64_t>(a.G) * a.NB);
    if (logical < 0) return;
    const int g = static_cast<int>(logical / a.NB), cb = static_cast<int>(logical % a.NB);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int j = lane & 15, q = lane >> 4;
    const int c_base = 16 * cb;
    const int n_kt = a.dp0 / 16;
    const bool vec = a.vec != 0;

    float* Xg = a.X + g * a.x_stride;
    float* Vg = a.V + g * a.x_stride;
    const float* Xrg = a.Xr + g * a.xr_stride;
    // ---- load the resident state
    f32x4 v1[kResTiles];   // V_1 at rows 16 kt + j, columns c_base + 4 q .. + 3, kt = wave + 16 i
    {
        // all tiles' loads first, with no branch around them (rows that do not exist read the last
        // row and are zeroed): one memory round trip instead of one per tile
        float4 wl[kResTiles], vl[kResTiles];
        if (vec && c_base + 16 <= a.d1) {   // the whole slice exists and is aligned (uniform over the workgroup)
#pragma unroll
            for (int i = 0; i < kResTiles; ++i) {
                const int k = 16 * (wave + kResWaves * i) + j, kc = k < a.d0 ? k : a.d0 - 1;
                const int64_t at = a.w1_off + static_cast<int64_t>(kc) * a.d1 + c_base + 4 * q;
                wl[i] = *reinterpret_cast<const float4*>(Xrg + at);
                vl[i] = *reinterpret_cast<const float4*>(Vg + at);
            }
        } else {
#pragma unroll
            for (int i = 0; i < kResTiles; ++i) {
                const int k = 16 * (wave + kResWaves * i) + j, kc = k < a.d0 ? k : a.d0 - 1;
                wl[i] = load_w4(Xrg + a.w1_off + static_cast<int64_t>(kc) * a.d1, c_base + 4 * q, a.d1, vec, false);
                vl[i] = load_w4(Vg + a.w1_off + static_cast<int64_t>(kc) * a.d1, c_base + 4 * q, a.d1, vec, false);
            }
        }
#pragma unroll
        for (int i = 0; i < kResTiles; ++i) {
            const int kt = wave + kResWaves * i, k = 16 * kt + j;
            const bool in = k < a.d0;
            v1[i] = in ? f32x4{vl[i].x, vl[i].y, vl[i].z, vl[i].w} : f32x4{0.f, 0.f, 0.f, 0.f};
            if (kt < n_kt) {
                w1s[4 * q + 0][k] = in ? wl[i].x : 0.f;
                w1s[4 * q + 1][k] = in ? wl[i].y : 0.f;
                w1s[4 * q + 2][k] = in ? wl[i].z : 0.f;
                w1s[4 * q + 3][k] = in ? wl[i].w : 0.f;
            }
        }
    }
    if (tid < 256) {   // own rows of the second layer
        const int kk = tid >> 4, c2 = tid & 15;
        const bool in = c_base + kk < a.d1 && c2 < a.d2;
        const int64_t at = a.w2_off + (in ? static_cast<int64_t>(c_base + kk) * a.d2 + c2 : 0);
        const float w = Xrg[at], v = Vg[at];
        w2s[c2][kk] = in ? w : 0.f;
        v2s[c2][kk] = in ? v : 0.f;
    }
    if (tid < 16) {
        const bool in1 = c_base + tid < a.d1, in2 = tid < a.d2;
        b1s[tid] = in1 ? Xrg[a.b1_off + c_base + tid] : 0.f;
        vb1s[tid] = in1 ? Vg[a.b1_off + c_base + tid] : 0.f;
        b2s[tid] = in2 ? Xrg[a.b2_off + tid] : 0.f;
        vb2s[tid] = in2 ? Vg[a.b2_off + tid] : 0.f;
    }
    __syncthreads();
    bool gave_up = false;   // thread 0: a barrier wait ran out of polls
    if (a.local_xcd && threadIdx.x == 0 && this_xcd() != ((a.xcc_of >> (4 * (blockIdx.x % kXcds))) & 15u))
        atomicOr(a.err, 2u);   // not where the probe saw such blocks run: the exchange cannot be trusted
    for (int s = 0; s < a.n_steps;) {
    // One period (the whole launch when it has no averaging steps).  What the steps derive from
    // the thread's id is derived afresh from an opaque copy per period, so that none of it is
    // held in registers across the averaging step, which needs them for its own loads.
    int tid_p = threadIdx.x;
    asm volatile("" : "+v"(tid_p));
    const int tid = tid_p, lane = tid & 63, wave = tid >> 6, j = lane & 15, q = lane >> 4;
    const int s_end = a.period > 0 ? s + a.period : a.n_steps;
    for (; s < s_end; ++s) {
        const float beta = s == 0 ? a.beta_first : a.beta;
        const int slot = a.slot0 + s;
        const OT* A0 = static_cast<const OT*>(a.a0_bm) + slot * a.a0_slot + static_cast<int64_t>(g) * Bp * a.dp0;
        const OT* A0T = static_cast<const OT*>(a.a0_fm) + slot * a.a0_slot + static_cast<int64_t>(g) * a.dp0 * Bp;
        const int32_t* lab = a.labels + (static_cast<int64_t>(slot) * a.G + g) * Bp;
        const int par = s & 1;
        float* xp = a.zx + (static_cast<int64_t>(par) * a.G + g) * Bp * a.dp1;   // [NB][Bp][16]
        // ---- (1) Z_1[:, C]: wavefront (mt, kpart) takes batch tile mt and the 32-wide k steps
        //      kpart, kpart + KP, ...
        const int mt = wave % MT, kpart = wave / MT;
        {
            f32x4 acc = f32x4{0.f, 0.f, 0.f, 0.f};
            const OT* arow = A0 + static_cast<int64_t>(16 * mt + j) * a.dp0 + 8 * q;
            const int n_st = (a.d0 + 31) / 32;   // (steps that hold only padding rows are skipped)
            Frag<OT> af = load8(arow + 32 * (kpart < n_st ? kpart : 0));
            for (int st = kpart; st < n_st; st += KP) {
                const int k0 = 32 * st + 8 * q;
                const int nx = st + KP < n_st ? st + KP : st;
                const Frag<OT> af_next = load8(arow + 32 * nx);   // next step's operand in flight
                const float4 x0 = *reinterpret_cast<const float4*>(&w1s[j][k0]);
                const float4 x1 = *reinterpret_cast<const float4*>(&w1s[j][k0 + 4]);
                const float x[8] = {x0.x, x0.y, x0.z, x0.w, x1.x, x1.y, x1.z, x1.w};
                Frag<OT> bf;
                pack8(bf, x);
                acc = mma8(af, bf, acc);
                af = af_next;
            }
#pragma unroll
            for (int r = 0; r < 4; ++r) part[kpart][16 * mt + 4 * q + r][j] = acc[r];
        }
        __syncthreads();
        for (int e = tid; e < Bp * 16; e += kResThreads) {
            const int b = e / 16, c = e % 16;
            float z = part[0][b][c];
#pragma unroll
            for (int p = 1; p < KP; ++p) z += part[p][b][c];
            z += b1s[c];
            float act = 0.f;
            if (b < a.B && c_base + c < a.d1) act = round_operand(z > 0.f ? z : 0.f, OT());
            a1s[b][c] = act;
        }
        __syncthreads();
        // ---- (2) this slice's share of the logits, A_1[:, C] W_2[C, :], handed to the replica
        if (tid < Bp * 16) {
            const int b = tid >> 4, c2 = tid & 15;
            float zp = 0.f;
#pragma unroll
            for (int kk = 0; kk < 16; ++kk) zp += a1s[b][kk] * round_operand(w2s[c2][kk], OT());
            float* px = xp + static_cast<int64_t>(cb) * (Bp * 16) + tid;
            if (a.local_xcd) __hip_atomic_store(px, zp, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);   // as far as the XCD's L2
            else __hip_atomic_store(px, zp, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // written through to device scope
        }
        // every wavefront's stores have arrived before the workgroup does
        __builtin_amdgcn_s_waitcnt(0);

        // ---- (2) replica-wide barrier
        __syncthreads();
        if (tid == 0 && a.NB > 1) {
            const unsigned target = a.ctr_base + static_cast<unsigned>(s + 1) * static_cast<unsigned>(a.NB);
            if (a.local_xcd) arrive_and_wait_same_xcd(&a.ctr[g], target, a.spin_limit, a.err, gave_up);
            else arrive_and_wait(&a.ctr[g], target, a.spin_limit, a.err, gave_up);
        }
        __syncthreads();
        // ---- (3) logits = sum of the slices' shares in slice order + b_2; softmax cross-entropy and
        //      dZ_2 (redundantly in every workgroup: a few hundred values)
        // one thread per (sample, class): 16-lane groups hold a sample's logits
        if (tid < Bp * 16) {
            const int b = tid >> 4, c = tid & 15;
            float z = 0.f;
            for (int o0 = 0; o0 < a.NB; o0 += 8) {   // eight loads in flight, added in slice order
                float r[8];
#pragma unroll
                for (int u = 0; u < 8; ++u)
                    if (o0 + u < a.NB) r[u] = xp[static_cast<int64_t>(o0 + u) * (Bp * 16) + tid];
#pragma unroll
                for (int u = 0; u < 8; ++u)
                    if (o0 + u < a.NB) z += r[u];
            }
            z += b2s[c];
            const int y = b < a.B ? lab[b] : -1;
            const bool valid = c < a.d2;
            float zmax = valid ? z : -INFINITY;
#pragma unroll
            for (int o = 8; o > 0; o >>= 1) zmax = fmaxf(zmax, __shfl_xor(zmax, o, 16));
            const float ex = valid ? expf(z - zmax) : 0.f;
            float s_other = c == y ? 0.f : ex;   // over the classes other than the label (see xent_loss)
#pragma unroll
            for (int o = 8; o > 0; o >>= 1) s_other += __shfl_xor(s_other, o, 16);
            const float zy = __shfl(z, y >= 0 ? y : 0, 16), sum = s_other + __shfl(ex, y >= 0 ? y : 0, 16);
            float dz = 0.f;
            if (y >= 0 && valid)
                dz = round_operand(xent_delta(ex, c == y, s_other, 1.f / sum) * (1.f / static_cast<float>(a.B)), OT());
            z2s[b][c] = dz;
            // (the step's own loss is a by-product here: the plain form, without the log1p of xent_loss)
            if (c == 0) lred[b] = y >= 0 ? -(zy - zmax - logf(sum)) : 0.f;
        }
        __syncthreads();
        if (cb == 0 && wave == 0) {
            float v = lane < Bp ? lred[lane] : 0.f;
#pragma unroll
            for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
            if (lane == 0) a.loss[static_cast<int64_t>(g) * kLossParts] = v / static_cast<float>(a.B);
        }
        // ---- (4) dZ_1[:, C] from the second layer's weights of before this step's update, and the
        //      column sums of dZ_1[:, C] and dZ_2 (bias gradients): first over each wavefront's
        //      four samples, then over the wavefronts
        if (tid < Bp * 16) {
            const int b = tid >> 4, c = tid & 15;
            float sum = 0.f;
            for (int c2 = 0; c2 < a.d2; ++c2) sum += z2s[b][c2] * round_operand(w2s[c2][c], OT());
            const OT d = static_cast<OT>(a1s[b][c] > 0.f ? sum : 0.f);   // rounds in bf16 mode
            dz1t[c][b] = d;
            float s1 = to_f32(d), s2 = z2s[b][c];
            s1 += __shfl_xor(s1, 16, 64); s1 += __shfl_xor(s1, 32, 64);
            s2 += __shfl_xor(s2, 16, 64); s2 += __shfl_xor(s2, 32, 64);
            if (lane < 16) {
                colsum1[wave][lane] = s1;
                colsum2[wave][lane] = s2;
            }
        }
        __syncthreads();
        // ---- bias updates (one thread per entry).  These small jobs go to the last wavefronts:
        //      when the tiles of step (6) do not divide evenly, those have one tile less to do
        if (tid >= kResThreads - 64 && tid < kResThreads - 32) {
            const int c = tid & 15;
            const bool first = tid < kResThreads - 48;
            float db = 0.f;
            for (int w = 0; w < Bp / 4; ++w) db += first ? colsum1[w][c] : colsum2[w][c];
            if (first) {
                if (c_base + c < a.d1) {
                    const float vb = momentum_update(beta, vb1s[c], db, a.wd, b1s[c]);
                    vb1s[c] = vb;
                    b1s[c] = weight_update(b1s[c], a.lr, vb);
                }
            } else if (c < a.d2) {
                const float vb = momentum_update(beta, vb2s[c], db, a.wd, b2s[c]);
                vb2s[c] = vb;
                b2s[c] = weight_update(b2s[c], a.lr, vb);
            }
        }
        // ---- (5) dW_2[C, :] = A_1[:, C]^T dZ_2 and the update of the own rows (16 x 16 values: plain FMAs)
        if (tid >= kResThreads - 320 && tid < kResThreads - 64) {
            const int kk = (tid - (kResThreads - 320)) >> 4, c2 = tid & 15;
            if (c_base + kk < a.d1 && c2 < a.d2) {
                float gw = 0.f;
                for (int b = 0; b < Bp; ++b) gw += a1s[b][kk] * z2s[b][c2];
                const float w = w2s[c2][kk];
                const float v = momentum_update(beta, v2s[c2][kk], gw, a.wd, w);
                v2s[c2][kk] = v;
                w2s[c2][kk] = weight_update(w, a.lr, v);
            }
        }
        // ---- (6) dW_1[:, C] = A_0^T dZ_1[:, C] and the update of the slice
#pragma unroll
        for (int i = 0; i < kResTiles; ++i) {
            const int kt = wave + kResWaves * i;
            if (16 * kt < a.d0) {   // (tiles that hold only padding rows have nothing to update)
                f32x4 acc = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int st = 0; st < NS; ++st) {
                    const int b0 = 32 * st + 8 * q;
                    const Frag<OT> af = *reinterpret_cast<const Frag<OT>*>(&dz1t[j][b0]);
                    const Frag<OT> bf = load8(A0T + static_cast<int64_t>(16 * kt + j) * Bp + b0);
                    acc = mma8(af, bf, acc);
                }
                const int k = 16 * kt + j;
                // rows k >= d0 and columns beyond d1 have zero gradient, weight and momentum,
                // and stay zero under the update
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const float w = w1s[4 * q + r][k];
                    const float v = momentum_update(beta, v1[i][r], acc[r], a.wd, w);
                    v1[i][r] = v;
                    w1s[4 * q + r][k] = weight_update(w, a.lr, v);
                }
            }
        }
        __syncthreads();
    }
    if (a.period > 0) average_resident(a, tid, s / a.period - 1, g, cb, w1s, w2s, b1s, b2s, gave_up);
    }

    // ---- write the state back
#pragma unroll
    for (int i = 0; i < kResTiles; ++i) {
        const int kt = wave + kResWaves * i;
        if (kt < n_kt) {
            const int k = 16 * kt + j, c = c_base + 4 * q;
            if (k < a.d0) {
                const float4 w = make_float4(w1s[4 * q + 0][k], w1s[4 * q + 1][k], w1s[4 * q + 2][k], w1s[4 * q + 3][k]);
                const float4 v = make_float4(v1[i][0], v1[i][1], v1[i][2], v1[i][3]);
                store_w4(Xg + a.w1_off + static_cast<int64_t>(k) * a.d1, c, a.d1, vec, false, w);
                store_w4(Vg + a.w1_off + static_cast<int64_t>(k) * a.d1, c, a.d1, vec, false, v);
            }
        }
    }
    if (tid < 16 && c_base + tid < a.d1) {
        Xg[a.b1_off + c_base + tid] = b1s[tid];
        Vg[a.b1_off + c_base + tid] = vb1s[tid];
    }
    if (tid >= 64 && tid < 320) {   // own rows of the second layer
        const int kk = (tid - 64) >> 4, c2 = tid & 15;
        if (c_base + kk < a.d1 && c2 < a.d2) {
            const int64_t at = a.w2_off + static_cast<int64_t>(c_base + kk) * a.d2 + c2;
            Xg[at] = w2s[c2][kk];
            Vg[at] = v2s[c2][kk];
        }
    }
    if (cb == 0 && tid < a.d2) {
        Xg[a.b2_off + tid] = b2s[tid];
        Vg[a.b2_off + tid] = vb2s[tid];
    }
}

// Softmax regression (one layer, d0 -> d1 with d1 <= 16 classes): the same idea without any
// exchange.  One workgroup per replica keeps W^T, V^T and the bias in LDS for all the steps of a
// launch; a step is logits (reduction split over the wavefronts), softmax cross-entropy, and
// dW = A_0^T dZ with the momentum update applied in place.
struct Res1Args {
    float* X;
    float* V;
    int64_t x_stride;
    const float* Xr;
    int64_t xr_stride;
    int64_t w_off, b_off;
    int d0, d1, dp0;
    int B, G;
    const void* a0_bm;      // [slots][G][Bp][dp0] of OT
    const void* a0_fm;      // [slots][G][dp0][Bp] of OT
    int64_t a0_slot;
    const int32_t* labels;  // [slots][G][Bp]
    int slot0, n_steps;
    float lr, beta_first, beta, wd;
    float* loss;            // [G][kLossParts], slot 0 written
    int period;             // averaging step after every `period` steps inside the launch; 0: none
    float* avx;             // [2][G][x_stride] models handed over at an averaging step
    unsigned* gctr;         // arrivals at averaging steps since attach
    unsigned gctr_base;
    unsigned* err;
    int spin_limit;
};

template <typename OT, int MT>
__global__ __launch_bounds__(kResThreads) void resident1_kernel(Res1Args a) {
    constexpr int Bp = 16 * MT;
    constexpr int NS = Bp / 32;
    constexpr int KP = kResWaves / MT;
    __shared__ __attribute__((aligned(16))) float ws[16][kResK2P];    // W^T (row = class)
    __shared__ __attribute__((aligned(16))) float vs[16][kResK2P];
    __shared__ __attribute__((aligned(16))) float part[KP][Bp][17];
    __shared__ float zs[Bp][17];                                       // dZ
    __shared__ __attribute__((aligned(16))) OT dzt[16][Bp + 8];        // dZ^T
    __shared__ float bs[16], vbs[16];
    __shared__ float lred[Bp];
    __shared__ float colsum[kResWaves][16];

    const int g = blockIdx.x;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int j = lane & 15, q = lane >> 4;
    float* Xg = a.X + g * a.x_stride;
    float* Vg = a.V + g * a.x_stride;
    const float* Xrg = a.Xr + g * a.xr_stride;

    for (int e = tid; e < 16 * a.dp0; e += kResThreads) {
        const int k = e / 16, c = e % 16;
        const bool in = k < a.d0 && c < a.d1;
        ws[c][k] = in ? Xrg[a.w_off + static_cast<int64_t>(k) * a.d1 + c] : 0.f;
        vs[c][k] = in ? Vg[a.w_off + static_cast<int64_t>(k) * a.d1 + c] : 0.f;
    }
    if (tid < 16) {
        bs[tid] = tid < a.d1 ? Xrg[a.b_off + tid] : 0.f;
        vbs[tid] = tid < a.d1 ? Vg[a.b_off + tid] : 0.f;
    }
    __syncthreads();

    const int mt = wave % MT, kpart = wave / MT;
    bool gave_up = false;   // thread 0: a barrier wait ran out of polls
    for (int s = 0; s < a.n_steps; ++s) {
        const float beta = s == 0 ? a.beta_first : a.beta;
        const int slot = a.slot0 + s;
        const OT* A0 = static_cast<const OT*>(a.a0_bm) + slot * a.a0_slot + static_cast<int64_t>(g) * Bp * a.dp0;
        const OT* A0T = static_cast<const OT*>(a.a0_fm) + slot * a.a0_slot + static_cast<int64_t>(g) * a.dp0 * Bp;
        const int32_t* lab = a.labels + (static_cast<int64_t>(slot) * a.G + g) * Bp;

        // ---- logits, partial over this wavefront's share of d0
        {
            f32x4 z = f32x4{0.f, 0.f, 0.f, 0.f};
            const OT* arow = A0 + static_cast<int64_t>(16 * mt + j) * a.dp0 + 8 * q;
            for (int st = kpart; st < a.dp0 / 32; st += KP) {
                const int k0 = 32 * st + 8 * q;
                const Frag<OT> af = load8(arow + 32 * st);
                const float4 x0 = *reinterpret_cast<const float4*>(&ws[j][k0]);
                const float4 x1 = *reinterpret_cast<const float4*>(&ws[j][k0 + 4]);
                const float x[8] = {x0.x, x0.y, x0.z, x0.w, x1.x, x1.y, x1.z, x1.w};
                Frag<OT> bf;
                pack8(bf, x);
                z = mma8(af, bf, z);
            }
#pragma unroll
            for (int r = 0; r < 4; ++r) part[kpart][16 * mt + 4 * q + r][j] = z[r];
        }
        __syncthreads();
        // ---- softmax cross-entropy and dZ, one thread per (sample, class); column sums of dZ
        if (tid < Bp * 16) {
            const int b = tid >> 4, c = tid & 15;
            float z = part[0][b][c];
#pragma unroll
            for (int p = 1; p < KP; ++p) z += part[p][b][c];
            z += bs[c];
            const int y = b < a.B ? lab[b] : -1;
            const bool valid = c < a.d1;
            float zmax = valid ? z : -INFINITY;
#pragma unroll
            for (int o = 8; o > 0; o >>= 1) zmax = fmaxf(zmax, __shfl_xor(zmax, o, 16));
            const float ex = valid ? expf(z - zmax) : 0.f;
            float s_other = c == y ? 0.f : ex;   // over the classes other than the label (see xent_loss)
#pragma unroll
            for (int o = 8; o > 0; o >>= 1) s_other += __shfl_xor(s_other, o, 16);
            const float zy = __shfl(z, y >= 0 ? y : 0, 16), sum = s_other + __shfl(ex, y >= 0 ? y : 0, 16);
            float dz = 0.f;
            if (y >= 0 && valid)
                dz = round_operand(xent_delta(ex, c == y, s_other, 1.f / sum) * (1.f / static_cast<float>(a.B)), OT());
            zs[b][c] = dz;
            dzt[c][b] = static_cast<OT>(dz);
            if (c == 0) lred[b] = y >= 0 ? -(zy - zmax - logf(sum)) : 0.f;
            float cs = dz;
            cs += __shfl_xor(cs, 16, 64);
            cs += __shfl_xor(cs, 32, 64);
            if (lane < 16) colsum[wave][lane] = cs;
        }
        __syncthreads();
        if (wave == 0) {
            float v = lane < Bp ? lred[lane] : 0.f;
#pragma unroll
            for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
            if (lane == 0) a.loss[static_cast<int64_t>(g) * kLossParts] = v / static_cast<float>(a.B);
        } else if (wave == 1 && lane < a.d1) {
            float db = 0.f;
            for (int w = 0; w < Bp / 4; ++w) db += colsum[w][lane];
            const float vb = momentum_update(beta, vbs[lane], db, a.wd, bs[lane]);
            vbs[lane] = vb;
            bs[lane] = weight_update(bs[lane], a.lr, vb);
        }
        // ---- dW = A_0^T dZ and the update; tile kt = 16 rows of W
        for (int kt = wave; kt < a.dp0 / 16; kt += kResWaves) {
            f32x4 acc = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int st = 0; st < NS; ++st) {
                const int b0 = 32 * st + 8 * q;
                const Frag<OT> af = load8(A0T + static_cast<int64_t>(16 * kt + j) * Bp + b0);
                const Frag<OT> bf = *reinterpret_cast<const Frag<OT>*>(&dzt[j][b0]);
                acc = mma8(af, bf, acc);
            }
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int k = 16 * kt + 4 * q + r;
                if (k < a.d0 && j < a.d1) {
                    const float w = ws[j][k];
                    const float v = momentum_update(beta, vs[j][k], acc[r], a.wd, w);
                    vs[j][k] = v;
                    ws[j][k] = weight_update(w, a.lr, v);
                }
            }
        }
        __syncthreads();
        if (a.period == 0 || (s + 1) % a.period != 0) continue;
        // ---- averaging step, as in the two-layer kernel: hand over the model, wait for all
        //      replicas, take the mean of the m copies
        const int pi = (s + 1) / a.period - 1;
        float* all = a.avx + static_cast<int64_t>(pi & 1) * a.G * a.x_stride;
        float* mine = all + g * a.x_stride;
        for (int e = tid; e < a.d0 * a.d1; e += kResThreads) mine[a.w_off + e] = ws[e % a.d1][e / a.d1];
        if (tid < a.d1) mine[a.b_off + tid] = bs[tid];
        __builtin_amdgcn_s_waitcnt(0);   // this wavefront's stores have left before the workgroup arrives
        __syncthreads();
        if (tid == 0)
            arrive_and_wait(a.gctr, a.gctr_base + static_cast<unsigned>(pi + 1) * static_cast<unsigned>(a.G),
                            a.spin_limit, a.err, gave_up);
        __syncthreads();
        for (int e = tid; e < a.d0 * a.d1; e += kResThreads)
            ws[e % a.d1][e / a.d1] = mean_of_replicas(all + a.w_off + e, a.x_stride, a.G);
        if (tid < a.d1) bs[tid] = mean_of_replicas(all + a.b_off + tid, a.x_stride, a.G);
        __syncthreads();
    }

    for (int e = tid; e < a.d0 * a.d1; e += kResThreads) {
        const int k = e / a.d1, c = e % a.d1;
        Xg[a.w_off + e] = ws[c][k];
        Vg[a.w_off + e] = vs[c][k];
    }
    if (tid < a.d1) {
        Xg[a.b_off + tid] = bs[tid];
        Vg[a.b_off + tid] = vbs[tid];
    }
}

}  // namespace

size_t resident_exchange_floats(const lc_handle* h) {
    // two step parities x (replicas x padded batch x padded hidden width); the single-layer form
    // exchanges nothing (a token amount keeps the buffer pointer non-null)
    if (h->L == 1) return 64;
    return 2 * static_cast<size_t>(h->m) * h->train.Bp * h->layer[1].dp_out;
}

// Workgroups of the resident kernel that can be on the chip at the same time: one per compute unit
// (16 wavefronts and 66 KB and more of LDS each) of the current device -- 256 on the MI355X this is
// written for, fewer on a partition of it.  Without a device (host-only use of the library) the
// full chip is assumed; the kernel's bounded barrier wait remains the last line of defence.
static int resident_workgroup_budget() {
    static const int budget = [] {
        int dev = 0, cus = 0;
        if (hipGetDevice(&dev) != hipSuccess) return 256;
        if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1) return 256;
        return cus < 256 ? cus : 256;   // (the exchange buffers and counters are sized for 256)
    }();
    return budget;
}

// Two layers, at most 16 classes and 64 samples, widths within the LDS budget, and few enough
// workgroups that all of them are on the chip at the same time (one per compute unit); or one
// layer of at most 256 (padded) inputs and 16 classes.
bool resident_shape_ok(const lc_handle* h) {
    if (h->md.kind != LC_KIND_MLP || h->md.B > 64) return false;
    if (h->L == 1) return h->layer[1].d_out <= 16 && h->layer[1].dp_in <= kResMaxD1;
    if (h->L != 2) return false;
    if (h->layer[2].d_out > 16) return false;
    if (h->layer[1].dp_in > kResMaxD0 || h->layer[1].dp_out > kResMaxD1) return false;
    return h->m <= 64 && static_cast<int64_t>(h->m) * (h->layer[1].dp_out / 16) <= resident_workgroup_budget();
}

namespace {

hipError_t launch_resident1(lc_handle* h, int slot0, int n_steps, int period) {
    const ActSet& S = h->train;
    const bool bf16 = h->md.gemm == LC_GEMM_BF16;
    Res1Args a;
    a.X = h->X;
    a.V = h->V;
    a.x_stride = h->Ps;
    a.Xr = h->lazy_rows ? h->xbar : h->X;
    a.xr_stride = h->lazy_rows ? 0 : h->Ps;
    a.w_off = h->layer[1].w_off;
    a.b_off = h->layer[1].b_off;
    a.d0 = h->layer[1].d_in;
    a.d1 = h->layer[1].d_out;
    a.dp0 = h->layer[1].dp_in;
    a.B = S.B;
    a.G = S.G;
    a.a0_bm = S.a_bm[0];
    a.a0_fm = S.a_fm[0];
    a.a0_slot = static_cast<int64_t>(S.G) * S.Bp * a.dp0;
    a.labels = S.labels;
    a.slot0 = slot0;
    a.n_steps = n_steps;
    a.lr = h->md.lr;
    a.beta_first = effective_beta(h);
    a.beta = h->md.beta;
    a.wd = h->md.wd;
    a.loss = S.loss;
    a.period = period;
    a.avx = h->res_avx;
    a.gctr = h->res_ctr + 65;
    a.gctr_base = h->res_garrivals;
    a.err = h->res_ctr + 64;
    a.spin_limit = h->res_spin_limit;
    if (slot0 < 0 || n_steps < 1 || slot0 + n_steps > S.slots) return hipErrorInvalidValue;
    if (period < 0 || (period > 0 && (n_steps % period != 0 || !h->res_avx || S.G > resident_workgroup_budget()))) return hipErrorInvalidValue;
    if (S.Bp != 32 && S.Bp != 64) return hipErrorInvalidValue;
    if (a.dp0 > kResMaxD1 || a.d1 > 16) return hipErrorInvalidValue;
    timing_start(h, kTimeBwd, 0, kBwdResident);
    const dim3 grid(static_cast<unsigned>(S.G)), block(kResThreads);
    if (S.Bp == 32) {
        if (bf16) hipLaunchKernelGGL((resident1_kernel<bf16_t, 2>), grid, block, 0, h->stream, a);
        else hipLaunchKernelGGL((resident1_kernel<float, 2>), grid, block, 0, h->stream, a);
    } else {
        if (bf16) hipLaunchKernelGGL((resident1_kernel<bf16_t, 4>), grid, block, 0, h->stream, a);
        else hipLaunchKernelGGL((resident1_kernel<float, 4>), grid, block, 0, h->stream, a);
    }
    h->loss_parts_train = 1;
    if (period > 0) h->res_garrivals += static_cast<unsigned>(n_steps / period) * static_cast<unsigned>(S.G);
    timing_stop(h, kTimeBwd, 0, kBwdResident);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_resident(lc_handle* h, int slot0, int n_steps, int period) {
    if (h->L == 1) return launch_resident1(h, slot0, n_steps, period);
    const ActSet& S = h->train;
    const bool bf16 = h->md.gemm == LC_GEMM_BF16;
    ResArgs a;
    a.X = h->X;
    a.V = h->V;
    a.x_stride = h->Ps;
    a.Xr = h->lazy_rows ? h->xbar : h->X;
    a.xr_stride = h->lazy_rows ? 0 : h->Ps;
    a.w1_off = h->layer[1].w_off;
    a.b1_off = h->layer[1].b_off;
    a.w2_off = h->layer[2].w_off;
    a.b2_off = h->layer[2].b_off;
    a.d0 = h->layer[1].d_in;
    a.d1 = h->layer[1].d_out;
    a.d2 = h->layer[2].d_out;
    a.dp0 = h->layer[1].dp_in;
    a.dp1 = h->layer[1].dp_out;
    a.B = S.B;
    a.G = S.G;
    a.NB = a.dp1 / 16;
    a.a0_bm = S.a_bm[0];
    a.a0_fm = S.a_fm[0];
    a.a0_slot = static_cast<int64_t>(S.G) * S.Bp * a.dp0;
    a.labels = S.labels;
    a.slot0 = slot0;
    a.n_steps = n_steps;
    a.lr = h->md.lr;
    a.beta_first = effective_beta(h);
    a.beta = h->md.beta;
    a.wd = h->md.wd;
    a.vec = (a.d1 % 4 == 0 && a.w1_off % 4 == 0) ? 1 : 0;
    a.zx = h->res_a1x;
    a.ctr = h->res_ctr;
    a.ctr_base = h->res_arrivals;
    a.err = h->res_ctr + 64;
    a.spin_limit = h->res_spin_limit;
    a.loss = S.loss;
    a.period = period;
    a.avx = h->res_avx;
    a.gctr = h->res_ctr + 65;
    a.gctr_base = h->res_garrivals;
    {
        // blocks are numbered so that each XCD works on a contiguous range of logical blocks: a
        // replica's NB workgroups share an XCD when the ranges are whole multiples of NB
        const int64_t per = (static_cast<int64_t>(a.G) * a.NB + kXcds - 1) / kXcds;
        a.local_xcd = (h->res_local_on && h->res_xcc_known && per % a.NB == 0) ? 1 : 0;
        a.xcc_of = h->res_xcc_of;
    }
    if (slot0 < 0 || n_steps < 1 || slot0 + n_steps > S.slots) return hipErrorInvalidValue;
    if (period < 0 || (period > 0 && (n_steps % period != 0 || !h->res_avx))) return hipErrorInvalidValue;
    const int64_t total = static_cast<int64_t>(a.G) * a.NB;
    if (total > resident_workgroup_budget() || a.G > 64 || !h->res_a1x) return hipErrorInvalidValue;
    const unsigned grid = static_cast<unsigned>((total + kXcds - 1) / kXcds * kXcds);
    if (S.Bp != 32 && S.Bp != 64) return hipErrorInvalidValue;
    timing_start(h, kTimeBwd, 0, kBwdResident);
    if (S.Bp == 32) {
        if (bf16) hipLaunchKernelGGL((resident_kernel<bf16_t, 2>), dim3(grid), dim3(kResThreads), 0, h->stream, a);
        else hipLaunchKernelGGL((resident_kernel<float, 2>), dim3(grid), dim3(kResThreads), 0, h->stream, a);
    } else {
        if (bf16) hipLaunchKernelGGL((resident_kernel<bf16_t, 4>), dim3(grid), dim3(kResThreads), 0, h->stream, a);
        else hipLaunchKernelGGL((resident_kernel<float, 4>), dim3(grid), dim3(kResThreads), 0, h->stream, a);
    }
    h->loss_parts_train = 1;
    h->res_arrivals += static_cast<unsigned>(n_steps) * static_cast<unsigned>(a.NB);   // wraps like the counters do
    if (period > 0) h->res_garrivals += static_cast<unsigned>(n_steps / period) * static_cast<unsigned>(total);
    timing_stop(h, kTimeBwd, 0, kBwdResident);
    return hipGetLastError();
}

// Where do blocks run?  Hardware block ids are dealt to the XCDs round-robin; the resident kernel's
// XCD-local exchange needs exactly that, so it is observed once per handle instead of assumed:
// 256 one-thread blocks report their XCD, and the rule holds if blocks with the same id mod 8
// agree and the 8 residues name 8 different XCDs.
hipError_t probe_block_placement(lc_handle* h) {
    h->res_xcc_known = false;
    h->res_xcc_of = 0;
    if (!h->res_ctr) return hipSuccess;
    unsigned* dev = h->res_ctr + 128;
    unsigned host[256];
    hipLaunchKernelGGL(xcd_probe_kernel, dim3(256), dim3(64), 0, h->stream, dev);
    hipError_t e = hipGetLastError();
    if (e == hipSuccess) e = hipMemcpyAsync(host, dev, sizeof(host), hipMemcpyDeviceToHost, h->stream);
    if (e == hipSuccess) e = hipStreamSynchronize(h->stream);
    if (e != hipSuccess) return e;
    unsigned seen = 0, packed = 0;
    for (int r = 0; r < kXcds; ++r) {
        for (int b = r; b < 256; b += kXcds)
            if (host[b] != host[r] || host[b] > 15u) return hipSuccess;   // no such rule here: agent-scope exchange
        if (seen & (1u << host[r])) return hipSuccess;
        seen |= 1u << host[r];
        packed |= host[r] << (4 * r);
    }
    h->res_xcc_known = true;
    h->res_xcc_of = packed;
    return hipSuccess;
}

}  // namespace lc
