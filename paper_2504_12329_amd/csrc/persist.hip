// Single-token decode step as ONE persistent kernel (paper Section 4, "decode" stage); an alternative to the
// kernel-per-stage step of decode.hip, chosen with ST_DECODE_PERSIST=1.
//
// One block per compute unit walks the stages of every layer (QKV, attention ranges, range merge, O projection,
// gate/up + SwiGLU, down projection) and then the LM head and the arg-max.  What a stage needs from the one before
// it -- a vector of a few thousand floats produced piecewise by all blocks -- travels through device memory as
// 8-byte words {value, epoch}: written with one relaxed 64-bit agent-scope atomic store, read with the matching load
// until the epoch is the expected one.  Value and flag share the word, so no fence, no read-modify-write atomic and
// no grid barrier is needed; a hand-over costs about 2.4 us, which is what a dependent dispatch costs.
//
// Why it exists: with one kernel per stage a small model pays ~170 dependent dispatches per token during which no
// weight byte moves.  Here weights are requested ahead of their stage (they do not depend on activations) and wait
// in registers.  Measured, the step is nevertheless 6-10 % slower than the separate kernels on the 1.5B / 7B / 32B
// shapes (the waits plus the arithmetic of one 8-wave block per compute unit outweigh the saved dispatches), so it
// is not the default; it is kept as a tested alternative.
//
// Work split: a block owns a contiguous range of rows of every matrix; a row (or, where rows are few and long, one of
// P parts of a row) is a task, wave w of the block takes the tasks w, w + 8, ...; a lane keeps one running sum per
// task, a task ends with one DPP wave sum into an LDS slot, and a row's slots are added in ascending order: every
// sum has a fixed order, results are reproducible.
//
// Every wait is bounded: a poll that exceeds its spin limit raises state[kPersistErr], which every other poll loop
// checks, and from then on no thread waits again -- every wave reaches the end of the kernel.
#include <hip/hip_ext.h>

#include <type_traits>

#include "st_device.h"
#include "st_internal.h"

namespace st {

namespace {

typedef unsigned long long u64;
// The step's arguments live in device memory and are read through the constant address space (scalar loads); the
// pointer is hidden from the optimiser at every stage, so a stage loads what it needs and nothing stays in scalar
// registers across the stages.
typedef const PersistArgs __attribute__((address_space(4))) *ArgsC;
#define ST_ARGS_FRESH() asm volatile("" : "+s"(a))

constexpr int kPT = kPersistThreads;  // threads of a block
constexpr int kPW = kPT / 64;         // waves of a block
// 16-byte loads per lane requested ahead of their stage (QKV / LM head, O, gate/up, down)
constexpr int kPFQ = 4, kPFO = 4, kPFG = 28, kPFD = 16;
constexpr int kPFG1 = 14;  // of the gate/up loads, those requested ahead of the attention (the rest ahead of the O stage)
constexpr int kRB = 6;                // groups per batch of the stream behind them (two batches in flight)
constexpr int kPollR = 6;             // words per thread and polling round (two rounds in flight)
constexpr int kTile = 64;             // keys per attention tile

// Pointers that reach the kernel through its argument record or the weight table carry no address space; every
// access through them is made as a global-memory access here.  (A generic access counts on the LDS counter as well
// as on the memory counter, and the compiler then waits for everything outstanding wherever a loaded value is used.)
#define ST_GLOBAL __attribute__((address_space(1)))
template <class T>
__device__ __forceinline__ const T ST_GLOBAL *as_global(const T *p) { return (const T ST_GLOBAL *)p; }
template <class T>
__device__ __forceinline__ T ST_GLOBAL *as_global(T *p) { return (T ST_GLOBAL *)p; }

__device__ __forceinline__ u32x4 ldw(const u32x4 *p) { return __builtin_nontemporal_load(as_global(p)); }
__device__ __forceinline__ u32x4 ldg16(const void *p) { return *as_global(reinterpret_cast<const u32x4 *>(p)); }

__device__ __forceinline__ void ll_put_bits(u64 *p, uint32_t bits, unsigned ep) {
    __hip_atomic_store(as_global(p), ((u64)ep << 32) | bits, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void ll_put(u64 *p, float v, unsigned ep) { ll_put_bits(p, __float_as_uint(v), ep); }
__device__ __forceinline__ u64 ll_get(const u64 *p) {
    return __hip_atomic_load(as_global(p), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Stage timestamps of three blocks (100 MHz wall clock), only in builds made with -DST_PERSIST_PROF for profiling.
#ifdef ST_PERSIST_PROF
__device__ unsigned long long g_prof[3][4096];
#define ST_STAMP()                                                                                                  \
    do {                                                                                                            \
        if (threadIdx.x == 0 && c.prof_slot >= 0 && c.prof_n < 4096) g_prof[c.prof_slot][c.prof_n++] = wall_clock64(); \
    } while (0)
#ifdef ST_PERSIST_PROF_IN
#define ST_STAMP_IN() ST_STAMP()
#else
#define ST_STAMP_IN() do { } while (0)
#endif
#else
#define ST_STAMP() do { } while (0)
#define ST_STAMP_IN() do { } while (0)
#endif

struct PCtx {
    int tid, lane, wave, b, nb;
    int spin_limit;
    int32_t *state;
    bool dead;  // a wait of this launch timed out: no thread waits any more
#ifdef ST_PERSIST_PROF
    int prof_slot, prof_n;
#endif
};

// Reads n hand-over words (word i at addr(i)) of epoch ep and hands every value to sink(i, bits).  All threads of the
// block take part; two rounds of kPollR words per thread are in flight, a round is re-read until all its words carry
// the epoch.
template <class Addr, class Sink>
__device__ __forceinline__ void ll_poll(PCtx &c, int n, unsigned ep, Addr addr, Sink sink) {
    u64 cur[kPollR], nxt[kPollR];
    const u64 filler = (u64)ep << 32;
    auto issue = [&](u64(&w)[kPollR], int i0) {
#pragma unroll
        for (int k = 0; k < kPollR; ++k) {
            const int i = i0 + c.tid + kPT * k;
            w[k] = i < n ? ll_get(addr(i)) : filler;
        }
    };
    issue(cur, 0);
    for (int i0 = 0; i0 < n; i0 += kPT * kPollR) {
        const bool more = i0 + kPT * kPollR < n;
        if (more) issue(nxt, i0 + kPT * kPollR);
        int spins = 0;
        while (!c.dead) {
            bool ok = true;
#pragma unroll
            for (int k = 0; k < kPollR; ++k) ok = ok && (uint32_t)(cur[k] >> 32) == ep;
            if (ok) break;
            ++spins;
            if (spins > c.spin_limit) {
                __hip_atomic_store(as_global(c.state + kPersistErr), 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                c.dead = true;
            } else if ((spins & 63) == 0 &&
                       __hip_atomic_load(as_global(c.state + kPersistErr), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) {
                c.dead = true;
            } else {
                issue(cur, i0);
            }
        }
#pragma unroll
        for (int k = 0; k < kPollR; ++k) {
            const int i = i0 + c.tid + kPT * k;
            if (i < n) sink(i, (uint32_t)cur[k]);
        }
        if (more) {
#pragma unroll
            for (int k = 0; k < kPollR; ++k) cur[k] = nxt[k];
        }
    }
}

// Split LDS layout of a K-vector the dot products read: elements 0-3 of every group of 8 as one float4 in the first
// half, elements 4-7 in the second; each half is K/8 + 1 float4 long and ends with a zero group, which lanes with
// nothing to add read instead of branching.
__device__ __forceinline__ int split_half(int K) { return (K >> 1) + 4; }
__device__ __forceinline__ int split_idx(int e, int K) { return ((e & 4) ? split_half(K) : 0) + ((e >> 3) << 2) + (e & 3); }
__device__ __forceinline__ void split_zero_pad(float *xs, int K, int tid) {
    if (tid < 4) xs[(K >> 1) + tid] = 0.f, xs[split_half(K) + (K >> 1) + tid] = 0.f;
}

// A block's share of a matrix: nrows whole rows in one or two segments (two: the gate rows and the up rows of the
// gate/up matrix), each segment contiguous in memory.  A row's K range is cut into P parts (a power of two); part q
// of row r is task r * P + q, and wave w of the block takes the tasks w, w + 8, w + 16, ...  A task is read with lpt
// loads of 64 lanes x 16 bytes along K: every load has a wave-uniform base and the lane offset lane * 16, a lane
// keeps one running sum per task, and a task ends with one wave sum into slots[task].
struct Flat {
    const char *p0, *p1;  // first row of each segment
    int nrows, seg_rows;  // rows in all, rows of the first segment
    int n8;               // 16-byte groups per row
    int lp;               // log2(P)
    int lpt;              // loads per task
    int ntask;            // nrows << lp
    unsigned row_bytes;
};
__device__ __forceinline__ Flat flat_make(const bf16_t *seg0, const bf16_t *seg1, int nrows, int seg_rows, int K, int lp) {
    Flat F;
    F.p0 = reinterpret_cast<const char *>(seg0);
    F.p1 = reinterpret_cast<const char *>(seg1);
    F.nrows = nrows, F.seg_rows = seg_rows, F.n8 = K >> 3, F.lp = lp;
    F.lpt = (((F.n8 + (1 << lp) - 1) >> lp) + 63) >> 6;
    F.ntask = nrows << lp;
    F.row_bytes = (unsigned)K * 2u;
    return F;
}
// Rows [r0, r1) of an N x K matrix.  An empty share still points at a row of the matrix (its loads are clamped
// there and add nothing).
__device__ __forceinline__ Flat flat_rows(const bf16_t *W, int N, int K, int r0, int r1, int lp) {
    const bf16_t *p = W + (size_t)min(r0, N - 1) * K;
    return flat_make(p, p, r1 - r0, r1 - r0, K, lp);
}
__device__ __forceinline__ Flat flat_pairs(const bf16_t *W, int K, int I, int u0, int u1, int lp) {
    const int ub = min(u0, I - 1);
    return flat_make(W + (size_t)ub * K, W + (size_t)(I + ub) * K, 2 * (u1 - u0), u1 - u0, K, lp);
}

// Position in a wave's sequence of loads: its task k, the load within the task, and what follows from k (kept up
// to date when k changes, not recomputed per load).  All of it is wave-uniform.  Past the wave's last task the
// cursor stays on a valid address with gn = 0: loads are never skipped (a load inside a branch would make the
// compiler wait for every outstanding load wherever a loaded register is used), they are clamped and add zero.
struct Cur {
    int k, sub;
    int gs, gn;        // first group of the task's part within its row, groups of the part (0: nothing left)
    int gclamp;        // last group a lane may read, relative to gs
    const char *base;  // address of group gs of the task's row
};
__device__ __forceinline__ void cur_task(const Flat &F, Cur &cu) {
    if (cu.k < F.ntask) {
        const int row = cu.k >> F.lp, q = cu.k & ((1 << F.lp) - 1);
        cu.gs = (q * F.n8) >> F.lp;
        cu.gn = (((q + 1) * F.n8) >> F.lp) - cu.gs;
        cu.gclamp = cu.gn - 1;
        const char *rb = row < F.seg_rows ? F.p0 + (size_t)((unsigned)row * F.row_bytes)
                                          : F.p1 + (size_t)((unsigned)(row - F.seg_rows) * F.row_bytes);
        cu.base = rb + (size_t)cu.gs * 16;
    } else {
        cu.gn = 0;
    }
}
__device__ __forceinline__ Cur cur_at(const Flat &F, int k, int sub) {
    Cur cu;
    cu.k = k, cu.sub = sub, cu.gs = 0, cu.gn = 0, cu.gclamp = 0, cu.base = F.p0;
    cur_task(F, cu);
    return cu;
}
__device__ __forceinline__ void cur_step(const Flat &F, Cur &cu) {
    if (++cu.sub == F.lpt) {
        cu.sub = 0, cu.k += kPW;
        cur_task(F, cu);
    }
}
__device__ __forceinline__ u32x4 cur_load(const Flat &F, Cur &cu, int lane) {
    const int g = min(cu.sub * 64 + lane, cu.gclamp);
    const u32x4 w = ldw(reinterpret_cast<const u32x4 *>(cu.base + (unsigned)g * 16u));
    cur_step(F, cu);
    return w;
}

template <int N>
struct Pre {
    u32x4 w[N];
};
// Requests the loads [J0, J1) of every wave's sequence.  Requests are placed right ahead of a wait for another
// stage's results: issuing a 1 KB load takes a wave ~0.15 us of the memory pipeline's time, which is free while it
// would wait anyway, and the wait ends no earlier than the hand-over takes.
template <int J0, int J1, int N>
__device__ __forceinline__ void prefetch_part(const Flat &F, const PCtx &c, Pre<N> &P) {
    static_assert(J0 >= 0 && J1 <= N, "part of the register set");
    Cur cu = cur_at(F, c.wave + kPW * (J0 / F.lpt), J0 % F.lpt);
#pragma unroll
    for (int j = J0; j < J1; ++j) P.w[j] = cur_load(F, cu, c.lane);
}
template <int N>
__device__ __forceinline__ void prefetch(const Flat &F, const PCtx &c, Pre<N> &P) {
    prefetch_part<0, N>(F, c, P);
}

// Dot products of the block's share with the K-vector xs (split layout); the first N loads of every wave are already
// in P, the rest streams in two batches of kRB loads.
template <int N>
__device__ __forceinline__ void gemv(PCtx &c, const Flat &F, const Pre<N> &P, const float *xs, int K, float *slots) {
    const float4 *xa = reinterpret_cast<const float4 *>(xs);
    const float4 *xb = reinterpret_cast<const float4 *>(xs + split_half(K));
    // cc: the load being multiplied; cn: the one after it, whose slice of x is read from LDS a load ahead
    Cur cc = cur_at(F, c.wave, 0), cn = cc;
    cur_step(F, cn);
    auto x_index = [&](const Cur &cu) {
        const int g = cu.sub * 64 + c.lane;
        return g < cu.gn ? cu.gs + g : F.n8;  // the zero group for lanes past the part
    };
    float4 xa_c = xa[x_index(cc)], xb_c = xb[x_index(cc)];
    float acc = 0.f;
    auto one = [&](const u32x4 &w) {
        const int xn = x_index(cn);
        const float4 xa_n = xa[xn], xb_n = xb[xn];
        acc = dot8(w, xa_c, xb_c, acc);
        if (cc.sub == F.lpt - 1 && cc.gn > 0) {  // wave-uniform: the task ends
            const float s = wave_sum(acc);
            if (c.lane == 0) slots[cc.k] = s;
            acc = 0.f;
        }
        cc = cn;
        cur_step(F, cn);
        xa_c = xa_n, xb_c = xb_n;
    };
#pragma unroll
    for (int j = 0; j < N; ++j) one(P.w[j]);
    ST_STAMP_IN();
    if (cc.gn > 0) {  // wave-uniform: this wave has more than N loads
        Cur lc = cur_at(F, c.wave + kPW * (N / F.lpt), N % F.lpt);
        u32x4 t0[kRB], t1[kRB];
#pragma unroll
        for (int k = 0; k < kRB; ++k) t0[k] = cur_load(F, lc, c.lane);
#pragma nounroll
        while (cc.gn > 0) {
#pragma unroll
            for (int k = 0; k < kRB; ++k) t1[k] = cur_load(F, lc, c.lane);
#pragma unroll
            for (int k = 0; k < kRB; ++k) one(t0[k]);
#pragma unroll
            for (int k = 0; k < kRB; ++k) t0[k] = cur_load(F, lc, c.lane);
#pragma unroll
            for (int k = 0; k < kRB; ++k) one(t1[k]);
        }
    }
}

// Adds the P slots of every row in ascending order and calls epi(row, sum); rows of the second segment follow those
// of the first.
template <class Epi>
__device__ __forceinline__ void reduce_rows(const PCtx &c, const Flat &F, const float *slots, Epi epi) {
    const int P = 1 << F.lp;
    for (int r = c.tid; r < F.nrows; r += kPT) {
        float s = slots[r << F.lp];
        for (int q = 1; q < P; ++q) s += slots[(r << F.lp) + q];
        epi(r, s);
    }
}

// Sum over the block in a fixed order (wave sums, then the waves in ascending order).  `red` is kPW floats of LDS;
// contains two barriers.
__device__ __forceinline__ float block_sum(const PCtx &c, float v, float *red) {
    v = wave_sum(v);
    __syncthreads();
    if (c.lane == 0) red[c.wave] = v;
    __syncthreads();
    float s = red[0];
#pragma unroll
    for (int w = 1; w < kPW; ++w) s += red[w];
    return s;
}

// rmsnorm(x) * g staged for the dot products: xs (split layout) = x * g, returns 1/rms which the caller applies to
// the sums.  x is the raw vector in LDS (n floats); gq holds this thread's gain groups (loaded before the wait).
__device__ __forceinline__ void load_gain(const bf16_t *g, int n8, int tid, u32x4 (&gq)[2]) {
#pragma unroll
    for (int k = 0; k < 2; ++k) {
        const int cg = tid + kPT * k;
        if (cg < n8) gq[k] = ldg16(reinterpret_cast<const u32x4 *>(g) + cg);
    }
}
__device__ __forceinline__ float stage_norm(const PCtx &c, const float *x, const u32x4 (&gq)[2], int n, float eps,
                                            float *xs, float *red) {
    const int n8 = n >> 3;
    float4 *xa = reinterpret_cast<float4 *>(xs);
    float4 *xb = reinterpret_cast<float4 *>(xs + split_half(n));
    split_zero_pad(xs, n, c.tid);
    float ss = 0.f;
#pragma unroll
    for (int k = 0; k < 2; ++k) {
        const int cg = c.tid + kPT * k;
        if (cg < n8) {
            const float4 a = reinterpret_cast<const float4 *>(x)[2 * cg], b = reinterpret_cast<const float4 *>(x)[2 * cg + 1];
            ss += a.x * a.x + a.y * a.y + a.z * a.z + a.w * a.w + b.x * b.x + b.y * b.y + b.z * b.z + b.w * b.w;
            const u32x4 g = gq[k];
            xa[cg] = make_float4(a.x * bf16_lo(g.x), a.y * bf16_hi(g.x), a.z * bf16_lo(g.y), a.w * bf16_hi(g.y));
            xb[cg] = make_float4(b.x * bf16_lo(g.z), b.y * bf16_hi(g.z), b.z * bf16_lo(g.w), b.w * bf16_hi(g.w));
        }
    }
    ss = block_sum(c, ss, red);
    return 1.0f / sqrtf(ss / (float)n + eps);
}

__device__ __forceinline__ float merge_weight(float m, float M) { return m == -INFINITY ? 0.f : exp2f(m - M); }
__device__ __forceinline__ void amax_take(float &v, int &i, float v2, int i2) {
    if (v2 > v || (v2 == v && i2 < i)) {
        v = v2;
        i = i2;
    }
}
__device__ __forceinline__ uint32_t pack2(float lo, float hi) { return pack_bf16x2(lo, hi); }

// ---------------------------------------------------------------------------------------
// Attention over the key range [k0, k1) of kv head g for its G query heads (64-key tiles):
//   scores : lane = key, wave = an eighth of head_dim (q broadcast from LDS), the eighths meet in LDS
//   softmax: wave = query head, lane = key (base 2, running max / sum per head)
//   P.V    : D/8 lanes share a key (16 bytes of V each)
// The K and V tiles are requested before the queries are waited for.  The queries arrive unrotated (the QKV stage is
// a plain matrix-vector product): they are rotated here; the block whose range ends with the new key also rotates
// that key, writes key and value to the cache and uses them from LDS.
// LDS (floats): raw[G*D + 2*D] | sc_part[kPW][G][64] | p_s[G][64] | run[3][8] | red_acc[kPW][G][D]
// ---------------------------------------------------------------------------------------
template <int D, int G>
__host__ __device__ constexpr int attn_lds_floats() {
    return G * D + 2 * D + kPW * G * kTile + G * kTile + 24 + kPW * G * D;
}

template <int D, int G>
__device__ __forceinline__ void attn_stage(PCtx &c, ArgsC a, int layer, int pos, int s, int g, int chunk,
                                           int s_act, unsigned ep, float *area, const Flat &Fnext, Pre<kPFG> &Pnext) {
    constexpr int LPK = D / 8, KSL = kPT / LPK, KPS = kTile / KSL, DS = D / kPW, HD = D / 2;
    static_assert(KPS >= 1 && DS >= 8, "tile mapping");
    float *raw = area;                          // q of the G heads, then the new key, then the new value
    float *knew = raw + G * D, *vnew = knew + D;
    float *sc_part = vnew + D;                  // [kPW][G][64]
    float *p_s = sc_part + kPW * G * kTile;     // [G][64]
    float *run_m = p_s + G * kTile, *run_l = run_m + 8, *corr_s = run_l + 8;
    float *red_acc = corr_s + 8;                // [kPW][G][D]

    const int tid = c.tid, lane = c.lane, wave = c.wave;
    const int t = pos + 1;
    const int k0 = s * chunk, k1 = min(t, k0 + chunk);
    const bool owner = s == s_act - 1;
    const size_t lofs = ((size_t)layer * a->nkv + g) * (size_t)a->max_seq * D;
    const bf16_t *kbase = a->kc + lofs, *vbase = a->vc + lofs;
    const int dl = tid % LPK, ks = tid / LPK;

    u32x4 kreg[DS / 8], vreg[KPS];
    auto issue = [&](int tile0) {
        const u32x4 *kp = reinterpret_cast<const u32x4 *>(kbase + (size_t)min(tile0 + lane, k1 - 1) * D + wave * DS);
#pragma unroll
        for (int i = 0; i < DS / 8; ++i) kreg[i] = ldg16(kp + i);
#pragma unroll
        for (int i = 0; i < KPS; ++i)
            vreg[i] = ldg16(vbase + (size_t)min(tile0 + ks + KSL * i, k1 - 1) * D + dl * 8);
    };
    // the cache row of the new key is not written yet: lanes that would read it take it from LDS instead
    auto patch = [&](int tile0) {
        if (!owner) return;
        if (min(tile0 + lane, k1 - 1) == pos) {
#pragma unroll
            for (int i = 0; i < DS / 8; ++i) {
                const float *kn = knew + wave * DS + 8 * i;
                kreg[i] = u32x4{pack2(kn[0], kn[1]), pack2(kn[2], kn[3]), pack2(kn[4], kn[5]), pack2(kn[6], kn[7])};
            }
        }
#pragma unroll
        for (int i = 0; i < KPS; ++i)
            if (min(tile0 + ks + KSL * i, k1 - 1) == pos) {
                const float *vn = vnew + dl * 8;
                vreg[i] = u32x4{pack2(vn[0], vn[1]), pack2(vn[2], vn[3]), pack2(vn[4], vn[5]), pack2(vn[6], vn[7])};
            }
    };
    issue(k0);
    // rotation of this thread's pair (i, i + D/2) of query head tid / HD; threads < HD also rotate the key
    static_assert(G * HD <= kPT, "one rotation pair per thread");
    const float ST_GLOBAL *cs_p = as_global(reinterpret_cast<const float *>(a->rope)) + 2 * ((size_t)pos * HD + (tid % HD));
    const float2 cs = make_float2(cs_p[0], cs_p[1]);
    if (tid < G) {
        run_m[tid] = -INFINITY;
        run_l[tid] = 0.f;
    }
    prefetch_part<0, kPFG1>(Fnext, c, Pnext);  // part of the next GEMV's weights, requested ahead of the wait
    {
        const int nq_words = G * D, n = nq_words + (owner ? 2 * D : 0);
        const u64 *qsrc = a->ll + a->off_qkv + (size_t)g * G * D;
        const u64 *ksrc = a->ll + a->off_qkv + (size_t)a->nq * D + (size_t)g * D;
        const u64 *vsrc = a->ll + a->off_qkv + (size_t)(a->nq + a->nkv) * D + (size_t)g * D;
        ll_poll(
            c, n, ep + 1,
            [&](int i) { return i < nq_words ? qsrc + i : (i < nq_words + D ? ksrc + (i - nq_words) : vsrc + (i - nq_words - D)); },
            [&](int i, uint32_t bits) { raw[i] = __uint_as_float(bits); });
    }
    ST_STAMP_IN();
    __syncthreads();
    const float scale = 1.4426950408889634f / sqrtf((float)D);
    if (tid < G * HD) {
        const int hh = tid / HD, i = tid % HD;
        const float lo = raw[hh * D + i], hi = raw[hh * D + i + HD];
        raw[hh * D + i] = (lo * cs.x - hi * cs.y) * scale;
        raw[hh * D + i + HD] = (hi * cs.x + lo * cs.y) * scale;
    }
    if (owner && tid < HD) {
        const float lo = knew[tid], hi = knew[tid + HD];
        knew[tid] = lo * cs.x - hi * cs.y;
        knew[tid + HD] = hi * cs.x + lo * cs.y;
    }
    __syncthreads();
    if (owner && tid < D) {
        bf16_t *kd = a->kc + lofs + (size_t)pos * D, *vd = a->vc + lofs + (size_t)pos * D;
        as_global(kd)[tid] = f32_to_bf16(knew[tid]);
        as_global(vd)[tid] = f32_to_bf16(vnew[tid]);
    }

    float acc[G][8];
#pragma unroll
    for (int hh = 0; hh < G; ++hh)
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[hh][e] = 0.f;
    ST_STAMP_IN();

    for (int tile0 = k0; tile0 < k1; tile0 += kTile) {
        const bool ok1 = tile0 + lane < k1;
        if (tile0 != k0) issue(tile0);
        patch(tile0);
        __syncthreads();  // the previous tile's p_s / sc_part are consumed
        {
            float pa[G];
#pragma unroll
            for (int hh = 0; hh < G; ++hh) pa[hh] = 0.f;
#pragma unroll
            for (int i = 0; i < DS / 8; ++i) {
                const u32x4 kw = kreg[i];
                const float kf[8] = {bf16_lo(kw.x), bf16_hi(kw.x), bf16_lo(kw.y), bf16_hi(kw.y),
                                     bf16_lo(kw.z), bf16_hi(kw.z), bf16_lo(kw.w), bf16_hi(kw.w)};
#pragma unroll
                for (int hh = 0; hh < G; ++hh) {
                    const float4 qa = *reinterpret_cast<const float4 *>(raw + hh * D + wave * DS + 8 * i);
                    const float4 qb = *reinterpret_cast<const float4 *>(raw + hh * D + wave * DS + 8 * i + 4);
                    float d0 = pa[hh];
                    d0 = fmaf(qa.x, kf[0], d0);
                    d0 = fmaf(qa.y, kf[1], d0);
                    d0 = fmaf(qa.z, kf[2], d0);
                    d0 = fmaf(qa.w, kf[3], d0);
                    d0 = fmaf(qb.x, kf[4], d0);
                    d0 = fmaf(qb.y, kf[5], d0);
                    d0 = fmaf(qb.z, kf[6], d0);
                    d0 = fmaf(qb.w, kf[7], d0);
                    pa[hh] = d0;
                }
            }
#pragma unroll
            for (int hh = 0; hh < G; ++hh) sc_part[(wave * G + hh) * kTile + lane] = pa[hh];
        }
        __syncthreads();
        for (int hh = wave; hh < G; hh += kPW) {
            float sc = sc_part[hh * kTile + lane];
#pragma unroll
            for (int w = 1; w < kPW; ++w) sc += sc_part[(w * G + hh) * kTile + lane];
            if (!ok1) sc = -INFINITY;
            const float m_old = run_m[hh];
            const float m_new = fmaxf(m_old, wave_max(sc));  // finite: the tile's first key is valid
            const float pr = exp2f(sc - m_new);
            const float ps = wave_sum(pr);
            p_s[hh * kTile + lane] = pr;
            if (lane == 0) {
                const float cf = merge_weight(m_old, m_new);
                corr_s[hh] = cf;
                run_l[hh] = run_l[hh] * cf + ps;
                run_m[hh] = m_new;
            }
        }
        __syncthreads();
#pragma unroll
        for (int hh = 0; hh < G; ++hh) {
            const float cf = corr_s[hh];
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[hh][e] *= cf;
        }
#pragma unroll
        for (int i = 0; i < KPS; ++i) {
            const u32x4 vw = vreg[i];
            const float vf[8] = {bf16_lo(vw.x), bf16_hi(vw.x), bf16_lo(vw.y), bf16_hi(vw.y),
                                 bf16_lo(vw.z), bf16_hi(vw.z), bf16_lo(vw.w), bf16_hi(vw.w)};
            const int kl = ks + KSL * i;
#pragma unroll
            for (int hh = 0; hh < G; ++hh) {
                const float pr = p_s[hh * kTile + kl];  // exactly 0 for keys past the range
#pragma unroll
                for (int e = 0; e < 8; ++e) acc[hh][e] = fmaf(pr, vf[e], acc[hh][e]);
            }
        }
    }
    ST_STAMP_IN();
    // the key slots of a wave are LPK lanes apart; then the waves meet in LDS
#pragma unroll
    for (int hh = 0; hh < G; ++hh)
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            float v = acc[hh][e];
            if (LPK == 8) v += __shfl_xor(v, 8, kWave);
            v = sum_xor16(v);
            acc[hh][e] = sum_xor32(v);
        }
    if (lane < LPK) {
#pragma unroll
        for (int hh = 0; hh < G; ++hh)
#pragma unroll
            for (int e = 0; e < 8; ++e) red_acc[(wave * G + hh) * D + lane * 8 + e] = acc[hh][e];
    }
    __syncthreads();
    for (int idx = tid; idx < G * D; idx += kPT) {
        const int hh = idx / D, e = idx - hh * D;
        float A = red_acc[hh * D + e];
#pragma unroll
        for (int w = 1; w < kPW; ++w) A += red_acc[(w * G + hh) * D + e];
        const int qh = g * G + hh;
        if (s_act == 1) {
            ll_put(a->ll + a->off_attn + (size_t)qh * D + e, A / run_l[hh], ep + 3);
        } else {
            u64 *rec = a->ll + a->off_part + ((size_t)qh * a->s_cap + s) * (D + 2);
            ll_put(rec + e, A, ep + 2);
            if (e == 0) {
                ll_put(rec + D, run_m[hh], ep + 2);
                ll_put(rec + D + 1, run_l[hh], ep + 2);
            }
        }
    }
    __syncthreads();  // the area is reused by the next stage
}

// Merges the s_act ranges of query head qh for the dsl output elements [e0, e0 + dsl): weights exp2(m_i - M) once,
// then the weighted sum over the ranges in a fixed order.
// LDS (floats): raw[s_act][dsl + 2] | wts[kAttnSplits] | part[kPT]
template <int D>
__device__ __forceinline__ void merge_stage(PCtx &c, ArgsC a, int qh, int e0, int s_act, unsigned ep,
                                            float *area, float *red) {
    const int dsl = a->dsl, W = dsl + 2, n = s_act * W;
    float *raw = area, *wts = raw + kAttnSplits * (D + 2), *part = wts + kAttnSplits;
    const u64 *recs = a->ll + a->off_part + (size_t)qh * a->s_cap * (D + 2);
    ll_poll(
        c, n, ep + 2,
        [&](int i) {
            const int r = i / W, k = i - r * W;
            return recs + (size_t)r * (D + 2) + (k < dsl ? e0 + k : D + (k - dsl));
        },
        [&](int i, uint32_t bits) { raw[i] = __uint_as_float(bits); });
    __syncthreads();
    ST_STAMP_IN();
    if (c.wave == 0) {
        static_assert(kAttnSplits <= 128, "two ranges per lane");
        const int r0 = c.lane, r1 = c.lane + 64;
        const float m0 = r0 < s_act ? raw[r0 * W + dsl] : -INFINITY, m1 = r1 < s_act ? raw[r1 * W + dsl] : -INFINITY;
        const float l0 = r0 < s_act ? raw[r0 * W + dsl + 1] : 0.f, l1 = r1 < s_act ? raw[r1 * W + dsl + 1] : 0.f;
        const float M = wave_max(fmaxf(m0, m1));
        const float w0 = merge_weight(m0, M), w1 = merge_weight(m1, M);
        wts[r0] = w0;
        wts[r1] = w1;
        const float L = wave_sum(w0 * l0) + wave_sum(w1 * l1);
        if (c.lane == 0) red[8] = L;
    }
    __syncthreads();
    const int e = c.tid % dsl, rr = c.tid / dsl, NR = kPT / dsl;
    float A = 0.f;
    for (int r = rr; r < s_act; r += NR) A += raw[r * W + e] * wts[r];
    part[c.tid] = A;
    __syncthreads();
    if (c.tid < dsl) {
        const int groups = min(NR, s_act);
        float S = part[c.tid];
        for (int r = 1; r < groups; ++r) S += part[r * dsl + c.tid];
        ll_put(a->ll + a->off_attn + (size_t)qh * D + e0 + c.tid, S / red[8], ep + 3);
    }
    __syncthreads();
}

template <int D>
__host__ __device__ constexpr int merge_lds_floats() {
    return kAttnSplits * (D + 2) + kAttnSplits + kPT;
}

// ---------------------------------------------------------------------------------------
// The step.  LDS (floats): red[64] | xres[h] | area: xs[kmax] | slots[...]
// (the attention and merge stages lay their own arrays over the area).
// Epochs: a launch owns 8 (L + 1) consecutive epochs; layer l uses base + 8 l + {0: x in, 1: q/k/v, 2: range records,
// 3: attention vector, 4: x after attention, 5: SwiGLU vector}, the LM head base + 8 L + {0: x, 1: candidates}.
// ---------------------------------------------------------------------------------------
template <int D, int G>
__global__ __launch_bounds__(kPT) void k_decode_persist(const PersistArgs *ap, const PersistRule rule) {
    ArgsC a = (ArgsC)ap;
    extern __shared__ __align__(16) float lds[];
    float *red = lds, *xres = lds + 64, *area = xres + a->h;
    float *xs = area, *slots = area + a->kmax;

    PCtx c;
    c.tid = threadIdx.x, c.lane = c.tid & 63, c.wave = c.tid >> 6, c.b = blockIdx.x, c.nb = gridDim.x;
    c.spin_limit = a->spin_limit, c.state = a->state, c.dead = false;
#ifdef ST_PERSIST_PROF
    c.prof_slot = blockIdx.x == 0 ? 0 : (blockIdx.x == 101 ? 1 : (blockIdx.x == gridDim.x - 1 ? 2 : -1));
    c.prof_n = 0;
#endif
    const int b = c.b, nb = c.nb;
    const int h = a->h, I = a->I, qd = a->nq * D, qkv_rows = (a->nq + 2 * a->nkv) * D;

    const int pos = __hip_atomic_load(as_global(a->state + kPos), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    int tok = __hip_atomic_load(as_global(a->state + kTok), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    tok = tok < 0 ? 0 : (tok >= a->V ? a->V - 1 : tok);
    const unsigned ep0 =
        (unsigned)__hip_atomic_load(as_global(a->state + kEpoch), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) * (unsigned)(8 * (a->L + 1)) + 64u;

    const int t = pos + 1;
    int chunk = (t + a->s_cap - 1) / a->s_cap;
    chunk = ((chunk + kTile - 1) / kTile) * kTile;
    const int s_act = (t + chunk - 1) / chunk;

    auto lo_of = [&](int N) { return (int)((long)N * b / nb); };
    auto hi_of = [&](int N) { return (int)((long)N * (b + 1) / nb); };
    int q_r0 = lo_of(qkv_rows), q_r1 = hi_of(qkv_rows);
    int o_r0 = lo_of(h), o_r1 = hi_of(h);          // rows of the O and down projections
    int u_r0 = lo_of(I), u_r1 = hi_of(I);
    const int v_r0 = lo_of(a->V), v_r1 = hi_of(a->V);

    // embedding row -> xres
    {
        const bf16_t *row = a->embed + (size_t)tok * h;
        for (int i = c.tid; i < h; i += kPT) xres[i] = bf16_to_f32(as_global(row)[i]);
    }
    // Weights requested ahead of their stage: the QKV (or LM-head) loads during the gate/up stage before, the O
    // loads during the QKV stage, the gate/up loads at the start of the attention, the down loads during the O stage.
    // Each request is issued after the stage's own wait, so that no wait queues behind it.
    Pre<kPFQ> PQ;
    Pre<kPFO> PO;
    Pre<kPFG> PG;
    Pre<kPFD> PD;
    prefetch(flat_rows(a->layers[0].wqkv, qkv_rows, h, q_r0, q_r1, a->lp_qkv), c, PQ);

    for (int l = 0; l < a->L; ++l) {
        // Everything a stage derives from the thread index is the same in every layer; hidden from the optimiser
        // here, or it computes all of it once ahead of the loop and keeps hundreds of values alive across it.
        {
            int t_ = threadIdx.x;
            asm volatile("" : "+v"(t_));
            c.tid = t_, c.lane = t_ & 63, c.wave = __builtin_amdgcn_readfirstlane(t_ >> 6);
            asm volatile("" : "+s"(q_r0), "+s"(q_r1), "+s"(o_r0), "+s"(o_r1), "+s"(u_r0), "+s"(u_r1));
        }
        const int nu = u_r1 - u_r0;
        const int tid = c.tid;
        const PersistLayer Lw = a->layers[l];
        const unsigned ep = ep0 + 8u * (unsigned)l;
        ST_STAMP();
        ST_ARGS_FRESH();
        // ---- QKV: q, k, v = W rmsnorm(x) g + bias, unrotated
        {
            const Flat Fq = flat_rows(Lw.wqkv, qkv_rows, h, q_r0, q_r1, a->lp_qkv);
            u32x4 gq[2];
            load_gain(Lw.norm_attn, h >> 3, tid, gq);
            const int my_row = q_r0 + tid;
            float bias_v = 0.f;
            if (Lw.bqkv && my_row < q_r1) bias_v = bf16_to_f32(as_global(Lw.bqkv)[my_row]);
            prefetch(flat_rows(Lw.wo, h, qd, o_r0, o_r1, a->lp_o), c, PO);
            if (l > 0)
                ll_poll(
                    c, h, ep, [&](int i) { return a->ll + a->off_x + i; },
                    [&](int i, uint32_t bits) { xres[i] = __uint_as_float(bits); });
            __syncthreads();
            ST_STAMP();
            const float inv = stage_norm(c, xres, gq, h, a->eps, xs, red);
            ST_STAMP();
            gemv(c, Fq, PQ, xs, h, slots);
            __syncthreads();
            ST_STAMP();
            reduce_rows(c, Fq, slots, [&](int lr, float s) {
                const int row = q_r0 + lr;
                float bv = bias_v;
                if (row != my_row) bv = Lw.bqkv ? bf16_to_f32(as_global(Lw.bqkv)[row]) : 0.f;
                ll_put(a->ll + a->off_qkv + row, s * inv + bv, ep + 1);
            });
            __syncthreads();
            ST_STAMP();
        }
        // ---- attention ranges and their merge (the gate/up weights start streaming under them)
        ST_ARGS_FRESH();
        {
            const Flat Fg = flat_pairs(Lw.wgu, h, I, u_r0, u_r1, a->lp_gu);
            if (b < s_act * a->nkv) attn_stage<D, G>(c, a, l, pos, b / a->nkv, b % a->nkv, chunk, s_act, ep, area, Fg, PG);
            else prefetch_part<0, kPFG1>(Fg, c, PG);
        }
        ST_STAMP();
        if (s_act > 1) {
            const int per_head = D / a->dsl, items = a->nq * per_head;
            for (int it = b; it < items; it += nb) merge_stage<D>(c, a, it / per_head, (it % per_head) * a->dsl, s_act, ep, area, red);
        }
        ST_STAMP();
        ST_ARGS_FRESH();
        // ---- O projection + residual
        {
            const Flat Fo = flat_rows(Lw.wo, h, qd, o_r0, o_r1, a->lp_o);
            prefetch_part<kPFG1, kPFG>(flat_pairs(Lw.wgu, h, I, u_r0, u_r1, a->lp_gu), c, PG);
            ll_poll(
                c, qd, ep + 3, [&](int i) { return a->ll + a->off_attn + i; },
                [&](int i, uint32_t bits) { xs[split_idx(i, qd)] = __uint_as_float(bits); });
            split_zero_pad(xs, qd, tid);
            __syncthreads();
            ST_STAMP();
            gemv(c, Fo, PO, xs, qd, slots);
            __syncthreads();
            ST_STAMP();
            reduce_rows(c, Fo, slots,
                        [&](int lr, float s) { ll_put(a->ll + a->off_x2 + o_r0 + lr, xres[o_r0 + lr] + s, ep + 4); });
            __syncthreads();
            ST_STAMP();
        }
        ST_ARGS_FRESH();
        // ---- gate/up + SwiGLU
        {
            const Flat Fg = flat_pairs(Lw.wgu, h, I, u_r0, u_r1, a->lp_gu);
            u32x4 gq[2];
            load_gain(Lw.norm_mlp, h >> 3, tid, gq);
            prefetch(flat_rows(Lw.wdown, h, I, o_r0, o_r1, a->lp_dn), c, PD);
            ll_poll(
                c, h, ep + 4, [&](int i) { return a->ll + a->off_x2 + i; },
                [&](int i, uint32_t bits) { xres[i] = __uint_as_float(bits); });
            __syncthreads();
            ST_STAMP();
            const float inv = stage_norm(c, xres, gq, h, a->eps, xs, red);
            ST_STAMP();
            gemv(c, Fg, PG, xs, h, slots);
            __syncthreads();
            ST_STAMP();
            for (int u = tid; u < nu; u += kPT) {
                const int P = 1 << a->lp_gu;
                float sg = slots[u << a->lp_gu], su = slots[(nu + u) << a->lp_gu];
                for (int q = 1; q < P; ++q) sg += slots[(u << a->lp_gu) + q], su += slots[((nu + u) << a->lp_gu) + q];
                const float gt = sg * inv, up = su * inv;
                ll_put(a->ll + a->off_act + u_r0 + u, gt / (1.0f + expf(-gt)) * up, ep + 5);
            }
            __syncthreads();
            ST_STAMP();
        }
        ST_ARGS_FRESH();
        // ---- down projection + residual -> x of the next layer (or of the LM head)
        {
            const Flat Fd = flat_rows(Lw.wdown, h, I, o_r0, o_r1, a->lp_dn);
            {   // the next layer's QKV rows, or the LM head's after the last layer (one request either way)
                const bool last = l + 1 >= a->L;
                const bf16_t *Wn = last ? a->lm_head : a->layers[last ? l : l + 1].wqkv;
                prefetch(flat_rows(Wn, last ? a->V : qkv_rows, h, last ? v_r0 : q_r0, last ? v_r1 : q_r1,
                                   last ? a->lp_lm : a->lp_qkv), c, PQ);
            }
            ll_poll(
                c, I, ep + 5, [&](int i) { return a->ll + a->off_act + i; },
                [&](int i, uint32_t bits) { xs[split_idx(i, I)] = __uint_as_float(bits); });
            split_zero_pad(xs, I, tid);
            __syncthreads();
            ST_STAMP();
            gemv(c, Fd, PD, xs, I, slots);
            __syncthreads();
            ST_STAMP();
            reduce_rows(c, Fd, slots,
                        [&](int lr, float s) { ll_put(a->ll + a->off_x + o_r0 + lr, xres[o_r0 + lr] + s, ep + 8); });
            __syncthreads();
            ST_STAMP();
        }
    }
    ST_ARGS_FRESH();
    // ---- LM head: logits and this block's arg-max candidate
    const unsigned epl = ep0 + 8u * (unsigned)a->L;
    const int tid = c.tid;
    {
        const Flat Fl = flat_rows(a->lm_head, a->V, h, v_r0, v_r1, a->lp_lm);
        u32x4 gq[2];
        load_gain(a->final_norm, h >> 3, tid, gq);
        ll_poll(
            c, h, epl, [&](int i) { return a->ll + a->off_x + i; },
            [&](int i, uint32_t bits) { xres[i] = __uint_as_float(bits); });
        __syncthreads();
        const float inv = stage_norm(c, xres, gq, h, a->eps, xs, red);
        gemv(c, Fl, PQ, xs, h, slots);
        __syncthreads();
        float best = -INFINITY;
        int besti = 0x7fffffff;
        reduce_rows(c, Fl, slots, [&](int lr, float s) {
            const float val = s * inv;
            as_global(a->logits)[v_r0 + lr] = val;
            if (val == val) amax_take(best, besti, val, v_r0 + lr);  // NaN never wins
        });
        for (int o = 32; o > 0; o >>= 1) {
            const float v2 = __shfl_xor(best, o, kWave);
            const int i2 = __shfl_xor(besti, o, kWave);
            amax_take(best, besti, v2, i2);
        }
        __syncthreads();
        if (c.lane == 0) {
            red[16 + c.wave] = best;
            red[32 + c.wave] = __int_as_float(besti);
        }
        __syncthreads();
        if (tid == 0) {
            for (int w = 1; w < kPW; ++w) amax_take(best, besti, red[16 + w], __float_as_int(red[32 + w]));
            ll_put(a->ll + a->off_cand + 2 * b, best, epl + 1);
            ll_put_bits(a->ll + a->off_cand + 2 * b + 1, (uint32_t)besti, epl + 1);
        }
    }
    // ---- block 0: arg-max over the candidates, trigger predicate on the winner, state update
    if (b == 0) {
        __syncthreads();
        uint32_t *cand = reinterpret_cast<uint32_t *>(xs);
        ll_poll(
            c, 2 * nb, epl + 1, [&](int i) { return a->ll + a->off_cand + i; }, [&](int i, uint32_t bits) { cand[i] = bits; });
        __syncthreads();
        if (c.wave == 0) {
            float best = -INFINITY;
            int besti = 0x7fffffff;
            for (int i = c.lane; i < nb; i += 64) amax_take(best, besti, __uint_as_float(cand[2 * i]), (int)cand[2 * i + 1]);
            for (int o = 32; o > 0; o >>= 1) {
                const float v2 = __shfl_xor(best, o, kWave);
                const int i2 = __shfl_xor(besti, o, kWave);
                amax_take(best, besti, v2, i2);
            }
            if (c.lane == 0) {
                const int win = besti == 0x7fffffff ? -1 : besti;
                int fired = 0;
                if (rule.kw && win >= 0 && win < rule.rule_vocab) {
                    fired = (rule.kw[win >> 5] >> (win & 31)) & 1u;
                    if (fired && rule.window == 2) fired = tok < rule.rule_vocab ? ((rule.delim[tok >> 5] >> (tok & 31)) & 1u) : 0;
                }
                a->state[kTok] = win;
                a->state[kFired] = fired;
                a->state[kFed] = tok;
                a->state[kPos] = pos + 1;
                a->state[kEpoch] = a->state[kEpoch] + 1;
                if (rule.out_seq) {
                    const int sidx = a->state[kStep];
                    rule.out_seq[sidx] = win;
                    a->state[kStep] = sidx + 1;
                }
            }
        }
    }
}

__global__ void k_persist_reset(u64 *ll, size_t words, int32_t *state) {
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < words; i += (size_t)gridDim.x * blockDim.x) ll[i] = 0;
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        state[kEpoch] = 0;
        state[kPersistErr] = 0;
    }
}

template <int D, int G>
hipError_t launch_t(const PersistArgs *a, const PersistRule &r, int nb, size_t lds_bytes, hipStream_t stream, bool set_attr) {
    if (set_attr) return hipFuncSetAttribute(reinterpret_cast<const void *>(&k_decode_persist<D, G>),
                                             hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
    hipLaunchKernelGGL((k_decode_persist<D, G>), dim3(nb), dim3(kPT), lds_bytes, stream, a, r);
    return hipSuccess;
}

template <int D>
hipError_t launch_d(int G, const PersistArgs *a, const PersistRule &r, int nb, size_t lds_bytes, hipStream_t stream, bool set_attr) {
    switch (G) {
        case 1: return launch_t<D, 1>(a, r, nb, lds_bytes, stream, set_attr);
        case 2: return launch_t<D, 2>(a, r, nb, lds_bytes, stream, set_attr);
        case 3: return launch_t<D, 3>(a, r, nb, lds_bytes, stream, set_attr);
        case 4: return launch_t<D, 4>(a, r, nb, lds_bytes, stream, set_attr);
        case 5: return launch_t<D, 5>(a, r, nb, lds_bytes, stream, set_attr);
        case 6: return launch_t<D, 6>(a, r, nb, lds_bytes, stream, set_attr);
        case 7: return launch_t<D, 7>(a, r, nb, lds_bytes, stream, set_attr);
        default: return launch_t<D, 8>(a, r, nb, lds_bytes, stream, set_attr);
    }
}

int attn_floats_of(int D, int G) {
    auto f = [&](auto d) {
        constexpr int DD = decltype(d)::value;
        switch (G) {
            case 1: return attn_lds_floats<DD, 1>();
            case 2: return attn_lds_floats<DD, 2>();
            case 3: return attn_lds_floats<DD, 3>();
            case 4: return attn_lds_floats<DD, 4>();
            case 5: return attn_lds_floats<DD, 5>();
            case 6: return attn_lds_floats<DD, 6>();
            case 7: return attn_lds_floats<DD, 7>();
            default: return attn_lds_floats<DD, 8>();
        }
    };
    return D == 128 ? f(std::integral_constant<int, 128>()) : f(std::integral_constant<int, 64>());
}

}  // namespace

#ifdef ST_PERSIST_PROF
extern "C" int st_debug_persist_prof(unsigned long long *out_host) {
    return (int)hipMemcpyFromSymbol(out_host, HIP_SYMBOL(g_prof), sizeof(unsigned long long) * 3 * 4096);
}
#endif

// Hand-over words of a model: x, q/k/v, range records, attention vector, x after attention, SwiGLU vector, arg-max
// candidates (layout in PersistPlan).
bool persist_plan(const st_config &c, int n_cu, PersistPlan *out) {
    PersistPlan p = {};
    const int h = c.hidden, D = c.head_dim, nq = c.n_q_heads, nkv = c.n_kv_heads, I = c.intermediate;
    const int qd = nq * D, qkv_rows = (nq + 2 * nkv) * D;
    p.nb = n_cu;
    if (n_cu < nkv || n_cu < 8 || n_cu > 1024) return false;
    // a wave's 64 groups must lie in at most three rows, and the gain of a row fits two groups per thread
    if ((h >> 3) < 32 || (qd >> 3) < 32 || (I >> 3) < 32 || h > 8192) return false;
    p.s_cap = n_cu / nkv < kAttnSplits ? n_cu / nkv : kAttnSplits;
    int dsl = 4;
    while (dsl < D && nq * (D / dsl) > n_cu) dsl <<= 1;
    p.dsl = dsl;
    auto share = [&](int N) { return (N + n_cu - 1) / n_cu; };
    // K parts per row of a stage: the P in {1, 2, 4, 8} (parts of at least 32 groups) with the fewest loads on the
    // busiest wave; returns log2(P) and counts the tasks
    int smax = 0;
    auto parts = [&](int rows, int K) {
        const int n8 = K >> 3;
        int best_lp = 0;
        long best_cost = -1;
        for (int lp = 0; lp <= 3; ++lp) {
            if (lp && (n8 >> lp) < 32) break;
            const int lpt = (((n8 + (1 << lp) - 1) >> lp) + 63) >> 6;
            const long cost = (long)(((rows << lp) + kPW - 1) / kPW) * lpt;
            if (best_cost < 0 || cost < best_cost) best_cost = cost, best_lp = lp;
        }
        if ((rows << best_lp) > smax) smax = rows << best_lp;
        return best_lp;
    };
    p.lp_qkv = parts(share(qkv_rows), h);
    p.lp_o = parts(share(h), qd);
    p.lp_gu = parts(2 * share(I), h);
    p.lp_dn = parts(share(h), I);
    p.lp_lm = parts(share(c.vocab), h);
    smax += 8;
    p.kmax = h > qd ? h : qd;
    if (I > p.kmax) p.kmax = I;
    p.kmax += 8;  // the two zero groups of the split layout
    int area = p.kmax + smax;
    const int af = attn_floats_of(D, nq / nkv);
    if (af > area) area = af;
    const int mf = D == 128 ? merge_lds_floats<128>() : merge_lds_floats<64>();
    if (mf > area) area = mf;
    if (2 * n_cu > area) area = 2 * n_cu;
    size_t lds = sizeof(float) * (size_t)(64 + h + area);
    if (lds > 160 * 1024) return false;
    if (lds < 84 * 1024) lds = 84 * 1024;  // more than half a CU's LDS: one block per compute unit
    p.lds_bytes = lds;
    size_t off = 0;
    auto take = [&](size_t words) {
        size_t o = off;
        off += (words + 31) & ~(size_t)31;
        return (int)o;
    };
    p.off_x = take(h);
    p.off_qkv = take(qkv_rows);
    p.off_part = take((size_t)nq * p.s_cap * (D + 2));
    p.off_attn = take(qd);
    p.off_x2 = take(h);
    p.off_act = take(I);
    p.off_cand = take(2 * (size_t)n_cu);
    p.ll_words = off;
    *out = p;
    return true;
}

hipError_t persist_prepare(const Model &m) {
    const int D = m.c.head_dim, G = m.c.n_q_heads / m.c.n_kv_heads;
    const PersistRule r = {};
    return D == 128 ? launch_d<128>(G, nullptr, r, 0, m.persist.lds_bytes, nullptr, true)
                    : launch_d<64>(G, nullptr, r, 0, m.persist.lds_bytes, nullptr, true);
}

void launch_persist_reset(const Model &m) {
    hipLaunchKernelGGL(k_persist_reset, dim3(64), dim3(256), 0, m.stream, reinterpret_cast<u64 *>(m.ws.ll),
                       m.persist.ll_words, m.ws.state);
}

// The per-model arguments of the step (everything but the trigger rule and the output buffer of a launch).
PersistArgs persist_args(const Model &m) {
    const st_config &c = m.c;
    const PersistPlan &p = m.persist;
    PersistArgs a = {};
    a.layers = m.ws.ptab;
    a.embed = m.embed, a.lm_head = m.lm_head, a.final_norm = m.final_norm;
    a.kc = m.kcache, a.vc = m.vcache;
    a.state = m.ws.state;
    a.rope = m.ws.rope;
    a.ll = reinterpret_cast<u64 *>(m.ws.ll);
    a.logits = m.ws.logits;
    a.L = c.n_layers, a.h = c.hidden, a.nq = c.n_q_heads, a.nkv = c.n_kv_heads, a.I = c.intermediate, a.V = c.vocab;
    a.max_seq = c.max_seq, a.eps = c.rms_eps;
    a.s_cap = p.s_cap, a.dsl = p.dsl, a.kmax = p.kmax;
    a.lp_qkv = p.lp_qkv, a.lp_o = p.lp_o, a.lp_gu = p.lp_gu, a.lp_dn = p.lp_dn, a.lp_lm = p.lp_lm;
    a.off_x = p.off_x, a.off_qkv = p.off_qkv, a.off_part = p.off_part, a.off_attn = p.off_attn, a.off_x2 = p.off_x2;
    a.off_act = p.off_act, a.off_cand = p.off_cand;
    a.spin_limit = m.persist_spin_limit;
    return a;
}

void launch_decode_persist(const Model &m, const st_trigger_rule *rule, int32_t *out_seq_dev, hipStream_t stream) {
    PersistRule r = {};
    r.kw = rule ? rule->kw_bitmap : nullptr;
    r.delim = rule ? rule->delim_bitmap : nullptr;
    r.window = rule ? rule->window : 1;
    r.rule_vocab = rule ? rule->vocab : 0;
    r.out_seq = out_seq_dev;
    const int G = m.c.n_q_heads / m.c.n_kv_heads;
    if (m.c.head_dim == 128) (void)launch_d<128>(G, m.ws.pargs, r, m.persist.nb, m.persist.lds_bytes, stream, false);
    else (void)launch_d<64>(G, m.ws.pargs, r, m.persist.nb, m.persist.lds_bytes, stream, false);
}

}  // namespace st
