// Single-token decode step (paper Section 4, "decode" stage): weight-streaming bf16
// matrix-vector products with fused RMSNorm / bias / RoPE / KV append / SwiGLU / residual
// epilogues, split-K GQA attention over the KV cache, LM head with greedy arg-max.
//
// Every kernel takes the position and the fed token from the model's device state block,
// so a step can be enqueued, captured into a graph and replayed without the host knowing
// either.  All kernels are latency-shaped for batch 1: weight loads are issued before anything
// that waits (the activation vector, the norm), and the RMSNorm scale is applied to the dot
// products afterwards as a scalar.
#include <hip/hip_ext.h>

#include "st_device.h"
#include "st_internal.h"

namespace st {

__device__ __forceinline__ u32x4 ldw(const u32x4 *p) { return __builtin_nontemporal_load(p); }

// ---------------------------------------------------------------------------------------
// Activation vector in LDS for the kernels whose input is rmsnorm(x) * g.  A lane consumes 8
// consecutive activations per 16-byte weight load; they are kept as two float4 arrays (elements
// 0-3 and 4-7 of every group of 8) so that 64 lanes read 64 consecutive float4 from each.
// The vector stored is x * g; the 1/rms factor is returned and applied to the dot products.
// n <= 8192, 256 threads.  Ends with the block's only barrier.
// ---------------------------------------------------------------------------------------
// XI = 16-byte groups of x per thread: 1 covers n <= 2048, 4 covers n <= 8192.
template <int XI>
struct XRegs {
    float4 a[XI], b[XI];
    u32x4 g[XI];
};

template <int XI>
__device__ __forceinline__ void xload(const float *__restrict__ x, const bf16_t *__restrict__ g, int n8,
                                      XRegs<XI> &r) {
#pragma unroll
    for (int i = 0; i < XI; ++i) {
        int c = threadIdx.x + i * 256;
        if (c < n8) {
            r.a[i] = reinterpret_cast<const float4 *>(x)[2 * c];
            r.b[i] = reinterpret_cast<const float4 *>(x)[2 * c + 1];
            r.g[i] = reinterpret_cast<const u32x4 *>(g)[c];
        }
    }
}

template <int XI>
__device__ __forceinline__ float xstage(const XRegs<XI> &r, int n, float eps, float *xs, float *red) {
    const int n8 = n >> 3;
    float4 *xa = reinterpret_cast<float4 *>(xs);
    float4 *xb = reinterpret_cast<float4 *>(xs + (n >> 1));
    float ss = 0.f;
#pragma unroll
    for (int i = 0; i < XI; ++i) {
        int c = threadIdx.x + i * 256;
        if (c < n8) {
            float4 a = r.a[i], b = r.b[i];
            ss += a.x * a.x + a.y * a.y + a.z * a.z + a.w * a.w + b.x * b.x + b.y * b.y + b.z * b.z + b.w * b.w;
            u32x4 g = r.g[i];
            xa[c] = make_float4(a.x * bf16_lo(g.x), a.y * bf16_hi(g.x), a.z * bf16_lo(g.y), a.w * bf16_hi(g.y));
            xb[c] = make_float4(b.x * bf16_lo(g.z), b.y * bf16_hi(g.z), b.z * bf16_lo(g.w), b.w * bf16_hi(g.w));
        }
    }
    ss = wave_sum(ss);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = ss;
    __syncthreads();
    ss = red[0] + red[1] + red[2] + red[3];
    return 1.0f / sqrtf(ss / (float)n + eps);
}

// Weight rows of one wave: the first PF 16-byte groups per lane are fetched up front (before the
// activation vector is waited for), the rest in the loop.
template <int NR, int PF>
struct RowFetch {
    const u32x4 *p[NR];
    u32x4 w[PF][NR];
    __device__ __forceinline__ void prefetch(int n8, int lane) {
        const u32x4 zero = {0, 0, 0, 0};
#pragma unroll
        for (int f = 0; f < PF; ++f)
#pragma unroll
            for (int r = 0; r < NR; ++r) w[f][r] = lane + 64 * f < n8 ? ldw(p[r] + lane + 64 * f) : zero;
    }
    __device__ __forceinline__ void dot(const float *xs, int n, int lane, float (&acc)[NR]) const {
        const int n8 = n >> 3;
        const float4 *xa = reinterpret_cast<const float4 *>(xs);
        const float4 *xb = reinterpret_cast<const float4 *>(xs + (n >> 1));
#pragma unroll
        for (int f = 0; f < PF; ++f) {
            int c = min(lane + 64 * f, n8 - 1);  // out-of-range lanes hold zero weights
            float4 a = xa[c], b = xb[c];
#pragma unroll
            for (int r = 0; r < NR; ++r) acc[r] = dot8(w[f][r], a, b, acc[r]);
        }
        int c = lane + 64 * PF;
        for (; c + 64 < n8; c += 128) {
            u32x4 u0[NR], u1[NR];
#pragma unroll
            for (int r = 0; r < NR; ++r) {
                u0[r] = ldw(p[r] + c);
                u1[r] = ldw(p[r] + c + 64);
            }
            float4 a0 = xa[c], b0 = xb[c], a1 = xa[c + 64], b1 = xb[c + 64];
#pragma unroll
            for (int r = 0; r < NR; ++r) {
                acc[r] = dot8(u0[r], a0, b0, acc[r]);
                acc[r] = dot8(u1[r], a1, b1, acc[r]);
            }
        }
        if (c < n8) {
            u32x4 u0[NR];
#pragma unroll
            for (int r = 0; r < NR; ++r) u0[r] = ldw(p[r] + c);
            float4 a0 = xa[c], b0 = xb[c];
#pragma unroll
            for (int r = 0; r < NR; ++r) acc[r] = dot8(u0[r], a0, b0, acc[r]);
        }
    }
};

// ---------------------------------------------------------------------------------------
// state / embedding
// ---------------------------------------------------------------------------------------
__global__ void k_init(int32_t *state, int32_t *counters, int nkv, float2 *rope, int max_seq, int half_d,
                       double theta) {
    int gid = blockIdx.x * blockDim.x + threadIdx.x;
    if (gid < kStateInts) state[gid] = 0;
    if (gid < nkv) counters[gid] = 0;
    long total = (long)max_seq * half_d;
    for (long i = gid; i < total; i += (long)gridDim.x * blockDim.x) {
        int p = (int)(i / half_d), f = (int)(i % half_d);
        double freq = pow(theta, -(double)f / (double)half_d);  // theta^(-2f/d)
        double s, c;
        sincos((double)p * freq, &s, &c);
        rope[i] = make_float2((float)c, (float)s);
    }
}

__global__ void k_set_token(int32_t *state, int32_t token) { state[kTok] = token; }
__global__ void k_set_token_from(int32_t *state, const int32_t *tokens, int32_t index) { state[kTok] = tokens[index]; }
__global__ void k_set_state(int32_t *state, int slot, int32_t value) { state[slot] = value; }

__global__ __launch_bounds__(256) void k_embed(const bf16_t *__restrict__ E, int32_t *state, float *__restrict__ x,
                                               int h, int vocab) {
    int tok = state[kTok];
    tok = tok < 0 ? 0 : (tok >= vocab ? vocab - 1 : tok);
    const bf16_t *row = E + (size_t)tok * h;
    for (int i = blockIdx.x * 256 + threadIdx.x; i < h; i += gridDim.x * 256) x[i] = bf16_to_f32(row[i]);
    if (blockIdx.x == 0 && threadIdx.x == 0) state[kFed] = tok;
}

// ---------------------------------------------------------------------------------------
// QKV projection: rmsnorm prologue, bias, rotate-half RoPE on q and k, K/V appended to the cache.
// A wave owns R "units"; unit u is the row pair (i, i + d/2) of one head so that the rotation
// needs no exchange.  One group of units per wave (the grid covers all of them).
// ---------------------------------------------------------------------------------------
template <int R, int XI>
__global__ __launch_bounds__(256) void k_qkv_rope(const bf16_t *__restrict__ W, const bf16_t *__restrict__ bias,
                                                  const float *__restrict__ x, const bf16_t *__restrict__ g,
                                                  const int32_t *__restrict__ state, const float2 *__restrict__ rope,
                                                  float *__restrict__ q_out, bf16_t *__restrict__ kc,
                                                  bf16_t *__restrict__ vc, int h, int nq, int nkv, int d,
                                                  int max_seq, float eps) {
    extern __shared__ __align__(16) float xs[];
    __shared__ float red[4];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int half_d = d >> 1, n8 = h >> 3;
    const int n_units = (nq + 2 * nkv) * half_d;
    const int u0 = (blockIdx.x * 4 + wave) * R;

    XRegs<XI> xr;
    xload(x, g, n8, xr);
    RowFetch<2 * R, (XI == 1 ? 3 : 2)> rf;
    int row0[R];
#pragma unroll
    for (int j = 0; j < R; ++j) {
        int u = min(u0 + j, n_units - 1);
        int head = u / half_d, i = u - head * half_d;
        row0[j] = head * d + i;
        rf.p[2 * j] = reinterpret_cast<const u32x4 *>(W + (size_t)row0[j] * h);
        rf.p[2 * j + 1] = reinterpret_cast<const u32x4 *>(W + (size_t)(row0[j] + half_d) * h);
    }
    rf.prefetch(n8, lane);
    const int pos = state[kPos];
    // lane j finishes unit j: its bias pair and rotation are fetched now, under the weight stream
    float b_lo = 0.f, b_hi = 0.f;
    float2 cs = make_float2(1.f, 0.f);
#pragma unroll
    for (int j = 0; j < R; ++j) {
        if (lane == j) {
            const int r0 = row0[j], head = r0 / d, i = r0 - head * d;
            if (bias) {
                b_lo = bf16_to_f32(bias[r0]);
                b_hi = bf16_to_f32(bias[r0 + half_d]);
            }
            if (head < nq + nkv) cs = rope[(size_t)pos * half_d + i];
        }
    }
    const float inv = xstage(xr, h, eps, xs, red);
    if (u0 >= n_units) return;

    float acc[2 * R];
#pragma unroll
    for (int r = 0; r < 2 * R; ++r) acc[r] = 0.f;
    rf.dot(xs, h, lane, acc);
#pragma unroll
    for (int r = 0; r < 2 * R; ++r) acc[r] = wave_sum(acc[r]);

#pragma unroll
    for (int j = 0; j < R; ++j) {
        if (lane == j && u0 + j < n_units) {
            int r0 = row0[j], r1 = r0 + half_d;
            int head = r0 / d, i = r0 - head * d;
            float lo = acc[2 * j] * inv + b_lo, hi = acc[2 * j + 1] * inv + b_hi;
            if (head < nq + nkv) {
                float nlo = lo * cs.x - hi * cs.y;
                float nhi = hi * cs.x + lo * cs.y;
                lo = nlo;
                hi = nhi;
            }
            if (head < nq) {
                q_out[r0] = lo;
                q_out[r1] = hi;
            } else if (head < nq + nkv) {
                bf16_t *dst = kc + ((size_t)(head - nq) * max_seq + pos) * d;
                dst[i] = f32_to_bf16(lo);
                dst[i + half_d] = f32_to_bf16(hi);
            } else {
                bf16_t *dst = vc + ((size_t)(head - nq - nkv) * max_seq + pos) * d;
                dst[i] = f32_to_bf16(lo);
                dst[i + half_d] = f32_to_bf16(hi);
            }
        }
    }
}

// ---------------------------------------------------------------------------------------
// a[i] = silu(Wg[i,:] . y) * (Wu[i,:] . y),  y = rmsnorm(x) * g.  Gate rows [0,I), up rows [I,2I).
// A wave owns a balanced contiguous range of pairs and walks it R pairs at a time.
// ---------------------------------------------------------------------------------------
template <int R, int XI, bool ONE>
__global__ __launch_bounds__(256) void k_gateup_swiglu(const bf16_t *__restrict__ W, const float *__restrict__ x,
                                                       const bf16_t *__restrict__ g, float *__restrict__ a, int h,
                                                       int I, float eps) {
    extern __shared__ __align__(16) float xs[];
    __shared__ float red[4];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int n8 = h >> 3;
    const long nw = (long)gridDim.x * 4, wg = (long)blockIdx.x * 4 + wave;
    // ONE: the grid has a wave for every group of R pairs; otherwise a balanced contiguous range per wave
    const int ub = ONE ? (int)min((long)I, wg * R) : (int)((long)I * wg / nw);
    const int ue = ONE ? min(I, ub + R) : (int)((long)I * (wg + 1) / nw);

    XRegs<XI> xr;
    xload(x, g, n8, xr);
    RowFetch<2 * R, (XI == 1 ? 3 : 2)> rf;
    auto point = [&](int u0) {
#pragma unroll
        for (int j = 0; j < R; ++j) {
            int u = min(u0 + j, I - 1);
            rf.p[2 * j] = reinterpret_cast<const u32x4 *>(W + (size_t)u * h);
            rf.p[2 * j + 1] = reinterpret_cast<const u32x4 *>(W + (size_t)(I + u) * h);
        }
    };
    point(ub);
    if (ub < ue) rf.prefetch(n8, lane);
    const float inv = xstage(xr, h, eps, xs, red);

    auto group = [&](int u0) {
        float acc[2 * R];
#pragma unroll
        for (int r = 0; r < 2 * R; ++r) acc[r] = 0.f;
        rf.dot(xs, h, lane, acc);
#pragma unroll
        for (int r = 0; r < 2 * R; ++r) acc[r] = wave_sum(acc[r]);
#pragma unroll
        for (int j = 0; j < R; ++j)
            if (lane == j && u0 + j < ue) {
                float gt = acc[2 * j] * inv, up = acc[2 * j + 1] * inv;
                a[u0 + j] = gt / (1.0f + expf(-gt)) * up;
            }
    };
    if (ONE) {
        if (ub < ue) group(ub);
    } else {
        for (int u0 = ub; u0 < ue; u0 += R) {
            if (u0 != ub) {
                point(u0);
                rf.prefetch(n8, lane);
            }
            group(u0);
        }
    }
}

// ---------------------------------------------------------------------------------------
// y[i] = res[i] + W[i,:] . v   (O projection and down projection; res may alias y).
// A block owns RB rows; its four waves split K and combine through LDS.  The activation vector is
// read straight from global memory (L2) next to the weights: no staging, no barrier before the loads.
// ---------------------------------------------------------------------------------------
template <int RB, int U>
__global__ __launch_bounds__(256) void k_gemv_residual(const bf16_t *__restrict__ W, const float *__restrict__ v,
                                                       const float *res, float *y, int N, int K) {
    __shared__ float part[4][RB];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int r0 = blockIdx.x * RB;
    const int n8 = K >> 3;
    const u32x4 *wrow[RB];
#pragma unroll
    for (int r = 0; r < RB; ++r) wrow[r] = reinterpret_cast<const u32x4 *>(W + (size_t)min(r0 + r, N - 1) * K);
    const float4 *xv = reinterpret_cast<const float4 *>(v);
    // the residual element this thread will add at the end: fetched now, under the weight stream
    const bool writer = threadIdx.x < RB && r0 + (int)threadIdx.x < N;
    const float res_v = writer ? res[r0 + threadIdx.x] : 0.f;
    float acc[RB];
#pragma unroll
    for (int r = 0; r < RB; ++r) acc[r] = 0.f;
    // the four waves interleave along K: together they read 4 KB of every row per step
    int c = wave * 64 + lane;
    for (; c + 256 * (U - 1) < n8; c += 256 * U) {  // U groups of 16 bytes per row in flight
        u32x4 w[U][RB];
        float4 a[U], b[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
#pragma unroll
            for (int r = 0; r < RB; ++r) w[u][r] = ldw(wrow[r] + c + 256 * u);
            a[u] = xv[2 * (c + 256 * u)];
            b[u] = xv[2 * (c + 256 * u) + 1];
        }
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int r = 0; r < RB; ++r) acc[r] = dot8(w[u][r], a[u], b[u], acc[r]);
    }
    for (; c < n8; c += 256) {
        u32x4 w0[RB];
#pragma unroll
        for (int r = 0; r < RB; ++r) w0[r] = ldw(wrow[r] + c);
        float4 a0 = xv[2 * c], b0 = xv[2 * c + 1];
#pragma unroll
        for (int r = 0; r < RB; ++r) acc[r] = dot8(w0[r], a0, b0, acc[r]);
    }
#pragma unroll
    for (int r = 0; r < RB; ++r) acc[r] = wave_sum(acc[r]);
    if (lane == 0) {
#pragma unroll
        for (int r = 0; r < RB; ++r) part[wave][r] = acc[r];
    }
    __syncthreads();
    if (writer) {
        int r = threadIdx.x;
        y[r0 + r] = res_v + ((part[0][r] + part[1][r]) + (part[2][r] + part[3][r]));
    }
}

// ---------------------------------------------------------------------------------------
// LM head: logits = W rmsnorm(x) * g, plus one (max, lowest index) candidate per block.
// ---------------------------------------------------------------------------------------
__device__ __forceinline__ void amax_merge(float &v, int &i, float v2, int i2) {
    if (v2 > v || (v2 == v && i2 < i)) {
        v = v2;
        i = i2;
    }
}

constexpr int kLmRows = 4;  // rows per wave per pass

template <int XI>
__global__ __launch_bounds__(256) void k_lm_head(const bf16_t *__restrict__ W, const float *__restrict__ x,
                                                 const bf16_t *__restrict__ g, float *__restrict__ logits,
                                                 float *__restrict__ pval, int32_t *__restrict__ pidx, int h, int V,
                                                 float eps) {
    extern __shared__ __align__(16) float xs[];
    __shared__ float red[4];
    __shared__ float bv[4];
    __shared__ int bi[4];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int n8 = h >> 3;
    const long nw = (long)gridDim.x * 4, wg = (long)blockIdx.x * 4 + wave;
    const int groups = (V + kLmRows - 1) / kLmRows;
    const int gb = (int)((long)groups * wg / nw), ge = (int)((long)groups * (wg + 1) / nw);

    XRegs<XI> xr;
    xload(x, g, n8, xr);
    RowFetch<kLmRows, (XI == 1 ? 3 : 2)> rf;
    auto point = [&](int r0) {
#pragma unroll
        for (int r = 0; r < kLmRows; ++r) rf.p[r] = reinterpret_cast<const u32x4 *>(W + (size_t)min(r0 + r, V - 1) * h);
    };
    point(gb * kLmRows);
    if (gb < ge) rf.prefetch(n8, lane);
    const float inv = xstage(xr, h, eps, xs, red);

    float best = -INFINITY;
    int besti = 0x7fffffff;
    for (int gi = gb; gi < ge; ++gi) {
        const int r0 = gi * kLmRows;
        if (gi != gb) {
            point(r0);
            rf.prefetch(n8, lane);
        }
        float acc[kLmRows];
#pragma unroll
        for (int r = 0; r < kLmRows; ++r) acc[r] = 0.f;
        rf.dot(xs, h, lane, acc);
#pragma unroll
        for (int r = 0; r < kLmRows; ++r) acc[r] = wave_sum(acc[r]);
#pragma unroll
        for (int r = 0; r < kLmRows; ++r)
            if (r0 + r < V) {
                float val = acc[r] * inv;
                if (lane == r) logits[r0 + r] = val;
                if (val == val) amax_merge(best, besti, val, r0 + r);  // NaN never wins
            }
    }
    // every lane of a wave holds the same candidate; merge the four waves
    if (lane == 0) {
        bv[wave] = best;
        bi[wave] = besti;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int w = 1; w < 4; ++w) amax_merge(best, besti, bv[w], bi[w]);
        pval[blockIdx.x] = best;
        pidx[blockIdx.x] = besti;
    }
}

// Final arg-max over the per-block candidates, trigger predicate on the winner, state update.
__global__ __launch_bounds__(256) void k_argmax_final(const float *__restrict__ pval, const int32_t *__restrict__ pidx,
                                                      int n, int32_t *state, const uint32_t *kw,
                                                      const uint32_t *delim, int window, int rule_vocab,
                                                      int advance, int32_t *out_seq) {
    __shared__ float sv[256];
    __shared__ int si[256];
    float best = -INFINITY;
    int besti = 0x7fffffff;
    for (int i = threadIdx.x; i < n; i += 256) amax_merge(best, besti, pval[i], pidx[i]);
    sv[threadIdx.x] = best;
    si[threadIdx.x] = besti;
    __syncthreads();
    for (int s = 128; s > 0; s >>= 1) {
        if ((int)threadIdx.x < s) {
            float v = sv[threadIdx.x];
            int i = si[threadIdx.x];
            amax_merge(v, i, sv[threadIdx.x + s], si[threadIdx.x + s]);
            sv[threadIdx.x] = v;
            si[threadIdx.x] = i;
        }
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        int tok = si[0] == 0x7fffffff ? -1 : si[0];
        int fired = 0;
        if (kw && tok >= 0 && tok < rule_vocab) {
            fired = (kw[tok >> 5] >> (tok & 31)) & 1u;
            if (fired && window == 2) {
                int prev = state[kFed];
                fired = (prev >= 0 && prev < rule_vocab) ? ((delim[prev >> 5] >> (prev & 31)) & 1u) : 0;
            }
        }
        state[kTok] = tok;
        state[kFired] = fired;
        state[kPos] += advance;
        if (out_seq) {
            int s = state[kStep];
            out_seq[s] = tok;
            state[kStep] = s + 1;
        }
    }
}

// ---------------------------------------------------------------------------------------
// GQA decode attention, split over the key range.  Block (s, g): kv head g, key range s, all G
// query heads of the group; keys are taken in tiles of 64.
//   scores : lane = key, wave = quarter of head_dim; q is read from LDS as broadcasts, so there is
//            no cross-lane reduction; the four quarters meet in LDS
//   softmax: wave = query head, lane = key (base 2, running max / sum per head across tiles)
//   P.V    : D/8 lanes share a key (16 bytes of V each), 64/(256/(D/8)) keys per lane group
// Each range publishes (max, sum, unnormalised output); a second kernel merges the ranges in a
// fixed order, so the result does not depend on timing.  A context that fits one range is
// finished by the first kernel alone.
// ---------------------------------------------------------------------------------------
__device__ __forceinline__ float merge_w(float m, float M) { return m == -INFINITY ? 0.f : exp2f(m - M); }

constexpr int kKeyTile = 64;

// One element of a row's attention output: fp32, or two bf16 terms where the consumer is a GEMM.
__device__ __forceinline__ void put_attn(const AttnRows &rows, float *out, size_t row_off, size_t i, float v) {
    if (rows.out_hi) {
        const bf16_t h = f32_to_bf16(v);
        rows.out_hi[row_off + i] = h;
        rows.out_lo[row_off + i] = f32_to_bf16(v - bf16_to_f32(h));
    } else {
        out[i] = v;
    }
}

__device__ __forceinline__ void unpack8(const u32x4 &w, float (&f)[8]) {
    f[0] = bf16_lo(w.x);
    f[1] = bf16_hi(w.x);
    f[2] = bf16_lo(w.y);
    f[3] = bf16_hi(w.y);
    f[4] = bf16_lo(w.z);
    f[5] = bf16_hi(w.z);
    f[6] = bf16_lo(w.w);
    f[7] = bf16_hi(w.w);
}

// Keys per range for a context of t keys split into at most S ranges (whole tiles).
__device__ __forceinline__ int attn_chunk(int t, int S) {
    int chunk = (t + S - 1) / S;
    return ((chunk + kKeyTile - 1) / kKeyTile) * kKeyTile;
}

// blockIdx.z is a row of a batch of independent sequences (one row, sequence 0, in the single-sequence step):
// rows.pos[z] is the position of that row's new token, rows.seq[z] the sequence whose cache it attends to.
template <int D, int G>
__global__ __launch_bounds__(256) void k_attn_partial(const float *__restrict__ q, const bf16_t *__restrict__ kc,
                                                      const bf16_t *__restrict__ vc, AttnRows rows, int max_seq, int S,
                                                      float *__restrict__ part_ml, float *__restrict__ part_acc,
                                                      float *__restrict__ out) {
    constexpr int LPK = D / 8;            // lanes sharing one key in the P.V phase
    constexpr int KSL = 256 / LPK;        // key slots of the block in the P.V phase
    constexpr int KPS = kKeyTile / KSL;   // keys per slot per tile
    constexpr int DS = D / 4;             // head_dim slice of one wave in the score phase
    __shared__ __align__(16) float q_s[G][D];
    __shared__ float sc_part[4][G][kKeyTile];
    __shared__ float p_s[G][kKeyTile];
    __shared__ float run_m[G], run_l[G], corr_s[G];
    __shared__ __align__(16) float red_acc[4][G][D];

    const int row = blockIdx.z;
    const int t = rows.pos[row] + 1;  // keys 0..pos, the new one included
    const int chunk = attn_chunk(t, S);
    const int s_active = (t + chunk - 1) / chunk;
    const int s = blockIdx.x, g = blockIdx.y;
    if (s >= s_active) return;
    const int k0 = s * chunk, k1 = min(t, k0 + chunk);
    {
        const size_t cache = (rows.seq ? (size_t)rows.seq[row] : 0) * rows.seq_stride;
        kc += cache;
        vc += cache;
        q += (size_t)row * rows.q_stride;
        out += (size_t)row * rows.q_stride;
        part_ml += (size_t)row * rows.ml_stride;
        part_acc += (size_t)row * rows.acc_stride;
    }

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int dl = tid % LPK, ks = tid / LPK;
    const float scale = 1.4426950408889634f / sqrtf((float)D);
    const bf16_t *kbase = kc + (size_t)g * max_seq * D;
    const bf16_t *vbase = vc + (size_t)g * max_seq * D;
    if (tid < G) {
        run_m[tid] = -INFINITY;
        run_l[tid] = 0.f;
    }
    float acc[G][8];
#pragma unroll
    for (int hh = 0; hh < G; ++hh)
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[hh][e] = 0.f;

    // Loads of a tile: rows past the range are read from the range's last key (in bounds, finite); their
    // scores are masked to -inf, so their probabilities are exactly 0.
    u32x4 kreg[DS / 8], vreg[KPS];
    auto issue = [&](int tile0) {
        const u32x4 *kp =
            reinterpret_cast<const u32x4 *>(kbase + (size_t)min(tile0 + lane, k1 - 1) * D + wave * DS);
#pragma unroll
        for (int i = 0; i < DS / 8; ++i) kreg[i] = kp[i];
#pragma unroll
        for (int i = 0; i < KPS; ++i)
            vreg[i] = *reinterpret_cast<const u32x4 *>(vbase + (size_t)min(tile0 + ks + KSL * i, k1 - 1) * D + dl * 8);
    };
    issue(k0);  // in flight while q is staged
    static_assert(G * D / 4 <= 256, "one float4 of q per thread");
    {
        float4 v = reinterpret_cast<const float4 *>(q + (size_t)g * G * D)[min(tid, G * D / 4 - 1)];
        if (tid < G * D / 4)
            reinterpret_cast<float4 *>(&q_s[0][0])[tid] =
                make_float4(v.x * scale, v.y * scale, v.z * scale, v.w * scale);
    }

    for (int tile0 = k0; tile0 < k1; tile0 += kKeyTile) {
        const bool ok1 = tile0 + lane < k1;
        if (tile0 != k0) issue(tile0);
        __syncthreads();  // q_s staged (first tile); previous tile's p_s / sc_part fully consumed
        {
            float pa[G];
#pragma unroll
            for (int hh = 0; hh < G; ++hh) pa[hh] = 0.f;
#pragma unroll
            for (int i = 0; i < DS / 8; ++i) {
                float kf[8];
                unpack8(kreg[i], kf);
#pragma unroll
                for (int hh = 0; hh < G; ++hh) {
                    const float4 qa = *reinterpret_cast<const float4 *>(&q_s[hh][wave * DS + 8 * i]);
                    const float4 qb = *reinterpret_cast<const float4 *>(&q_s[hh][wave * DS + 8 * i + 4]);
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
            for (int hh = 0; hh < G; ++hh) sc_part[wave][hh][lane] = pa[hh];
        }
        __syncthreads();
        for (int hh = wave; hh < G; hh += 4) {
            float sc = (sc_part[0][hh][lane] + sc_part[1][hh][lane]) + (sc_part[2][hh][lane] + sc_part[3][hh][lane]);
            if (!ok1) sc = -INFINITY;
            const float m_old = run_m[hh];
            const float m_new = fmaxf(m_old, wave_max(sc));  // finite: the tile's first key is valid
            const float p = exp2f(sc - m_new);
            const float ps = wave_sum(p);
            p_s[hh][lane] = p;
            if (lane == 0) {
                const float c = merge_w(m_old, m_new);
                corr_s[hh] = c;
                run_l[hh] = run_l[hh] * c + ps;
                run_m[hh] = m_new;
            }
        }
        __syncthreads();
#pragma unroll
        for (int hh = 0; hh < G; ++hh) {
            const float c = corr_s[hh];
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[hh][e] *= c;
        }
#pragma unroll
        for (int i = 0; i < KPS; ++i) {
            float vf[8];
            unpack8(vreg[i], vf);
            const int kl = ks + KSL * i;
#pragma unroll
            for (int hh = 0; hh < G; ++hh) {
                const float p = p_s[hh][kl];  // exactly 0 for keys past the range
#pragma unroll
                for (int e = 0; e < 8; ++e) acc[hh][e] = fmaf(p, vf[e], acc[hh][e]);
            }
        }
    }
    // sum the key slots of a wave (LPK lanes apart: whole 16- / 32-lane rows), then the four waves
    static_assert(LPK == 16 || LPK == 8, "key slots are rows of 16 lanes, or halves of them");
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
            for (int e = 0; e < 8; ++e) red_acc[wave][hh][lane * 8 + e] = acc[hh][e];
    }
    __syncthreads();
    // four consecutive output elements per thread: 16-byte LDS reads and one 16-byte store
    for (int idx = tid; idx < G * D / 4; idx += 256) {
        const int hh = idx / (D / 4), e = (idx - hh * (D / 4)) * 4;
        const float4 a0 = *reinterpret_cast<const float4 *>(&red_acc[0][hh][e]);
        const float4 a1 = *reinterpret_cast<const float4 *>(&red_acc[1][hh][e]);
        const float4 a2 = *reinterpret_cast<const float4 *>(&red_acc[2][hh][e]);
        const float4 a3 = *reinterpret_cast<const float4 *>(&red_acc[3][hh][e]);
        const float4 A = make_float4((a0.x + a1.x) + (a2.x + a3.x), (a0.y + a1.y) + (a2.y + a3.y),
                                     (a0.z + a1.z) + (a2.z + a3.z), (a0.w + a1.w) + (a2.w + a3.w));
        if (s_active == 1) {
            const float inv_l = 1.0f / run_l[hh];
            const size_t row_off = (size_t)row * rows.q_stride, i0 = (size_t)(g * G + hh) * D + e;
            if (rows.out_hi) {
                put_attn(rows, out, row_off, i0 + 0, A.x * inv_l);
                put_attn(rows, out, row_off, i0 + 1, A.y * inv_l);
                put_attn(rows, out, row_off, i0 + 2, A.z * inv_l);
                put_attn(rows, out, row_off, i0 + 3, A.w * inv_l);
            } else {
                *reinterpret_cast<float4 *>(out + i0) = make_float4(A.x * inv_l, A.y * inv_l, A.z * inv_l, A.w * inv_l);
            }
        } else {
            const size_t pi = (size_t)(g * G + hh) * S + s;
            *reinterpret_cast<float4 *>(part_acc + pi * D + e) = A;
            if (e == 0) {
                part_ml[pi * 2] = run_m[hh];
                part_ml[pi * 2 + 1] = run_l[hh];
            }
        }
    }
}

// Merges the ranges of one query head.  Block = head; 256 threads = 1024/D groups x D/4 quads of output elements:
// group j sums the ranges i = j (mod 1024/D) in ascending order with 16-byte loads, and the groups are added in a
// fixed order.  The per-range weights exp2(m_i - M) are computed once into LDS.
template <int D>
__global__ __launch_bounds__(256) void k_attn_combine(AttnRows rows, int S, const float *__restrict__ part_ml,
                                                      const float *__restrict__ part_acc, float *__restrict__ out) {
    constexpr int Q = D / 4, NG = 256 / Q;  // quads per row, groups of ranges
    __shared__ float m_s[2], wl_s[kAttnSplits][2];  // wl_s[i][0]: weight of range i; wl_s[0..1][1]: the waves' sums
    __shared__ float4 red[NG][Q];
    const int row = blockIdx.z;
    const int t = rows.pos[row] + 1;
    const int chunk = attn_chunk(t, S);
    const int s_active = (t + chunk - 1) / chunk;
    if (s_active == 1) return;  // the first kernel already wrote the result
    part_ml += (size_t)row * rows.ml_stride;
    part_acc += (size_t)row * rows.acc_stride;
    out += (size_t)row * rows.q_stride;
    const int hh = blockIdx.x, tid = threadIdx.x, q = tid % Q, grp = tid / Q;
    const size_t p0 = (size_t)hh * S;
    // this thread's slice of the unnormalised outputs, issued before anything waits
    constexpr int BATCH = kAttnSplits / NG;
    float4 aa[BATCH];
#pragma unroll
    for (int u = 0; u < BATCH; ++u) {
        const int i = grp + NG * u;
        aa[u] = i < s_active ? reinterpret_cast<const float4 *>(part_acc + (p0 + i) * D)[q] : make_float4(0.f, 0.f, 0.f, 0.f);
    }
    // thread i < 128 holds range i's (max, sum); the overall max and the rescaled sum are two-level reductions
    // (wave, then the two waves that hold ranges) in a fixed order
    static_assert(kAttnSplits == 128, "ranges live in the first two waves");
    float2 ml = make_float2(-INFINITY, 0.f);
    if (tid < s_active) ml = reinterpret_cast<const float2 *>(part_ml)[p0 + tid];
    const int lane = tid & 63, wave = tid >> 6;
    const float mx = wave_max(ml.x);
    if (lane == 0 && wave < 2) m_s[wave] = mx;
    __syncthreads();
    const float M = fmaxf(m_s[0], m_s[1]);
    const float w = merge_w(ml.x, M);
    if (tid < kAttnSplits) wl_s[tid][0] = w;
    const float ls = wave_sum(w * ml.y);
    if (lane == 0 && wave < 2) wl_s[wave][1] = ls;
    __syncthreads();
    const float L = wl_s[0][1] + wl_s[1][1];
    float4 A = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
    for (int u = 0; u < BATCH; ++u) {
        const int i = grp + NG * u;
        if (i < s_active) {
            const float wi = wl_s[i][0];
            A.x += aa[u].x * wi, A.y += aa[u].y * wi, A.z += aa[u].z * wi, A.w += aa[u].w * wi;
        }
    }
    red[grp][q] = A;
    __syncthreads();
    if (grp == 0) {
#pragma unroll
        for (int j = 1; j < NG; ++j) {
            const float4 o = red[j][q];
            A.x += o.x, A.y += o.y, A.z += o.z, A.w += o.w;
        }
        const size_t row_off = (size_t)row * rows.q_stride, i0 = (size_t)hh * D + 4 * q;
        put_attn(rows, out, row_off, i0 + 0, A.x / L);
        put_attn(rows, out, row_off, i0 + 1, A.y / L);
        put_attn(rows, out, row_off, i0 + 2, A.z / L);
        put_attn(rows, out, row_off, i0 + 3, A.w / L);
    }
}

// ---------------------------------------------------------------------------------------
// launchers
// ---------------------------------------------------------------------------------------
void launch_init(const Model &m) {
    const st_config &c = m.c;
    hipLaunchKernelGGL(k_init, dim3(256), dim3(256), 0, m.stream, m.ws.state, m.ws.counters, c.n_kv_heads,
                       m.ws.rope, c.max_seq, c.head_dim / 2, (double)c.rope_theta);
}
void launch_set_token(const Model &m, int32_t token) {
    hipLaunchKernelGGL(k_set_token, dim3(1), dim3(1), 0, m.stream, m.ws.state, token);
}
void launch_set_token_from(const Model &m, const int32_t *tokens_dev, int32_t index) {
    hipLaunchKernelGGL(k_set_token_from, dim3(1), dim3(1), 0, m.stream, m.ws.state, tokens_dev, index);
}
void launch_set_state(const Model &m, int slot, int32_t value) {
    hipLaunchKernelGGL(k_set_state, dim3(1), dim3(1), 0, m.stream, m.ws.state, slot, value);
}

template <int D>
static void launch_attn_t(const Model &m, int layer, hipStream_t stream, int attn_blocks, const AttnRows &rows,
                          int n_rows, const float *q, float *part_ml, float *part_acc, float *out) {
    const st_config &c = m.c;
    const int G = c.n_q_heads / c.n_kv_heads;
    size_t lofs = (size_t)layer * c.n_kv_heads * c.max_seq * c.head_dim;
    dim3 grid(attn_blocks, c.n_kv_heads, n_rows), block(256);
#define ST_ATTN_CASE(GG)                                                                                           \
    case GG:                                                                                                       \
        hipLaunchKernelGGL((k_attn_partial<D, GG>), grid, block, 0, stream, q, m.kcache + lofs, m.vcache + lofs,   \
                           rows, c.max_seq, kAttnSplits, part_ml, part_acc, out);                                  \
        break;
    switch (G) {
        ST_ATTN_CASE(1) ST_ATTN_CASE(2) ST_ATTN_CASE(3) ST_ATTN_CASE(4)
        ST_ATTN_CASE(5) ST_ATTN_CASE(6) ST_ATTN_CASE(7) ST_ATTN_CASE(8)
    }
#undef ST_ATTN_CASE
    if (attn_blocks > 1)  // a single range is finished by the first kernel
        hipLaunchKernelGGL(k_attn_combine<D>, dim3(c.n_q_heads, 1, n_rows), dim3(256), 0, stream, rows, kAttnSplits,
                           part_ml, part_acc, out);
}

// the single-sequence step: one row whose position is state[kPos], sequence 0
template <int D>
static void launch_attn(const Model &m, int layer, hipStream_t stream, int attn_blocks) {
    const AttnRows rows = {m.ws.state + kPos, nullptr, 0, 0, 0, 0, nullptr, nullptr};
    launch_attn_t<D>(m, layer, stream, attn_blocks, rows, 1, m.ws.q1, m.ws.part_ml, m.ws.part_acc, m.ws.o1);
}

void launch_attn_rows(const Model &m, int layer, hipStream_t stream, int attn_blocks, const AttnRows &rows, int n_rows,
                      const float *q, float *part_ml, float *part_acc, float *out) {
    if (m.c.head_dim == 128)
        launch_attn_t<128>(m, layer, stream, attn_blocks, rows, n_rows, q, part_ml, part_acc, out);
    else
        launch_attn_t<64>(m, layer, stream, attn_blocks, rows, n_rows, q, part_ml, part_acc, out);
}

// Rows per block of the residual GEMV: five where that gives 480..1024 blocks (measured at 3584 rows x 18944:
// 24.4 us against 26.0 with four rows, 25.7 with three, 28.4 with seven; 5120 rows take five by the next rule too);
// otherwise, among the candidates that give 480..1024 blocks, the one with the least padding, then the most
// blocks; small matrices take the smallest candidate.
static int pick_rb(int N) {
    if ((N + 4) / 5 >= 480 && (N + 4) / 5 <= 1024) return 5;
    const int cand[] = {8, 7, 5, 4, 3, 2};
    int best = 2, best_blocks = 0;
    long best_waste = -1;
    for (int rb : cand) {
        int blocks = (N + rb - 1) / rb;
        if (blocks < 480 || blocks > 1024) continue;
        long waste = (long)blocks * rb - N;
        if (best_waste < 0 || waste < best_waste || (waste == best_waste && blocks > best_blocks)) {
            best = rb;
            best_waste = waste;
            best_blocks = blocks;
        }
    }
    return best;
}

static void launch_gemv_residual(const Model &m, const bf16_t *W, const float *v, float *x, int N, int K,
                                 hipStream_t stream) {
    const int rb = pick_rb(N);
    const bool deep = K >= 16384;  // long rows: four 16-byte groups per row in flight instead of two
    dim3 grid((N + rb - 1) / rb), block(256);
#define ST_RB_CASE(RBV)                                                                              \
    case RBV:                                                                                        \
        if (deep)                                                                                    \
            hipLaunchKernelGGL((k_gemv_residual<RBV, 4>), grid, block, 0, stream, W, v, x, x, N, K); \
        else                                                                                         \
            hipLaunchKernelGGL((k_gemv_residual<RBV, 2>), grid, block, 0, stream, W, v, x, x, N, K); \
        break;
    switch (rb) {
        ST_RB_CASE(8) ST_RB_CASE(7) ST_RB_CASE(5) ST_RB_CASE(4) ST_RB_CASE(3) ST_RB_CASE(2)
    }
#undef ST_RB_CASE
}

void launch_head(const Model &m, const float *x_row, const st_trigger_rule *rule, int32_t advance,
                 int32_t *out_seq_dev, hipStream_t stream) {
    const st_config &c = m.c;
    size_t lds = sizeof(float) * (size_t)c.hidden;
    int blocks = (c.vocab + 4 * kLmRows - 1) / (4 * kLmRows);
    if (blocks > kLmBlocks) blocks = kLmBlocks;
    if (c.hidden <= 2048)
        hipLaunchKernelGGL(k_lm_head<1>, dim3(blocks), dim3(256), lds, stream, m.lm_head, x_row, m.final_norm,
                           m.ws.logits, m.ws.amax_val, m.ws.amax_idx, c.hidden, c.vocab, c.rms_eps);
    else
        hipLaunchKernelGGL(k_lm_head<4>, dim3(blocks), dim3(256), lds, stream, m.lm_head, x_row, m.final_norm,
                           m.ws.logits, m.ws.amax_val, m.ws.amax_idx, c.hidden, c.vocab, c.rms_eps);
    hipLaunchKernelGGL(k_argmax_final, dim3(1), dim3(256), 0, stream, m.ws.amax_val, m.ws.amax_idx, blocks,
                       m.ws.state, rule ? rule->kw_bitmap : nullptr, rule ? rule->delim_bitmap : nullptr,
                       rule ? rule->window : 1, rule ? rule->vocab : 0, advance, out_seq_dev);
}

// Pairs per wave-group of the gate/up kernel and its grid: one group per wave while the whole grid
// can be resident (3 blocks of 256 threads per CU), a balanced walk over 768 blocks otherwise.
static void gateup_shape(int I, int k_iters, int *r_out, int *blocks_out, bool *one_out) {
    // keeps the up-front loads within the register file; from hidden 3584 on single pairs measured best
    int r = k_iters <= 4 ? 3 : (k_iters <= 6 ? 2 : 1);
    int groups = (I + r - 1) / r;
    int blocks = (groups + 3) / 4;
    *one_out = blocks <= 768;
    if (blocks > 768) blocks = 768;
    *r_out = r;
    *blocks_out = blocks;
}

int attn_bucket(int t) {
    int need = (t + kKeyTile - 1) / kKeyTile;
    if (need >= kAttnSplits) return kAttnSplits;
    if (need > 16) return (need + 7) & ~7;  // multiples of 8 ranges above 1024 keys
    int b = 1;
    while (b < need) b <<= 1;
    return b;
}

void launch_decode_layers(const Model &m, float *x, hipStream_t stream, int attn_blocks) {
    const st_config &c = m.c;
    const int h = c.hidden, d = c.head_dim, nq = c.n_q_heads, nkv = c.n_kv_heads, I = c.intermediate;
    size_t lds_h = sizeof(float) * (size_t)h;
    hipLaunchKernelGGL(k_embed, dim3((h + 255) / 256), dim3(256), 0, stream, m.embed, m.ws.state, x, h, c.vocab);
    const int qkv_units = (nq + 2 * nkv) * (d / 2);
    // two units per wave only where that still leaves 1.5 blocks per CU (measured: 3584 units 14.9 us against 15.2
    // with one unit per wave; 2304 units 10.1 us against 8.9, its 288 blocks sit unevenly on 256 CUs)
    const int r_qkv = qkv_units >= 3072 ? 2 : 1;
    const bool small_h = h <= 2048;
    int r_gu, gu_blocks;
    bool gu_one;
    gateup_shape(I, (h + 511) / 512, &r_gu, &gu_blocks, &gu_one);
    for (int l = 0; l < c.n_layers; ++l) {
        size_t lofs = (size_t)l * nkv * c.max_seq * d;
        {
            dim3 grid((qkv_units + 4 * r_qkv - 1) / (4 * r_qkv)), block(256);
#define ST_QKV(RR, XX)                                                                                       \
    hipLaunchKernelGGL((k_qkv_rope<RR, XX>), grid, block, lds_h, stream, m.wqkv[l], m.bqkv[l], x,          \
                       m.norm_attn[l], m.ws.state, m.ws.rope, m.ws.q1, m.kcache + lofs, m.vcache + lofs, h, \
                       nq, nkv, d, c.max_seq, c.rms_eps)
            if (r_qkv == 2 && small_h) ST_QKV(2, 1);
            else if (r_qkv == 2) ST_QKV(2, 4);
            else if (small_h) ST_QKV(1, 1);
            else ST_QKV(1, 4);
#undef ST_QKV
        }
        if (d == 128)
            launch_attn<128>(m, l, stream, attn_blocks);
        else
            launch_attn<64>(m, l, stream, attn_blocks);
        launch_gemv_residual(m, m.wo[l], m.ws.o1, x, h, nq * d, stream);
        {
            dim3 grid(gu_blocks), block(256);
            hipEvent_t e0 = m.timers ? m.timers->ev[2 + 2 * l] : nullptr;
            hipEvent_t e1 = m.timers ? m.timers->ev[3 + 2 * l] : nullptr;
#define ST_GU(RR, XX)                                                                                     \
    do {                                                                                                  \
        if (!m.timers && gu_one)                                                                          \
            hipLaunchKernelGGL((k_gateup_swiglu<RR, XX, true>), grid, block, lds_h, stream, m.wgu[l], x,  \
                               m.norm_mlp[l], m.ws.a1, h, I, c.rms_eps);                                  \
        else if (!m.timers)                                                                               \
            hipLaunchKernelGGL((k_gateup_swiglu<RR, XX, false>), grid, block, lds_h, stream, m.wgu[l], x, \
                               m.norm_mlp[l], m.ws.a1, h, I, c.rms_eps);                                  \
        else if (gu_one)                                                                                  \
            hipExtLaunchKernelGGL((k_gateup_swiglu<RR, XX, true>), grid, block, lds_h, stream, e0, e1, 0, \
                                  m.wgu[l], x, m.norm_mlp[l], m.ws.a1, h, I, c.rms_eps);                  \
        else                                                                                              \
            hipExtLaunchKernelGGL((k_gateup_swiglu<RR, XX, false>), grid, block, lds_h, stream, e0, e1, 0, \
                                  m.wgu[l], x, m.norm_mlp[l], m.ws.a1, h, I, c.rms_eps);                  \
    } while (0)
            if (r_gu == 3 && small_h) ST_GU(3, 1);
            else if (r_gu == 3) ST_GU(3, 4);
            else if (r_gu == 2) ST_GU(2, 4);
            else ST_GU(1, 4);
#undef ST_GU
        }
        launch_gemv_residual(m, m.wdown[l], m.ws.a1, x, h, I, stream);
    }
}

void launch_decode_step(const Model &m, const st_trigger_rule *rule, int32_t *out_seq_dev, hipStream_t stream,
                        int attn_blocks) {
    if (m.persist_on && !m.timers) {
        launch_decode_persist(m, rule, out_seq_dev, stream);
        return;
    }
    launch_decode_layers(m, m.ws.x, stream, attn_blocks);
    launch_head(m, m.ws.x, rule, 1, out_seq_dev, stream);
}

}  // namespace st
