// Single-token decode step (paper Section 4, "decode" stage): weight-streaming bf16
// matrix-vector products with fused RMSNorm / bias / RoPE / KV append / SwiGLU / residual
// epilogues, split-K GQA attention over the KV cache, LM head with greedy arg-max.
//
// Every kernel takes the position and the fed token from the model's device state block,
// so a step can be enqueued (or replayed) without the host knowing either.
#include <hip/hip_ext.h>

#include "st_device.h"
#include "st_internal.h"

namespace st {

// ---------------------------------------------------------------------------------------
// x vector in LDS.  A lane consumes 8 consecutive activations per 16-byte weight load; they
// are stored as two float4 arrays (elements 0-3 and 4-7 of every group of 8) so that the
// 64 lanes of a wave read 64 consecutive float4 from each array.
// ---------------------------------------------------------------------------------------
__device__ __forceinline__ int xs_slot(int e, int half) { return ((e >> 3) << 2) + (e & 3) + ((e >> 2) & 1) * half; }

constexpr int kMaxChunk = 8192;  // floats of x staged at once

// Dot products of NR weight rows with the staged x chunk.  wrow[r] points at the first
// 16-byte group of row r inside the chunk; n8 = number of 8-element groups in the chunk.
template <int NR>
__device__ __forceinline__ void wave_rows_dot(const u32x4 *const (&wrow)[NR], const float *xs, int half,
                                              int n8, int lane, float (&acc)[NR]) {
    const float4 *xa = reinterpret_cast<const float4 *>(xs);
    const float4 *xb = reinterpret_cast<const float4 *>(xs + half);
    int c = lane;
    for (; c + 64 < n8; c += 128) {
        u32x4 w0[NR], w1[NR];
#pragma unroll
        for (int r = 0; r < NR; ++r) {
            w0[r] = __builtin_nontemporal_load(wrow[r] + c);
            w1[r] = __builtin_nontemporal_load(wrow[r] + c + 64);
        }
        float4 a0 = xa[c], b0 = xb[c], a1 = xa[c + 64], b1 = xb[c + 64];
#pragma unroll
        for (int r = 0; r < NR; ++r) {
            acc[r] = dot8(w0[r], a0, b0, acc[r]);
            acc[r] = dot8(w1[r], a1, b1, acc[r]);
        }
    }
    if (c < n8) {
        u32x4 w0[NR];
#pragma unroll
        for (int r = 0; r < NR; ++r) w0[r] = __builtin_nontemporal_load(wrow[r] + c);
        float4 a0 = xa[c], b0 = xb[c];
#pragma unroll
        for (int r = 0; r < NR; ++r) acc[r] = dot8(w0[r], a0, b0, acc[r]);
    }
}

// Stages rmsnorm(x) * g (whole vector, n <= kMaxChunk) into xs.  256 threads.
__device__ __forceinline__ void stage_rmsnorm(const float *__restrict__ x, const bf16_t *__restrict__ g, int n,
                                              float eps, float *xs, float *red) {
    int half = n >> 1;
    float ss = 0.f;
    for (int i = threadIdx.x; i < n; i += 256) {
        float v = x[i];
        ss = fmaf(v, v, ss);
        xs[xs_slot(i, half)] = v;
    }
    ss = block_sum_256(ss, red);
    float inv = 1.0f / sqrtf(ss / (float)n + eps);
    for (int i = threadIdx.x; i < n; i += 256) {
        int s = xs_slot(i, half);
        xs[s] = xs[s] * inv * bf16_to_f32(g[i]);
    }
    __syncthreads();
}

__device__ __forceinline__ void stage_plain(const float *__restrict__ v, int n, float *xs) {
    int half = n >> 1;
    for (int i = threadIdx.x; i < n; i += 256) xs[xs_slot(i, half)] = v[i];
    __syncthreads();
}

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
// needs no exchange.
// ---------------------------------------------------------------------------------------
template <int R>
__global__ __launch_bounds__(256) void k_qkv_rope(const bf16_t *__restrict__ W, const bf16_t *__restrict__ bias,
                                                  const float *__restrict__ x, const bf16_t *__restrict__ g,
                                                  const int32_t *__restrict__ state, const float2 *__restrict__ rope,
                                                  float *__restrict__ q_out, bf16_t *__restrict__ kc,
                                                  bf16_t *__restrict__ vc, int h, int nq, int nkv, int d,
                                                  int max_seq, float eps) {
    extern __shared__ __align__(16) float xs[];
    __shared__ float red[4];
    stage_rmsnorm(x, g, h, eps, xs, red);

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int half_d = d >> 1;
    const int n_units = (nq + 2 * nkv) * half_d;
    const int u0 = (blockIdx.x * 4 + wave) * R;
    if (u0 >= n_units) return;
    const int n8 = h >> 3;
    const u32x4 *wrow[2 * R];
    float acc[2 * R];
    int row0[R];
#pragma unroll
    for (int j = 0; j < R; ++j) {
        int u = min(u0 + j, n_units - 1);
        int head = u / half_d, i = u - head * half_d;
        row0[j] = head * d + i;
        wrow[2 * j] = reinterpret_cast<const u32x4 *>(W + (size_t)row0[j] * h);
        wrow[2 * j + 1] = reinterpret_cast<const u32x4 *>(W + (size_t)(row0[j] + half_d) * h);
        acc[2 * j] = acc[2 * j + 1] = 0.f;
    }
    wave_rows_dot<2 * R>(wrow, xs, h >> 1, n8, lane, acc);
#pragma unroll
    for (int r = 0; r < 2 * R; ++r) acc[r] = wave_sum(acc[r]);

    const int pos = state[kPos];
#pragma unroll
    for (int j = 0; j < R; ++j) {
        if (lane == j && u0 + j < n_units) {
            int r0 = row0[j], r1 = r0 + half_d;
            int head = r0 / d, i = r0 - head * d;
            float lo = acc[2 * j], hi = acc[2 * j + 1];
            if (bias) {
                lo += bf16_to_f32(bias[r0]);
                hi += bf16_to_f32(bias[r1]);
            }
            if (head < nq + nkv) {
                float2 cs = rope[(size_t)pos * half_d + i];
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
// y[i] = res[i] + W[i,:] . v   (O projection and down projection; res may alias y)
// ---------------------------------------------------------------------------------------
template <int NR>
__global__ __launch_bounds__(256) void k_gemv_residual(const bf16_t *__restrict__ W, const float *__restrict__ v,
                                                       const float *res, float *y, int N, int K) {
    extern __shared__ __align__(16) float xs[];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int r0 = (blockIdx.x * 4 + wave) * NR;
    float acc[NR];
#pragma unroll
    for (int r = 0; r < NR; ++r) acc[r] = 0.f;
    for (int k0 = 0; k0 < K; k0 += kMaxChunk) {
        int kc = min(kMaxChunk, K - k0);
        if (k0 > 0) __syncthreads();
        stage_plain(v + k0, kc, xs);
        if (r0 < N) {
            const u32x4 *wrow[NR];
#pragma unroll
            for (int r = 0; r < NR; ++r)
                wrow[r] = reinterpret_cast<const u32x4 *>(W + (size_t)min(r0 + r, N - 1) * K + k0);
            wave_rows_dot<NR>(wrow, xs, kc >> 1, kc >> 3, lane, acc);
        }
    }
    if (r0 >= N) return;
#pragma unroll
    for (int r = 0; r < NR; ++r) acc[r] = wave_sum(acc[r]);
#pragma unroll
    for (int r = 0; r < NR; ++r)
        if (lane == r && r0 + r < N) y[r0 + r] = res[r0 + r] + acc[r];
}

// ---------------------------------------------------------------------------------------
// a[i] = silu(Wg[i,:] . y) * (Wu[i,:] . y),  y = rmsnorm(x) * g.  Gate rows [0,I), up rows [I,2I).
// ---------------------------------------------------------------------------------------
template <int R>
__global__ __launch_bounds__(256) void k_gateup_swiglu(const bf16_t *__restrict__ W, const float *__restrict__ x,
                                                       const bf16_t *__restrict__ g, float *__restrict__ a, int h,
                                                       int I, float eps) {
    extern __shared__ __align__(16) float xs[];
    __shared__ float red[4];
    stage_rmsnorm(x, g, h, eps, xs, red);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int u0 = (blockIdx.x * 4 + wave) * R;
    if (u0 >= I) return;
    const u32x4 *wrow[2 * R];
    float acc[2 * R];
#pragma unroll
    for (int j = 0; j < R; ++j) {
        int u = min(u0 + j, I - 1);
        wrow[2 * j] = reinterpret_cast<const u32x4 *>(W + (size_t)u * h);
        wrow[2 * j + 1] = reinterpret_cast<const u32x4 *>(W + (size_t)(I + u) * h);
        acc[2 * j] = acc[2 * j + 1] = 0.f;
    }
    wave_rows_dot<2 * R>(wrow, xs, h >> 1, h >> 3, lane, acc);
#pragma unroll
    for (int r = 0; r < 2 * R; ++r) acc[r] = wave_sum(acc[r]);
#pragma unroll
    for (int j = 0; j < R; ++j)
        if (lane == j && u0 + j < I) {
            float gt = acc[2 * j], up = acc[2 * j + 1];
            a[u0 + j] = gt / (1.0f + expf(-gt)) * up;
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

__global__ __launch_bounds__(256) void k_lm_head(const bf16_t *__restrict__ W, const float *__restrict__ x,
                                                 const bf16_t *__restrict__ g, float *__restrict__ logits,
                                                 float *__restrict__ pval, int32_t *__restrict__ pidx, int h, int V,
                                                 float eps) {
    extern __shared__ __align__(16) float xs[];
    __shared__ float red[4];
    __shared__ float bv[4];
    __shared__ int bi[4];
    stage_rmsnorm(x, g, h, eps, xs, red);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    float best = -INFINITY;
    int besti = 0x7fffffff;
    const int rows_per_pass = gridDim.x * 4 * kLmRows;
    for (int r0 = (blockIdx.x * 4 + wave) * kLmRows; r0 < V; r0 += rows_per_pass) {
        const u32x4 *wrow[kLmRows];
        float acc[kLmRows];
#pragma unroll
        for (int r = 0; r < kLmRows; ++r) {
            wrow[r] = reinterpret_cast<const u32x4 *>(W + (size_t)min(r0 + r, V - 1) * h);
            acc[r] = 0.f;
        }
        wave_rows_dot<kLmRows>(wrow, xs, h >> 1, h >> 3, lane, acc);
#pragma unroll
        for (int r = 0; r < kLmRows; ++r) acc[r] = wave_sum(acc[r]);
#pragma unroll
        for (int r = 0; r < kLmRows; ++r)
            if (r0 + r < V) {
                float val = acc[r];
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
// query heads of the group.  D/8 lanes share one key (16 bytes of K and of V each); online
// softmax in base 2 per lane group; groups, then waves, are merged; the last block to finish
// for a kv head merges the ranges (fixed order, so the result does not depend on timing).
// ---------------------------------------------------------------------------------------
__device__ __forceinline__ float merge_w(float m, float M) { return m == -INFINITY ? 0.f : exp2f(m - M); }

template <int D, int G>
__global__ __launch_bounds__(256) void k_attn_decode(const float *__restrict__ q, const bf16_t *__restrict__ kc,
                                                     const bf16_t *__restrict__ vc, const int32_t *__restrict__ state,
                                                     int max_seq, int S, float *part_ml, float *part_acc,
                                                     int32_t *counters, float *__restrict__ out) {
    constexpr int LPK = D / 8;     // lanes per key
    constexpr int KPW = 64 / LPK;  // keys per wave per pass
    __shared__ float sm_ml[4][G][2];
    __shared__ float sm_acc[4][G][D];
    __shared__ int is_last;

    const int t = state[kPos] + 1;  // keys 0..pos, the new one included
    int chunk = (t + S - 1) / S;
    chunk = max(64, (chunk + 15) & ~15);
    const int s_active = (t + chunk - 1) / chunk;
    const int s = blockIdx.x, g = blockIdx.y;
    if (s >= s_active) return;
    const int k0 = s * chunk, k1 = min(t, k0 + chunk);

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int slot = lane / LPK, dl = lane % LPK;
    const float scale = 1.4426950408889634f / sqrtf((float)D);

    float qf[G][8], acc[G][8], m[G], l[G];
#pragma unroll
    for (int hh = 0; hh < G; ++hh) {
        const float *qp = q + (size_t)(g * G + hh) * D + dl * 8;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            qf[hh][e] = qp[e] * scale;
            acc[hh][e] = 0.f;
        }
        m[hh] = -INFINITY;
        l[hh] = 0.f;
    }
    const uint4 *kb = reinterpret_cast<const uint4 *>(kc + (size_t)g * max_seq * D);
    const uint4 *vb = reinterpret_cast<const uint4 *>(vc + (size_t)g * max_seq * D);
    for (int j = k0 + wave * KPW + slot; j < k1; j += 4 * KPW) {
        uint4 kk = kb[(size_t)j * LPK + dl];
        uint4 vv = vb[(size_t)j * LPK + dl];
        float kf[8] = {bf16_lo(kk.x), bf16_hi(kk.x), bf16_lo(kk.y), bf16_hi(kk.y),
                       bf16_lo(kk.z), bf16_hi(kk.z), bf16_lo(kk.w), bf16_hi(kk.w)};
        float vf[8] = {bf16_lo(vv.x), bf16_hi(vv.x), bf16_lo(vv.y), bf16_hi(vv.y),
                       bf16_lo(vv.z), bf16_hi(vv.z), bf16_lo(vv.w), bf16_hi(vv.w)};
#pragma unroll
        for (int hh = 0; hh < G; ++hh) {
            float sc = 0.f;
#pragma unroll
            for (int e = 0; e < 8; ++e) sc = fmaf(qf[hh][e], kf[e], sc);
#pragma unroll
            for (int o = 1; o < LPK; o <<= 1) sc += __shfl_xor(sc, o, kWave);
            float mn = fmaxf(m[hh], sc);
            float c = merge_w(m[hh], mn);
            float p = exp2f(sc - mn);
            l[hh] = l[hh] * c + p;
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[hh][e] = acc[hh][e] * c + p * vf[e];
            m[hh] = mn;
        }
    }
    // merge the KPW lane groups of the wave
#pragma unroll
    for (int o = LPK; o < 64; o <<= 1) {
#pragma unroll
        for (int hh = 0; hh < G; ++hh) {
            float m2 = __shfl_xor(m[hh], o, kWave), l2 = __shfl_xor(l[hh], o, kWave);
            float M = fmaxf(m[hh], m2);
            float w1 = merge_w(m[hh], M), w2 = merge_w(m2, M);
            l[hh] = l[hh] * w1 + l2 * w2;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                float a2 = __shfl_xor(acc[hh][e], o, kWave);
                acc[hh][e] = acc[hh][e] * w1 + a2 * w2;
            }
            m[hh] = M;
        }
    }
    if (lane < LPK) {
#pragma unroll
        for (int hh = 0; hh < G; ++hh) {
            if (lane == 0) {
                sm_ml[wave][hh][0] = m[hh];
                sm_ml[wave][hh][1] = l[hh];
            }
#pragma unroll
            for (int e = 0; e < 8; ++e) sm_acc[wave][hh][lane * 8 + e] = acc[hh][e];
        }
    }
    __syncthreads();
    // merge the four waves and publish this range's partial result
    for (int idx = threadIdx.x; idx < G * D; idx += 256) {
        int hh = idx / D, e = idx - hh * D;
        float M = fmaxf(fmaxf(sm_ml[0][hh][0], sm_ml[1][hh][0]), fmaxf(sm_ml[2][hh][0], sm_ml[3][hh][0]));
        float L = 0.f, A = 0.f;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            float ww = merge_w(sm_ml[w][hh][0], M);
            L += sm_ml[w][hh][1] * ww;
            A += sm_acc[w][hh][e] * ww;
        }
        size_t pi = (size_t)(g * G + hh) * S + s;
        part_acc[pi * D + e] = A;
        if (e == 0) {
            part_ml[pi * 2] = M;
            part_ml[pi * 2 + 1] = L;
        }
    }
    __threadfence();
    __syncthreads();
    if (threadIdx.x == 0) {
        int prev = atomicAdd(&counters[g], 1);
        is_last = (prev == s_active - 1);
    }
    __syncthreads();
    if (!is_last) return;
    __threadfence();
    for (int idx = threadIdx.x; idx < G * D; idx += 256) {
        int hh = idx / D, e = idx - hh * D;
        size_t p0 = (size_t)(g * G + hh) * S;
        float M = -INFINITY;
        for (int i = 0; i < s_active; ++i) M = fmaxf(M, part_ml[(p0 + i) * 2]);
        float L = 0.f, A = 0.f;
        for (int i = 0; i < s_active; ++i) {
            float ww = merge_w(part_ml[(p0 + i) * 2], M);
            L += part_ml[(p0 + i) * 2 + 1] * ww;
            A += part_acc[(p0 + i) * D + e] * ww;
        }
        out[(size_t)(g * G + hh) * D + e] = A / L;
    }
    if (threadIdx.x == 0) counters[g] = 0;
}

// ---------------------------------------------------------------------------------------
// launchers
// ---------------------------------------------------------------------------------------
static int pick_rows(int units, int max_r) {
    // most rows per wave that still leaves >= 2048 waves (8 per CU), at least 1
    int r = max_r;
    while (r > 1 && (units + r - 1) / r < 2048) r >>= 1;
    return r;
}

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
static void launch_attn(const Model &m, int layer) {
    const st_config &c = m.c;
    const int G = c.n_q_heads / c.n_kv_heads;
    size_t lofs = (size_t)layer * c.n_kv_heads * c.max_seq * c.head_dim;
    dim3 grid(kAttnSplits, c.n_kv_heads), block(256);
#define ST_ATTN_CASE(GG)                                                                                   \
    case GG:                                                                                               \
        hipLaunchKernelGGL((k_attn_decode<D, GG>), grid, block, 0, m.stream, m.ws.q1, m.kcache + lofs,     \
                           m.vcache + lofs, m.ws.state, c.max_seq, kAttnSplits, m.ws.part_ml, m.ws.part_acc, \
                           m.ws.counters, m.ws.o1);                                                        \
        break;
    switch (G) {
        ST_ATTN_CASE(1) ST_ATTN_CASE(2) ST_ATTN_CASE(3) ST_ATTN_CASE(4)
        ST_ATTN_CASE(5) ST_ATTN_CASE(6) ST_ATTN_CASE(7) ST_ATTN_CASE(8)
    }
#undef ST_ATTN_CASE
}

static void launch_gemv_residual(const Model &m, const bf16_t *W, const float *v, float *x, int N, int K) {
    int nr = pick_rows(N, 4);
    size_t lds = sizeof(float) * (size_t)(K < kMaxChunk ? K : kMaxChunk);
    int rows_per_block = 4 * nr;
    dim3 grid((N + rows_per_block - 1) / rows_per_block), block(256);
    switch (nr) {
        case 4: hipLaunchKernelGGL(k_gemv_residual<4>, grid, block, lds, m.stream, W, v, x, x, N, K); break;
        case 2: hipLaunchKernelGGL(k_gemv_residual<2>, grid, block, lds, m.stream, W, v, x, x, N, K); break;
        default: hipLaunchKernelGGL(k_gemv_residual<1>, grid, block, lds, m.stream, W, v, x, x, N, K); break;
    }
}

void launch_head(const Model &m, const float *x_row, const st_trigger_rule *rule, int32_t advance,
                 int32_t *out_seq_dev) {
    const st_config &c = m.c;
    size_t lds = sizeof(float) * (size_t)c.hidden;
    int blocks = (c.vocab + 4 * kLmRows - 1) / (4 * kLmRows);
    if (blocks > kLmBlocks) blocks = kLmBlocks;
    hipLaunchKernelGGL(k_lm_head, dim3(blocks), dim3(256), lds, m.stream, m.lm_head, x_row, m.final_norm,
                       m.ws.logits, m.ws.amax_val, m.ws.amax_idx, c.hidden, c.vocab, c.rms_eps);
    hipLaunchKernelGGL(k_argmax_final, dim3(1), dim3(256), 0, m.stream, m.ws.amax_val, m.ws.amax_idx, blocks,
                       m.ws.state, rule ? rule->kw_bitmap : nullptr, rule ? rule->delim_bitmap : nullptr,
                       rule ? rule->window : 1, rule ? rule->vocab : 0, advance, out_seq_dev);
}

void launch_decode_layers(const Model &m, float *x) {
    const st_config &c = m.c;
    const int h = c.hidden, d = c.head_dim, nq = c.n_q_heads, nkv = c.n_kv_heads, I = c.intermediate;
    size_t lds_h = sizeof(float) * (size_t)h;
    hipLaunchKernelGGL(k_embed, dim3((h + 255) / 256), dim3(256), 0, m.stream, m.embed, m.ws.state, x, h, c.vocab);
    const int qkv_units = (nq + 2 * nkv) * (d / 2);
    const int r_qkv = pick_rows(qkv_units, 2);
    const int r_gu = pick_rows(I, 4);
    for (int l = 0; l < c.n_layers; ++l) {
        size_t lofs = (size_t)l * nkv * c.max_seq * d;
        {
            dim3 grid((qkv_units + 4 * r_qkv - 1) / (4 * r_qkv)), block(256);
            if (r_qkv == 2)
                hipLaunchKernelGGL(k_qkv_rope<2>, grid, block, lds_h, m.stream, m.wqkv[l], m.bqkv[l], x,
                                   m.norm_attn[l], m.ws.state, m.ws.rope, m.ws.q1, m.kcache + lofs,
                                   m.vcache + lofs, h, nq, nkv, d, c.max_seq, c.rms_eps);
            else
                hipLaunchKernelGGL(k_qkv_rope<1>, grid, block, lds_h, m.stream, m.wqkv[l], m.bqkv[l], x,
                                   m.norm_attn[l], m.ws.state, m.ws.rope, m.ws.q1, m.kcache + lofs,
                                   m.vcache + lofs, h, nq, nkv, d, c.max_seq, c.rms_eps);
        }
        if (d == 128)
            launch_attn<128>(m, l);
        else
            launch_attn<64>(m, l);
        launch_gemv_residual(m, m.wo[l], m.ws.o1, x, h, nq * d);
        {
            dim3 grid((I + 4 * r_gu - 1) / (4 * r_gu)), block(256);
            hipEvent_t e0 = m.timers ? m.timers->ev[2 + 2 * l] : nullptr;
            hipEvent_t e1 = m.timers ? m.timers->ev[3 + 2 * l] : nullptr;
            switch (r_gu) {
                case 4:
                    hipExtLaunchKernelGGL(k_gateup_swiglu<4>, grid, block, lds_h, m.stream, e0, e1, 0, m.wgu[l], x,
                                          m.norm_mlp[l], m.ws.a1, h, I, c.rms_eps);
                    break;
                case 2:
                    hipExtLaunchKernelGGL(k_gateup_swiglu<2>, grid, block, lds_h, m.stream, e0, e1, 0, m.wgu[l], x,
                                          m.norm_mlp[l], m.ws.a1, h, I, c.rms_eps);
                    break;
                default:
                    hipExtLaunchKernelGGL(k_gateup_swiglu<1>, grid, block, lds_h, m.stream, e0, e1, 0, m.wgu[l], x,
                                          m.norm_mlp[l], m.ws.a1, h, I, c.rms_eps);
                    break;
            }
        }
        launch_gemv_residual(m, m.wdown[l], m.ws.a1, x, h, I);
    }
}

void launch_decode_step(const Model &m, const st_trigger_rule *rule, int32_t *out_seq_dev) {
    launch_decode_layers(m, m.ws.x);
    launch_head(m, m.ws.x, rule, 1, out_seq_dev);
}

}  // namespace st
