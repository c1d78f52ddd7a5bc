// Catch-up ("prefix") pass over a chunk of m tokens on top of an existing KV cache (paper
// Section 4, Table 3, Eq. 1): the dense part of the path.  bf16 MFMA GEMMs with fused bias /
// residual / SwiGLU epilogues, RoPE + KV append, and causal flash attention with a key offset.
#include "st_device.h"
#include "st_internal.h"

namespace st {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ bf16x8 as_bf16x8(u32x4 v) { return __builtin_bit_cast(bf16x8, v); }

// ---------------------------------------------------------------------------------------
// rows: embedding gather and RMSNorm
// ---------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_embed_rows(const bf16_t *__restrict__ E, const int32_t *__restrict__ tokens,
                                                    float *__restrict__ X, int h, int vocab) {
    int tok = tokens[blockIdx.x];
    tok = tok < 0 ? 0 : (tok >= vocab ? vocab - 1 : tok);
    const bf16_t *row = E + (size_t)tok * h;
    float *x = X + (size_t)blockIdx.x * h;
    for (int i = threadIdx.x; i < h; i += 256) x[i] = bf16_to_f32(row[i]);
}

// Records the last fed token for the trigger's one-token look-back.
__global__ void k_note_fed(int32_t *state, const int32_t *tokens, int index, int vocab) {
    int tok = tokens[index];
    state[kFed] = tok < 0 ? 0 : (tok >= vocab ? vocab - 1 : tok);
}

__global__ __launch_bounds__(256) void k_rmsnorm_rows(const float *__restrict__ X, const bf16_t *__restrict__ g,
                                                      bf16_t *__restrict__ Y, int h, float eps) {
    __shared__ float red[4];
    const float *x = X + (size_t)blockIdx.x * h;
    bf16_t *y = Y + (size_t)blockIdx.x * h;
    float ss = 0.f;
    for (int i = threadIdx.x; i < h; i += 256) {
        float v = x[i];
        ss = fmaf(v, v, ss);
    }
    ss = block_sum_256(ss, red);
    float inv = 1.0f / sqrtf(ss / (float)h + eps);
    for (int i = threadIdx.x; i < h; i += 256) y[i] = f32_to_bf16(x[i] * inv * bf16_to_f32(g[i]));
}

// ---------------------------------------------------------------------------------------
// C[M][N] = A[M][K] * B[N][K]^T on MFMA 32x32x16 bf16.  Block 256 threads = 2x2 waves, block
// tile 128 x 128 (B-tile rows), wave tile 64 x 64, K step 32, LDS double-buffered.
//   EPI 0: out_f32 = acc + bias        EPI 1: out_f32 += acc (residual)
//   EPI 2: the B tile holds 64 gate rows then the matching 64 up rows; out_bf16 = silu(gate)*up
// ---------------------------------------------------------------------------------------
constexpr int kBM = 128, kBN = 128, kBK = 32, kLdsStride = kBK + 8;  // 80-byte rows: conflict-free 16-byte reads

template <int EPI>
__global__ __launch_bounds__(256) void k_gemm(const bf16_t *__restrict__ A, int lda, const bf16_t *__restrict__ B,
                                              int M, int N, int K, float *outf, bf16_t *__restrict__ outb, int ldo,
                                              const bf16_t *__restrict__ bias) {
    __shared__ __align__(16) bf16_t As[2][kBM * kLdsStride];
    __shared__ __align__(16) bf16_t Bs[2][kBN * kLdsStride];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int m0 = blockIdx.y * kBM;
    const int n0 = blockIdx.x * (EPI == 2 ? kBN / 2 : kBN);
    const int l32 = lane & 31, kg = lane >> 5;

    // global -> register staging: every thread owns chunks q = tid and tid + 256 of both tiles
    const bf16_t *ga[2], *gb[2];
    bool va[2], vb[2];
    int soff[2], kcol[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        int q = tid + i * 256, row = q >> 2, kc = q & 3;
        kcol[i] = kc * 8;
        soff[i] = row * kLdsStride + kc * 8;
        int am = m0 + row;
        va[i] = am < M;
        ga[i] = A + (size_t)(va[i] ? am : 0) * lda + kc * 8;
        int bn;
        if (EPI == 2) {
            int half = row >> 6, r = row & 63;
            vb[i] = n0 + r < N;  // N is the number of output columns (I)
            bn = (vb[i] ? n0 + r : 0) + half * N;
        } else {
            vb[i] = n0 + row < N;
            bn = vb[i] ? n0 + row : 0;
        }
        gb[i] = B + (size_t)bn * K + kc * 8;
    }
    u32x4 ra[2], rb[2];
    const u32x4 zero = {0, 0, 0, 0};
    auto fetch = [&](int k0) {
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            bool kin = k0 + kcol[i] < K;
            ra[i] = (va[i] && kin) ? *reinterpret_cast<const u32x4 *>(ga[i] + k0) : zero;
            rb[i] = (vb[i] && kin) ? *reinterpret_cast<const u32x4 *>(gb[i] + k0) : zero;
        }
    };
    auto stash = [&](int buf) {
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            *reinterpret_cast<u32x4 *>(&As[buf][soff[i]]) = ra[i];
            *reinterpret_cast<u32x4 *>(&Bs[buf][soff[i]]) = rb[i];
        }
    };

    f32x16 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    int brow[2];
#pragma unroll
    for (int j = 0; j < 2; ++j) brow[j] = (EPI == 2 ? j * 64 + wn * 32 : wn * 64 + j * 32) + l32;

    const int nk = (K + kBK - 1) / kBK;
    fetch(0);
    stash(0);
    __syncthreads();
    for (int kt = 0; kt < nk; ++kt) {
        const int buf = kt & 1;
        if (kt + 1 < nk) fetch((kt + 1) * kBK);
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            bf16x8 af[2], bfr[2];
#pragma unroll
            for (int i = 0; i < 2; ++i)
                af[i] = as_bf16x8(*reinterpret_cast<const u32x4 *>(
                    &As[buf][(wm * 64 + i * 32 + l32) * kLdsStride + ks * 16 + kg * 8]));
#pragma unroll
            for (int j = 0; j < 2; ++j)
                bfr[j] = as_bf16x8(
                    *reinterpret_cast<const u32x4 *>(&Bs[buf][brow[j] * kLdsStride + ks * 16 + kg * 8]));
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0);
        }
        if (kt + 1 < nk) stash(buf ^ 1);
        __syncthreads();
    }

    // epilogue: register r of a 32x32 tile is row 8*(r/4) + 4*(lane/32) + r%4, column lane%32
#pragma unroll
    for (int i = 0; i < 2; ++i) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            int row = m0 + wm * 64 + i * 32 + 8 * (r >> 2) + 4 * kg + (r & 3);
            if (row >= M) continue;
            if (EPI == 2) {
                int col = n0 + wn * 32 + l32;
                if (col < N) {
                    float gt = acc[i][0][r], up = acc[i][1][r];
                    outb[(size_t)row * ldo + col] = f32_to_bf16(gt / (1.0f + expf(-gt)) * up);
                }
            } else {
#pragma unroll
                for (int j = 0; j < 2; ++j) {
                    int col = n0 + wn * 64 + j * 32 + l32;
                    if (col >= N) continue;
                    float *o = outf + (size_t)row * ldo + col;
                    if (EPI == 0)
                        *o = acc[i][j][r] + (bias ? bf16_to_f32(bias[col]) : 0.f);
                    else
                        *o += acc[i][j][r];
                }
            }
        }
    }
}

// ---------------------------------------------------------------------------------------
// RoPE on q and k at absolute positions pos0 + row, K/V appended to the cache, q kept as bf16.
// grid (rows, heads), block d/2 threads: one rotation pair per thread.
// ---------------------------------------------------------------------------------------
__global__ void k_rope_append(const float *__restrict__ qkv, const float2 *__restrict__ rope,
                              bf16_t *__restrict__ qb, bf16_t *__restrict__ kc, bf16_t *__restrict__ vc, int pos0,
                              int nq, int nkv, int d, int max_seq) {
    const int row = blockIdx.x, head = blockIdx.y, i = threadIdx.x, half = d >> 1;
    const int pos = pos0 + row;
    const float *src = qkv + (size_t)row * (nq + 2 * nkv) * d + head * d;
    float lo = src[i], hi = src[i + half];
    if (head < nq + nkv) {
        float2 cs = rope[(size_t)pos * half + i];
        float nlo = lo * cs.x - hi * cs.y;
        float nhi = hi * cs.x + lo * cs.y;
        lo = nlo;
        hi = nhi;
    }
    bf16_t *dst;
    if (head < nq)
        dst = qb + (size_t)row * nq * d + head * d;
    else if (head < nq + nkv)
        dst = kc + ((size_t)(head - nq) * max_seq + pos) * d;
    else
        dst = vc + ((size_t)(head - nq - nkv) * max_seq + pos) * d;
    dst[i] = f32_to_bf16(lo);
    dst[i + half] = f32_to_bf16(hi);
}

// ---------------------------------------------------------------------------------------
// Causal flash attention of m query rows at absolute positions kv0 + row over keys [0, kv0 + row].
// Block = 4 waves x 32 queries of one head; keys go through LDS in tiles of 32 (V transposed).
// Each wave computes S^T = K Q^T, so a lane owns one query column: the online-softmax statistics
// are per-lane scalars, and P^T feeds the second MFMA (O^T = V^T P^T) straight from registers.
// ---------------------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(256) void k_flash_prefill(const bf16_t *__restrict__ qb, const bf16_t *__restrict__ kc,
                                                       const bf16_t *__restrict__ vc, bf16_t *__restrict__ out, int m,
                                                       int kv0, int nq, int G, int max_seq) {
    constexpr int KS = D + 8;  // K tile row stride (elements): 16-byte reads conflict-free
    constexpr int VS = 36;     // V^T row stride (elements): 8-byte reads conflict-free
    constexpr int CH = D / 8;  // 16-byte chunks per key
    __shared__ __align__(16) bf16_t Ks[32 * KS];
    __shared__ __align__(16) bf16_t Vt[D * VS];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, kg = lane >> 5;
    const int head = blockIdx.y, g = head / G;
    const int q0 = blockIdx.x * 128, qw0 = q0 + wave * 32;
    const int ldq = nq * D;
    const bool wave_active = qw0 < m;
    const int qrow = min(qw0 + l32, m - 1);
    const int q_abs = kv0 + qrow;
    const int wave_last_key = kv0 + min(qw0 + 31, m - 1);
    const int n_keys = kv0 + min(q0 + 128, m);
    const int n_tiles = (n_keys + 31) >> 5;
    const float scale = 1.4426950408889634f / sqrtf((float)D);

    bf16x8 qf[D / 16];
#pragma unroll
    for (int s = 0; s < D / 16; ++s)
        qf[s] = as_bf16x8(*reinterpret_cast<const u32x4 *>(qb + (size_t)qrow * ldq + head * D + 16 * s + 8 * kg));

    f32x16 o[D / 32];
#pragma unroll
    for (int t = 0; t < D / 32; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[t][r] = 0.f;
    float m_i = -INFINITY, l_i = 0.f;

    const bf16_t *kbase = kc + (size_t)g * max_seq * D;
    const bf16_t *vbase = vc + (size_t)g * max_seq * D;
    const u32x4 zero = {0, 0, 0, 0};

    for (int t = 0; t < n_tiles; ++t) {
        const int key0 = t * 32;
        __syncthreads();
        for (int c = tid; c < 32 * CH; c += 256) {
            int key = c / CH, ch = c - key * CH;
            int kabs = key0 + key;
            u32x4 v = kabs < n_keys ? *reinterpret_cast<const u32x4 *>(kbase + (size_t)kabs * D + ch * 8) : zero;
            *reinterpret_cast<u32x4 *>(&Ks[key * KS + ch * 8]) = v;
        }
        for (int c = tid; c < 32 * CH; c += 256) {
            int key = c & 31, ch = c >> 5;
            int kabs = key0 + key;
            u32x4 v = kabs < n_keys ? *reinterpret_cast<const u32x4 *>(vbase + (size_t)kabs * D + ch * 8) : zero;
            bf16_t *dst = &Vt[(ch * 8) * VS + key];
            dst[0 * VS] = (bf16_t)(v.x & 0xffff);
            dst[1 * VS] = (bf16_t)(v.x >> 16);
            dst[2 * VS] = (bf16_t)(v.y & 0xffff);
            dst[3 * VS] = (bf16_t)(v.y >> 16);
            dst[4 * VS] = (bf16_t)(v.z & 0xffff);
            dst[5 * VS] = (bf16_t)(v.z >> 16);
            dst[6 * VS] = (bf16_t)(v.w & 0xffff);
            dst[7 * VS] = (bf16_t)(v.w >> 16);
        }
        __syncthreads();
        if (!wave_active || key0 > wave_last_key) continue;

        f32x16 sacc;
#pragma unroll
        for (int r = 0; r < 16; ++r) sacc[r] = 0.f;
#pragma unroll
        for (int s = 0; s < D / 16; ++s) {
            bf16x8 kf = as_bf16x8(*reinterpret_cast<const u32x4 *>(&Ks[l32 * KS + 16 * s + 8 * kg]));
            sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[s], sacc, 0, 0, 0);
        }
        // lane = query column l32; register r = key 8*(r/4) + 4*kg + r%4 of the tile
        float mx = -INFINITY;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            int kabs = key0 + 8 * (r >> 2) + 4 * kg + (r & 3);
            float sc = kabs > q_abs ? -INFINITY : sacc[r] * scale;
            sacc[r] = sc;
            mx = fmaxf(mx, sc);
        }
        mx = fmaxf(mx, __shfl_xor(mx, 32, kWave));
        const float m_new = fmaxf(m_i, mx);  // finite: key 0 is visible to every query
        const float corr = exp2f(m_i - m_new);
        float rs = 0.f;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            float p = exp2f(sacc[r] - m_new);
            sacc[r] = p;
            rs += p;
        }
        rs += __shfl_xor(rs, 32, kWave);
        l_i = l_i * corr + rs;
        m_i = m_new;
#pragma unroll
        for (int tt = 0; tt < D / 32; ++tt)
#pragma unroll
            for (int r = 0; r < 16; ++r) o[tt][r] *= corr;
        // P^T as the B operand: k-step s2 covers keys 16*s2 .. 16*s2+15, this lane holds registers 8*s2 .. 8*s2+7
        bf16x8 pf[2];
#pragma unroll
        for (int s2 = 0; s2 < 2; ++s2) {
            u32x4 pk = {pack_bf16x2(sacc[8 * s2 + 0], sacc[8 * s2 + 1]), pack_bf16x2(sacc[8 * s2 + 2], sacc[8 * s2 + 3]),
                        pack_bf16x2(sacc[8 * s2 + 4], sacc[8 * s2 + 5]), pack_bf16x2(sacc[8 * s2 + 6], sacc[8 * s2 + 7])};
            pf[s2] = as_bf16x8(pk);
        }
#pragma unroll
        for (int tt = 0; tt < D / 32; ++tt) {
#pragma unroll
            for (int s2 = 0; s2 < 2; ++s2) {
                const bf16_t *vrow = &Vt[(tt * 32 + l32) * VS + 16 * s2 + 4 * kg];
                u32x2 a0 = *reinterpret_cast<const u32x2 *>(vrow);
                u32x2 a1 = *reinterpret_cast<const u32x2 *>(vrow + 8);
                u32x4 vv = {a0.x, a0.y, a1.x, a1.y};
                o[tt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(vv), pf[s2], o[tt], 0, 0, 0);
            }
        }
    }
    if (!wave_active || qw0 + l32 >= m) return;
    const float inv = 1.0f / l_i;
    bf16_t *orow = out + (size_t)(qw0 + l32) * ldq + head * D;
#pragma unroll
    for (int tt = 0; tt < D / 32; ++tt)
#pragma unroll
        for (int rq = 0; rq < 4; ++rq) {
            int dcol = tt * 32 + 8 * rq + 4 * kg;
            u32x2 pk = {pack_bf16x2(o[tt][4 * rq + 0] * inv, o[tt][4 * rq + 1] * inv),
                        pack_bf16x2(o[tt][4 * rq + 2] * inv, o[tt][4 * rq + 3] * inv)};
            *reinterpret_cast<u32x2 *>(orow + dcol) = pk;
        }
}

// ---------------------------------------------------------------------------------------
// launcher
// ---------------------------------------------------------------------------------------
template <int EPI>
static void gemm(const Model &m, const bf16_t *A, int lda, const bf16_t *B, int M, int N, int K, float *outf,
                 bf16_t *outb, int ldo, const bf16_t *bias) {
    const int bn = EPI == 2 ? kBN / 2 : kBN;
    dim3 grid((N + bn - 1) / bn, (M + kBM - 1) / kBM), block(256);
    hipLaunchKernelGGL(k_gemm<EPI>, grid, block, 0, m.stream, A, lda, B, M, N, K, outf, outb, ldo, bias);
}

void launch_prefill_layers(const Model &m, int32_t pos0, int32_t n) {
    const st_config &c = m.c;
    const int h = c.hidden, d = c.head_dim, nq = c.n_q_heads, nkv = c.n_kv_heads, I = c.intermediate;
    const int qd = nq * d, qkv = m.qkv_dim;
    const Workspace &w = m.ws;
    hipLaunchKernelGGL(k_embed_rows, dim3(n), dim3(256), 0, m.stream, m.embed, w.tokens, w.x, h, c.vocab);
    hipLaunchKernelGGL(k_note_fed, dim3(1), dim3(1), 0, m.stream, w.state, w.tokens, n - 1, c.vocab);
    for (int l = 0; l < c.n_layers; ++l) {
        size_t lofs = (size_t)l * nkv * c.max_seq * d;
        hipLaunchKernelGGL(k_rmsnorm_rows, dim3(n), dim3(256), 0, m.stream, w.x, m.norm_attn[l], w.xn, h, c.rms_eps);
        gemm<0>(m, w.xn, h, m.wqkv[l], n, qkv, h, w.qkv, nullptr, qkv, m.bqkv[l]);
        hipLaunchKernelGGL(k_rope_append, dim3(n, nq + 2 * nkv), dim3(d / 2), 0, m.stream, w.qkv, w.rope, w.qb,
                           m.kcache + lofs, m.vcache + lofs, pos0, nq, nkv, d, c.max_seq);
        dim3 fgrid((n + 127) / 128, nq);
        if (d == 128)
            hipLaunchKernelGGL(k_flash_prefill<128>, fgrid, dim3(256), 0, m.stream, w.qb, m.kcache + lofs,
                               m.vcache + lofs, w.attn, n, pos0, nq, nq / nkv, c.max_seq);
        else
            hipLaunchKernelGGL(k_flash_prefill<64>, fgrid, dim3(256), 0, m.stream, w.qb, m.kcache + lofs,
                               m.vcache + lofs, w.attn, n, pos0, nq, nq / nkv, c.max_seq);
        gemm<1>(m, w.attn, qd, m.wo[l], n, h, qd, w.x, nullptr, h, nullptr);
        hipLaunchKernelGGL(k_rmsnorm_rows, dim3(n), dim3(256), 0, m.stream, w.x, m.norm_mlp[l], w.xn, h, c.rms_eps);
        gemm<2>(m, w.xn, h, m.wgu[l], n, I, h, nullptr, w.act, I, nullptr);
        gemm<1>(m, w.act, I, m.wdown[l], n, h, I, w.x, nullptr, h, nullptr);
    }
}

}  // namespace st
