// Catch-up ("prefix") pass over a chunk of m tokens on top of an existing KV cache (paper
// Section 4, Table 3, Eq. 1): the dense part of the path.  bf16 MFMA GEMMs with fused bias /
// residual / SwiGLU epilogues, RoPE + KV append, and causal flash attention with a key offset.
#include "st_device.h"
#include "st_internal.h"
#include <vector>

#include <type_traits>

namespace st {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ bf16x8 as_bf16x8(u32x4 v) { return __builtin_bit_cast(bf16x8, v); }

// fp16 operand mode of the long-chunk GEMMs (see st_model_attach_f16): the same 16-bit containers hold IEEE half
// numbers and the MFMA is the f16 one (same rate as bf16, 11 mantissa bits instead of 8).
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ f16x8 as_f16x8(u32x4 v) { return __builtin_bit_cast(f16x8, v); }
// fp32 -> fp16, round to nearest even, saturating at the largest finite half (activations are O(1); the clamp only
// keeps a stray huge value from becoming an infinity inside a dot product); a NaN stays a NaN
__device__ __forceinline__ float clamp_f16(float v) { return v != v ? v : fminf(fmaxf(v, -65504.f), 65504.f); }
__device__ __forceinline__ uint32_t pack_f16x2(float lo, float hi) {
    lo = clamp_f16(lo), hi = clamp_f16(hi);
    const f16x2_t v = {(_Float16)lo, (_Float16)hi};
    return __builtin_bit_cast(uint32_t, v);
}
__device__ __forceinline__ uint32_t pack_16x2(bool f16, float lo, float hi) {
    return f16 ? pack_f16x2(lo, hi) : pack_bf16x2(lo, hi);
}
__device__ __forceinline__ uint16_t to_16(bool f16, float v) {
    return f16 ? (uint16_t)(pack_f16x2(v, 0.f) & 0xffffu) : f32_to_bf16(v);
}

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

// Extra K slices for the last columns of a split-K result (the ring GEMM's tail): columns >= col0 have n more
// slices, slice t of row r at part[base + t * stride + r * ld + (column - col0)]; n = 0: none.
struct PartTail {
    int col0, n, ld;
    long long base, stride;
};
// the same for a view whose part pointer has been advanced to row `row` of an [rows][h] slice
static inline PartTail tail_at_row(PartTail t, int row, int h) {
    t.base += (long long)row * (t.ld - h);
    return t;
}

// Threads per row of k_rmsnorm_rows: with few rows a row is one block's serial walk, so the block is made wide.
static inline int norm_threads(int rows) { return rows <= 512 ? 1024 : 256; }

// x[row] += sum of the pending split-K partial results (fixed order), then y[row] = bf16(rmsnorm(x) * g).
// part is [n_part][rows][h] (plus the extra slices `tail` describes); with g == nullptr only the residual update is done.  With Ylo the
// normalised row is written as a sum of two bf16 numbers (Y + Ylo), which keeps 16 mantissa bits; with f16 (and no
// Ylo) as one fp16 number.
__global__ __launch_bounds__(1024) void k_rmsnorm_rows(float *__restrict__ X, const float *__restrict__ part,
                                                       int n_part, size_t part_stride, const bf16_t *__restrict__ g,
                                                       bf16_t *__restrict__ Y, bf16_t *__restrict__ Ylo, int h,
                                                       float eps, PartTail tail, int f16) {
    __shared__ float red[16];
    float4 *x = reinterpret_cast<float4 *>(X + (size_t)blockIdx.x * h);
    const float4 *p0 = reinterpret_cast<const float4 *>(part + (size_t)blockIdx.x * h);
    const size_t ps4 = part_stride / 4;
    const int n4 = h >> 2;  // h is a multiple of 8
    const int nthr = blockDim.x;  // 256, or 1024 where the rows are few and each would be a long serial walk
    // a thread's updated residual elements stay in registers between the two passes: kKeep groups of four cover
    // the longest row the library accepts (hidden 8192) at 256 threads; the trailing loops would re-read anything
    // beyond that from x
    constexpr int kKeep = 8;
    float4 keep[kKeep];
    float ss = 0.f;
    auto update = [&](int i) {
        float4 v = x[i];
        for (int s0 = 0; s0 < n_part; s0 += 8) {  // slices in ascending order, eight loads in flight
            float4 q[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) q[u] = s0 + u < n_part ? p0[(size_t)(s0 + u) * ps4 + i] : make_float4(0, 0, 0, 0);
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                v.x += q[u].x;
                v.y += q[u].y;
                v.z += q[u].z;
                v.w += q[u].w;
            }
        }
        if (tail.n && 4 * i >= tail.col0) {
            const float4 *pt = reinterpret_cast<const float4 *>(part + tail.base + (long long)blockIdx.x * tail.ld +
                                                                (4 * i - tail.col0));
            for (int t = 0; t < tail.n; ++t) {
                const float4 q = pt[t * (tail.stride / 4)];
                v.x += q.x, v.y += q.y, v.z += q.z, v.w += q.w;
            }
        }
        if (n_part) x[i] = v;
        ss += v.x * v.x + v.y * v.y + v.z * v.z + v.w * v.w;
        return v;
    };
#pragma unroll
    for (int k = 0; k < kKeep; ++k) {
        const int i = threadIdx.x + k * nthr;
        if (i < n4) keep[k] = update(i);
    }
    for (int i = threadIdx.x + kKeep * nthr; i < n4; i += nthr) update(i);
    if (!g) return;
    ss = wave_sum(ss);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = ss;
    __syncthreads();
    ss = 0.f;
    for (int w = 0; w < nthr / 64; ++w) ss += red[w];
    const float inv = 1.0f / sqrtf(ss / (float)h + eps);
    u32x2 *y = reinterpret_cast<u32x2 *>(Y + (size_t)blockIdx.x * h);
    u32x2 *ylo = Ylo ? reinterpret_cast<u32x2 *>(Ylo + (size_t)blockIdx.x * h) : nullptr;
    const u32x2 *g2 = reinterpret_cast<const u32x2 *>(g);
    auto emit = [&](int i, const float4 &v) {
        u32x2 gg = g2[i];
        float a = v.x * inv * bf16_lo(gg.x), b = v.y * inv * bf16_hi(gg.x);
        float c = v.z * inv * bf16_lo(gg.y), d = v.w * inv * bf16_hi(gg.y);
        u32x2 hi = {pack_16x2(f16, a, b), pack_16x2(f16, c, d)};  // fp16 for the fp16 operand mode (then no low term)
        y[i] = hi;
        if (ylo) {  // second bf16 term of the activation
            u32x2 lo = {pack_bf16x2(a - bf16_lo(hi.x), b - bf16_hi(hi.x)), pack_bf16x2(c - bf16_lo(hi.y), d - bf16_hi(hi.y))};
            ylo[i] = lo;
        }
    };
#pragma unroll
    for (int k = 0; k < kKeep; ++k) {
        const int i = threadIdx.x + k * nthr;
        if (i < n4) emit(i, keep[k]);
    }
    for (int i = threadIdx.x + kKeep * nthr; i < n4; i += nthr) emit(i, x[i]);
}

// ---------------------------------------------------------------------------------------
// C[M][N] = A[M][K] * B[N][K]^T on MFMA 32x32x16 bf16.  Block 256 threads = 2x2 waves, block tile
// BM x 128 (B-tile rows), wave tile BM/2 x 64, K step 32, LDS double-buffered.
//   plain: raw fp32 accumulators of K-slice z go to part[z][M][N]; the consumer kernel adds the
//          slices (fixed order), bias and residual.  Slices give small-M problems enough blocks to
//          stream the weights with every CU and keep the result independent of timing.
//   DUAL : the B tile holds 64 gate rows then the matching 64 up rows; out_bf16 = silu(gate) * up.
//   SPLITA: activations arrive as two bf16 terms (A + Alo, 16 mantissa bits) and each weight fragment is
//          multiplied by both; used for short chunks, where the weight stream, not the MFMA rate, sets the
//          time, so catch-up passes of paper-like length keep near-fp32 activations for free.
// Block ids map to tiles XCD-aware: ids are dealt round-robin to the 8 XCDs, and inside an XCD 32
// consecutive blocks form a TY x TX patch of tiles over a strided set of weight columns, so the
// weight and activation panels a patch streams are shared in that XCD's L2.
// ---------------------------------------------------------------------------------------
constexpr int kBK = 32, kLdsStride = kBK + 8;  // 80-byte rows: conflict-free 16-byte reads

struct GemmGrid {
    int My, Nx, TY, TX, YB, blocks;
};

// BM x BNR block tile (BNR = rows of the weight tile), WGM x WGN waves, wave tile (BM/WGM) x (BNR/WGN).
// The general-shape kernel (any K that is a multiple of 8): 128 x 128 with 2 x 2 waves, or 32- / 64-row tiles with
// two waves for the shortest chunks.  Where K is a multiple of 64 -- every model shape of the paper -- chunks of
// up to 256 rows go to k_gemm_stream and longer ones to k_gemm_ring below.
template <int BM, int BNR, int WGM, int WGN, bool DUAL, bool SPLITA>
__global__ __launch_bounds__(64 * WGM * WGN) void k_gemm(const bf16_t *__restrict__ A, const bf16_t *__restrict__ Alo,
                                                         int lda, const bf16_t *__restrict__ B, int M, int N, int K,
                                                         int kps, float *__restrict__ part,
                                                         bf16_t *__restrict__ outb, bf16_t *__restrict__ outlo,
                                                         int ldo, GemmGrid gg) {
    constexpr int NTH = 64 * WGM * WGN;
    constexpr int MT = BM / WGM / 32, NT = BNR / WGN / 32;
    constexpr int ACH = BM * 4 / NTH, BCH = BNR * 4 / NTH;  // 16-byte chunks per thread per tile
    constexpr int RPP = NTH / 4;                            // tile rows covered per staging pass
    constexpr int BNO = DUAL ? BNR / 2 : BNR;               // output columns per block
    static_assert(!DUAL || NT == 2, "fused SwiGLU pairs the wave's two column tiles");
    constexpr int A_ELEMS = BM * kLdsStride, B_ELEMS = BNR * kLdsStride;
    extern __shared__ __align__(16) bf16_t lds[];
    bf16_t *As = lds;                                       // [2][A_ELEMS]
    bf16_t *Al = lds + 2 * A_ELEMS;                         // [2][A_ELEMS] low terms (SPLITA only)
    bf16_t *Bs = lds + (SPLITA ? 4 : 2) * A_ELEMS;          // [2][B_ELEMS]
    int x, y;
    {
        const int id = blockIdx.x, xcd = id & 7, j = id >> 3;
        const int st = j >> 5, r = j & 31;
        const int tx = r % gg.TX, ty = r / gg.TX;
        const int yb = st % gg.YB, xb = st / gg.YB;
        y = yb * gg.TY + ty;
        x = (xb * gg.TX + tx) * 8 + xcd;
        if (y >= gg.My || x >= gg.Nx) return;
    }
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WGN, wn = wave % WGN;
    const int m0 = y * BM, n0 = x * BNO;
    const int l32 = lane & 31, kg = lane >> 5;
    const int kbeg = blockIdx.y * kps, kend = min(K, kbeg + kps);

    // global -> register staging: thread owns chunks (row = tid/4 + i*RPP, 8 columns at (tid%4)*8)
    const bf16_t *ga[ACH], *gl[ACH], *gb[BCH];
    bool va[ACH], vb[BCH];
    const int kcol = (tid & 3) * 8;
    const int so = (tid >> 2) * kLdsStride + kcol;
#pragma unroll
    for (int i = 0; i < ACH; ++i) {
        int am = m0 + (tid >> 2) + i * RPP;
        va[i] = am < M;
        ga[i] = A + (size_t)(va[i] ? am : 0) * lda + kcol;
        gl[i] = SPLITA ? Alo + (size_t)(va[i] ? am : 0) * lda + kcol : nullptr;
    }
#pragma unroll
    for (int i = 0; i < BCH; ++i) {
        int row = (tid >> 2) + i * RPP;
        int bn;
        if (DUAL) {
            int half = row / (BNR / 2), r = row % (BNR / 2);
            vb[i] = n0 + r < N;  // N is the number of output columns (I)
            bn = (vb[i] ? n0 + r : 0) + half * N;
        } else {
            vb[i] = n0 + row < N;
            bn = vb[i] ? n0 + row : 0;
        }
        gb[i] = B + (size_t)bn * K + kcol;
    }
    u32x4 ra[ACH], rl[SPLITA ? ACH : 1], rb[BCH];
    const u32x4 zero = {0, 0, 0, 0};
    auto fetch = [&](int k0) {
        const bool kin = k0 + kcol < kend;
#pragma unroll
        for (int i = 0; i < ACH; ++i) ra[i] = (va[i] && kin) ? *reinterpret_cast<const u32x4 *>(ga[i] + k0) : zero;
        if (SPLITA) {
#pragma unroll
            for (int i = 0; i < ACH; ++i)
                rl[i] = (va[i] && kin) ? *reinterpret_cast<const u32x4 *>(gl[i] + k0) : zero;
        }
#pragma unroll
        for (int i = 0; i < BCH; ++i) rb[i] = (vb[i] && kin) ? *reinterpret_cast<const u32x4 *>(gb[i] + k0) : zero;
    };
    auto stash = [&](int buf) {
#pragma unroll
        for (int i = 0; i < ACH; ++i)
            *reinterpret_cast<u32x4 *>(&As[buf * A_ELEMS + so + i * RPP * kLdsStride]) = ra[i];
        if (SPLITA) {
#pragma unroll
            for (int i = 0; i < ACH; ++i)
                *reinterpret_cast<u32x4 *>(&Al[buf * A_ELEMS + so + i * RPP * kLdsStride]) = rl[i];
        }
#pragma unroll
        for (int i = 0; i < BCH; ++i)
            *reinterpret_cast<u32x4 *>(&Bs[buf * B_ELEMS + so + i * RPP * kLdsStride]) = rb[i];
    };

    f32x16 acc[MT][NT];
#pragma unroll
    for (int i = 0; i < MT; ++i)
#pragma unroll
        for (int j = 0; j < NT; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    int brow[NT];
#pragma unroll
    for (int j = 0; j < NT; ++j) brow[j] = (DUAL ? j * (BNR / 2) + wn * 32 : wn * (BNR / WGN) + j * 32) + l32;
    const int arow = wm * (BM / WGM) + l32;

    const int nk = (kend - kbeg + kBK - 1) / kBK;
    fetch(kbeg);
    stash(0);
    __syncthreads();
    for (int kt = 0; kt < nk; ++kt) {
        const int buf = kt & 1;
        if (kt + 1 < nk) fetch(kbeg + (kt + 1) * kBK);
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            bf16x8 af[MT], bfr[NT];
#pragma unroll
            for (int i = 0; i < MT; ++i)
                af[i] = as_bf16x8(*reinterpret_cast<const u32x4 *>(
                    &As[buf * A_ELEMS + (arow + i * 32) * kLdsStride + ks * 16 + kg * 8]));
#pragma unroll
            for (int j = 0; j < NT; ++j)
                bfr[j] = as_bf16x8(*reinterpret_cast<const u32x4 *>(
                    &Bs[buf * B_ELEMS + brow[j] * kLdsStride + ks * 16 + kg * 8]));
#pragma unroll
            for (int i = 0; i < MT; ++i)
#pragma unroll
                for (int j = 0; j < NT; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0);
            if (SPLITA) {
#pragma unroll
                for (int i = 0; i < MT; ++i) {
                    bf16x8 al = as_bf16x8(*reinterpret_cast<const u32x4 *>(
                        &Al[buf * A_ELEMS + (arow + i * 32) * kLdsStride + ks * 16 + kg * 8]));
#pragma unroll
                    for (int j = 0; j < NT; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(al, bfr[j], acc[i][j], 0, 0, 0);
                }
            }
        }
        if (kt + 1 < nk) stash(buf ^ 1);
        __syncthreads();
    }

    // epilogue: register r of a 32x32 tile is row 8*(r/4) + 4*(lane/32) + r%4, column lane%32
    float *pz = DUAL ? nullptr : part + (size_t)blockIdx.y * M * N;
#pragma unroll
    for (int i = 0; i < MT; ++i) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            int row = m0 + wm * (BM / WGM) + i * 32 + 8 * (r >> 2) + 4 * kg + (r & 3);
            if (row >= M) continue;
            if (DUAL) {
                int col = n0 + wn * 32 + l32;
                if (col < N) {
                    float gt = acc[i][0][r], up = acc[i][NT - 1][r];
                    float a = gt / (1.0f + expf(-gt)) * up;
                    bf16_t hi = f32_to_bf16(a);
                    outb[(size_t)row * ldo + col] = hi;
                    if (outlo) outlo[(size_t)row * ldo + col] = f32_to_bf16(a - bf16_to_f32(hi));
                }
            } else {
#pragma unroll
                for (int j = 0; j < NT; ++j) {
                    int col = n0 + wn * (BNR / WGN) + j * 32 + l32;
                    if (col < N) pz[(size_t)row * N + col] = acc[i][j][r];
                }
            }
        }
    }
}

// ---------------------------------------------------------------------------------------
// Long chunks: the same contraction with a 256 x 256 block tile, K step 64, on four waves that each own
// a 128 x 128 tile (256 accumulator registers), built around the three limits measured on this chip:
//   * tile traffic from L2 moves about 40 % faster in whole 128-byte lines, hence K step 64;
//   * LDS delivers 128 bytes per clock, so fragments are read once per 128 x 128 wave tile (half the
//     LDS bytes per MFMA of a 128 x 64 wave tile), from rows whose 16-byte chunks are XOR-swizzled so
//     that the reads are conflict-free without padding;
//   * the vector memory path accepts one 1 KB load per 16 clocks per CU and stalls the issuing wave
//     beyond that, and with one wave per SIMD a stalled wave is an idle MFMA pipe.  Tiles therefore
//     go global -> LDS directly (no staging registers), one load instruction per four MFMAs, all
//     through the K loop.  That needs slots freed early: the ring has five 32 KB slots, one operand of
//     one K step each (A0 B0 A1 B1 A2 ...), so loads run up to two and a half steps ahead of the math.
// Per K step of 64: 64 MFMAs, 32 fragment reads (fetched one 16-wide step ahead into a second register
// set), 16 direct loads and one barrier.  Needs K % 64 == 0 and at least two steps per K slice.
// ---------------------------------------------------------------------------------------
constexpr int kRingBK = 64, kRingSlot = 256 * kRingBK * 2, kRingSlots = 5;
constexpr int kRingLds = kRingSlot * kRingSlots;  // 160 KB: all of a CU's LDS

__device__ __forceinline__ int ring_swz(int row) { return (row + (row >> 3)) & 7; }

// 64 lanes x 16 bytes from per-lane global addresses to 1 KB of LDS starting at lds_off (wave-uniform)
__device__ __forceinline__ void load_to_lds16(const void *g, uint32_t lds_off) {
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(g),
                 "s"(__builtin_amdgcn_readfirstlane(lds_off))
                 : "memory");
}
// the same from a wave-uniform base and a 32-bit byte offset per lane (half the address registers to read)
__device__ __forceinline__ void load_to_lds16(const void *base, uint32_t byte_off, uint32_t lds_off) {
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(byte_off), "s"(base),
                 "s"(__builtin_amdgcn_readfirstlane(lds_off))
                 : "memory");
}
template <int N>
__device__ __forceinline__ void wait_loads() {  // until at most N of this wave's direct loads are outstanding
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}
template <int V>
using ic = std::integral_constant<int, V>;
template <int N, int I = 0, class F>
__device__ __forceinline__ void static_for(F &&f) {  // f(ic<0>{}), ..., f(ic<N-1>{})
    if constexpr (I < N) {
        f(ic<I>{});
        static_for<N, I + 1>(f);
    }
}

// Block ids -> work of the ring kernel.  Main part: S K slices of kps columns over My x Nx tiles, numbered slice by
// slice, inside a slice by groups of TX column tiles, inside a group by TY x TX patches down the rows (narrower
// patches at the edges, so the numbering has no gaps); XCD e (= block id % 8) takes the `per` consecutive numbers
// from e * per on.  The 32 blocks an XCD runs together are then one patch of one K slice -- the panels they stream
// are shared in that XCD's L2 -- and every XCD gets the same number of blocks.  Ids that are dealt out but return at
// once must not be interleaved with working ones (measured: with two of every four ids returning, the O / down
// projections of a 4096-row chunk took 40 % longer -- as if the working blocks sat on half an XCD's shader engines).
// Tail (block ids from `blocks` on): the column tiles from tail_x0 on, their K range cut into tail_s slices of
// tail_kps columns; a unit is one slice of 32 tiles (column-major) and unit u runs on XCD u % 8.
struct RingGrid {
    int My, Nx, x0, TY, TX, S, kps, per, blocks;  // x0: column tile of the launch's first column (in its own tiles)
    int tail_x0, tail_tiles, tail_s, tail_kps;
};
// What block `bid` of a launch works on: tile (x, y) in the launch's own tiles (x before adding x0), K range
// [kbeg, kend), and for the plain form where its fp32 tile goes: part + part_off, row stride ldp (the offset
// already discounts the tail's first column).  False: the id has no work.  Shared by the kernel and the host-side
// check of the numbering.
struct RingBlock {
    int x, y, kbeg, kend, ldp;
    long long part_off;
};
__host__ __device__ inline bool ring_block(const RingGrid &gg, int bid, int M, int N, int K, RingBlock *o) {
    o->ldp = N;
    if (bid < gg.blocks) {
        const int j = bid >> 3, T = gg.My * gg.Nx;
        const int f = (bid & 7) * gg.per + j;
        if (j >= gg.per || f >= gg.S * T) return false;  // only at the end of an XCD's range
        const int sl = f / T, fs = f % T;
        const int full_c = gg.Nx / gg.TX * gg.TX, full_r = gg.My / gg.TY * gg.TY;
        int cols, c0, jj;
        if (fs < full_c * gg.My)
            cols = gg.TX, c0 = fs / (cols * gg.My) * cols, jj = fs % (cols * gg.My);
        else
            cols = gg.Nx - full_c, c0 = full_c, jj = fs - full_c * gg.My;
        int r, y0;
        if (jj < cols * full_r)
            y0 = jj / (cols * gg.TY) * gg.TY, r = jj % (cols * gg.TY);
        else
            y0 = full_r, r = jj - cols * full_r;
        o->y = y0 + r / cols, o->x = c0 + r % cols;
        o->kbeg = sl * gg.kps, o->kend = o->kbeg + gg.kps < K ? o->kbeg + gg.kps : K;
        o->part_off = (long long)sl * M * N;
        return true;
    }
    // tail: a unit is one K slice of a patch of 32 tiles (column-major over the tail's columns); unit u runs on
    // XCD u % 8, so the blocks that share panels at the same K positions share an L2
    const int t = bid - gg.blocks, xcd = t & 7, j = t >> 3;
    const int u = (j >> 5) * 8 + xcd, q = (u / gg.tail_s) * 32 + (j & 31), sl = u % gg.tail_s;
    if (q >= gg.tail_tiles) return false;
    o->x = gg.tail_x0 + q / gg.My, o->y = q % gg.My;
    o->kbeg = sl * gg.tail_kps, o->kend = o->kbeg + gg.tail_kps < K ? o->kbeg + gg.tail_kps : K;
    const int col0 = gg.tail_x0 * 256;
    o->part_off = 0;
    if (sl > 0) o->ldp = N - col0, o->part_off = (long long)M * N + (long long)(sl - 1) * M * o->ldp - col0;
    return true;
}

// HALF (fused SwiGLU form only): the block tile is 256 x (64 gate + 64 up) weight rows -- half the columns, half the
// MFMAs per fragment of activations -- for the tiles left over after whole rounds of full tiles (one more round of
// half the length instead of a round that leaves half the chip idle).
// F16: A and B hold fp16 numbers (single-term activations, the model's fp16 copy of the weights).  out_f16: the
// fused epilogue writes fp16 (one term) instead of bf16 (+ its low term).
template <bool DUAL, bool HALF = false, bool F16 = false>
__global__ __launch_bounds__(256) void k_gemm_ring(const bf16_t *__restrict__ A, const bf16_t *__restrict__ Alo, int lda,
                                                   const bf16_t *__restrict__ B, int M, int N, int K,
                                                   float *__restrict__ part, bf16_t *__restrict__ outb,
                                                   bf16_t *__restrict__ outlo, int ldo, RingGrid gg, int out_f16) {
    extern __shared__ __align__(16) unsigned char ring[];
    RingBlock rb;
    // Two-term activations (Alo != nullptr): the contraction runs over 2K columns, [A | Alo] against [B | B]; K step
    // ka >= K / 64 takes its activations from Alo and wraps round in the weights.
    if (!ring_block(gg, blockIdx.x, M, N, Alo ? 2 * K : K, &rb)) return;
    const int x = rb.x, y = rb.y, kbeg = rb.kbeg, kend = rb.kend, ldp = rb.ldp;
    float *pz = DUAL ? nullptr : part + rb.part_off;  // where this block's fp32 tile goes (plain form)
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave >> 1, wn = wave & 1;
    const int l32 = lane & 31, kg = lane >> 5;
    static_assert(DUAL || !HALF, "the half-width tile exists for the fused form only");
    constexpr int NB = HALF ? 2 : 4;   // 32-row weight fragments per wave
    constexpr int NLB = HALF ? 4 : 8;  // direct loads per wave for one weight slot
    const int m0 = y * 256, n0 = (x + gg.x0) * (HALF ? 64 : DUAL ? 128 : 256);
    const int nk = (kend - kbeg) / kRingBK;
    const uint32_t ring0 = (uint32_t)(uintptr_t)ring;  // LDS byte offset of the ring (low half of the flat address)

    // direct loads: instruction i of a wave fills LDS rows [(wave*8+i)*8, +8) of a slot, lane -> (row lane/8,
    // 16-byte position lane%8, which holds global chunk position ^ swizzle(row)); rows past the edge re-read
    // the last valid row (their results are never stored)
    uint32_t pa[8], pb[NLB];  // byte offsets from A / B (every operand of the library is far below 4 GB)
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const int row = (wave * 8 + i) * 8 + (lane >> 3);
        const int c = (lane & 7) ^ ring_swz(row);
        pa[i] = (uint32_t)(((size_t)min(m0 + row, M - 1) * lda + c * 8) * sizeof(bf16_t));
    }
#pragma unroll
    for (int i = 0; i < NLB; ++i) {
        const int row = (wave * NLB + i) * 8 + (lane >> 3);
        const int c = (lane & 7) ^ ring_swz(row);
        int bn;
        if (HALF)  // rows 0..63 of the tile are gate rows, 64..127 the matching up rows
            bn = min(n0 + (row & 63), N - 1) + (row >> 6) * N;
        else if (DUAL)  // rows 0..127 of the tile are gate rows, 128..255 the matching up rows (N = I)
            bn = min(n0 + (row & 127), N - 1) + (row >> 7) * N;
        else
            bn = min(n0 + row, N - 1);
        pb[i] = (uint32_t)(((size_t)bn * K + c * 8) * sizeof(bf16_t));
    }
    // the K position of a step is a wave-uniform base (scalar registers), the lane offsets above never change
    const int nkw = K / kRingBK, k0 = kbeg / kRingBK;  // K steps of the weights; first step of this block
    auto baseA = [&](int kt) {
        const int ka = k0 + kt;
        return ka < nkw ? A + (size_t)ka * kRingBK : Alo + (size_t)(ka - nkw) * kRingBK;
    };
    auto baseB = [&](int kt) {
        const int ka = k0 + kt;
        return B + (size_t)(ka < nkw ? ka : ka - nkw) * kRingBK;
    };
    auto loadA = [&](auto i_c, int slot, const bf16_t *base) {
        constexpr int i = decltype(i_c)::value;
        load_to_lds16(base, pa[i], ring0 + slot * kRingSlot + (wave * 8 + i) * 1024);
    };
    auto loadB = [&](auto i_c, int slot, const bf16_t *base) {
        constexpr int i = decltype(i_c)::value;
        if constexpr (i < NLB) load_to_lds16(base, pb[i], ring0 + slot * kRingSlot + (wave * NLB + i) * 1024);
    };

    f32x16 acc[4][NB];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < NB; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    // fragment reads: lane (row l32, K half kg) of 32-row block t reads chunk (2*ks + kg) ^ swizzle; the
    // swizzle of row 32*t + l32 is swizzle(l32) ^ 4*(t & 1)
    const int a_off = (wm * 128 + l32) * 128;
    int b_off[NB];
#pragma unroll
    for (int j = 0; j < NB; ++j)
        b_off[j] = (HALF   ? (j * 64 + wn * 32 + l32)
                    : DUAL ? ((j >> 1) * 128 + wn * 64 + (j & 1) * 32 + l32)
                           : (wn * 128 + j * 32 + l32)) * 128;
    const int ch_even = (kg ^ ring_swz(l32)) * 16, ch_odd = ch_even ^ 64;
    const int ch_half = wn ? ch_odd : ch_even;  // HALF: both weight fragments of a wave sit in 32-row block wn or 2 + wn

    u32x4 fa[2][4], fb[2][NB];
    // fragment q of a 16-wide step: q = 0..3 weight fragments (0..1 with HALF), 4..7 activation fragments
    auto fetch = [&](auto buf_c, auto q_c, int slotA, int slotB, int ks) {
        constexpr int buf = decltype(buf_c)::value, q = decltype(q_c)::value;
        if constexpr (q < 4) {
            if constexpr (q < NB) {
                const int ch = (HALF ? ch_half : (q & 1) ? ch_odd : ch_even) ^ (ks * 32);
                fb[buf][q] = *reinterpret_cast<const u32x4 *>(ring + slotB * kRingSlot + b_off[q] + ch);
            }
        } else {
            const int ch = ((q & 1) ? ch_odd : ch_even) ^ (ks * 32);
            fa[buf][q & 3] = *reinterpret_cast<const u32x4 *>(ring + slotA * kRingSlot + a_off + (q & 3) * 4096 + ch);
        }
    };
    auto mma_one = [&](auto buf_c, auto i_c, auto j_c) {
        constexpr int buf = decltype(buf_c)::value, i = decltype(i_c)::value, j = decltype(j_c)::value;
        if constexpr (j < NB) {
            if constexpr (F16)
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(as_f16x8(fa[buf][i]), as_f16x8(fb[buf][j]),
                                                                   acc[i][j], 0, 0, 0);
            else
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(fa[buf][i]), as_bf16x8(fb[buf][j]),
                                                                    acc[i][j], 0, 0, 0);
        }
    };
    // One 16-wide step: four groups of { one direct load (KIND 1: weight instruction D0+g, 2: activation
    // instruction D0+g, 0: none), two fragment reads for the following step, four MFMAs }; the scheduling
    // fences keep that interleave.
    auto step = [&](auto cur_c, auto fetch_c, int slotA, int slotB, int ks_next, auto kind_c, auto d0_c, int dslot,
                    const bf16_t *dbase) {
        constexpr int cur = decltype(cur_c)::value, kind = decltype(kind_c)::value, d0 = decltype(d0_c)::value;
        constexpr bool FETCH = decltype(fetch_c)::value != 0;
        // the two reads and the load sit between the group's MFMAs, each issued while the MFMA before it runs
#define ST_GEMM_GROUP(g)                                                      \
    mma_one(ic<cur>{}, ic<g>{}, ic<0>{});                                     \
    __builtin_amdgcn_sched_barrier(0);                                        \
    if (FETCH) fetch(ic<cur ^ 1>{}, ic<2 * g>{}, slotA, slotB, ks_next);      \
    __builtin_amdgcn_sched_barrier(0);                                        \
    mma_one(ic<cur>{}, ic<g>{}, ic<1>{});                                     \
    __builtin_amdgcn_sched_barrier(0);                                        \
    if (FETCH) fetch(ic<cur ^ 1>{}, ic<2 * g + 1>{}, slotA, slotB, ks_next);  \
    __builtin_amdgcn_sched_barrier(0);                                        \
    mma_one(ic<cur>{}, ic<g>{}, ic<2>{});                                     \
    __builtin_amdgcn_sched_barrier(0);                                        \
    if (kind == 1) loadB(ic<d0 + g>{}, dslot, dbase);                         \
    if (kind == 2) loadA(ic<d0 + g>{}, dslot, dbase);                         \
    __builtin_amdgcn_sched_barrier(0);                                        \
    mma_one(ic<cur>{}, ic<g>{}, ic<3>{});                                     \
    __builtin_amdgcn_sched_barrier(0);
        ST_GEMM_GROUP(0) ST_GEMM_GROUP(1) ST_GEMM_GROUP(2) ST_GEMM_GROUP(3)
#undef ST_GEMM_GROUP
    };

    // prologue: A0 B0 A1 whole and the first half of B1 (nk >= 2)
    {
        const bf16_t *a0 = baseA(0), *b0 = baseB(0), *a1 = baseA(1), *b1 = baseB(1);
        loadA(ic<0>{}, 0, a0), loadA(ic<1>{}, 0, a0), loadA(ic<2>{}, 0, a0), loadA(ic<3>{}, 0, a0);
        loadA(ic<4>{}, 0, a0), loadA(ic<5>{}, 0, a0), loadA(ic<6>{}, 0, a0), loadA(ic<7>{}, 0, a0);
        loadB(ic<0>{}, 1, b0), loadB(ic<1>{}, 1, b0), loadB(ic<2>{}, 1, b0), loadB(ic<3>{}, 1, b0);
        loadB(ic<4>{}, 1, b0), loadB(ic<5>{}, 1, b0), loadB(ic<6>{}, 1, b0), loadB(ic<7>{}, 1, b0);
        loadA(ic<0>{}, 2, a1), loadA(ic<1>{}, 2, a1), loadA(ic<2>{}, 2, a1), loadA(ic<3>{}, 2, a1);
        loadA(ic<4>{}, 2, a1), loadA(ic<5>{}, 2, a1), loadA(ic<6>{}, 2, a1), loadA(ic<7>{}, 2, a1);
        loadB(ic<0>{}, 3, b1), loadB(ic<1>{}, 3, b1), loadB(ic<2>{}, 3, b1), loadB(ic<3>{}, 3, b1);
    }
    wait_loads<12>();  // A0 and B0 are in
    __builtin_amdgcn_s_barrier();
    fetch(ic<0>{}, ic<0>{}, 0, 1, 0), fetch(ic<0>{}, ic<1>{}, 0, 1, 0), fetch(ic<0>{}, ic<2>{}, 0, 1, 0);
    fetch(ic<0>{}, ic<3>{}, 0, 1, 0), fetch(ic<0>{}, ic<4>{}, 0, 1, 0), fetch(ic<0>{}, ic<5>{}, 0, 1, 0);
    fetch(ic<0>{}, ic<6>{}, 0, 1, 0), fetch(ic<0>{}, ic<7>{}, 0, 1, 0);
    __builtin_amdgcn_sched_barrier(0);

    const bf16_t *bn1 = baseB(1), *an2 = baseA(2), *bn2 = baseB(2);  // bases of B(kt+1), A(kt+2), B(kt+2)
    int wrap_in = nkw - (k0 + 2);  // K steps until A(kt+2) crosses into the low term (<= 0: never in this block)
    int sA = 0;  // ring slot of this K step's activations; its weights sit in the next slot, and so on round
    auto fwd = [](int s, int d) { return s + d >= kRingSlots ? s + d - kRingSlots : s + d; };
    // AHEAD: 2 = K steps kt+1 and kt+2 exist, 1 = only kt+1, 0 = this is the last
    auto kstep = [&](int, auto ahead_c) {
        constexpr int AHEAD = decltype(ahead_c)::value;
        const int sB = fwd(sA, 1), sA1 = fwd(sA, 2), sB1 = fwd(sA, 3), sA2 = fwd(sA, 4);
        step(ic<0>{}, ic<1>{}, sA, sB, 1, ic<(AHEAD >= 1 ? 1 : 0)>{}, ic<4>{}, sB1, bn1);  // rest of B(kt+1)
        step(ic<1>{}, ic<1>{}, sA, sB, 2, ic<(AHEAD >= 2 ? 2 : 0)>{}, ic<0>{}, sA2, an2);  // A(kt+2), first half
        step(ic<0>{}, ic<1>{}, sA, sB, 3, ic<(AHEAD >= 2 ? 2 : 0)>{}, ic<4>{}, sA2, an2);  // A(kt+2), second half
        if (AHEAD >= 1) {
            // all fragments of this K step are in registers and K step kt+1 has landed (only A(kt+2) may
            // still be in flight); after the barrier that holds for every wave, so both slots are free
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
            if (AHEAD >= 2) wait_loads<8>(); else wait_loads<0>();
            __builtin_amdgcn_s_barrier();
            __builtin_amdgcn_sched_barrier(0);
            step(ic<1>{}, ic<1>{}, sA1, sB1, 0, ic<(AHEAD >= 2 ? 1 : 0)>{}, ic<0>{}, sA, bn2);  // B(kt+2), first half
        } else {
            step(ic<1>{}, ic<0>{}, sA1, sB1, 0, ic<0>{}, ic<0>{}, sA, bn2);
        }
        sA = sA1;
        // bases of the next step's loads: B(kt+2) becomes B(kt+1), the other two move on by one K step and cross
        // from the high to the low term (and back to the weights' first column) at most once in a block's range
        bn1 = bn2, an2 += kRingBK, bn2 += kRingBK;
        if (--wrap_in == 0) an2 = Alo, bn2 = B;
    };
    int kt = 0;
    for (; kt + 2 < nk; ++kt) kstep(kt, ic<2>{});
    kstep(kt++, ic<1>{});
    kstep(kt++, ic<0>{});

    // epilogue: register r of a 32x32 tile is row 8*(r/4) + 4*(lane/32) + r%4, column lane%32
    if constexpr (DUAL) {
        // Two rows at a time: neighbouring lanes (columns c, c + 1) swap one value each, so that the even lane holds
        // both columns of the first row and the odd lane both of the second -- one 4-byte store per lane instead of
        // two 2-byte ones.  silu goes through the hardware exp2 and reciprocal (1 ulp each, far below bf16).
        const bool odd = l32 & 1;
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < NB / 2; ++j)
#pragma unroll
                for (int r = 0; r < 16; r += 2) {
                    float a[2];
#pragma unroll
                    for (int e = 0; e < 2; ++e) {
                        const float gt = acc[i][j][r + e], up = acc[i][j + NB / 2][r + e];
                        a[e] = gt * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(-1.4426950408889634f * gt)) * up;
                    }
                    const float other = dpp_move<0xB1, 0xf>(0.f, odd ? a[0] : a[1]);  // quad_perm [1,0,3,2]
                    const float x0 = odd ? other : a[0], x1 = odd ? a[1] : other;
                    const uint32_t pk = out_f16 ? pack_f16x2(x0, x1) : pack_bf16x2(x0, x1);
                    const int row = m0 + wm * 128 + i * 32 + 8 * (r >> 2) + 4 * kg + (r & 3) + (odd ? 1 : 0);
                    const int col = n0 + wn * (NB * 16) + j * 32 + (l32 & ~1);
                    if (row < M && col + 1 < N)
                        *reinterpret_cast<uint32_t *>(outb + (size_t)row * ldo + col) = pk;
                    else if (row < M && col < N)  // an odd width: the last column alone
                        outb[(size_t)row * ldo + col] = (bf16_t)(pk & 0xffffu);
                    if (!out_f16 && outlo) {  // second bf16 term of the activation (feeds a two-term down projection)
                        const uint32_t lo = pack_bf16x2(x0 - bf16_lo(pk), x1 - bf16_hi(pk));
                        if (row < M && col + 1 < N)
                            *reinterpret_cast<uint32_t *>(outlo + (size_t)row * ldo + col) = lo;
                        else if (row < M && col < N)
                            outlo[(size_t)row * ldo + col] = (bf16_t)(lo & 0xffffu);
                    }
                }
    } else {
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int row = m0 + wm * 128 + i * 32 + 8 * (r >> 2) + 4 * kg + (r & 3);
                if (row >= M) continue;
#pragma unroll
                for (int j = 0; j < NB; ++j) {
                    const int col = n0 + wn * 128 + j * 32 + l32;
                    if (col < N) pz[(size_t)row * ldp + col] = acc[i][j][r];
                }
            }
    }
}

// ---------------------------------------------------------------------------------------
// Weight-streaming GEMM for chunks of at most 256 rows (two-term activations).  A block owns nt <= 8 tiles of 32
// weight rows and a K slice; K advances BK columns per stage.  Every block re-reads the activation rows from L2,
// and direct loads of L2-resident data cost as much load-path time as the weights from HBM do (measured: adding
// 24 KB of activations to 16 KB of weights per stage takes the weight stream from 6.0 to 4.2 TB/s), so the block
// is made tall -- 256 weight rows per activation fetch -- and LDS is split into two rings: weights, nw stages,
// filled by waves 0-1, and activations, na stages, filled by waves 2-3.  The two kinds of loads sit in different
// waves because a wave's load counter retires in order: one wave cannot wait for a recent activation load
// without also waiting for every older weight load.  BK = 64 (128-byte row segments, which HBM streams a fifth
// faster than 64-byte ones) up to 128 rows; BK = 32 above, where the activation stages would not leave room for
// three weight stages.  All four waves multiply: wave w owns weight tiles w and w + 4 against every 32-row
// activation tile (C^T = W A^T, a lane owns an activation row); raw fp32 partial sums of the K slice go to
// part[z][M][N].  Needs K % BK == 0 and (nw - 2) * (loads per weight wave per stage) <= 63.
// ---------------------------------------------------------------------------------------
__device__ __forceinline__ void wait_loads_rt(int n) {  // s_waitcnt takes an immediate only
#define ST_W1(v) case v: wait_loads<v>(); break;
#define ST_W8(v) ST_W1(v) ST_W1(v + 1) ST_W1(v + 2) ST_W1(v + 3) ST_W1(v + 4) ST_W1(v + 5) ST_W1(v + 6) ST_W1(v + 7)
    switch (n) {
        ST_W8(0) ST_W8(8) ST_W8(16) ST_W8(24) ST_W8(32) ST_W8(40) ST_W8(48) ST_W8(56)
        default: wait_loads<0>(); break;
    }
#undef ST_W8
#undef ST_W1
}

template <int BK>
struct StreamGeom {
    static constexpr int kSeg = BK * 2;          // bytes of a row per stage
    static constexpr int kLpr = kSeg / 16;       // lanes per row in a direct load
    static constexpr int kRpi = 64 / kLpr;       // rows per 1 KB instruction
    static constexpr int kWTile = 32 * kSeg;     // bytes of one 32-row weight tile per stage
    static constexpr int kARows = 32 * kSeg;     // bytes of 32 activation rows per stage (a tile holds one such block
                                                 // per term: high, low)
    // 16-byte chunk swizzle of LDS row `row` (conflict-free fragment reads)
    __device__ static int swz(int row) { return BK == 32 ? (row >> 2) & 3 : ring_swz(row); }
};

// TERMS = 2: activations as two bf16 terms (A + Alo).  TERMS = 1 with F16: single fp16 activations against the
// model's fp16 copy of the weights on the f16 MFMA (half the activation traffic and half the MFMAs per weight byte).
template <int MT, int BK, bool SPEC, int TERMS = 2, bool F16 = false>
__global__ __launch_bounds__(SPEC ? 512 : 256) void k_gemm_stream(const bf16_t *__restrict__ A,
                                                                  const bf16_t *__restrict__ Alo, int lda,
                                                                  const bf16_t *__restrict__ B, int M, int N, int K,
                                                                  int kps, int nt, int nw, int na,
                                                                  float *__restrict__ part) {
    using G = StreamGeom<BK>;
    static_assert(TERMS == 1 || TERMS == 2, "one or two activation terms");
    constexpr int RT = 32 * TERMS;                   // LDS rows of one activation tile
    constexpr int kAStage = MT * TERMS * G::kARows;
    constexpr int kALoads = MT * RT / G::kRpi / 2;   // activation instructions per stage of each activation wave
    constexpr int kWLoadsMax = 8 * 32 / G::kRpi / 2; // weight instructions per stage of each weight wave at nt = 8
    constexpr int NL = kALoads > kWLoadsMax ? kALoads : kWLoadsMax;
    extern __shared__ __align__(16) unsigned char ring[];
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l32 = lane & 31, kg = lane >> 5;
    const int n0 = blockIdx.x * nt * 32;
    const int kbeg = blockIdx.y * kps;
    const int nk = (min(K, kbeg + kps) - kbeg) / BK;
    const uint32_t ring0 = (uint32_t)(uintptr_t)ring;
    const int wstage = nt * G::kWTile, a_ring = na * kAStage;
    // SPEC: eight waves, 0-3 multiply and 4-7 load (a wave is held ~70 clocks at every direct load it issues, time
    // the multiplying waves then do not lose); otherwise four waves do both.
    const bool computes = !SPEC || wave < 4, loads = !SPEC || wave >= 4;
    const int lw = SPEC ? (wave - 4) & 3 : wave;  // loader index: 0, 1 weights; 2, 3 activations

    // direct loads: a 1 KB instruction fills kRpi LDS rows; lane -> (row lane/kLpr, 16-byte position lane%kLpr
    // holding global chunk position ^ swz(row)).  Activations: LDS row RT*t + 32*term + r is row 32*t + r of term
    // (0 = high, 1 = low); rows past the edge re-read the last valid row and are never stored.
    const bool w_loader = lw < 2;
    const int n_loads = w_loader ? nt * 32 / G::kRpi / 2 : kALoads;
    const int depth = w_loader ? nw : na;
    const uint32_t my_ring = ring0 + (w_loader ? a_ring : 0), my_stage = w_loader ? wstage : kAStage;
    const bf16_t *pl[NL];
    int l_off[NL];
#pragma unroll
    for (int i = 0; i < NL; ++i) {
        const int inst = (w_loader ? lw : lw - 2) * n_loads + i;
        const int row = inst * G::kRpi + lane / G::kLpr;
        const int piece = ((lane % G::kLpr) ^ G::swz(row)) * 8;
        if (w_loader) {
            pl[i] = B + (size_t)min(n0 + row, N - 1) * K + kbeg + piece;
        } else {
            const int t = min(row / RT, MT - 1), term = (row >> 5) % TERMS, r = row & 31;
            pl[i] = (term ? Alo : A) + (size_t)min(t * 32 + r, M - 1) * lda + kbeg + piece;
        }
        l_off[i] = inst * 1024;
    }
    int iss_st = 0, iss_slot = 0;  // next stage this wave loads and its ring slot
    auto issue_one = [&](auto i_c) {
        constexpr int i = decltype(i_c)::value;
        if constexpr (i < NL)
            if (i < n_loads) load_to_lds16(pl[i] + iss_st * BK, my_ring + iss_slot * my_stage + l_off[i]);
    };
    auto issued = [&]() {
        ++iss_st;
        if (++iss_slot == depth) iss_slot = 0;
    };

    f32x16 acc[2][MT];
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int t = 0; t < MT; ++t)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[j][t][r] = 0.f;
    const bool second = wave + 4 < nt;  // this (multiplying) wave's second weight tile exists
    // swizzles of LDS rows 32*b + l32 for even / odd b (weight tile w and w + 4 have the parity of w)
    const int sw_even = G::swz(l32), sw_odd = G::swz(32 + l32), sw_w = (wave & 1) ? sw_odd : sw_even;

    if (loads)
        for (int st = 0; st < depth - 1 && st < nk; ++st) {
            static_for<NL>([&](auto i_c) { issue_one(i_c); });
            issued();
        }
    int wslot = 0, aslot = 0;
    constexpr int KS = BK / 16, GROUPS = 2 * KS, PER = (NL + GROUPS - 1) / GROUPS;
    for (int st = 0; st < nk; ++st) {
        // stage st has landed once only the stages this wave issued after it are outstanding
        if (loads) wait_loads_rt((iss_st - (st + 1)) * n_loads);
        __builtin_amdgcn_s_barrier();  // stage st complete for every wave; every wave is done with stage st-1
        const bool more = loads && iss_st < nk;
        if (SPEC && more) static_for<NL>([&](auto i_c) { issue_one(i_c); });
        if (computes) {
            const unsigned char *wb = ring + a_ring + wslot * wstage, *ab = ring + aslot * kAStage;
            // fragments of K step ks + 1 are read while the MFMAs of step ks run: one 16-byte read behind each of the
            // first MFMAs, pinned there -- issued as one run ahead of the MFMAs they cost the matrix pipe their issue
            // time
            u32x4 wf[2][2], af[2][TERMS][MT];
            constexpr int NR = 2 + TERMS * MT, NM = 2 * TERMS * MT;  // reads and MFMAs of a 16-wide step
            // read r of a step: 0 = the first weight tile, 1 .. TERMS = activation tile 0 (high, low), TERMS + 1 = the
            // second weight tile, then the other activation tiles
            auto frag = [&](auto ks_c, auto r_c) {
                constexpr int ks = decltype(ks_c)::value, b = ks & 1, r = decltype(r_c)::value;
                const int c = 2 * ks + kg;
                if constexpr (r == 0) {
                    wf[b][0] = *reinterpret_cast<const u32x4 *>(wb + (wave * 32 + l32) * G::kSeg + (c ^ sw_w) * 16);
                } else if constexpr (r == TERMS + 1) {
                    if (second)
                        wf[b][1] =
                            *reinterpret_cast<const u32x4 *>(wb + ((wave + 4) * 32 + l32) * G::kSeg + (c ^ sw_w) * 16);
                } else {
                    constexpr int q = r <= TERMS ? r - 1 : r - 2, t = q / TERMS, term = q % TERMS;
                    constexpr int blk = t * TERMS + term;  // 32-row block of the activation stage
                    af[b][term][t] = *reinterpret_cast<const u32x4 *>(
                        ab + (blk * 32 + l32) * G::kSeg + (c ^ ((blk & 1) ? sw_odd : sw_even)) * 16);
                }
            };
            static_for<NR>([&](auto r_c) { frag(ic<0>{}, r_c); });
            static_for<KS>([&](auto ks_c) {
                constexpr int ks = decltype(ks_c)::value, b = ks & 1;
                static_for<NM>([&](auto m_c) {
                    constexpr int m = decltype(m_c)::value, j = m / (TERMS * MT), t = (m % (TERMS * MT)) / TERMS;
                    constexpr int term = m % TERMS;
                    // a share of this wave's loads for the stage it fills, ahead of each weight tile's MFMAs
                    if constexpr (m % (TERMS * MT) == 0)
                        if (!SPEC && more)
                            static_for<PER>([&](auto q_c) { issue_one(ic<(2 * ks + j) * PER + decltype(q_c)::value>{}); });
                    if (j == 0 || second) {
                        if constexpr (F16)
                            acc[j][t] = __builtin_amdgcn_mfma_f32_32x32x16_f16(as_f16x8(wf[b][j]), as_f16x8(af[b][term][t]),
                                                                               acc[j][t], 0, 0, 0);
                        else
                            acc[j][t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                                as_bf16x8(wf[b][j]), as_bf16x8(af[b][term][t]), acc[j][t], 0, 0, 0);
                    }
                    if constexpr (ks + 1 < KS && m < NR) frag(ic<ks + 1>{}, m_c);
                    __builtin_amdgcn_sched_barrier(0);
                });
                // (one activation tile in one term has more reads than MFMAs: the rest follow the last MFMA)
                if constexpr (ks + 1 < KS && NR > NM)
                    static_for<NR - NM>([&](auto e_c) { frag(ic<ks + 1>{}, ic<NM + decltype(e_c)::value>{}); });
            });
        }
        if (more) issued();
        if (++wslot == nw) wslot = 0;
        if (++aslot == na) aslot = 0;
    }
    if (!computes) return;
    // C^T tile: lane = activation row (column of the MFMA result), register r = weight row 8*(r/4) + 4*kg + r%4
    float *pz = part + (size_t)blockIdx.y * M * N;
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        if (j == 1 && !second) break;
#pragma unroll
        for (int t = 0; t < MT; ++t) {
            const int m = t * 32 + l32;
            if (m >= M) continue;
#pragma unroll
            for (int rq = 0; rq < 4; ++rq) {
                const int n = n0 + (wave + 4 * j) * 32 + 8 * rq + 4 * kg;
                float *dst = pz + (size_t)m * N + n;
                if (n + 3 < N && (N & 3) == 0) {
                    *reinterpret_cast<float4 *>(dst) = make_float4(acc[j][t][4 * rq + 0], acc[j][t][4 * rq + 1],
                                                                   acc[j][t][4 * rq + 2], acc[j][t][4 * rq + 3]);
                } else {
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        if (n + e < N) dst[e] = acc[j][t][4 * rq + e];
                }
            }
        }
    }
}

// ---------------------------------------------------------------------------------------
// RoPE on q and k at absolute positions pos0 + row, K/V appended to the cache, q kept as bf16.
// A thread owns four neighbouring rotation pairs (i, i + d/2) of one head: 16-byte loads of the partial sums and
// the rotation table, 8-byte stores; d/8 threads per head, 256 / (d/8) heads per block, grid (rows, head groups).
// ---------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_rope_append(const float *__restrict__ part, int n_part, size_t part_stride,
                                                     const bf16_t *__restrict__ bias, const float2 *__restrict__ rope,
                                                     bf16_t *__restrict__ qb, bf16_t *__restrict__ qb_lo,
                                                     bf16_t *__restrict__ kc, bf16_t *__restrict__ vc, int pos0, int nq,
                                                     int nkv, int d, int max_seq, PartTail tail) {
    const int half = d >> 1, tph = d >> 3, row = blockIdx.x;  // tph: threads per head
    const int head = blockIdx.y * (256 / tph) + threadIdx.x / tph, i = 4 * (threadIdx.x % tph);
    if (head >= nq + 2 * nkv) return;
    const int pos = pos0 + row;
    const size_t off = (size_t)row * (nq + 2 * nkv) * d + head * d;
    float lo[4] = {0.f, 0.f, 0.f, 0.f}, hi[4] = {0.f, 0.f, 0.f, 0.f};
    auto add = [&](const float *src) {
        const float4 a = *reinterpret_cast<const float4 *>(src + i), b = *reinterpret_cast<const float4 *>(src + i + half);
        lo[0] += a.x, lo[1] += a.y, lo[2] += a.z, lo[3] += a.w;
        hi[0] += b.x, hi[1] += b.y, hi[2] += b.z, hi[3] += b.w;
    };
    for (int s = 0; s < n_part; ++s) add(part + (size_t)s * part_stride + off);
    if (tail.n && head * d >= tail.col0) {  // col0 is a multiple of 256, so a head lies on one side of it
        const float *src = part + tail.base + (long long)row * tail.ld + (head * d - tail.col0);
        for (int t = 0; t < tail.n; ++t, src += tail.stride) add(src);
    }
    if (bias) {
        const u32x2 bl = *reinterpret_cast<const u32x2 *>(bias + head * d + i);
        const u32x2 bh = *reinterpret_cast<const u32x2 *>(bias + head * d + i + half);
        lo[0] += bf16_lo(bl.x), lo[1] += bf16_hi(bl.x), lo[2] += bf16_lo(bl.y), lo[3] += bf16_hi(bl.y);
        hi[0] += bf16_lo(bh.x), hi[1] += bf16_hi(bh.x), hi[2] += bf16_lo(bh.y), hi[3] += bf16_hi(bh.y);
    }
    if (head < nq + nkv) {
        const float4 *cs4 = reinterpret_cast<const float4 *>(rope + (size_t)pos * half + i);
        const float4 c01 = cs4[0], c23 = cs4[1];  // (cos, sin) of pairs i, i+1 and i+2, i+3
        const float cx[4] = {c01.x, c01.z, c23.x, c23.z}, sy[4] = {c01.y, c01.w, c23.y, c23.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const float nlo = lo[e] * cx[e] - hi[e] * sy[e];
            const float nhi = hi[e] * cx[e] + lo[e] * sy[e];
            lo[e] = nlo, hi[e] = nhi;
        }
    }
    bf16_t *dst;
    if (head < nq)
        dst = qb + (size_t)row * nq * d + head * d;
    else if (head < nq + nkv)
        dst = kc + ((size_t)(head - nq) * max_seq + pos) * d;
    else
        dst = vc + ((size_t)(head - nq - nkv) * max_seq + pos) * d;
    const u32x2 plo = {pack_bf16x2(lo[0], lo[1]), pack_bf16x2(lo[2], lo[3])};
    const u32x2 phi = {pack_bf16x2(hi[0], hi[1]), pack_bf16x2(hi[2], hi[3])};
    *reinterpret_cast<u32x2 *>(dst + i) = plo;
    *reinterpret_cast<u32x2 *>(dst + i + half) = phi;
    if (head < nq && qb_lo) {  // short chunks: the query keeps 16 mantissa bits as a second bf16 term
        bf16_t *dl = qb_lo + (size_t)row * nq * d + head * d;
        const u32x2 rlo = {pack_bf16x2(lo[0] - bf16_lo(plo.x), lo[1] - bf16_hi(plo.x)),
                           pack_bf16x2(lo[2] - bf16_lo(plo.y), lo[3] - bf16_hi(plo.y))};
        const u32x2 rhi = {pack_bf16x2(hi[0] - bf16_lo(phi.x), hi[1] - bf16_hi(phi.x)),
                           pack_bf16x2(hi[2] - bf16_lo(phi.y), hi[3] - bf16_hi(phi.y))};
        *reinterpret_cast<u32x2 *>(dl + i) = rlo;
        *reinterpret_cast<u32x2 *>(dl + i + half) = rhi;
    }
}

// a[row][i] = silu(gate) * up from the K slices of the gate/up projection of a short chunk
// (part is [n_part][rows][2I]: gate columns [0,I), up columns [I,2I)), written as two bf16 terms.
__global__ __launch_bounds__(256) void k_swiglu_rows(const float *__restrict__ part, int n_part, size_t part_stride,
                                                     int I, bf16_t *__restrict__ act, bf16_t *__restrict__ act_lo,
                                                     int f16) {
    const int row = blockIdx.y;
    const int i4 = blockIdx.x * 256 + threadIdx.x;  // group of four columns
    if (i4 * 4 >= I) return;
    const float4 *p0 = reinterpret_cast<const float4 *>(part + (size_t)row * 2 * I);
    const size_t ps4 = part_stride / 4;
    float4 gt = make_float4(0, 0, 0, 0), up = gt;
    for (int s0 = 0; s0 < n_part; s0 += 4) {
        float4 a[4], b[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            bool ok = s0 + u < n_part;
            a[u] = ok ? p0[(size_t)(s0 + u) * ps4 + i4] : make_float4(0, 0, 0, 0);
            b[u] = ok ? p0[(size_t)(s0 + u) * ps4 + I / 4 + i4] : make_float4(0, 0, 0, 0);
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            gt.x += a[u].x; gt.y += a[u].y; gt.z += a[u].z; gt.w += a[u].w;
            up.x += b[u].x; up.y += b[u].y; up.z += b[u].z; up.w += b[u].w;
        }
    }
    const float v0 = gt.x / (1.0f + expf(-gt.x)) * up.x, v1 = gt.y / (1.0f + expf(-gt.y)) * up.y;
    const float v2 = gt.z / (1.0f + expf(-gt.z)) * up.z, v3 = gt.w / (1.0f + expf(-gt.w)) * up.w;
    if (f16) {  // fp16 operand mode: one fp16 number, no low term
        const u32x2 h16 = {pack_f16x2(v0, v1), pack_f16x2(v2, v3)};
        reinterpret_cast<u32x2 *>(act + (size_t)row * I)[i4] = h16;
        return;
    }
    u32x2 hi = {pack_bf16x2(v0, v1), pack_bf16x2(v2, v3)};
    u32x2 lo = {pack_bf16x2(v0 - bf16_lo(hi.x), v1 - bf16_hi(hi.x)), pack_bf16x2(v2 - bf16_lo(hi.y), v3 - bf16_hi(hi.y))};
    reinterpret_cast<u32x2 *>(act + (size_t)row * I)[i4] = hi;
    reinterpret_cast<u32x2 *>(act_lo + (size_t)row * I)[i4] = lo;
}

// ---------------------------------------------------------------------------------------
// Causal flash attention of m query tokens at absolute positions kv0 + q over keys [0, kv0 + q].
// The G query heads that share a kv head are folded into the row dimension: row r of kv head g is
// (token r / G, head g*G + r % G), so one staged K/V tile serves all of them.  Block = 4 waves x 32
// rows; keys go through LDS in tiles of 64 (V transposed on the way in), the next tile is already
// in registers while the current one is multiplied.  Each wave computes S^T = K Q^T, so a lane owns
// one row: the online-softmax statistics are per-lane scalars, and P^T feeds the second MFMA
// (O^T = V^T P^T) straight from registers.  grid.z splits the key range; with more than one
// split each block publishes (max, sum, unnormalised output) and k_flash_combine merges them in a
// fixed order -- that is what gives a 20-token catch-up chunk on a 4k context enough blocks.
// ---------------------------------------------------------------------------------------
constexpr int kFlashKeys = 64;

// Resolves blockIdx.x to (segment, row block inside it); all values are wave-uniform.
struct FlashWhere {
    int m, kv0, row_base, bx, nbx;
    size_t cache;
};
__device__ __forceinline__ FlashWhere flash_where(const FlashSeg *segs, int n_seg, size_t seq_stride, int m, int kv0) {
    FlashWhere w = {m, kv0, 0, (int)blockIdx.x, (int)gridDim.x, 0};
    if (segs) {
        int j = 0;
        while (j + 1 < n_seg && w.bx >= segs[j + 1].blk0) ++j;
        const FlashSeg sg = segs[j];
        w.m = sg.len, w.kv0 = sg.kv0, w.row_base = sg.row0, w.bx -= sg.blk0, w.nbx = sg.nblk;
        w.cache = (size_t)sg.seq * seq_stride;
    }
    return w;
}

template <int D>
__global__ __launch_bounds__(256) void k_flash_prefill(const bf16_t *__restrict__ qb, const bf16_t *__restrict__ kc,
                                                       const bf16_t *__restrict__ vc, bf16_t *__restrict__ out,
                                                       bf16_t *__restrict__ outlo, float *__restrict__ part_o,
                                                       float *__restrict__ part_ml, int m, int kv0, int nq, int G,
                                                       int max_seq, const FlashSeg *__restrict__ segs, int n_seg,
                                                       size_t seq_stride, int m_total, int f16) {
    constexpr int KS = D + 8;             // K tile row stride (elements): 16-byte reads conflict-free
    constexpr int VS = kFlashKeys + 4;    // V^T row stride (elements)
    constexpr int CH = D / 8;             // 16-byte chunks per key
    constexpr int CPT = kFlashKeys * CH / 256;  // chunks per thread per tile (4 for D=128, 2 for D=64)
    __shared__ __align__(16) bf16_t Ks[kFlashKeys * KS];
    __shared__ __align__(16) bf16_t Vt[D * VS];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, kg = lane >> 5;
    const int g = blockIdx.y, n_split = gridDim.z, z = blockIdx.z;
    const FlashWhere fw = flash_where(segs, n_seg, seq_stride, m, kv0);
    m = fw.m, kv0 = fw.kv0;
    kc += fw.cache, vc += fw.cache;
    const int rows = m * G;
    const int r0 = fw.bx * 128, rw0 = r0 + wave * 32;
    const int ldq = nq * D;
    const bool wave_active = rw0 < rows;
    const int row = min(rw0 + l32, rows - 1);
    const int qtok = row / G, head = g * G + row % G;
    const int q_abs = kv0 + qtok;
    const int wave_last_key = kv0 + min(rw0 + 31, rows - 1) / G;
    const int n_keys = kv0 + min(r0 + 127, rows - 1) / G + 1;       // keys any row of the block may see
    const int n_tiles = (n_keys + kFlashKeys - 1) / kFlashKeys;
    const int tps = (n_tiles + n_split - 1) / n_split;             // tiles per split
    const int t_begin = z * tps, t_end = min(n_tiles, t_begin + tps);
    const float scale = 1.4426950408889634f / sqrtf((float)D);

    bf16x8 qf[D / 16];
#pragma unroll
    for (int s = 0; s < D / 16; ++s)
        qf[s] = as_bf16x8(*reinterpret_cast<const u32x4 *>(qb + (size_t)(fw.row_base + qtok) * ldq + head * D + 16 * s + 8 * kg));

    f32x16 o[D / 32];
#pragma unroll
    for (int t = 0; t < D / 32; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[t][r] = 0.f;
    float m_i = -INFINITY, l_i = 0.f;

    const bf16_t *kbase = kc + (size_t)g * max_seq * D;
    const bf16_t *vbase = vc + (size_t)g * max_seq * D;
    // staging ownership: K chunk c = tid + 256*i is (key c / CH, columns 8*(c % CH) .. +7); V: consecutive
    // keys of one chunk column per thread, so the transposed tile is written four (two) keys at a time
    u32x4 kr[CPT], vr[CPT];
    auto fetch = [&](int t) {
        const int key0 = t * kFlashKeys;
#pragma unroll
        for (int i = 0; i < CPT; ++i) {
            int c = tid + i * 256;
            int kabs = min(key0 + c / CH, n_keys - 1);  // clamped rows are masked by the causal test
            kr[i] = *reinterpret_cast<const u32x4 *>(kbase + (size_t)kabs * D + (c % CH) * 8);
        }
        // V: D = 128 -> keys 4*kq + p (p < 4) of chunk column tid/16;
        //    D = 64  -> keys 4*kq + 2*pair + p (p < 2) of chunk column (tid/16) % 8, pair = tid/128
        const int kq = tid & 15;
        const int col = CPT == 4 ? tid >> 4 : (tid >> 4) & (CH - 1);
        const int kfirst = CPT == 4 ? 4 * kq : 4 * kq + 2 * ((tid >> 4) / CH);
#pragma unroll
        for (int p = 0; p < CPT; ++p) {
            int kabs = min(key0 + kfirst + p, n_keys - 1);
            vr[p] = *reinterpret_cast<const u32x4 *>(vbase + (size_t)kabs * D + col * 8);
        }
    };
    auto stash = [&]() {
#pragma unroll
        for (int i = 0; i < CPT; ++i) {
            int c = tid + i * 256;
            *reinterpret_cast<u32x4 *>(&Ks[(c / CH) * KS + (c % CH) * 8]) = kr[i];
        }
        if (CPT == 4) {
            // four keys x eight d of one chunk column -> eight 8-byte writes of four consecutive keys
            const int kq = tid & 15, col = tid >> 4;
            const uint32_t w[4][4] = {{vr[0].x, vr[0].y, vr[0].z, vr[0].w},
                                      {vr[1].x, vr[1].y, vr[1].z, vr[1].w},
                                      {vr[2].x, vr[2].y, vr[2].z, vr[2].w},
                                      {vr[3].x, vr[3].y, vr[3].z, vr[3].w}};
#pragma unroll
            for (int e = 0; e < 4; ++e) {  // d = 8*col + 2e (low halves) and 2e+1 (high halves)
                u32x2 lo = {(w[0][e] & 0xffffu) | (w[1][e] << 16), (w[2][e] & 0xffffu) | (w[3][e] << 16)};
                u32x2 hi = {(w[0][e] >> 16) | (w[1][e] & 0xffff0000u), (w[2][e] >> 16) | (w[3][e] & 0xffff0000u)};
                *reinterpret_cast<u32x2 *>(&Vt[(8 * col + 2 * e) * VS + 4 * kq]) = lo;
                *reinterpret_cast<u32x2 *>(&Vt[(8 * col + 2 * e + 1) * VS + 4 * kq]) = hi;
            }
        } else {
            // D = 64: two keys x eight d per thread -> eight 4-byte writes of two consecutive keys
            const int kq = tid & 15, col = (tid >> 4) & (CH - 1), pair = (tid >> 4) / CH;
            const uint32_t w[2][4] = {{vr[0].x, vr[0].y, vr[0].z, vr[0].w}, {vr[1].x, vr[1].y, vr[1].z, vr[1].w}};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                uint32_t lo = (w[0][e] & 0xffffu) | (w[1][e] << 16);
                uint32_t hi = (w[0][e] >> 16) | (w[1][e] & 0xffff0000u);
                *reinterpret_cast<uint32_t *>(&Vt[(8 * col + 2 * e) * VS + 4 * kq + 2 * pair]) = lo;
                *reinterpret_cast<uint32_t *>(&Vt[(8 * col + 2 * e + 1) * VS + 4 * kq + 2 * pair]) = hi;
            }
        }
    };

    if (t_begin < t_end) fetch(t_begin);
    for (int t = t_begin; t < t_end; ++t) {
        const int key0 = t * kFlashKeys;
        __syncthreads();  // previous tile fully consumed
        stash();
        __syncthreads();
        if (t + 1 < t_end) fetch(t + 1);
        if (!wave_active || key0 > wave_last_key) continue;

        // S^T: two 32-key sub-tiles x 32 rows
        f32x16 sacc[2];
#pragma unroll
        for (int u = 0; u < 2; ++u) {
#pragma unroll
            for (int r = 0; r < 16; ++r) sacc[u][r] = 0.f;
#pragma unroll
            for (int s = 0; s < D / 16; ++s) {
                bf16x8 kf = as_bf16x8(*reinterpret_cast<const u32x4 *>(&Ks[(u * 32 + l32) * KS + 16 * s + 8 * kg]));
                sacc[u] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[s], sacc[u], 0, 0, 0);
            }
        }
        // lane = row l32; register r of sub-tile u = key 32*u + 8*(r/4) + 4*kg + r%4 of the tile
        float mx = -INFINITY;
#pragma unroll
        for (int u = 0; u < 2; ++u)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                int kabs = key0 + 32 * u + 8 * (r >> 2) + 4 * kg + (r & 3);
                float sc = kabs > q_abs ? -INFINITY : sacc[u][r] * scale;
                sacc[u][r] = sc;
                mx = fmaxf(mx, sc);
            }
        mx = max_xor32(mx);
        const float m_new = fmaxf(m_i, mx);
        const float m_use = m_new == -INFINITY ? 0.f : m_new;  // a row may see no key of this split yet
        const float corr = exp2f(m_i - m_use);                 // m_i = -inf gives 0
        float rs = 0.f;
#pragma unroll
        for (int u = 0; u < 2; ++u)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                float p = exp2f(sacc[u][r] - m_use);
                sacc[u][r] = p;
                rs += p;
            }
        rs = sum_xor32(rs);
        l_i = l_i * corr + rs;
        m_i = m_new;
#pragma unroll
        for (int tt = 0; tt < D / 32; ++tt)
#pragma unroll
            for (int r = 0; r < 16; ++r) o[tt][r] *= corr;
        // P^T as the B operand: k-step s2 covers keys 16*s2 .. +15 of the tile; this lane holds registers
        // 8*(s2%2) .. +7 of sub-tile s2/2, i.e. keys 16*s2 + {4kg..4kg+3, 8+4kg..8+4kg+3}
        bf16x8 pf[4];
#pragma unroll
        for (int s2 = 0; s2 < 4; ++s2) {
            const int u = s2 >> 1, b = 8 * (s2 & 1);
            u32x4 pk = {pack_bf16x2(sacc[u][b + 0], sacc[u][b + 1]), pack_bf16x2(sacc[u][b + 2], sacc[u][b + 3]),
                        pack_bf16x2(sacc[u][b + 4], sacc[u][b + 5]), pack_bf16x2(sacc[u][b + 6], sacc[u][b + 7])};
            pf[s2] = as_bf16x8(pk);
        }
#pragma unroll
        for (int tt = 0; tt < D / 32; ++tt) {
#pragma unroll
            for (int s2 = 0; s2 < 4; ++s2) {
                const bf16_t *vrow = &Vt[(tt * 32 + l32) * VS + 16 * s2 + 4 * kg];
                u32x2 a0 = *reinterpret_cast<const u32x2 *>(vrow);
                u32x2 a1 = *reinterpret_cast<const u32x2 *>(vrow + 8);
                u32x4 vv = {a0.x, a0.y, a1.x, a1.y};
                o[tt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(vv), pf[s2], o[tt], 0, 0, 0);
            }
        }
    }
    if (!wave_active || rw0 + l32 >= rows) return;
    if (n_split == 1) {
        const float inv = 1.0f / l_i;
        bf16_t *orow = out + (size_t)(fw.row_base + qtok) * ldq + head * D;
        bf16_t *lrow = outlo ? outlo + (size_t)(fw.row_base + qtok) * ldq + head * D : nullptr;
#pragma unroll
        for (int tt = 0; tt < D / 32; ++tt)
#pragma unroll
            for (int rq = 0; rq < 4; ++rq) {
                int dcol = tt * 32 + 8 * rq + 4 * kg;
                float v0 = o[tt][4 * rq + 0] * inv, v1 = o[tt][4 * rq + 1] * inv;
                float v2 = o[tt][4 * rq + 2] * inv, v3 = o[tt][4 * rq + 3] * inv;
                u32x2 pk = {pack_16x2(f16, v0, v1), pack_16x2(f16, v2, v3)};  // output: bf16, or fp16 (no low term)
                *reinterpret_cast<u32x2 *>(orow + dcol) = pk;
                if (lrow) {
                    u32x2 lo = {pack_bf16x2(v0 - bf16_lo(pk.x), v1 - bf16_hi(pk.x)),
                                pack_bf16x2(v2 - bf16_lo(pk.y), v3 - bf16_hi(pk.y))};
                    *reinterpret_cast<u32x2 *>(lrow + dcol) = lo;
                }
            }
    } else {
        // partial result of this key split for (token, head): [z][token*nq + head]
        const size_t pr = (size_t)z * m_total * nq + (size_t)(fw.row_base + qtok) * nq + head;
        float *po = part_o + pr * D;
#pragma unroll
        for (int tt = 0; tt < D / 32; ++tt)
#pragma unroll
            for (int rq = 0; rq < 4; ++rq) {
                int dcol = tt * 32 + 8 * rq + 4 * kg;
                *reinterpret_cast<float4 *>(po + dcol) =
                    make_float4(o[tt][4 * rq + 0], o[tt][4 * rq + 1], o[tt][4 * rq + 2], o[tt][4 * rq + 3]);
            }
        if (kg == 0) {
            part_ml[pr * 2] = m_i;
            part_ml[pr * 2 + 1] = l_i;
        }
    }
}

// head_dim 128 (every chunk length): the same attention with at most 256 registers per lane, so that two waves
// share a SIMD and one wave's softmax runs under another's MFMAs, and one barrier per 64-key tile:
//   * K tiles go global -> LDS directly into two 16 KB slots whose 16-byte chunks are XOR-swizzled by the key
//     row, so the S^T fragment reads need neither staging registers nor padding;
//   * the S^T fragment of lane i reads key row swap(i) (bits 2 and 3 of i exchanged): the 32x32 MFMA output
//     then leaves every lane with eight *consecutive* keys per 16-key step, so P^T feeds the second MFMA
//     straight from registers and each V^T fragment is one 16-byte read;
//   * the running maximum is raised only when it would grow by more than 2^8 (softmax is shift-invariant and
//     the final division by the row sum absorbs the reference), which makes the rescale of the 64 output
//     registers rare; tiles wholly below the diagonal skip the causal compare.
// Interface and key-split partial results are those of k_flash_prefill.
// ---------------------------------------------------------------------------------------
template <int NW, bool TWO>  // NW waves per block, 32 folded rows each; TWO: queries arrive as two bf16 terms
__global__ __launch_bounds__(64 * NW, 2) void k_flash_long(const bf16_t *__restrict__ qb,
                                                    const bf16_t *__restrict__ qb_lo, const bf16_t *__restrict__ kc,
                                                    const bf16_t *__restrict__ vc, bf16_t *__restrict__ out,
                                                    bf16_t *__restrict__ outlo, float *__restrict__ part_o,
                                                    float *__restrict__ part_ml, int m, int kv0, int nq, int G,
                                                    int max_seq, const FlashSeg *__restrict__ segs, int n_seg,
                                                    size_t seq_stride, int m_total, int f16) {
    constexpr int D = 128, VS = kFlashKeys + 8;  // V^T rows of 144 bytes: 16-byte reads conflict-free
    __shared__ __align__(16) unsigned char Ks[2][kFlashKeys * D * 2];
    __shared__ __align__(16) bf16_t Vt[2][D * VS];

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l32 = lane & 31, kg = lane >> 5;
    const int g = blockIdx.y, n_split = gridDim.z, z = blockIdx.z;
    const FlashWhere fw = flash_where(segs, n_seg, seq_stride, m, kv0);
    m = fw.m, kv0 = fw.kv0;
    kc += fw.cache, vc += fw.cache;
    const int rows = m * G;
    constexpr int kLongRows = 32 * NW, NT = 64 * NW;
    // blocks with the most keys (the last rows) are dispatched first, so the causal tail is made of short blocks
    const int r0 = (fw.nbx - 1 - fw.bx) * kLongRows, rw0 = r0 + wave * 32;
    const int ldq = nq * D;
    const bool wave_active = rw0 < rows;
    const int row = min(rw0 + l32, rows - 1);
    const int qtok = row / G, head = g * G + row % G;
    const int q_abs = kv0 + qtok;
    const int wave_first_q = kv0 + min(rw0, rows - 1) / G;          // smallest position among the wave's rows
    const int wave_last_key = kv0 + min(rw0 + 31, rows - 1) / G;
    const int n_keys = kv0 + min(r0 + kLongRows - 1, rows - 1) / G + 1;
    const int n_tiles = (n_keys + kFlashKeys - 1) / kFlashKeys;
    const int tps = (n_tiles + n_split - 1) / n_split;
    const int t_begin = z * tps, t_end = min(n_tiles, t_begin + tps);
    const float scale = 1.4426950408889634f / sqrtf((float)D);

    bf16x8 qf[D / 16], ql[TWO ? D / 16 : 1];
#pragma unroll
    for (int s = 0; s < D / 16; ++s) {
        qf[s] = as_bf16x8(*reinterpret_cast<const u32x4 *>(qb + (size_t)(fw.row_base + qtok) * ldq + head * D + 16 * s + 8 * kg));
        if constexpr (TWO)
            ql[s] = as_bf16x8(*reinterpret_cast<const u32x4 *>(qb_lo + (size_t)(fw.row_base + qtok) * ldq + head * D + 16 * s + 8 * kg));
    }

    f32x16 o[D / 32];
#pragma unroll
    for (int t = 0; t < D / 32; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[t][r] = 0.f;
    float m_i = -INFINITY, l_i = 0.f;

    const bf16_t *kbase = kc + (size_t)g * max_seq * D;
    const bf16_t *vbase = vc + (size_t)g * max_seq * D;
    const uint32_t ks0 = (uint32_t)(uintptr_t)&Ks[0][0];
    // K: a wave loads 64/NW key rows of the tile with 1 KB instructions of four 256-byte rows each;
    // lane -> (row lane/16, 16-byte position lane%16 holding chunk position ^ (row & 15))
    constexpr int KI = 16 / NW;  // K instructions per wave per tile
    auto load_k = [&](int t) {
        const int key0 = t * kFlashKeys;
#pragma unroll
        for (int i = 0; i < KI; ++i) {
            const int r4 = (wave * KI + i) * 4, r = r4 + (lane >> 4);
            const int c = (lane & 15) ^ (r & 15);
            const int kabs = min(key0 + r, n_keys - 1);  // clamped rows lie above the diagonal: masked
            load_to_lds16(kbase + (size_t)kabs * D + c * 8, ks0 + (t & 1) * (kFlashKeys * D * 2) + r4 * 256);
        }
    };
    // V: thread -> keys 2*(tid%32), +1 of 8-column groups tid/32 + (NT/32)*q; written transposed, two keys per word
    constexpr int VQ = 16 / (NT / 32);
    u32x4 vr[VQ][2];
    auto load_v = [&](int t) {
        const int key0 = t * kFlashKeys;
#pragma unroll
        for (int q = 0; q < VQ; ++q)
#pragma unroll
            for (int p = 0; p < 2; ++p) {
                const int kabs = min(key0 + 2 * (tid & 31) + p, n_keys - 1);
                vr[q][p] = *reinterpret_cast<const u32x4 *>(vbase + (size_t)kabs * D + ((tid >> 5) + (NT / 32) * q) * 8);
            }
    };
    auto stash_v = [&](int t) {
        bf16_t *vt = &Vt[t & 1][0];
        const int kp = tid & 31;
#pragma unroll
        for (int q = 0; q < VQ; ++q) {
            const int col = (tid >> 5) + (NT / 32) * q;
            const uint32_t a[4] = {vr[q][0].x, vr[q][0].y, vr[q][0].z, vr[q][0].w};
            const uint32_t b[4] = {vr[q][1].x, vr[q][1].y, vr[q][1].z, vr[q][1].w};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                *reinterpret_cast<uint32_t *>(&vt[(8 * col + 2 * e) * VS + 2 * kp]) = (a[e] & 0xffffu) | (b[e] << 16);
                *reinterpret_cast<uint32_t *>(&vt[(8 * col + 2 * e + 1) * VS + 2 * kp]) =
                    (a[e] >> 16) | (b[e] & 0xffff0000u);
            }
        }
    };

    // S^T fragment rows: lane i of a 32-key sub-tile reads key swap(i)
    const int krow = (l32 & 19) | ((l32 & 4) << 1) | ((l32 & 8) >> 1);
    const int k_swz = krow & 15;

    f32x16 sacc[2];
    bf16x8 pf[4];
    auto tile_active = [&](int t) { return wave_active && t * kFlashKeys <= wave_last_key; };
    // S^T of tile t: two 32-key sub-tiles x 32 rows
    // (fragment reads run kAhead MFMAs ahead of their use, one read pinned behind each MFMA: an LDS read takes
    // longer than the one or two MFMAs the compiler's own schedule leaves between a read and its use)
    constexpr int kAhead = 4;
    auto scores = [&](int t) {
        if (!tile_active(t)) return;
        const unsigned char *kt = &Ks[t & 1][0];
#pragma unroll
        for (int u = 0; u < 2; ++u)
#pragma unroll
            for (int r = 0; r < 16; ++r) sacc[u][r] = 0.f;
        constexpr int NS = D / 16;  // 16-wide steps of a sub-tile; fragment i is sub-tile i / NS, step i % NS
        bf16x8 kf[kAhead];
        auto kread = [&](auto i_c) {
            constexpr int i = decltype(i_c)::value, u = i / NS, s = i % NS;
            kf[i % kAhead] = as_bf16x8(
                *reinterpret_cast<const u32x4 *>(kt + (u * 32 + krow) * 256 + (((2 * s + kg) ^ k_swz) * 16)));
        };
        static_for<kAhead>([&](auto i_c) { kread(i_c); });
        __builtin_amdgcn_sched_barrier(0);
        static_for<2 * NS>([&](auto i_c) {
            constexpr int i = decltype(i_c)::value, u = i / NS, s = i % NS;
            sacc[u] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[i % kAhead], qf[s], sacc[u], 0, 0, 0);
            if constexpr (TWO) sacc[u] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[i % kAhead], ql[s], sacc[u], 0, 0, 0);
            if constexpr (i + kAhead < 2 * NS) kread(ic<i + kAhead>{});
            __builtin_amdgcn_sched_barrier(0);
        });
    };
    // online softmax of tile t: lane = query row; register r of sub-tile u is key 32u + 16*(r/8) + 8*kg + r%8
    auto softmax = [&](int t) {
        if (!tile_active(t)) return;
        const int key0 = t * kFlashKeys;
        if (key0 + kFlashKeys - 1 > wave_first_q) {  // the tile touches the diagonal for some row of this wave
#pragma unroll
            for (int u = 0; u < 2; ++u)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int kabs = key0 + 32 * u + 16 * (r >> 3) + 8 * kg + (r & 7);
                    if (kabs > q_abs) sacc[u][r] = -INFINITY;
                }
        }
        float mx = sacc[0][0];
#pragma unroll
        for (int u = 0; u < 2; ++u)
#pragma unroll
            for (int r = 0; r < 16; ++r) mx = fmaxf(mx, sacc[u][r]);
        mx = max_xor32(mx);
        const float m_cand = mx * scale;
        const bool raise = m_cand > m_i + 8.0f;                    // also the first keys a row sees (m_i = -inf)
        const float m_new = raise ? m_cand : m_i;
        const float base = m_new == -INFINITY ? 0.f : m_new;       // a row may have seen no key yet
        float rs = 0.f;
#pragma unroll
        for (int u = 0; u < 2; ++u)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const float p = __builtin_amdgcn_exp2f(fmaf(sacc[u][r], scale, -base));
                sacc[u][r] = p;
                rs += p;
            }
        rs = sum_xor32(rs);
        if (__builtin_amdgcn_ballot_w64(raise) != 0) {
            const float corr = raise ? __builtin_amdgcn_exp2f(m_i - base) : 1.0f;  // m_i = -inf gives 0
            l_i *= corr;
#pragma unroll
            for (int tt = 0; tt < D / 32; ++tt)
#pragma unroll
                for (int r = 0; r < 16; ++r) o[tt][r] *= corr;
        }
        l_i += rs;
        m_i = m_new;
        // P^T as the B operand: 16-key step s2 = registers 8*(s2%2) .. +7 of sub-tile s2/2 = keys 16*s2 + 8*kg .. +7
#pragma unroll
        for (int s2 = 0; s2 < 4; ++s2) {
            const int u = s2 >> 1, b = 8 * (s2 & 1);
            u32x4 pk = {pack_bf16x2(sacc[u][b + 0], sacc[u][b + 1]), pack_bf16x2(sacc[u][b + 2], sacc[u][b + 3]),
                        pack_bf16x2(sacc[u][b + 4], sacc[u][b + 5]), pack_bf16x2(sacc[u][b + 6], sacc[u][b + 7])};
            pf[s2] = as_bf16x8(pk);
        }
    };
    // O^T += V^T P^T for tile t
    auto weighted_values = [&](int t) {
        if (!tile_active(t)) return;
        const bf16_t *vt = &Vt[t & 1][0];
        constexpr int NV = (D / 32) * 4;  // fragment i: output tile i / 4, 16-key step i % 4
        bf16x8 vf[kAhead];
        auto vread = [&](auto i_c) {
            constexpr int i = decltype(i_c)::value, tt = i / 4, s2 = i % 4;
            vf[i % kAhead] = as_bf16x8(*reinterpret_cast<const u32x4 *>(&vt[(tt * 32 + l32) * VS + 16 * s2 + 8 * kg]));
        };
        static_for<kAhead>([&](auto i_c) { vread(i_c); });
        __builtin_amdgcn_sched_barrier(0);
        static_for<NV>([&](auto i_c) {
            constexpr int i = decltype(i_c)::value, tt = i / 4, s2 = i % 4;
            o[tt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[i % kAhead], pf[s2], o[tt], 0, 0, 0);
            if constexpr (i + kAhead < NV) vread(ic<i + kAhead>{});
            __builtin_amdgcn_sched_barrier(0);
        });
    };

    // One barrier per tile: before it a wave writes its part of V^T(t) and waits for its part of K(t); after it
    // the loads of tile t+1 start into the other slots, which every wave finished reading before the barrier.
    if (t_begin < t_end) {
        load_k(t_begin);
        load_v(t_begin);
    }
    for (int t = t_begin; t < t_end; ++t) {
        stash_v(t);
        wait_loads<0>();
        __builtin_amdgcn_s_barrier();
        if (t + 1 < t_end) {
            load_k(t + 1);
            load_v(t + 1);
        }
        scores(t);
        softmax(t);
        weighted_values(t);
    }
    if (!wave_active || rw0 + l32 >= rows) return;
    if (n_split == 1) {
        const float inv = 1.0f / l_i;
        bf16_t *orow = out + (size_t)(fw.row_base + qtok) * ldq + head * D;
#pragma unroll
        for (int tt = 0; tt < D / 32; ++tt)
#pragma unroll
            for (int rq = 0; rq < 4; ++rq) {
                const int dcol = tt * 32 + 8 * rq + 4 * kg;
                const float v0 = o[tt][4 * rq + 0] * inv, v1 = o[tt][4 * rq + 1] * inv;
                const float v2 = o[tt][4 * rq + 2] * inv, v3 = o[tt][4 * rq + 3] * inv;
                u32x2 pk = {pack_16x2(f16, v0, v1), pack_16x2(f16, v2, v3)};  // output: bf16, or fp16 (no low term)
                *reinterpret_cast<u32x2 *>(orow + dcol) = pk;
                if (outlo) {  // second bf16 term of the activation (short chunks)
                    u32x2 lo = {pack_bf16x2(v0 - bf16_lo(pk.x), v1 - bf16_hi(pk.x)),
                                pack_bf16x2(v2 - bf16_lo(pk.y), v3 - bf16_hi(pk.y))};
                    *reinterpret_cast<u32x2 *>(outlo + (size_t)(fw.row_base + qtok) * ldq + head * D + dcol) = lo;
                }
            }
    } else {
        const size_t pr = (size_t)z * m_total * nq + (size_t)(fw.row_base + qtok) * nq + head;
        float *po = part_o + pr * D;
#pragma unroll
        for (int tt = 0; tt < D / 32; ++tt)
#pragma unroll
            for (int rq = 0; rq < 4; ++rq) {
                const int dcol = tt * 32 + 8 * rq + 4 * kg;
                *reinterpret_cast<float4 *>(po + dcol) =
                    make_float4(o[tt][4 * rq + 0], o[tt][4 * rq + 1], o[tt][4 * rq + 2], o[tt][4 * rq + 3]);
            }
        if (kg == 0) {
            part_ml[pr * 2] = m_i;
            part_ml[pr * 2 + 1] = l_i;
        }
    }
}

// Merges the key splits of one (token, head): block = 256 threads = 256/D rows x D elements.  The (max, sum) pairs
// of all splits (at most 32) are fetched by the first threads of each row in one go and turned into weights in
// LDS; the partial outputs are then loaded eight splits at a time, so nothing waits on a chain of dependent loads.
// Splits are added in ascending order.
template <int D>
__global__ __launch_bounds__(256) void k_flash_combine(const float *__restrict__ part_o,
                                                       const float *__restrict__ part_ml, int n_split, int n_rows,
                                                       bf16_t *__restrict__ out, bf16_t *__restrict__ outlo, int f16) {
    constexpr int RPB = 256 / D, kMaxSplits = 32;
    __shared__ float m_s[RPB][kMaxSplits], w_s[RPB][kMaxSplits], l_s[RPB];
    const int g = threadIdx.x / D, e = threadIdx.x % D;
    const int r = blockIdx.x * RPB + g;
    const bool live = r < n_rows;
    float2 ml = make_float2(-INFINITY, 0.f);
    if (live && e < n_split) ml = reinterpret_cast<const float2 *>(part_ml)[(size_t)e * n_rows + r];
    if (e < kMaxSplits) m_s[g][e] = ml.x;
    __syncthreads();
    float M = -INFINITY;
    for (int z = 0; z < n_split; ++z) M = fmaxf(M, m_s[g][z]);
    if (e < kMaxSplits) {
        const float w = ml.x == -INFINITY ? 0.f : exp2f(ml.x - M);
        w_s[g][e] = w;
        m_s[g][e] = w * ml.y;   // reused: weighted row sums
    }
    __syncthreads();
    if (e == 0) {
        float L = 0.f;
        for (int z = 0; z < n_split; ++z) L += m_s[g][z];
        l_s[g] = L;
    }
    float A = 0.f;
    if (live) {
        for (int z0 = 0; z0 < n_split; z0 += 8) {
            float v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u)
                v[u] = z0 + u < n_split ? part_o[((size_t)(z0 + u) * n_rows + r) * D + e] : 0.f;
#pragma unroll
            for (int u = 0; u < 8; ++u)
                if (z0 + u < n_split) A += v[u] * w_s[g][z0 + u];
        }
    }
    __syncthreads();
    if (!live) return;
    const float v = A / l_s[g];
    const bf16_t hi = to_16(f16, v);
    out[(size_t)r * D + e] = hi;
    if (outlo) outlo[(size_t)r * D + e] = f32_to_bf16(v - bf16_to_f32(hi));
}

// ---------------------------------------------------------------------------------------
// launcher
// ---------------------------------------------------------------------------------------
constexpr int kLongWaves = 4;  // waves per block of k_flash_long

constexpr int kInvariantRows = 64;  // most rows of a batched decode step (see stream_shape)

// Floats the split-K partial buffer (ws.qkv) holds (the workspace is carved with the same figure).
size_t partial_floats(const st_config &c) {
    size_t rows = c.max_chunk > 1024 ? c.max_chunk : 1024;
    size_t qkv = (size_t)(c.n_q_heads + 2 * c.n_kv_heads) * c.head_dim;
    size_t cols = qkv > (size_t)c.hidden ? qkv : (size_t)c.hidden;
    size_t short_chunk = (size_t)1024 * 2 * c.intermediate;  // gate/up slices of chunks up to 256 rows
    size_t long_chunk = rows * cols + rows * cols / 4;         // one full-width slice + the extra slices of tail columns
    size_t head_rows = (size_t)kInvariantRows * c.vocab;       // LM-head GEMM of a batched step / ragged pass (one slice)
    size_t need = long_chunk > short_chunk ? long_chunk : short_chunk;
    return need > head_rows ? need : head_rows;
}

// Launches one GEMM; returns the number of K slices written to ws.qkv (0 for the fused SwiGLU form).
// Alo != nullptr selects the two-term activation form.
constexpr int kSplitRows = 256;  // most rows the weight-streaming kernel takes (eight 32-row activation tiles)

template <int BM, int BNR, int WGM, int WGN, bool DUAL, bool SPLITA>
static void gemm_launch(const Model &m, dim3 grid, const bf16_t *A, const bf16_t *Alo, int lda, const bf16_t *B, int M,
                        int N, int K, int kps, bf16_t *outb, bf16_t *outlo, int ldo, const GemmGrid &gg) {
    auto kern = k_gemm<BM, BNR, WGM, WGN, DUAL, SPLITA>;
    constexpr size_t lds = sizeof(bf16_t) * 2 * ((SPLITA ? 2 : 1) * BM + BNR) * kLdsStride;
    static_assert(lds <= 65536, "more dynamic LDS than a kernel gets without raising its limit");
    hipLaunchKernelGGL(kern, grid, dim3(64 * WGM * WGN), lds, m.stream, A, Alo, lda, B, M, N, K, kps, m.ws.qkv, outb,
                       outlo, ldo, gg);
}

template <bool DUAL, bool HALF = false>
static void ring_launch(const Model &m, bool f16, bool out_f16, dim3 grid, const bf16_t *A, const bf16_t *Alo, int lda,
                        const bf16_t *B, int M, int N, int K, bf16_t *outb, bf16_t *outlo, int ldo, const RingGrid &gg) {
    if (f16)
        hipLaunchKernelGGL((k_gemm_ring<DUAL, HALF, true>), grid, dim3(256), kRingLds, m.stream, A, Alo, lda, B, M, N, K,
                           m.ws.qkv, outb, outlo, ldo, gg, (int)out_f16);
    else
        hipLaunchKernelGGL((k_gemm_ring<DUAL, HALF, false>), grid, dim3(256), kRingLds, m.stream, A, Alo, lda, B, M, N, K,
                           m.ws.qkv, outb, outlo, ldo, gg, (int)out_f16);
}

// The ring and streaming kernels use more dynamic LDS than a kernel gets by default; the limit is raised once per
// process for every instantiation (called under std::call_once when the first model is created, so the launchers,
// which may run on several host threads, never touch it).
template <class K>
static hipError_t raise_one(K kern) {
    return hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                               kRingLds);
}
hipError_t raise_lds_limits() {
    hipError_t e = hipSuccess;
    auto take = [&](hipError_t r) {
        if (e == hipSuccess) e = r;
    };
    take(raise_one(k_gemm_ring<false, false, false>)), take(raise_one(k_gemm_ring<true, false, false>));
    take(raise_one(k_gemm_ring<true, true, false>));
    take(raise_one(k_gemm_ring<false, false, true>)), take(raise_one(k_gemm_ring<true, false, true>));
    take(raise_one(k_gemm_ring<true, true, true>));
    take(raise_one(k_gemm_stream<1, 64, true, 1, true>)), take(raise_one(k_gemm_stream<2, 64, true, 1, true>));
    take(raise_one(k_gemm_stream<3, 64, true, 1, true>)), take(raise_one(k_gemm_stream<4, 64, false, 1, true>));
    take(raise_one(k_gemm_stream<5, 64, false, 1, true>)), take(raise_one(k_gemm_stream<6, 64, false, 1, true>));
    take(raise_one(k_gemm_stream<7, 64, false, 1, true>)), take(raise_one(k_gemm_stream<8, 64, false, 1, true>));
    take(raise_one(k_gemm_stream<1, 64, true, 1, false>)), take(raise_one(k_gemm_stream<2, 64, true, 1, false>));
    take(raise_one(k_gemm_stream<3, 64, true, 1, false>)), take(raise_one(k_gemm_stream<4, 64, false, 1, false>));
    take(raise_one(k_gemm_stream<5, 64, false, 1, false>)), take(raise_one(k_gemm_stream<6, 64, false, 1, false>));
    take(raise_one(k_gemm_stream<7, 64, false, 1, false>)), take(raise_one(k_gemm_stream<8, 64, false, 1, false>));
    take(raise_one(k_gemm_stream<1, 64, true>)), take(raise_one(k_gemm_stream<2, 64, true>));
    take(raise_one(k_gemm_stream<3, 64, true>)), take(raise_one(k_gemm_stream<4, 64, false>));
    take(raise_one(k_gemm_stream<5, 32, false>)), take(raise_one(k_gemm_stream<6, 32, false>));
    take(raise_one(k_gemm_stream<7, 32, false>)), take(raise_one(k_gemm_stream<8, 32, false>));
    return e;
}

// Shape of a streaming GEMM launch: K columns per stage, weight tiles per block (4..8), K slices, ring depths.
struct StreamShape {
    int bk, nt, splits, kps, nw, na;
};

template <int MT, int BK, int TERMS = 2, bool F16 = false>
static void stream_launch(const Model &m, const StreamShape &sh, const bf16_t *A, const bf16_t *Alo, int lda,
                          const bf16_t *B, int M, int N, int K) {
    constexpr bool SPEC = MT <= 3;  // eight waves fit the register file up to three activation tiles (measured: a
                                    // few percent faster there, slower with four)
    auto kern = k_gemm_stream<MT, BK, SPEC, TERMS, F16>;
    using G = StreamGeom<BK>;
    const int lds = sh.na * MT * TERMS * G::kARows + sh.nw * sh.nt * G::kWTile;
    dim3 grid((N + 32 * sh.nt - 1) / (32 * sh.nt), sh.splits);
    hipLaunchKernelGGL(kern, grid, dim3(SPEC ? 512 : 256), lds, m.stream, A, Alo, lda, B, M, N, K, sh.kps, sh.nt, sh.nw,
                       sh.na, m.ws.qkv);
}

// One block per CU at a time, so the time is (rounds of 256 blocks) x (bytes a block loads, weights and activations
// alike, + a fixed cost per block); the partial sums written and read again are charged per CU as well.
// Up to kInvariantRows rows (the most a batched decode step holds) the K slices are those of a 16-row launch whatever
// M is, and only the tile count per block follows M: a row's sums are then formed in the same order in every batch,
// so its logits do not depend on which or how many other rows share the step.
static StreamShape stream_shape(const Model &m, int M, int N, int K, int terms = 2) {
    const int MT = (M + 31) / 32;
    const int bk = MT * terms <= 8 ? 64 : 32, seg = bk * 2, nk = K / bk;  // 128-byte row segments while the tiles fit
    const int fixed = 640 / seg;  // stages' worth of time a block spends filling its ring and storing its tile
    const size_t cap = partial_floats(m.c);
    // cheapest (tiles per block, K slices) for cost_rows rows in mt activation tiles; cap_rows rows must fit the
    // partial buffer; only_steps > 0 admits only slices of that many stages
    auto search = [&](int cost_rows, int mt, int cap_rows, int only_steps) {
        StreamShape best = {bk, 8, 1, K, 2, 2};
        double best_cost = -1;
        for (int nt = 8; nt >= 4; --nt) {
            const int tiles = (N + 32 * nt - 1) / (32 * nt);
            for (int s = 1; s <= 32; ++s) {
                const int steps = (nk + s - 1) / s;
                if (s > 1 && (steps * bk < 256 || (size_t)s * cap_rows * N > cap)) break;
                if (only_steps > 0 && steps != only_steps) continue;
                const int used = (nk + steps - 1) / steps;  // slices that are not empty
                const int rounds = (tiles * used + 255) / 256;
                const double cost = (double)rounds * (steps + fixed) * (nt * 32 + mt * 32 * terms) * seg +
                                    (double)used * cost_rows * N * 8 / 256;
                if (best_cost < 0 || cost < best_cost) {
                    best_cost = cost;
                    best.nt = nt, best.splits = used, best.kps = steps * bk;
                }
            }
        }
        return best;
    };
    StreamShape best;
    if (M <= kInvariantRows) {
        const StreamShape canon = search(16, 1, kInvariantRows, 0);
        best = search(M, MT, kInvariantRows, canon.kps / bk);
    } else {
        best = search(M, MT, M, 0);
    }
    const int a_stage = MT * 32 * terms * seg, w_stage = best.nt * 32 * seg;
    best.na = kRingLds - 3 * a_stage >= 3 * w_stage ? 3 : 2;
    int nw = (kRingLds - best.na * a_stage) / w_stage;
    const int w_loads = best.nt * 32 / (64 / (seg / 16)) / 2;  // per weight wave per stage
    if (nw > 2 + 63 / w_loads) nw = 2 + 63 / w_loads;
    best.nw = nw;
    return best;
}

// Launches of the 256 x 256 ring kernel for one GEMM of a chunk of more than kSplitRows rows: K slices, leftover
// tiles and block numbering.  Pure host arithmetic (ring_plan_check walks it without a GPU).
struct RingPlan {
    int n;             // launches: 1, or 2 for the fused form with half-width leftover tiles
    RingGrid g[2];
    bool half[2];
    int grid_x[2];
    int slices;        // full-width K slices written to the partial buffer (0 for the fused form)
    PartTail tail;     // extra slices of the tail columns
};

static RingPlan ring_plan(bool dual, int M, int N, int K, size_t cap, bool allow_tail) {
    RingPlan p{};
    RingGrid gg;
    gg.My = (M + 255) / 256;
    gg.Nx = (N + (dual ? 128 : 256) - 1) / (dual ? 128 : 256);
    gg.TY = 1;
    while (gg.TY * 2 <= gg.My && gg.TY < 8) gg.TY *= 2;
    gg.TX = 32 / gg.TY;
    gg.S = 1, gg.kps = K, gg.x0 = 0;
    gg.tail_x0 = gg.tail_tiles = 0, gg.tail_s = 1, gg.tail_kps = K;
    const int tiles = gg.My * gg.Nx, nk = K / kRingBK;
    p.n = 1;
    if (dual) {
        // Whole rounds of 256 full tiles, then the column tiles left over as half-width tiles in a launch of their
        // own: twice the blocks at half the length each, so the last round keeps every CU busy for half a round
        // instead of half the CUs for a whole one.
        if (tiles > 256 && tiles % 256 && 256 % gg.My == 0) {
            const int nx_main = tiles / 256 * 256 / gg.My;
            RingGrid th = gg;
            th.Nx = 2 * (gg.Nx - nx_main), th.x0 = 2 * nx_main;
            if (th.x0 * 64 + th.Nx * 64 > N + 63) th.Nx = (N - th.x0 * 64 + 63) / 64;  // a ragged last column tile
            th.per = (th.My * th.Nx + 7) / 8, th.blocks = 8 * th.per;
            gg.Nx = nx_main;
            p.n = 2, p.g[1] = th, p.half[1] = true, p.grid_x[1] = th.blocks;
        }
    } else {
        // One block per CU at a time: pick the K slices that minimise (rounds of 256 blocks) x (K steps per
        // slice + a fixed cost for filling the ring and writing the tile)
        // Short passes (one or two row tiles) have few tiles, so they may take up to 16 slices; there the partial
        // sums every slice writes and the consumer reads again (8 bytes per element at ~4 TB/s, in units of a
        // 1.4 us K step) are part of the price.
        long best = -1;
        const int max_s = M <= 512 ? 16 : 8;
        const double slice_steps = M <= 512 ? (double)M * N * 8 / 4e12 / 1.4e-6 : 0.0;
        for (int s = 1; s <= max_s; ++s) {
            const int steps = (nk + s - 1) / s;
            if (steps < 4 && s > 1) break;
            if (s > 1 && (size_t)s * M * N > cap) break;
            const long cost = (long)((tiles * s + 255) / 256) * (steps + 6) + (long)(s * slice_steps);
            if (best < 0 || cost < best) best = cost, gg.S = s;
        }
        gg.kps = (nk + gg.S - 1) / gg.S * kRingBK;
        gg.S = (K + gg.kps - 1) / gg.kps;
        if (K - (gg.S - 1) * gg.kps < 2 * kRingBK) gg.S = 1, gg.kps = K;  // a last slice of one step: do not split
        // Or: whole rounds of 256 tiles at full K, and only the column tiles left over cut into K slices (a
        // consumer that takes a PartTail adds their extra slices).  320 tiles with K = 432 steps: three rounds of
        // half the K range each become one round at full K plus one round of quarter slices.
        if (allow_tail && tiles > 256 && tiles % 256 && 256 % gg.My == 0) {
            const int nx_main = tiles / 256 * 256 / gg.My, tail_tiles = (gg.Nx - nx_main) * gg.My;
            const int ld = N - nx_main * 256;
            long tbest = -1;
            int ts = 1;
            for (int s = 1; s <= 8; ++s) {
                const int steps = (nk + s - 1) / s;
                if (s > 1 && (steps < 4 || nk - (s - 1) * steps < 2)) break;
                if ((size_t)M * N + (size_t)(s - 1) * M * ld > cap) break;
                const long cost = (long)((tail_tiles * s + 255) / 256) * (steps + 6);
                if (tbest < 0 || cost < tbest) tbest = cost, ts = s;
            }
            if ((long)(tiles / 256) * (nk + 6) + tbest < best) {
                gg.tail_x0 = nx_main, gg.tail_tiles = tail_tiles, gg.tail_s = ts;
                gg.tail_kps = (nk + ts - 1) / ts * kRingBK;
                gg.Nx = nx_main, gg.S = 1, gg.kps = K;  // the main part: the first nx_main column tiles at full K
                p.tail = PartTail{nx_main * 256, ts - 1, ld, (long long)M * N, (long long)M * ld};
            }
        }
        p.slices = gg.S;
    }
    gg.per = (gg.S * gg.My * gg.Nx + 7) / 8;
    gg.blocks = 8 * gg.per;
    const int tail_units = (gg.tail_tiles + 31) / 32 * gg.tail_s;
    p.g[0] = gg, p.half[0] = false, p.grid_x[0] = gg.blocks + (tail_units + 7) / 8 * 256;
    return p;
}

// Alo != nullptr: two-term activations, the plan covers the doubled contraction [A | Alo] x [B | B].
template <bool DUAL>
static int ring_gemm(const Model &m, bool f16, bool out_f16, const bf16_t *A, const bf16_t *Alo, int lda, const bf16_t *B,
                     int M, int N, int K, bf16_t *outb, bf16_t *outlo, int ldo, PartTail *tail) {
    const RingPlan p = ring_plan(DUAL, M, N, Alo ? 2 * K : K, partial_floats(m.c), tail != nullptr);
    ring_launch<DUAL, false>(m, f16, out_f16, dim3(p.grid_x[0]), A, Alo, lda, B, M, N, K, outb, outlo, ldo, p.g[0]);
    if constexpr (DUAL)
        if (p.n == 2)
            ring_launch<true, true>(m, f16, out_f16, dim3(p.grid_x[1]), A, Alo, lda, B, M, N, K, outb, outlo, ldo,
                                    p.g[1]);
    if (tail) *tail = p.tail;
    return p.slices;
}

// Walks every block id of the plan on the host: 0 if each (output tile, 64-column K step) of the GEMM is covered by
// exactly one block, every block has at least two K steps, and (plain form) every partial-sum tile lies inside
// cap_floats; a negative code names the first failure.  blocks_out: working blocks, ids_out: ids launched.
int ring_plan_check(int dual, int M, int N, int K, long long cap_floats, int allow_tail, int *launches_out,
                    int *blocks_out, int *ids_out) {
    if (M <= 0 || N <= 0 || K < 2 * kRingBK || K % kRingBK) return -1;
    const RingPlan p = ring_plan(dual != 0, M, N, K, (size_t)cap_floats, allow_tail != 0);
    const int nk = K / kRingBK, my = (M + 255) / 256;
    const int out_cols = dual ? 64 : 256;  // count output columns in units every tile width is a multiple of
    const int ncu = (N + out_cols - 1) / out_cols;
    std::vector<unsigned char> seen((size_t)my * ncu * nk, 0);
    int working = 0, ids = 0;
    for (int l = 0; l < p.n; ++l) {
        const int width = p.half[l] ? 64 : dual ? 128 : 256, per_tile = width / out_cols;
        ids += p.grid_x[l];
        for (int bid = 0; bid < p.grid_x[l]; ++bid) {
            RingBlock rb;
            if (!ring_block(p.g[l], bid, M, N, K, &rb)) continue;
            ++working;
            const int n0 = (rb.x + p.g[l].x0) * width;
            if (rb.y < 0 || rb.y >= my || n0 < 0 || n0 >= N) return -2;
            if (rb.kbeg < 0 || rb.kend > K || (rb.kend - rb.kbeg) % kRingBK || rb.kend - rb.kbeg < 2 * kRingBK) return -3;
            for (int c = 0; c < per_tile; ++c) {
                const int cu = n0 / out_cols + c;
                if (cu >= ncu) break;  // the ragged part of a last tile
                for (int ks = rb.kbeg / kRingBK; ks < rb.kend / kRingBK; ++ks) {
                    unsigned char &cell = seen[((size_t)rb.y * ncu + cu) * nk + ks];
                    if (cell) return -4;
                    cell = 1;
                }
            }
            if (!dual) {
                const int rows = (rb.y * 256 + 256 < M ? rb.y * 256 + 256 : M), cols = (n0 + 256 < N ? n0 + 256 : N);
                const long long lo = rb.part_off + (long long)rb.y * 256 * rb.ldp + n0;
                const long long hi = rb.part_off + (long long)(rows - 1) * rb.ldp + cols - 1;
                if (lo < 0 || hi >= cap_floats) return -5;
                if (rb.part_off > 0 && p.tail.n > 0 && rb.ldp != N &&
                    hi >= p.tail.base + (long long)p.tail.n * p.tail.stride)
                    return -6;
            }
        }
    }
    for (unsigned char c : seen)
        if (!c) return -7;
    if (launches_out) *launches_out = p.n;
    if (blocks_out) *blocks_out = working;
    if (ids_out) *ids_out = ids;
    return 0;
}

// Chunks below the model's ring threshold (two-term, at most kSplitRows rows) use the streaming kernel and an unfused
// SwiGLU wherever K is a multiple of 64; otherwise the register-staged kernel, with many K slices and an unfused
// SwiGLU up to kSmallRows rows.
constexpr int kSmallRows = 64;

// f16: the operands hold fp16 numbers (only the ring kernel has that form: the caller has made sure this GEMM takes it).
template <bool DUAL>
static int gemm(const Model &m, const bf16_t *A, const bf16_t *Alo, int lda, const bf16_t *B, int M, int N, int K,
                bf16_t *outb, bf16_t *outlo, int ldo, PartTail *tail = nullptr, bool f16 = false, bool out_f16 = false) {
    if (tail) *tail = PartTail{};
    // (the ring kernel addresses its operands with 32-bit byte offsets)
    const bool fits32 = (size_t)M * lda * sizeof(bf16_t) < ((size_t)1 << 32) &&
                        (size_t)(DUAL ? 2 : 1) * N * K * sizeof(bf16_t) < ((size_t)1 << 32);
    const bool big = M >= m.ring_min_rows && K % kRingBK == 0 && K >= 2 * kRingBK && fits32;
    if (!big && !DUAL && !Alo && M <= kSplitRows && K % kRingBK == 0) {
        // one activation term below the ring threshold: fp16 operands, or single bf16 (ST_PREFILL_FAST)
        const StreamShape sh = stream_shape(m, M, N, K, 1);
#define ST_STREAM1(MTV)                                                                   \
    case MTV:                                                                             \
        if (f16)                                                                          \
            stream_launch<MTV, 64, 1, true>(m, sh, A, nullptr, lda, B, M, N, K);          \
        else                                                                              \
            stream_launch<MTV, 64, 1, false>(m, sh, A, nullptr, lda, B, M, N, K);         \
        break;
        switch ((M + 31) / 32) {
            ST_STREAM1(1) ST_STREAM1(2) ST_STREAM1(3) ST_STREAM1(4) ST_STREAM1(5) ST_STREAM1(6) ST_STREAM1(7)
            default: ST_STREAM1(8)
        }
#undef ST_STREAM1
        return sh.splits;
    }
    if (!big && !DUAL && Alo && M <= kSplitRows && K % kRingBK == 0) {
        const StreamShape sh = stream_shape(m, M, N, K);
        switch ((M + 31) / 32) {
            case 1: stream_launch<1, 64>(m, sh, A, Alo, lda, B, M, N, K); break;
            case 2: stream_launch<2, 64>(m, sh, A, Alo, lda, B, M, N, K); break;
            case 3: stream_launch<3, 64>(m, sh, A, Alo, lda, B, M, N, K); break;
            case 4: stream_launch<4, 64>(m, sh, A, Alo, lda, B, M, N, K); break;
            case 5: stream_launch<5, 32>(m, sh, A, Alo, lda, B, M, N, K); break;
            case 6: stream_launch<6, 32>(m, sh, A, Alo, lda, B, M, N, K); break;
            case 7: stream_launch<7, 32>(m, sh, A, Alo, lda, B, M, N, K); break;
            default: stream_launch<8, 32>(m, sh, A, Alo, lda, B, M, N, K); break;
        }
        return sh.splits;
    }
    if (big) return ring_gemm<DUAL>(m, f16, out_f16, A, Alo, lda, B, M, N, K, outb, outlo, ldo, tail);
    // (K not a multiple of 64) two-term chunks of at most 32 / 64 rows use 32- / 64-row tiles with two waves: less
    // LDS per block, so more blocks per CU keep more of the weight stream in flight
    const int BM = (Alo && M <= 32) ? 32 : (Alo && M <= 64) ? 64 : 128;
    const int BNO = 128 / (DUAL ? 2 : 1);
    GemmGrid gg;
    gg.My = (M + BM - 1) / BM;
    gg.Nx = (N + BNO - 1) / BNO;
    gg.TY = 1;
    while (gg.TY * 2 <= gg.My && gg.TY < 8) gg.TY *= 2;
    gg.TX = 32 / gg.TY;
    gg.YB = (gg.My + gg.TY - 1) / gg.TY;
    const int nxl = (gg.Nx + 7) / 8, xb = (nxl + gg.TX - 1) / gg.TX;
    gg.blocks = 8 * xb * gg.YB * 32;
    int splits = 1, kps = K;
    const int tiles = gg.My * gg.Nx;
    const size_t cap = partial_floats(m.c);
    if (!DUAL) {
        // K slices: enough blocks to keep every CU streaming weights (the small tiles have two waves
        // each, so they need more of them), bounded by the partial-result buffer
        const bool small = BM <= 64;
        const int want = small ? 2048 : 640;
        splits = (want + tiles - 1) / tiles;
        if (splits > (small ? 32 : 8)) splits = small ? 32 : 8;
        while (splits > 1 && (size_t)splits * M * N > cap) --splits;
        kps = ((K + splits - 1) / splits + kBK - 1) / kBK * kBK;
        if (kps < 256) kps = 256;
        splits = (K + kps - 1) / kps;
    }
    dim3 grid(gg.blocks, splits);
    if (Alo && BM == 32)
        gemm_launch<32, 128, 1, 2, DUAL, true>(m, grid, A, Alo, lda, B, M, N, K, kps, outb, outlo, ldo, gg);
    else if (Alo && BM == 64)
        gemm_launch<64, 128, 1, 2, DUAL, true>(m, grid, A, Alo, lda, B, M, N, K, kps, outb, outlo, ldo, gg);
    else if (Alo)
        gemm_launch<128, 128, 2, 2, DUAL, true>(m, grid, A, Alo, lda, B, M, N, K, kps, outb, outlo, ldo, gg);
    else
        gemm_launch<128, 128, 2, 2, DUAL, false>(m, grid, A, Alo, lda, B, M, N, K, kps, outb, outlo, ldo, gg);
    return DUAL ? 0 : splits;
}

// Which GEMM and attention inputs of a pass over n rows carry a second bf16 term (x = hi + lo, 16 mantissa bits).
// By default all of them, at every pass length: the pass then rounds nothing the decode step does not round either
// (only the bf16 K/V cache is left), and measured against the CPU oracle its logit error is the decode step's at
// every depth tried.  Up to kSplitRows rows the second term is free (the weight stream sets the time); longer
// passes are MFMA-bound and pay twice the MFMA work.  m.long_terms == 0 (ST_PREFILL_FAST) drops the second terms
// of those longer passes: single bf16 inputs, about 1.8x faster, about twice the logit error.
struct PassTerms {
    bf16_t *xn_lo, *attn_lo, *act_lo, *qb_lo;  // where the producers write the low terms (nullptr: not needed)
    bool qkv_two, gu_two;                      // xn_lo feeds the QKV / the gate-up projection
    // fp16 operand mode: the inputs of the gate/up, O and down projections (normalised rows of the MLP block,
    // attention output, SwiGLU output) are single fp16 numbers multiplied with the model's fp16 weights
    bool f16_xg, f16_attn, f16_act;
};
static PassTerms pass_terms(const Model &m, int n) {
    const Workspace &w = m.ws;
    int terms = n <= 128 ? kTermAll : m.long_terms;  // up to 128 rows the second term is free in every mode
    PassTerms t;
    // Default-precision passes of a model that has its fp16 weight copy: at every pass length the inputs of the
    // gate/up, O and down projections are single fp16 numbers.  The input of the QKV projection and the queries keep
    // two bf16 terms: what reaches the attention logits is exponentiated, and through 64 layers of the 32B shape a
    // pass with fp16 QKV inputs ended 2.1-2.5e-2 from the decode step where this form ends 1.3-1.6e-2, the same as
    // two bf16 terms everywhere (fp16 in any of the other three inputs made no difference), for 5 % of the time.
    t.f16_xg = t.f16_attn = t.f16_act = m.f16_pass;
    if (t.f16_xg) terms &= ~kTermGateUp;
    if (t.f16_attn) terms &= ~kTermO;
    if (t.f16_act) terms &= ~kTermDown;
    t.qkv_two = terms & kTermQKV, t.gu_two = terms & kTermGateUp;
    t.xn_lo = (t.qkv_two || t.gu_two) ? w.xn_lo : nullptr;
    t.attn_lo = terms & kTermO ? w.attn_lo : nullptr;
    t.act_lo = terms & kTermDown ? w.act_lo : nullptr;
    t.qb_lo = (terms & kTermQuery) && m.c.head_dim == 128 ? w.qb_lo : nullptr;  // rotated queries (k_flash_long)
    return t;
}

// ---------------------------------------------------------------------------------------
// fp16 copy of the projection weights (st_model_attach_f16).  A bf16 number of magnitude in [2^-16, 65504] is an
// fp16 number too (8 significant bits fit the 11 of a half; below 2^-14 the half is subnormal with spacing 2^-24),
// smaller ones round to a multiple of 2^-24 (absolute error <= 3e-8), larger ones or NaNs are counted in *bad.
// ---------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_bf16_to_f16(const bf16_t *__restrict__ src, bf16_t *__restrict__ dst, size_t n8,
                                                     int32_t *__restrict__ bad) {
    int n_bad = 0;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n8; i += (size_t)gridDim.x * 256) {
        const u32x4 v = reinterpret_cast<const u32x4 *>(src)[i];
        const float f[8] = {bf16_lo(v.x), bf16_hi(v.x), bf16_lo(v.y), bf16_hi(v.y),
                            bf16_lo(v.z), bf16_hi(v.z), bf16_lo(v.w), bf16_hi(v.w)};
#pragma unroll
        for (int e = 0; e < 8; ++e) n_bad += !(fabsf(f[e]) <= 65504.f);  // too large for a half, or NaN
        const u32x4 o = {pack_f16x2(f[0], f[1]), pack_f16x2(f[2], f[3]), pack_f16x2(f[4], f[5]), pack_f16x2(f[6], f[7])};
        reinterpret_cast<u32x4 *>(dst)[i] = o;
    }
    if (n_bad) atomicAdd(bad, n_bad);
}
void launch_f16_copy(const Model &m, const bf16_t *src, bf16_t *dst, size_t n, int32_t *bad) {
    const size_t n8 = n / 8;  // every projection matrix has a multiple of 8 elements (K is a multiple of 64)
    int blocks = (int)((n8 + 255) / 256 < 4096 ? (n8 + 255) / 256 : 4096);
    hipLaunchKernelGGL(k_bf16_to_f16, dim3(blocks), dim3(256), 0, m.stream, src, dst, n8, bad);
}
// The fp16 operand mode runs only in the ring kernel: every projection's K must suit it and its 32-bit offsets.
bool f16_shape_ok(const st_config &c) {
    const size_t h = c.hidden, qd = (size_t)c.n_q_heads * c.head_dim, I = c.intermediate;
    const size_t qkv = (size_t)(c.n_q_heads + 2 * c.n_kv_heads) * c.head_dim, mc = c.max_chunk, lim = (size_t)1 << 32;
    for (size_t K : {h, qd, I})
        if (K % kRingBK || K < 2 * kRingBK || mc * K * sizeof(bf16_t) >= lim) return false;
    return qkv * h * 2 < lim && h * qd * 2 < lim && 2 * I * h * 2 < lim && h * I * 2 < lim;
}

int flash_row_blocks(const st_config &c, int len) {
    const int G = c.n_q_heads / c.n_kv_heads;
    return (len * G + 127) / 128;  // both attention kernels take 128 folded rows per block
}

// Causal attention of n query rows at positions pos0 .. pos0+n-1 over one sequence's cache (kc / vc of one layer) --
// or, with `ragged`, of the R rows of several sequences in one launch (kc / vc are then sequence 0's caches).
struct RaggedPass {
    const FlashSeg *segs_dev;  // device table, n_seg entries
    int n_seg, R, total_blocks, max_tiles;
    size_t seq_stride;
};
static void launch_flash(const Model &m, const bf16_t *qb, const bf16_t *qb_lo, const bf16_t *kc, const bf16_t *vc,
                         bf16_t *attn, bf16_t *attn_lo, int n, int pos0, const RaggedPass *ragged = nullptr,
                         bool f16_out = false) {
    const st_config &c = m.c;
    const int d = c.head_dim, nq = c.n_q_heads, nkv = c.n_kv_heads;
    const Workspace &w = m.ws;
    const bool long_chunk = d == 128;  // head_dim 128: k_flash_long at every chunk length
    const int G = nq / nkv;
    const int rblocks = ragged ? ragged->total_blocks : flash_row_blocks(c, n);
    const int n_tiles = ragged ? ragged->max_tiles : (pos0 + n + kFlashKeys - 1) / kFlashKeys;
    const int n_rows_all = ragged ? ragged->R : n;  // rows the partial buffers are sized for
    // key splits: enough blocks for every CU, bounded by the tiles and by the partial buffer
    int splits = (512 + rblocks * nkv - 1) / (rblocks * nkv);
    if (splits > n_tiles) splits = n_tiles;
    if (splits > 32) splits = 32;
    const size_t cap = partial_floats(c);
    if (long_chunk && !ragged) {
        // k_flash_long: the count that minimises (rounds of resident blocks) x (tiles per block + 2 for the set-up
        // and the store) x the time of a tile step, plus the merge pass over the partial results (its bytes at
        // 4 TB/s + a launch).  640 blocks of 42 tiles on 512 slots are two rounds; 960 blocks of 27 are two shorter ones.
        const int slots = 512;                      // two blocks per CU
        const double step_us = qb_lo ? 2.2 : 1.7;   // a tile step with / without the second term of the queries
        double best = -1;
        // (from two rounds of blocks on, the causal spread of their lengths, longest first, balances the CUs
        // better than splitting does, and the merge pass would cost more than it saves: measured at 4096 rows)
        const int sp_max = rblocks * nkv >= 2 * slots ? 1 : (n_tiles < 32 ? n_tiles : 32);
        for (int sp = 1; sp <= sp_max; ++sp) {
            if (sp > 1 && (size_t)sp * n * nq * (d + 2) > cap) break;
            const int tps = (n_tiles + sp - 1) / sp, used = (n_tiles + tps - 1) / tps;
            if (used != sp) continue;  // the same blocks as a smaller count
            const int rounds = (rblocks * nkv * sp + slots - 1) / slots;
            const double merge = sp > 1 ? 3.0 + (double)n * nq * d * 4 * (sp + 1) / 4e6 : 0.0;
            const double cost = rounds * (tps + 2) * step_us + merge;
            if (best < 0 || cost < best) best = cost, splits = sp;
        }
    }
    while (splits > 1 && (size_t)splits * n_rows_all * nq * (d + 2) > cap) --splits;
    float *part_o = w.qkv, *part_ml = w.qkv + (size_t)splits * n_rows_all * nq * d;
    dim3 fgrid(rblocks, nkv, splits);
    const FlashSeg *segs = ragged ? ragged->segs_dev : nullptr;
    const int n_seg = ragged ? ragged->n_seg : 0;
    const size_t seq_stride = ragged ? ragged->seq_stride : 0;
    if (long_chunk && qb_lo)
        hipLaunchKernelGGL((k_flash_long<kLongWaves, true>), fgrid, dim3(64 * kLongWaves), 0, m.stream, qb, qb_lo, kc, vc,
                           attn, attn_lo, part_o, part_ml, n, pos0, nq, G, c.max_seq, segs, n_seg, seq_stride, n_rows_all,
                           (int)f16_out);
    else if (long_chunk)
        hipLaunchKernelGGL((k_flash_long<kLongWaves, false>), fgrid, dim3(64 * kLongWaves), 0, m.stream, qb, qb_lo, kc, vc,
                           attn, attn_lo, part_o, part_ml, n, pos0, nq, G, c.max_seq, segs, n_seg, seq_stride, n_rows_all,
                           (int)f16_out);
    else
        hipLaunchKernelGGL(k_flash_prefill<64>, fgrid, dim3(256), 0, m.stream, qb, kc, vc, attn, attn_lo, part_o,
                           part_ml, n, pos0, nq, G, c.max_seq, segs, n_seg, seq_stride, n_rows_all, (int)f16_out);
    if (splits > 1) {
        const int n_rows = n_rows_all * nq;
        if (d == 128)
            hipLaunchKernelGGL(k_flash_combine<128>, dim3((n_rows + 1) / 2), dim3(256), 0, m.stream, part_o, part_ml,
                               splits, n_rows, attn, attn_lo, (int)f16_out);
        else
            hipLaunchKernelGGL(k_flash_combine<64>, dim3((n_rows + 3) / 4), dim3(256), 0, m.stream, part_o, part_ml,
                               splits, n_rows, attn, attn_lo, (int)f16_out);
    }
}

void launch_prefill_layers(const Model &m, int32_t pos0, int32_t n) {
    const st_config &c = m.c;
    const int h = c.hidden, d = c.head_dim, nq = c.n_q_heads, nkv = c.n_kv_heads, I = c.intermediate;
    const int qd = nq * d, qkv = m.qkv_dim;
    const Workspace &w = m.ws;
    const PassTerms t = pass_terms(m, n);
    bf16_t *xn_lo = t.xn_lo, *attn_lo = t.attn_lo, *act_lo = t.act_lo, *qb_lo = t.qb_lo;
    hipLaunchKernelGGL(k_embed_rows, dim3(n), dim3(256), 0, m.stream, m.embed, w.tokens, w.x, h, c.vocab);
    hipLaunchKernelGGL(k_note_fed, dim3(1), dim3(1), 0, m.stream, w.state, w.tokens, n - 1, c.vocab);
    int pending = 0;  // K slices of the previous layer's down projection still to be added to x
    PartTail pend_tail{}, tq{}, to{};  // extra slices of the tail columns (long chunks only)
    for (int l = 0; l < c.n_layers; ++l) {
        size_t lofs = (size_t)l * nkv * c.max_seq * d;
        hipLaunchKernelGGL(k_rmsnorm_rows, dim3(n), dim3(norm_threads(n)), 0, m.stream, w.x, w.qkv, pending, (size_t)n * h,
                           m.norm_attn[l], w.xn, t.qkv_two ? xn_lo : nullptr, h, c.rms_eps, pend_tail, 0);
        int sq = gemm<false>(m, w.xn, t.qkv_two ? xn_lo : nullptr, h, m.wqkv[l], n, qkv, h, nullptr, nullptr, 0, &tq);
        hipLaunchKernelGGL(k_rope_append, dim3(n, ((nq + 2 * nkv) * (d / 8) + 255) / 256), dim3(256), 0, m.stream,
                           w.qkv, sq,
                           (size_t)n * qkv, m.bqkv[l], w.rope, w.qb, qb_lo, m.kcache + lofs, m.vcache + lofs, pos0, nq, nkv,
                           d, c.max_seq, tq);
        launch_flash(m, w.qb, qb_lo, m.kcache + lofs, m.vcache + lofs, w.attn, attn_lo, n, pos0, nullptr, t.f16_attn);
        int so = gemm<false>(m, w.attn, attn_lo, qd, t.f16_attn ? m.wo16[l] : m.wo[l], n, h, qd, nullptr, nullptr, 0, &to,
                             t.f16_attn);
        hipLaunchKernelGGL(k_rmsnorm_rows, dim3(n), dim3(norm_threads(n)), 0, m.stream, w.x, w.qkv, so, (size_t)n * h,
                           m.norm_mlp[l], w.xn, t.f16_xg ? nullptr : xn_lo, h, c.rms_eps, to, (int)t.f16_xg);
        if (n < (h % kRingBK == 0 ? m.ring_min_rows : kSmallRows + 1)) {  // small chunk: gate/up as a plain split-K
                                                                           // GEMM over all 2I rows, SwiGLU in the consumer
            int sg = gemm<false>(m, w.xn, t.f16_xg ? nullptr : xn_lo, h, t.f16_xg ? m.wgu16[l] : m.wgu[l], n, 2 * I, h,
                                 nullptr, nullptr, 0, nullptr, t.f16_xg);
            hipLaunchKernelGGL(k_swiglu_rows, dim3((I / 4 + 255) / 256, n), dim3(256), 0, m.stream, w.qkv, sg,
                               (size_t)n * 2 * I, I, w.act, w.act_lo, (int)t.f16_act);
        } else {
            gemm<true>(m, w.xn, t.gu_two ? xn_lo : nullptr, h, t.f16_xg ? m.wgu16[l] : m.wgu[l], n, I, h, w.act, act_lo, I,
                       nullptr, t.f16_xg, t.f16_act);
        }
        pending = gemm<false>(m, w.act, act_lo, I, t.f16_act ? m.wdown16[l] : m.wdown[l], n, h, I, nullptr, nullptr, 0,
                              &pend_tail, t.f16_act);
    }
    // the head needs the last row only: fold the last down projection into it
    hipLaunchKernelGGL(k_rmsnorm_rows, dim3(1), dim3(norm_threads(1)), 0, m.stream, w.x + (size_t)(n - 1) * h,
                       w.qkv + (size_t)(n - 1) * h, pending, (size_t)n * h, nullptr, nullptr, nullptr, h, c.rms_eps,
                       tail_at_row(pend_tail, n - 1, h), 0);
}

// ---------------------------------------------------------------------------------------
// One decode step for a batch of independent sequences sharing the weights (the "many sequences at once" regime):
// the rows of the step are different sequences at their own positions, so the projections are the short-chunk
// GEMMs above (the weights are streamed once for all rows), RoPE / KV append go row by row to each sequence's
// cache, attention is the split decode attention with one grid plane per row, and the LM head is one more GEMM
// followed by a per-row arg-max.
// ---------------------------------------------------------------------------------------
// RoPE at each row's own position, K/V appended to each row's own cache; q kept in fp32 (decode rows, as in the
// single step) or, with qb != nullptr, written as bf16 (catch-up rows).
__global__ void k_rope_append_rows(const float *__restrict__ part, int n_part, size_t part_stride,
                                   const bf16_t *__restrict__ bias, const float2 *__restrict__ rope,
                                   float *__restrict__ q_rows, bf16_t *__restrict__ qb, bf16_t *__restrict__ qb_lo,
                                   bf16_t *__restrict__ kc,
                                   bf16_t *__restrict__ vc, const int32_t *__restrict__ row_pos,
                                   const int32_t *__restrict__ row_seq,
                                   size_t seq_stride, int nq, int nkv, int d, int max_seq) {
    const int row = blockIdx.x, head = blockIdx.y, i = threadIdx.x, half = d >> 1;
    const int pos = row_pos[row];
    const size_t cache = (size_t)row_seq[row] * seq_stride;
    const size_t off = (size_t)row * (nq + 2 * nkv) * d + head * d;
    float lo = 0.f, hi = 0.f;
    for (int s = 0; s < n_part; ++s) {
        const float *src = part + (size_t)s * part_stride + off;
        lo += src[i];
        hi += src[i + half];
    }
    if (bias) {
        lo += bf16_to_f32(bias[head * d + i]);
        hi += bf16_to_f32(bias[head * d + i + half]);
    }
    if (head < nq + nkv) {
        float2 cs = rope[(size_t)pos * half + i];
        float nlo = lo * cs.x - hi * cs.y;
        float nhi = hi * cs.x + lo * cs.y;
        lo = nlo;
        hi = nhi;
    }
    if (head < nq) {
        if (qb) {  // catch-up rows: bf16 queries for the flash kernels
            bf16_t *dq = qb + (size_t)row * nq * d + head * d;
            const bf16_t blo = f32_to_bf16(lo), bhi = f32_to_bf16(hi);
            dq[i] = blo;
            dq[i + half] = bhi;
            if (qb_lo) {
                bf16_t *dl = qb_lo + (size_t)row * nq * d + head * d;
                dl[i] = f32_to_bf16(lo - bf16_to_f32(blo));
                dl[i + half] = f32_to_bf16(hi - bf16_to_f32(bhi));
            }
        } else {
            float *dst = q_rows + (size_t)row * nq * d + head * d;
            dst[i] = lo;
            dst[i + half] = hi;
        }
        return;
    }
    bf16_t *dst = head < nq + nkv ? kc + cache + ((size_t)(head - nq) * max_seq + pos) * d
                                  : vc + cache + ((size_t)(head - nq - nkv) * max_seq + pos) * d;
    dst[i] = f32_to_bf16(lo);
    dst[i + half] = f32_to_bf16(hi);
}

// Row r: logits[r][:] = sum of the K slices (also stored when logits != nullptr), next[r] = arg-max, lowest id on ties.
// Two passes: grid (rows, kArgSegs) blocks each reduce one segment of a row to a (value, id) pair, then one wave per
// row picks among the pairs (one 1024-thread block per row walked 152064 columns in 148 dependent steps: 127 us).
constexpr int kArgSegs = 16;  // rows * kArgSegs pairs must fit the kLmBlocks-entry scratch arrays (rows <= 64)
static_assert(64 * kArgSegs <= kLmBlocks, "the per-segment arg-max pairs use the LM head's scratch arrays");
__device__ __forceinline__ void argmax_take(float &best, int &arg, float v, int id) {
    if (v > best || (v == best && id < arg)) best = v, arg = id;
}
__global__ __launch_bounds__(256) void k_argmax_rows_part(const float *__restrict__ part, int n_part, size_t part_stride,
                                                          int V, bool vec4, float *__restrict__ logits,
                                                          float *__restrict__ pv, int32_t *__restrict__ pi) {
    __shared__ float bv[4];
    __shared__ int bi[4];
    const int row = blockIdx.x, seg = blockIdx.y, lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int per = ((V + kArgSegs - 1) / kArgSegs + 3) & ~3;  // columns per segment, a multiple of four
    const int v0 = seg * per, v1 = min(V, v0 + per);
    const float *p = part + (size_t)row * V;
    float best = -INFINITY;
    int arg = 0x7fffffff;
    if (vec4) {
        for (int v = v0 + 4 * threadIdx.x; v < v1; v += 1024) {
            float4 a = *reinterpret_cast<const float4 *>(p + v);
            for (int s = 1; s < n_part; ++s) {
                const float4 q = *reinterpret_cast<const float4 *>(p + (size_t)s * part_stride + v);
                a.x += q.x, a.y += q.y, a.z += q.z, a.w += q.w;
            }
            if (logits) *reinterpret_cast<float4 *>(logits + (size_t)row * V + v) = a;
            argmax_take(best, arg, a.x, v), argmax_take(best, arg, a.y, v + 1);
            argmax_take(best, arg, a.z, v + 2), argmax_take(best, arg, a.w, v + 3);
        }
    } else {
        for (int v = v0 + threadIdx.x; v < v1; v += 256) {
            float a = 0.f;
            for (int s = 0; s < n_part; ++s) a += p[(size_t)s * part_stride + v];
            if (logits) logits[(size_t)row * V + v] = a;
            argmax_take(best, arg, a, v);
        }
    }
    for (int o = 32; o > 0; o >>= 1) argmax_take(best, arg, __shfl_xor(best, o, kWave), __shfl_xor(arg, o, kWave));
    if (lane == 0) bv[wave] = best, bi[wave] = arg;
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int w = 1; w < 4; ++w) argmax_take(best, arg, bv[w], bi[w]);
        pv[row * kArgSegs + seg] = best, pi[row * kArgSegs + seg] = arg;
    }
}
__global__ __launch_bounds__(64) void k_argmax_rows_final(const float *__restrict__ pv, const int32_t *__restrict__ pi,
                                                          int V, int32_t *__restrict__ next) {
    const int row = blockIdx.x, lane = threadIdx.x;
    float best = lane < kArgSegs ? pv[row * kArgSegs + lane] : -INFINITY;
    int arg = lane < kArgSegs ? pi[row * kArgSegs + lane] : 0x7fffffff;
    for (int o = 32; o > 0; o >>= 1) argmax_take(best, arg, __shfl_xor(best, o, kWave), __shfl_xor(arg, o, kWave));
    if (lane == 0) next[row] = arg < V ? arg : 0;  // a row of NaNs compares false everywhere: keep the id in range
}
static void launch_argmax_rows(const Model &m, int rows, int n_part, float *logits, int32_t *next) {
    const int V = m.c.vocab;
    const bool vec4 = (V & 3) == 0 && ((uintptr_t)logits & 15) == 0;  // 16-byte accesses need both
    hipLaunchKernelGGL(k_argmax_rows_part, dim3(rows, kArgSegs), dim3(256), 0, m.stream, m.ws.qkv, n_part,
                       (size_t)rows * V, V, vec4, logits, m.ws.amax_val, m.ws.amax_idx);
    hipLaunchKernelGGL(k_argmax_rows_final, dim3(rows), dim3(64), 0, m.stream, m.ws.amax_val, m.ws.amax_idx, V, next);
}

void launch_batch_step(const Model &m, const BatchRows &b, int n, int attn_blocks) {
    const st_config &c = m.c;
    const int h = c.hidden, d = c.head_dim, nq = c.n_q_heads, nkv = c.n_kv_heads, I = c.intermediate;
    const int qd = nq * d, qkv = m.qkv_dim;
    const Workspace &w = m.ws;
    const AttnRows rows = {b.row_pos, b.row_seq, b.seq_stride, qd, (size_t)nq * kAttnSplits * 2,
                           (size_t)nq * kAttnSplits * d, w.attn, w.attn_lo};  // result straight into the O GEMM's input
    hipLaunchKernelGGL(k_embed_rows, dim3(n), dim3(256), 0, m.stream, m.embed, b.row_tok, w.x, h, c.vocab);
    int pending = 0;
    for (int l = 0; l < c.n_layers; ++l) {
        const size_t lofs = (size_t)l * nkv * c.max_seq * d;
        hipLaunchKernelGGL(k_rmsnorm_rows, dim3(n), dim3(norm_threads(n)), 0, m.stream, w.x, w.qkv, pending, (size_t)n * h,
                           m.norm_attn[l], w.xn, w.xn_lo, h, c.rms_eps, PartTail{}, 0);
        const int sq = gemm<false>(m, w.xn, w.xn_lo, h, m.wqkv[l], n, qkv, h, nullptr, nullptr, 0);
        hipLaunchKernelGGL(k_rope_append_rows, dim3(n, nq + 2 * nkv), dim3(d / 2), 0, m.stream, w.qkv, sq,
                           (size_t)n * qkv, m.bqkv[l], w.rope, b.q_rows, (bf16_t *)nullptr, (bf16_t *)nullptr,
                           m.kcache + lofs, m.vcache + lofs, b.row_pos, b.row_seq, b.seq_stride, nq, nkv, d, c.max_seq);
        launch_attn_rows(m, l, m.stream, attn_blocks, rows, n, b.q_rows, b.part_ml, b.part_acc, b.o_rows);
        const int so = gemm<false>(m, w.attn, w.attn_lo, qd, m.wo[l], n, h, qd, nullptr, nullptr, 0);
        hipLaunchKernelGGL(k_rmsnorm_rows, dim3(n), dim3(norm_threads(n)), 0, m.stream, w.x, w.qkv, so, (size_t)n * h,
                           m.norm_mlp[l], w.xn, w.xn_lo, h, c.rms_eps, PartTail{}, 0);
        const int sg = gemm<false>(m, w.xn, w.xn_lo, h, m.wgu[l], n, 2 * I, h, nullptr, nullptr, 0);
        hipLaunchKernelGGL(k_swiglu_rows, dim3((I / 4 + 255) / 256, n), dim3(256), 0, m.stream, w.qkv, sg,
                           (size_t)n * 2 * I, I, w.act, w.act_lo, 0);
        pending = gemm<false>(m, w.act, w.act_lo, I, m.wdown[l], n, h, I, nullptr, nullptr, 0);
    }
    hipLaunchKernelGGL(k_rmsnorm_rows, dim3(n), dim3(norm_threads(n)), 0, m.stream, w.x, w.qkv, pending, (size_t)n * h,
                       m.final_norm, w.xn, w.xn_lo, h, c.rms_eps, PartTail{}, 0);
    const int sl = gemm<false>(m, w.xn, w.xn_lo, h, m.lm_head, n, c.vocab, h, nullptr, nullptr, 0);
    launch_argmax_rows(m, n, sl, b.logits, b.row_next);
}

// Xg[j][:] = X[idx[j]][:] + the K slices of the last down projection for that row
__global__ __launch_bounds__(256) void k_gather_rows(const float *__restrict__ X, const float *__restrict__ part,
                                                     int n_part, size_t part_stride, const int32_t *__restrict__ idx,
                                                     float *__restrict__ Xg, int h) {
    const size_t src = (size_t)idx[blockIdx.x] * h;
    for (int i = threadIdx.x; i < h; i += 256) {
        float v = X[src + i];
        for (int s = 0; s < n_part; ++s) v += part[(size_t)s * part_stride + src + i];
        Xg[(size_t)blockIdx.x * h + i] = v;
    }
}

// Catch-up pass over rows of several sequences at once (ragged): R rows in all, the rows of segment j are
// contiguous (segs[j].row0 .. +len) at positions kv0 .. kv0+len-1 of sequence segs[j].seq.  Projections see one
// R-row chunk (the weights are streamed once for all sequences); RoPE / KV append go by the per-row (sequence,
// position) arrays; attention is one launch over all segments (a device table tells every block its segment: rows,
// positions and cache), with one key-split count for the whole pass; the LM head runs on the gathered last rows of
// the segments.  `segs` is the host copy of the table at b.seg_tab.
void launch_prefill_varlen(const Model &m, const BatchRows &b, const FlashSeg *segs, int n_seg, int R) {
    const st_config &c = m.c;
    RaggedPass ragged = {b.seg_tab, n_seg, R, 0, 0, b.seq_stride};
    for (int j = 0; j < n_seg; ++j) {
        ragged.total_blocks = segs[j].blk0 + segs[j].nblk;
        const int tiles = (segs[j].kv0 + segs[j].len + kFlashKeys - 1) / kFlashKeys;
        if (tiles > ragged.max_tiles) ragged.max_tiles = tiles;
    }
    const int h = c.hidden, d = c.head_dim, nq = c.n_q_heads, nkv = c.n_kv_heads, I = c.intermediate;
    const int qd = nq * d, qkv = m.qkv_dim;
    const Workspace &w = m.ws;
    const PassTerms t = pass_terms(m, R);
    bf16_t *xn_lo = t.xn_lo, *attn_lo = t.attn_lo, *act_lo = t.act_lo, *qb_lo = t.qb_lo;
    hipLaunchKernelGGL(k_embed_rows, dim3(R), dim3(256), 0, m.stream, m.embed, b.row_tok, w.x, h, c.vocab);
    int pending = 0;
    for (int l = 0; l < c.n_layers; ++l) {
        const size_t lofs = (size_t)l * nkv * c.max_seq * d;
        hipLaunchKernelGGL(k_rmsnorm_rows, dim3(R), dim3(norm_threads(R)), 0, m.stream, w.x, w.qkv, pending, (size_t)R * h,
                           m.norm_attn[l], w.xn, t.qkv_two ? xn_lo : nullptr, h, c.rms_eps, PartTail{}, 0);
        const int sq = gemm<false>(m, w.xn, t.qkv_two ? xn_lo : nullptr, h, m.wqkv[l], R, qkv, h, nullptr, nullptr, 0);
        hipLaunchKernelGGL(k_rope_append_rows, dim3(R, nq + 2 * nkv), dim3(d / 2), 0, m.stream, w.qkv, sq,
                           (size_t)R * qkv, m.bqkv[l], w.rope, (float *)nullptr, w.qb, qb_lo, m.kcache + lofs,
                           m.vcache + lofs, b.row_pos, b.row_seq, b.seq_stride, nq, nkv, d, c.max_seq);
        launch_flash(m, w.qb, qb_lo, m.kcache + lofs, m.vcache + lofs, w.attn, attn_lo, 0, 0, &ragged, t.f16_attn);
        const int so = gemm<false>(m, w.attn, attn_lo, qd, t.f16_attn ? m.wo16[l] : m.wo[l], R, h, qd, nullptr, nullptr, 0,
                                   nullptr, t.f16_attn);
        hipLaunchKernelGGL(k_rmsnorm_rows, dim3(R), dim3(norm_threads(R)), 0, m.stream, w.x, w.qkv, so, (size_t)R * h,
                           m.norm_mlp[l], w.xn, t.f16_xg ? nullptr : xn_lo, h, c.rms_eps, PartTail{}, (int)t.f16_xg);
        if (R < (h % kRingBK == 0 ? m.ring_min_rows : kSmallRows + 1)) {
            const int sg = gemm<false>(m, w.xn, t.f16_xg ? nullptr : xn_lo, h, t.f16_xg ? m.wgu16[l] : m.wgu[l], R, 2 * I, h,
                                       nullptr, nullptr, 0, nullptr, t.f16_xg);
            hipLaunchKernelGGL(k_swiglu_rows, dim3((I / 4 + 255) / 256, R), dim3(256), 0, m.stream, w.qkv, sg,
                               (size_t)R * 2 * I, I, w.act, w.act_lo, (int)t.f16_act);
        } else {
            gemm<true>(m, w.xn, t.gu_two ? xn_lo : nullptr, h, t.f16_xg ? m.wgu16[l] : m.wgu[l], R, I, h, w.act, act_lo, I,
                       nullptr, t.f16_xg, t.f16_act);
        }
        pending = gemm<false>(m, w.act, act_lo, I, t.f16_act ? m.wdown16[l] : m.wdown[l], R, h, I, nullptr, nullptr, 0,
                              nullptr, t.f16_act);
    }
    // head on the last row of every segment (their row indices are in b.row_next on entry)
    hipLaunchKernelGGL(k_gather_rows, dim3(n_seg), dim3(256), 0, m.stream, w.x, w.qkv, pending, (size_t)R * h,
                       b.row_next, b.o_rows, h);
    hipLaunchKernelGGL(k_rmsnorm_rows, dim3(n_seg), dim3(norm_threads(n_seg)), 0, m.stream, b.o_rows, (const float *)nullptr, 0,
                       (size_t)0, m.final_norm, w.xn, w.xn_lo, h, c.rms_eps, PartTail{}, 0);
    const int sl = gemm<false>(m, w.xn, w.xn_lo, h, m.lm_head, n_seg, c.vocab, h, nullptr, nullptr, 0);
    launch_argmax_rows(m, n_seg, sl, b.logits, b.row_next);
}

}  // namespace st
