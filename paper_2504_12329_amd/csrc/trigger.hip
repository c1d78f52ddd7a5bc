// Token-level takeover trigger (paper Section 3 (1), keyword sets of Appendix C as id bitmaps; window > 2
// is the n1-token sentence after a delimiter): an ordered, exact scan of a token range.  One 1024-thread block walks the range in tiles and
// compacts the firing positions in ascending order with wave ballots.
#include "st_device.h"
#include "st_internal.h"

namespace st {

__device__ __forceinline__ bool in_set(const uint32_t *bm, int id, int vocab) {
    return id >= 0 && id < vocab && ((bm[id >> 5] >> (id & 31)) & 1u);
}

__global__ __launch_bounds__(1024) void k_trigger_scan(const int32_t *__restrict__ tokens, int lo, int hi,
                                                       const uint32_t *__restrict__ kw,
                                                       const uint32_t *__restrict__ delim, int window, int vocab,
                                                       int32_t *__restrict__ positions, int cap,
                                                       int32_t *__restrict__ n_found) {
    __shared__ int wave_total[16];
    __shared__ int base;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (threadIdx.x == 0) base = 0;
    __syncthreads();
    for (int start = lo; start < hi; start += 1024) {
        int p = start + (int)threadIdx.x;
        bool fire = false;
        if (p < hi) {
            if (window == 1) {
                fire = in_set(kw, tokens[p], vocab);
            } else {
                // the sentence of window - 1 tokens ending at p: delimiter right before it, none inside it
                // before its last token, a keyword somewhere in it
                const int first = p - (window - 1) + 1;
                if (first >= 1 && in_set(delim, tokens[first - 1], vocab)) {
                    bool ok = true, any = false;
                    for (int q = first; q <= p; ++q) {
                        const int t = tokens[q];
                        if (q < p && in_set(delim, t, vocab)) ok = false;
                        any |= in_set(kw, t, vocab);
                    }
                    fire = ok && any;
                }
            }
        }
        unsigned long long mask = __ballot(fire);
        int before = __popcll(mask & ((1ull << lane) - 1ull));
        if (lane == 0) wave_total[wave] = __popcll(mask);
        __syncthreads();
        int off = base + before;
        for (int w = 0; w < wave; ++w) off += wave_total[w];
        if (fire && off < cap) positions[off] = p;
        __syncthreads();
        if (threadIdx.x == 0) {
            int tot = 0;
            for (int w = 0; w < 16; ++w) tot += wave_total[w];
            base += tot;
        }
        __syncthreads();
    }
    if (threadIdx.x == 0) *n_found = base;
}

void launch_trigger_scan(const st_trigger_rule &rule, const int32_t *tokens, int32_t lo, int32_t hi,
                         int32_t *positions, int32_t cap, int32_t *n_found, hipStream_t stream) {
    hipLaunchKernelGGL(k_trigger_scan, dim3(1), dim3(1024), 0, stream, tokens, lo, hi, rule.kw_bitmap,
                       rule.delim_bitmap, rule.window, rule.vocab, positions, cap, n_found);
}

}  // namespace st
