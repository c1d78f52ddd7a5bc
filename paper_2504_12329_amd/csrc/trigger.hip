// Token-level takeover trigger (paper Section 3 (1), keyword sets of Appendix C as id bitmaps; window > 2
// is the n1-token sentence after a delimiter): an ordered, exact scan of a token range.
//
// The rule is evaluated as two running maxima instead of a look-back loop per position.  With w = window - 1,
//   lastD(q) = largest index j <= q whose token is a delimiter (-1: none),
//   lastK(q) = largest index j <= q whose token is a keyword   (-1: none),
// position p fires exactly when  p - w >= 0,  lastD(p - 1) == p - w  (a delimiter right before the sentence and none
// inside it before its last token)  and  lastK(p) > p - w  (a keyword inside it).  Both maxima are prefix scans, so
// a position costs O(1) whatever the window; the scan starts w tokens before `lo`, which is as far back as any
// position of the range looks.  One 1024-thread block walks the tokens in tiles, carries the two maxima from tile
// to tile and compacts the firing positions in ascending order with wave ballots.
#include <mutex>

#include "st_device.h"
#include "st_internal.h"

namespace st {

__device__ __forceinline__ bool in_set(const uint32_t *bm, int id, int vocab) {
    return id >= 0 && id < vocab && ((bm[id >> 5] >> (id & 31)) & 1u);
}

// inclusive running maximum over the lanes of a wave
__device__ __forceinline__ int wave_running_max(int v, int lane) {
#pragma unroll
    for (int o = 1; o < kWave; o <<= 1) {
        const int u = __shfl_up(v, o, kWave);
        if (lane >= o) v = max(v, u);
    }
    return v;
}

__global__ __launch_bounds__(1024) void k_trigger_scan(const int32_t *__restrict__ tokens, int lo, int hi,
                                                       const uint32_t *__restrict__ kw,
                                                       const uint32_t *__restrict__ delim, int window, int vocab,
                                                       int32_t *__restrict__ positions, int cap,
                                                       int32_t *__restrict__ n_found) {
    __shared__ int wave_d[16], wave_k[16], wave_n[16];
    __shared__ int carry_d, carry_k, base;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int w = window - 1;
    const int scan_from = w == 0 ? lo : max(0, lo - w);
    if (threadIdx.x == 0) carry_d = carry_k = -1, base = 0;
    __syncthreads();
    for (int start = scan_from; start < hi; start += 1024) {
        const int p = start + (int)threadIdx.x;
        const int id = p < hi ? tokens[p] : -1;  // -1 belongs to no set
        const bool is_k = in_set(kw, id, vocab), is_d = w > 0 && in_set(delim, id, vocab);
        const int run_d = wave_running_max(is_d ? p : -1, lane), run_k = wave_running_max(is_k ? p : -1, lane);
        int before_d = __shfl_up(run_d, 1, kWave);  // lastD(p - 1) within this wave
        if (lane == 0) before_d = -1;
        if (lane == kWave - 1) wave_d[wave] = run_d, wave_k[wave] = run_k;
        __syncthreads();
        int pre_d = carry_d, pre_k = carry_k;  // maxima over everything before this wave
        for (int v = 0; v < wave; ++v) pre_d = max(pre_d, wave_d[v]), pre_k = max(pre_k, wave_k[v]);
        const int last_d = max(pre_d, before_d), last_k = max(pre_k, run_k);
        const bool fire = p >= lo && p < hi && (w == 0 ? is_k : (p - w >= 0 && last_d == p - w && last_k > p - w));
        const unsigned long long mask = __ballot(fire);
        if (lane == 0) wave_n[wave] = __popcll(mask);
        __syncthreads();
        int off = base + __popcll(mask & ((1ull << lane) - 1ull));
        for (int v = 0; v < wave; ++v) off += wave_n[v];
        if (fire && off < cap) positions[off] = p;
        __syncthreads();
        if (threadIdx.x == 0) {
            int tot = 0, md = carry_d, mk = carry_k;
            for (int v = 0; v < 16; ++v) tot += wave_n[v], md = max(md, wave_d[v]), mk = max(mk, wave_k[v]);
            base += tot, carry_d = md, carry_k = mk;
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

// ---------------------------------------------------------------------------------------
// The scan for callers that cannot allocate device memory: the result staging (count + positions) lives in a
// file-scope device array instead of a caller-provided scratch buffer.  Every GPU the library runs on holds its
// own copy of the array until the process ends; its address is looked up once per device.
// ---------------------------------------------------------------------------------------
static __device__ __align__(256) int32_t scratch[1 + ST_SCAN_STATIC_MAX_CAP];

constexpr int kMaxDevices = 64;
static std::mutex g_scratch_mutex;
static int32_t *g_scratch_ptr[kMaxDevices];  // device address of `scratch` on each device (nullptr: not looked up yet)

// Device address of this device's copy of the staging array (the array's name is only a host-side handle).
static int scratch_address(int32_t **out) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return fail(ST_EHIP, "hipGetDevice: %s", hipGetErrorString(e));
    if (dev < 0 || dev >= kMaxDevices) return fail(ST_EHIP, "device index %d outside [0, %d)", dev, kMaxDevices);
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p)
            return fail(ST_EHIP, "hipGetSymbolAddress(scratch): %s", hipGetErrorString(e));
        g_scratch_ptr[dev] = static_cast<int32_t *>(p);
    }
    *out = g_scratch_ptr[dev];
    return ST_OK;
}

}  // namespace st

using namespace st;

extern "C" int st_trigger_scan_static(const st_trigger_rule *rule, const int32_t *tokens, int32_t lo, int32_t hi,
                                      int32_t *positions, int32_t cap, int32_t *n_found, void *stream) {
    if (!rule || !rule->kw_bitmap || !tokens || !n_found) return fail(ST_EINVAL, "rule, bitmap, tokens or n_found is NULL");
    if (rule->window < 1 || rule->window > ST_MAX_SCAN_WINDOW) return fail(ST_EINVAL, "window must be in [1, %d]", ST_MAX_SCAN_WINDOW);
    if (rule->window >= 2 && !rule->delim_bitmap) return fail(ST_EINVAL, "a window above 1 needs a delimiter bitmap");
    if (rule->vocab <= 0) return fail(ST_EINVAL, "rule vocab must be positive");
    if (cap < 0 || (cap > 0 && !positions)) return fail(ST_EINVAL, "cap < 0, or positions is NULL with cap > 0");
    if (cap > ST_SCAN_STATIC_MAX_CAP)
        return fail(ST_ERANGE, "cap %d exceeds the static staging array (%d positions)", cap, ST_SCAN_STATIC_MAX_CAP);
    if (lo < 0 || hi < lo) return fail(ST_ERANGE, "bad range [%d,%d)", lo, hi);
    int32_t *stage = nullptr;
    if (int rc = scratch_address(&stage)) return rc;
    hipStream_t s = (hipStream_t)stream;
    // the kernel writes the count and the first min(count, cap) positions on every call: nothing of the previous
    // call's contents is read, so nothing has to be cleared
    launch_trigger_scan(*rule, tokens, lo, hi, stage + 1, cap, stage, s);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(ST_EHIP, "trigger scan: %s", hipGetErrorString(e));
    e = hipMemcpyAsync(n_found, stage, sizeof(int32_t), hipMemcpyDeviceToHost, s);
    if (e == hipSuccess) e = hipStreamSynchronize(s);
    if (e != hipSuccess) return fail(ST_EHIP, "reading the count back: %s", hipGetErrorString(e));
    const int32_t k = *n_found < cap ? *n_found : cap;
    if (k > 0) {
        e = hipMemcpyAsync(positions, stage + 1, sizeof(int32_t) * k, hipMemcpyDeviceToHost, s);
        if (e == hipSuccess) e = hipStreamSynchronize(s);
        if (e != hipSuccess) return fail(ST_EHIP, "reading the positions back: %s", hipGetErrorString(e));
    }
    return ST_OK;
}
