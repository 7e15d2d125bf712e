// Adaptive mini-batch selection on gfx950 (TASER, arXiv 2402.05396, Sec. 3.1):
// an importance score per training edge, batches drawn with probability
// proportional to the scores, the scores of a batch overwritten after the
// iteration.
//
// An iteration changes only a batch's worth of scores, so nothing here is
// linear in the number of training edges per iteration: the scores carry two
// levels of partial sums (1024 scores per level-1 sum, 1024 level-1 sums per
// level-2 sum) that an update adjusts by the difference it makes, and a draw
// descends the three levels with one wavefront: at most 32 + 16 + 16 rows of
// 64 values for 2^31 edges, 1 + 16 + 16 for a million.
#include <new>

#include "sampling_device.h"
#include "taser_internal.h"

struct taser_selector {
    int64_t n;          // training edges
    int64_t n1, n2;     // level-1 and level-2 sums
    uint32_t* score;    // device uint32[n]
    uint64_t* sum1;     // device uint64[n1]: sum of score[1024*i .. 1024*i+1023]
    uint64_t* sum2;     // device uint64[n2]: sum of sum1[1024*i .. 1024*i+1023]
    int32_t* owner;     // device int32[n], -1 between calls: latest batch position that names an edge
};

namespace {

constexpr int kThreads = 256;
constexpr int kFan = 1024;             // values per partial sum
constexpr uint32_t kDrawTag = 0x4253454Cu;

// First index i in [begin, end) whose running sum over a[begin..i] exceeds x, by
// one wavefront, 64 values per step; x is reduced by the sum before a[i]. The
// caller guarantees that the whole range sums to more than x. Wave-uniform.
// Used for the top level, whose length varies.
template <typename T>
__device__ __forceinline__ int64_t wave_descend(const T* __restrict__ a, int64_t begin, int64_t end, uint64_t& x,
                                                int lane) {
    uint64_t before = 0;
    for (int64_t row = begin; row < end; row += kWave) {
        const int64_t i = row + lane;
        const uint64_t v = i < end ? (uint64_t)a[i] : 0;
        const uint64_t inc = wave_inclusive_scan64(v);
        const uint64_t hit = __ballot(before + inc > x);
        if (hit) {
            const int first = __ffsll((long long)hit) - 1;
            x -= before + wave_get64(inc - v, first);
            return row + first;
        }
        before += wave_get64(inc, kWave - 1);
    }
    return end - 1;   // not reached while the guarantee holds
}

// The same for one group of up to 1024 values starting at a[begin]: lane l loads
// values 16 l .. 16 l + 15 at once (all loads of the group in flight together),
// one wave scan of the lane totals finds the lane, that lane walks its 16 values.
template <typename T>
__device__ __forceinline__ int64_t wave_descend_group(const T* __restrict__ a, int64_t begin, int64_t end, uint64_t& x,
                                                      int lane) {
    constexpr int kPer = kFan / kWave;   // 16
    T v[kPer];
    const int64_t mine = begin + (int64_t)lane * kPer;
    if (begin + kFan <= end) {   // a whole group (wave-uniform): 16-byte loads; the arrays come from hipMalloc and
                                 // `mine` is a multiple of 16 values, so the address is 64-byte aligned
        typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
        constexpr int kVec = kPer * (int)sizeof(T) / 16;
        u32x4 raw[kVec];
        const u32x4* p = reinterpret_cast<const u32x4*>(a + mine);
#pragma unroll
        for (int i = 0; i < kVec; ++i) raw[i] = p[i];
        __builtin_memcpy(v, raw, sizeof(v));
    } else {
#pragma unroll
        for (int i = 0; i < kPer; ++i) v[i] = mine + i < end ? a[mine + i] : (T)0;
    }
    uint64_t own = 0;
#pragma unroll
    for (int i = 0; i < kPer; ++i) own += (uint64_t)v[i];
    const uint64_t inc = wave_inclusive_scan64(own);
    const uint64_t hit = __ballot(inc > x);
    const int first = hit ? __ffsll((long long)hit) - 1 : kWave - 1;   // hit is never 0 while the guarantee holds
    uint64_t rest = x - wave_get64(inc - own, first);                  // what is left inside that lane
    int found = kPer - 1;
    uint64_t left = rest;
    bool done = false;
#pragma unroll
    for (int i = 0; i < kPer; ++i) {
        if (!done) {
            if ((uint64_t)v[i] > rest) {
                found = i;
                left = rest;
                done = true;
            } else {
                rest -= (uint64_t)v[i];
            }
        }
    }
    x = wave_get64(left, first);
    return begin + (int64_t)first * kPer + __shfl(found, first, kWave);
}

// One block per partial sum: out[b] = sum of in[1024*b .. 1024*b+1023].
template <typename T>
__global__ __launch_bounds__(kThreads) void partial_sums_kernel(const T* __restrict__ in, int64_t n,
                                                                uint64_t* __restrict__ out) {
    __shared__ uint64_t part[kThreads / kWave];
    const int64_t base = (int64_t)blockIdx.x * kFan;
    uint64_t s = 0;
    for (int j = threadIdx.x; j < kFan; j += kThreads)
        if (base + j < n) s += (uint64_t)in[base + j];
    s = wave_sum64(s);
    if ((threadIdx.x & (kWave - 1)) == 0) part[threadIdx.x >> 6] = s;
    __syncthreads();
    if (threadIdx.x == 0) {
        uint64_t t = 0;
        for (int w = 0; w < kThreads / kWave; ++w) t += part[w];
        out[blockIdx.x] = t;
    }
}

__global__ __launch_bounds__(kThreads) void fill_u32_kernel(uint32_t* __restrict__ a, int64_t n, uint32_t v) {
    for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < n; i += (int64_t)gridDim.x * kThreads) a[i] = v;
}

// One wavefront per draw.
__global__ __launch_bounds__(kThreads) void batch_draw_kernel(const uint32_t* __restrict__ score, int64_t n,
                                                              const uint64_t* __restrict__ sum1, int64_t n1,
                                                              const uint64_t* __restrict__ sum2, int64_t n2, int64_t b,
                                                              uint32_t seed_lo, uint32_t seed_hi, uint64_t iteration,
                                                              int32_t* __restrict__ out) {
    const int lane = threadIdx.x & (kWave - 1);
    const int64_t j = (int64_t)blockIdx.x * (kThreads / kWave) + (threadIdx.x >> 6);
    if (j >= b) return;   // wave-uniform
    uint64_t total = 0;
    for (int64_t i = lane; i < n2; i += kWave) total += sum2[i];
    total = wave_sum64(total);
    if (total == 0) {
        if (lane == 0) out[j] = -1;
        return;
    }
    uint64_t x = __umul64hi(draw64(seed_lo, seed_hi, kDrawTag, iteration, (uint32_t)j), total);
    const int64_t i2 = wave_descend(sum2, 0, n2, x, lane);
    const int64_t end1 = (i2 + 1) * kFan < n1 ? (i2 + 1) * kFan : n1;
    const int64_t i1 = wave_descend_group(sum1, i2 * kFan, end1, x, lane);
    const int64_t end0 = (i1 + 1) * kFan < n ? (i1 + 1) * kFan : n;
    const int64_t e = wave_descend_group(score, i1 * kFan, end0, x, lane);
    if (lane == 0) out[j] = (int32_t)e;
}

// Update, step 1: for every named edge remember the latest batch position that names it.
__global__ __launch_bounds__(kThreads) void claim_kernel(const int32_t* __restrict__ idx, int64_t b, int64_t n,
                                                         int32_t* __restrict__ owner) {
    const int64_t j = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (j >= b) return;
    const int32_t e = idx[j];
    if (e >= 0 && e < n) atomicMax(&owner[e], (int32_t)j);
}

// Update, step 2: that position writes its value, moves the partial sums by the
// difference (integer adds: any order gives the same sums) and releases the edge.
__global__ __launch_bounds__(kThreads) void apply_kernel(const int32_t* __restrict__ idx,
                                                         const uint32_t* __restrict__ value, int64_t b, int64_t n,
                                                         uint32_t* __restrict__ score, uint64_t* __restrict__ sum1,
                                                         uint64_t* __restrict__ sum2, int32_t* __restrict__ owner) {
    const int64_t j = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    const int lane = threadIdx.x & (kWave - 1);
    uint64_t diff = 0;   // modulo 2^64: adding it is the signed change
    int32_t e = -1;
    if (j < b) {
        e = idx[j];
        if (e >= 0 && e < n && owner[e] == (int32_t)j) {
            const uint32_t old = score[e], now = value[j];
            score[e] = now;
            owner[e] = -1;
            diff = (uint64_t)now - (uint64_t)old;
        }
    }
    if (diff) atomicAdd((unsigned long long*)&sum1[e / kFan], (unsigned long long)diff);
    // A million edges share one level-2 sum: thousands of atomics on one address would
    // run one after the other. Lanes of a wavefront that change the same level-2 sum
    // as its first changing lane add up first and issue a single atomic.
    const uint64_t changing = __ballot(diff != 0);
    if (changing == 0) return;   // wave-uniform
    const int leader = __ffsll((long long)changing) - 1;
    const int32_t top = diff ? e / (kFan * kFan) : -1;
    const int32_t leader_top = __shfl(top, leader, kWave);
    const uint64_t together = wave_sum64(top == leader_top ? diff : 0);
    if (lane == leader) {
        if (together) atomicAdd((unsigned long long*)&sum2[leader_top], (unsigned long long)together);
    } else if (diff && top != leader_top) {
        atomicAdd((unsigned long long*)&sum2[top], (unsigned long long)diff);
    }
}

void free_all(taser_selector* s) {
    if (!s) return;
    (void)hipFree(s->score);
    (void)hipFree(s->sum1);
    (void)hipFree(s->sum2);
    (void)hipFree(s->owner);
    delete s;
}

void rebuild_sums(taser_selector* s, hipStream_t stream) {
    hipLaunchKernelGGL((partial_sums_kernel<uint32_t>), dim3((unsigned)s->n1), dim3(kThreads), 0, stream, s->score, s->n, s->sum1);
    hipLaunchKernelGGL((partial_sums_kernel<uint64_t>), dim3((unsigned)s->n2), dim3(kThreads), 0, stream, s->sum1, s->n1, s->sum2);
}

}  // namespace

extern "C" int taser_selector_init(const uint32_t* scores, int64_t n, uint32_t initial_score, void* hip_stream,
                                   taser_selector** out) {
    if (!out) return taser_fail(TASER_E_ARG, "selector_init: null out");
    *out = nullptr;
    if (n < 1 || n >= ((int64_t)1 << 31)) return taser_fail(TASER_E_RANGE, "selector_init: n = %lld outside [1, 2^31)", (long long)n);
    taser_clear_stale_hip_error();
    hipStream_t stream = (hipStream_t)hip_stream;
    taser_selector* s = new (std::nothrow) taser_selector();
    if (!s) return taser_fail(TASER_E_OOM, "selector_init: out of host memory");
    s->n = n;
    s->n1 = (n + kFan - 1) / kFan;
    s->n2 = (s->n1 + kFan - 1) / kFan;
    hipError_t e = hipMalloc(&s->score, (size_t)n * sizeof(uint32_t));
    if (e == hipSuccess) e = hipMalloc(&s->sum1, (size_t)s->n1 * sizeof(uint64_t));
    if (e == hipSuccess) e = hipMalloc(&s->sum2, (size_t)s->n2 * sizeof(uint64_t));
    if (e == hipSuccess) e = hipMalloc(&s->owner, (size_t)n * sizeof(int32_t));
    if (e == hipSuccess) {
        if (scores) e = hipMemcpyAsync(s->score, scores, (size_t)n * sizeof(uint32_t), hipMemcpyDeviceToDevice, stream);
        else hipLaunchKernelGGL(fill_u32_kernel, dim3(1024), dim3(kThreads), 0, stream, s->score, n, initial_score);
    }
    if (e == hipSuccess) {
        hipLaunchKernelGGL(fill_u32_kernel, dim3(1024), dim3(kThreads), 0, stream, (uint32_t*)s->owner, n, 0xFFFFFFFFu);
        rebuild_sums(s, stream);
        e = hipGetLastError();
    }
    if (e == hipSuccess) e = hipStreamSynchronize(stream);
    if (e != hipSuccess) {
        free_all(s);
        return taser_fail_hip(e, "selector_init");
    }
    *out = s;
    return TASER_OK;
}

extern "C" int taser_selector_draw(const taser_selector* s, int64_t b, uint64_t seed, uint64_t iteration,
                                   int32_t* batch, void* hip_stream) {
    if (!s) return taser_fail(TASER_E_ARG, "selector_draw: null selector");
    if (b < 0 || b >= ((int64_t)1 << 31)) return taser_fail(TASER_E_RANGE, "selector_draw: b = %lld outside [0, 2^31)", (long long)b);
    if (b == 0) return TASER_OK;
    if (!batch) return taser_fail(TASER_E_ARG, "selector_draw: null batch");
    taser_clear_stale_hip_error();
    hipStream_t stream = (hipStream_t)hip_stream;
    TaserProfileSpan span(stream, "selector_draw");
    const int64_t blocks = (b + kThreads / kWave - 1) / (kThreads / kWave);
    hipLaunchKernelGGL(batch_draw_kernel, dim3((unsigned)blocks), dim3(kThreads), 0, stream, s->score, s->n, s->sum1,
                       s->n1, s->sum2, s->n2, b, (uint32_t)seed, (uint32_t)(seed >> 32), iteration, batch);
    TASER_HIP_TRY(hipGetLastError());
    return TASER_OK;
}

extern "C" int taser_selector_update(taser_selector* s, const int32_t* batch, const uint32_t* new_scores, int64_t b,
                                     void* hip_stream) {
    if (!s) return taser_fail(TASER_E_ARG, "selector_update: null selector");
    if (b < 0 || b >= ((int64_t)1 << 31)) return taser_fail(TASER_E_RANGE, "selector_update: b = %lld outside [0, 2^31)", (long long)b);
    if (b == 0) return TASER_OK;
    if (!batch || !new_scores) return taser_fail(TASER_E_ARG, "selector_update: null batch or new_scores");
    taser_clear_stale_hip_error();
    hipStream_t stream = (hipStream_t)hip_stream;
    TaserProfileSpan span(stream, "selector_update");
    const unsigned blocks = (unsigned)((b + kThreads - 1) / kThreads);
    hipLaunchKernelGGL(claim_kernel, dim3(blocks), dim3(kThreads), 0, stream, batch, b, s->n, s->owner);
    hipLaunchKernelGGL(apply_kernel, dim3(blocks), dim3(kThreads), 0, stream, batch, new_scores, b, s->n, s->score,
                       s->sum1, s->sum2, s->owner);
    TASER_HIP_TRY(hipGetLastError());
    return TASER_OK;
}

extern "C" int taser_selector_scores(const taser_selector* s, uint32_t* scores, uint64_t* total, void* hip_stream) {
    if (!s) return taser_fail(TASER_E_ARG, "selector_scores: null selector");
    taser_clear_stale_hip_error();
    hipStream_t stream = (hipStream_t)hip_stream;
    if (scores) TASER_HIP_TRY(hipMemcpyAsync(scores, s->score, (size_t)s->n * sizeof(uint32_t), hipMemcpyDeviceToDevice, stream));
    if (total) {
        // sum of the level-2 sums, read back: at most 2048 values
        uint64_t host2[2048];
        TASER_HIP_TRY(hipMemcpyAsync(host2, s->sum2, (size_t)s->n2 * sizeof(uint64_t), hipMemcpyDeviceToHost, stream));
        TASER_HIP_TRY(hipStreamSynchronize(stream));
        uint64_t t = 0;
        for (int64_t i = 0; i < s->n2; ++i) t += host2[i];
        *total = t;
    }
    return TASER_OK;
}

extern "C" int taser_selector_size(const taser_selector* s, int64_t* n) {
    if (!s || !n) return taser_fail(TASER_E_ARG, "selector_size: null argument");
    *n = s->n;
    return TASER_OK;
}

extern "C" void taser_selector_free(taser_selector* s) { free_all(s); }
