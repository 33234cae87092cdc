// 1-D average pooling of the importance scores (the "pooling configurations" the paper's
// Section 5.1 shares with its baselines), fused with the first radix histogram that the top-B
// selection needs, plus two small helpers (fill, standalone histogram).
//
//   pooled[l,g,t] = (1/k) * sum_{|u| <= (k-1)/2} scores[l,g,t+u],  zero outside t's own sequence.
//
// Memory-bound and tiny next to the K passes.  Device-scope atomics are the expensive part on a
// multi-die GPU, so blocks are large (8192 positions) and flush one LDS histogram each.  A block stages its span plus halo in LDS (zeros
// where the sequence ends), so every score is fetched from global memory once; blocks that
// straddle two sequences, or kernels wider than the staged halo, take a direct per-thread path.
#include "jq_common.h"

namespace jq {

constexpr int kPoolThreads = 1024;  // big blocks: few device-scope atomics per histogram bin
constexpr int kPoolPerThread = 8;
constexpr int kPoolBlockPos = kPoolThreads * kPoolPerThread;
constexpr int kPoolMaxHalo = 32;  // (pool_k - 1) / 2 up to here uses the LDS path

struct PoolArgs {
    const float* in;   // [n_layers][h_kv][T]
    float* out;        // same shape (null for the histogram-only kernel)
    uint32_t* hist;    // [n_layers][n_seq][h_kv][kHistStride] or null
    int32_t n_layers, h_kv, pool_k;
    float inv_k;
    int64_t T;
    SeqTab tab;
};

// Neighbouring scores mostly share a bin: count each distinct bin of the wave once instead of
// letting 64 lanes serialise on the same LDS word.  Must be called by all 64 lanes (pass
// `active` = false for lanes without an element).
__device__ __forceinline__ void wave_hist_add(uint32_t* bins, uint32_t bin, bool active) {
    const int lane = threadIdx.x & 63;
    uint64_t todo = __ballot(active);
    while (todo) {
        const int leader = __ffsll((unsigned long long)todo) - 1;
        const uint32_t lb = __shfl(bin, leader);
        const uint64_t same = __ballot(active && bin == lb);
        if (lane == leader) atomicAdd(&bins[lb], (uint32_t)__popcll(same));
        todo &= ~same;
    }
}

template <bool POOL>
__global__ __launch_bounds__(kPoolThreads) void jq_pool_kernel(PoolArgs a) {
    __shared__ uint32_t bins[kHistBins];
    __shared__ float tile[POOL ? kPoolBlockPos + 2 * kPoolMaxHalo : 1];
    const int g = blockIdx.y, layer = blockIdx.z;
    const int64_t row = ((int64_t)layer * a.h_kv + g) * a.T;
    const float* in_row = a.in + row;
    const int64_t p0 = (int64_t)blockIdx.x * kPoolBlockPos;
    const int64_t p1 = min(a.T, p0 + kPoolBlockPos);
    const int s_first = find_seq(a.tab.cu_seq, a.tab.n_seq, p0);
    const int s_last = find_seq(a.tab.cu_seq, a.tab.n_seq, p1 - 1);
    const bool one_seq = (s_first == s_last);  // uniform over the block
    const bool do_hist = a.hist != nullptr;
    const int r = (a.pool_k - 1) / 2;
    const bool staged = POOL && one_seq && r <= kPoolMaxHalo;  // uniform
    if (do_hist && one_seq) {
        for (int b = threadIdx.x; b < kHistBins; b += kPoolThreads) bins[b] = 0;
    }
    if (staged) {
        const int64_t lo = a.tab.cu_seq[s_first], hi = a.tab.cu_seq[s_first + 1];
        const int n = (int)(p1 - p0) + 2 * r;
        for (int i = threadIdx.x; i < n; i += kPoolThreads) {
            const int64_t q = p0 - r + i;
            tile[i] = (q >= lo && q < hi) ? in_row[q] : 0.f;
        }
    }
    __syncthreads();
#pragma unroll
    for (int e = 0; e < kPoolPerThread; ++e) {
        const int j = e * kPoolThreads + threadIdx.x;
        const int64_t p = p0 + j;
        const bool in = p < p1;
        int s = s_first;
        float v = 0.f;
        if (in) {
            if (!POOL) {
                v = in_row[p];
                if (!one_seq) s = find_seq(a.tab.cu_seq, a.tab.n_seq, p);
            } else if (staged) {
                float acc = 0.f;
                for (int u = 0; u <= 2 * r; ++u) acc += tile[j + u];  // ascending position order
                v = acc * a.inv_k;
                a.out[row + p] = v;
            } else {
                if (!one_seq) s = find_seq(a.tab.cu_seq, a.tab.n_seq, p);
                const int64_t lo = max((int64_t)a.tab.cu_seq[s], p - r);
                const int64_t hi = min((int64_t)a.tab.cu_seq[s + 1] - 1, p + r);
                float acc = 0.f;
                for (int64_t q = lo; q <= hi; ++q) acc += in_row[q];
                v = acc * a.inv_k;
                a.out[row + p] = v;
            }
        }
        if (do_hist) {  // uniform
            const uint32_t bin = sortable_key(v) >> 21;
            if (one_seq) wave_hist_add(bins, bin, in);  // uniform branch, all lanes take part
            else if (in) atomicAdd(a.hist + (((int64_t)layer * a.tab.n_seq + s) * a.h_kv + g) * kHistStride + bin, 1u);
        }
    }
    if (do_hist && one_seq) {
        __syncthreads();
        uint32_t* gh = a.hist + (((int64_t)layer * a.tab.n_seq + s_first) * a.h_kv + g) * kHistStride;
        for (int b = threadIdx.x; b < kHistBins; b += kPoolThreads) {
            const uint32_t c = bins[b];
            if (c) atomicAdd(gh + b, c);
        }
    }
}

__global__ __launch_bounds__(256) void jq_fill_u32_kernel(uint32_t* dst, size_t n, uint32_t v) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (; i < n; i += stride) dst[i] = v;
}

static PoolArgs make_args(const Plan& p, const float* in, float* out, uint32_t* hist) {
    PoolArgs a;
    a.in = in; a.out = out; a.hist = hist;
    a.n_layers = p.n_layers; a.h_kv = p.h_kv; a.pool_k = p.pool_k;
    a.inv_k = 1.0f / (float)p.pool_k;
    a.T = p.T;
    a.tab = p.tab;
    return a;
}

hipError_t launch_pool(const Plan& p, const float* scores, float* pooled, uint32_t* hist_or_null, hipStream_t st) {
    const PoolArgs a = make_args(p, scores, pooled, hist_or_null);
    dim3 grid((unsigned)((p.T + kPoolBlockPos - 1) / kPoolBlockPos), p.h_kv, p.n_layers);
    return launch_kernel(jq_pool_kernel<true>, grid, dim3(kPoolThreads), 0, st, p.marks, kTrPool, a);
}

hipError_t launch_hist(const Plan& p, const float* pooled, uint32_t* hist, hipStream_t st) {
    const PoolArgs a = make_args(p, pooled, nullptr, hist);
    dim3 grid((unsigned)((p.T + kPoolBlockPos - 1) / kPoolBlockPos), p.h_kv, p.n_layers);
    return launch_kernel(jq_pool_kernel<false>, grid, dim3(kPoolThreads), 0, st, nullptr, -1, a);
}

hipError_t launch_fill_u32(uint32_t* dst, size_t n, uint32_t v, hipStream_t st) {
    if (n == 0) return hipSuccess;
    const size_t want = (n + 255) / 256;
    const unsigned blocks = (unsigned)(want < 1024 ? want : 1024);
    return launch_kernel(jq_fill_u32_kernel, dim3(blocks), dim3(256), 0, st, nullptr, -1, dst, n, v);
}

}  // namespace jq
