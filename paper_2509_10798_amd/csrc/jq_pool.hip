// 1-D average pooling of the importance scores (the pooling settings the paper's
// Section 5.1 shares with its baselines), fused with the first radix histogram that the top-B
// selection needs, plus two small helpers (fill, standalone histogram).
//
//   pooled[l,g,t] = (1/k) * sum_{|u| <= (k-1)/2} scores[l,g,t+u],  zero outside t's own sequence.
//
// Memory-bound and tiny next to the K passes.  A block stages its span plus halo in LDS (zeros
// where the sequence ends), so every score is fetched from global memory once; a block whose span
// crosses a sequence boundary handles one sequence's part after the other, and pooling widths beyond
// the staged halo read their taps straight from global memory.
#include "jq_common.h"

namespace jq {

constexpr int kPoolThreads = 256;
constexpr int kPoolPerThread = 4;                              // a multiple of 4
constexpr int kPoolBlockPos = kPoolThreads * kPoolPerThread;  // 1024 positions per block (2048 and 8192 were slower:
                                                              // the kernel is one latency chain per block, and more,
                                                              // shorter chains overlap better)
constexpr int kPoolMaxHalo = 32;                               // (pool_k - 1) / 2 up to here uses the LDS path
constexpr int kWinBins = 128;                                  // histogram window below the block's top bin
constexpr int kWinCopies = 16;
constexpr int kWinStride = kWinBins + 1;                       // +1: copies of one bin fall into different banks

struct PoolArgs {
    const float* in;   // [n_layers][h_kv][T]
    float* out;        // same shape (null for the histogram-only kernel)
    uint32_t* hist;    // [n_layers][n_seq][h_kv][kHistStride] or null
    int32_t n_layers, h_kv, pool_k;
    int32_t keep_first, keep_last;  // always-kept positions (they land in the histogram's top bin)
    float inv_k;
    int64_t T;
    SeqTab tab;
};

// Histogram of the block's values.  Neighbouring scores crowd into a few bins, which would serialise
// LDS atomics on one word; so the 128 bins below the block's highest bin are kept in 16 interleaved
// copies (lane & 15 picks the copy) and merged into the problem's global histogram with one
// device-scope atomic per non-empty bin.  Values more than 32 octaves below the block's maximum
// (the far tail of a peaked softmax, exact zeros) are counted in a single full-width LDS histogram
// that is cleared, filled and flushed only by blocks that meet such a value.
template <bool POOL, int K>  // K: pool_k known at compile time (taps unrolled), or 0 for any
__global__ __launch_bounds__(kPoolThreads) void jq_pool_kernel(PoolArgs a) {
    __shared__ uint32_t win[kWinCopies * kWinStride];
    __shared__ uint32_t wave_top[kPoolThreads / 64];
    // staged inputs; once the block's values are in registers the same memory serves as the full-width
    // histogram `low` of the far tail
    __shared__ __attribute__((aligned(16))) float tile[(POOL ? kPoolBlockPos + 2 * kPoolMaxHalo + 8 : 4) > kHistBins
                                                           ? (POOL ? kPoolBlockPos + 2 * kPoolMaxHalo + 8 : 4) : kHistBins];
    uint32_t* low = (uint32_t*)tile;
    const int g = blockIdx.y, layer = blockIdx.z;
    const int64_t row = ((int64_t)layer * a.h_kv + g) * a.T;
    const float* in_row = a.in + row;
    const int64_t b0 = (int64_t)blockIdx.x * kPoolBlockPos;
    const int64_t b1 = min(a.T, b0 + kPoolBlockPos);
    const int s_first = find_seq(a.tab.cu_seq, a.tab.n_seq, b0);
    const int s_last = find_seq(a.tab.cu_seq, a.tab.n_seq, b1 - 1);
    const bool do_hist = a.hist != nullptr;
    const int r = K ? (K - 1) / 2 : (a.pool_k - 1) / 2;
    const bool staged = POOL && r <= kPoolMaxHalo;  // uniform

    // The block's span is handled one sequence at a time (nearly always there is just one), so pooling
    // windows stop at sequence ends and every count goes to its own problem's histogram.
    for (int s = s_first; s <= s_last; ++s) {
        const int64_t lo = a.tab.cu_seq[s], hi = a.tab.cu_seq[s + 1];
        const int64_t p0 = max(b0, lo), p1 = min(b1, hi);  // this sequence's part of the span
        if (do_hist)
            for (int b = threadIdx.x; b < kWinCopies * kWinStride; b += kPoolThreads) win[b] = 0;
        if (staged) {
            const int n = (int)(p1 - p0) + 2 * r;
            for (int i = threadIdx.x; i < n; i += kPoolThreads) {
                const int64_t q = p0 - r + i;
                tile[i] = (q >= lo && q < hi) ? in_row[q] : 0.f;
            }
        }
        __syncthreads();
        // Thread t owns runs of four consecutive positions (4t.., then 4 * threads + 4t.., ...): with the taps unrolled
        // a run reads its 4 + 2r inputs as a few 16-byte LDS loads (lanes 16 B apart: no bank conflict) instead
        // of 2r + 1 loads per output, and stores one 16-byte vector when the row allows it.
        uint32_t bin[kPoolPerThread];
        uint32_t top = 0;
        const bool vec_store = ((row + p0) & 3) == 0;  // uniform
#pragma unroll
        for (int h = 0; h < kPoolPerThread / 4; ++h) {
            const int j0 = h * (kPoolThreads * 4) + threadIdx.x * 4;
            float v[4] = {0.f, 0.f, 0.f, 0.f};
            if (p0 + j0 < p1) {
                if (!POOL) {
#pragma unroll
                    for (int u = 0; u < 4; ++u)
                        if (p0 + j0 + u < p1) v[u] = in_row[p0 + j0 + u];
                } else if (staged && K > 0 && K <= 13) {
                    constexpr int kNeed = 4 + (K > 0 ? K - 1 : 0);  // inputs of the run
                    float x[16];
#pragma unroll
                    for (int q = 0; q < (kNeed + 3) / 4; ++q) {
                        const float4 f = *(const float4*)&tile[j0 + 4 * q];
                        x[4 * q] = f.x; x[4 * q + 1] = f.y; x[4 * q + 2] = f.z; x[4 * q + 3] = f.w;
                    }
#pragma unroll
                    for (int u = 0; u < 4; ++u) {
                        float acc = 0.f;
#pragma unroll
                        for (int k = 0; k < (K > 0 ? K : 1); ++k) acc += x[u + k];  // ascending position order
                        v[u] = acc * a.inv_k;
                    }
                } else if (staged) {
#pragma unroll
                    for (int u = 0; u < 4; ++u) {
                        float acc = 0.f;
                        for (int k = 0; k <= 2 * r; ++k) acc += tile[j0 + u + k];
                        v[u] = acc * a.inv_k;
                    }
                } else {
#pragma unroll
                    for (int u = 0; u < 4; ++u) {
                        const int64_t p = p0 + j0 + u;
                        const int64_t q0 = max(lo, p - r), q1 = min(hi - 1, p + r);
                        float acc = 0.f;
                        for (int64_t q = q0; q <= q1 && p < p1; ++q) acc += in_row[q];
                        v[u] = acc * a.inv_k;
                    }
                }
                if (POOL) {
                    if (vec_store && p0 + j0 + 3 < p1) {
                        *(float4*)&a.out[row + p0 + j0] = make_float4(v[0], v[1], v[2], v[3]);
                    } else {
#pragma unroll
                        for (int u = 0; u < 4; ++u)
                            if (p0 + j0 + u < p1) a.out[row + p0 + j0 + u] = v[u];
                    }
                }
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const bool in = p0 + j0 + u < p1;
                bin[4 * h + u] = in ? (select_key(v[u], (int)(p0 - lo) + j0 + u, (int)(hi - lo), a.keep_first, a.keep_last) >> 21)
                                    : 0xFFFFFFFFu;  // 0xFFFFFFFF: no element
                if (in) top = max(top, bin[4 * h + u]);
            }
        }
        if (!do_hist) {  // uniform
            __syncthreads();
            continue;
        }

#pragma unroll
        for (int d = 32; d >= 1; d >>= 1) top = max(top, (uint32_t)__shfl_xor((int)top, d));
        if ((threadIdx.x & 63) == 0) wave_top[threadIdx.x >> 6] = top;
        __syncthreads();
#pragma unroll
        for (int wv = 0; wv < kPoolThreads / 64; ++wv) top = max(top, wave_top[wv]);
        const uint32_t base = top >= kWinBins - 1 ? top - (kWinBins - 1) : 0u;  // window = [base, base + 127]
        uint32_t* gh = a.hist + (((int64_t)layer * a.tab.n_seq + s) * a.h_kv + g) * kHistStride;
        uint32_t* my = win + (threadIdx.x & (kWinCopies - 1)) * kWinStride;
        bool below = false;
#pragma unroll
        for (int e = 0; e < kPoolPerThread; ++e) below |= bin[e] < base;  // the "no element" marker is never below
        const bool any_below = __syncthreads_or(below);                    // uniform over the block
        if (any_below) {
            for (uint32_t b = threadIdx.x; b < base; b += kPoolThreads) low[b] = 0;
            __syncthreads();
        }
#pragma unroll
        for (int e = 0; e < kPoolPerThread; ++e) {
            if (bin[e] == 0xFFFFFFFFu) continue;
            if (bin[e] >= base) atomicAdd(&my[bin[e] - base], 1u);
            else atomicAdd(&low[bin[e]], 1u);
        }
        __syncthreads();
        if (any_below) {
            for (uint32_t b = threadIdx.x; b < base; b += kPoolThreads) {
                const uint32_t c = low[b];
                if (c) atomicAdd(gh + b, c);
            }
        }
        if (threadIdx.x < kWinBins) {
            uint32_t c = 0;
#pragma unroll
            for (int k = 0; k < kWinCopies; ++k) c += win[k * kWinStride + threadIdx.x];
            if (c) atomicAdd(gh + base + threadIdx.x, c);
        }
        __syncthreads();  // win, low, tile and wave_top are reused by the next sequence
    }
}

// Forward value of the training objective (paper Section 4.2, Eq. 3-5): mean squared difference of two averaged
// attention maps, map = scores / rows.  One workgroup per (layer, sequence, KV head); every thread sums its
// strided share in fp64 (the terms span many orders of magnitude), then a fixed-order tree in LDS.
constexpr int kMseThreads = 1024;
struct MseArgs {
    const float* a; const float* b;  // [n_layers][h_kv][T]
    float* mse;                      // [n_layers][n_seq][h_kv]
    float inv_rows_a, inv_rows_b;
    int32_t h_kv;
    int64_t T;
    SeqTab tab;
};

__global__ __launch_bounds__(kMseThreads) void jq_map_mse_kernel(MseArgs a) {
    __shared__ double part[kMseThreads];
    const int g = blockIdx.x % a.h_kv;
    const int s = (blockIdx.x / a.h_kv) % a.tab.n_seq;
    const int layer = blockIdx.x / (a.h_kv * a.tab.n_seq);
    const int L = a.tab.cu_seq[s + 1] - a.tab.cu_seq[s];
    const int64_t row = ((int64_t)layer * a.h_kv + g) * a.T + a.tab.cu_seq[s];
    double acc = 0.0;
    for (int j = threadIdx.x; j < L; j += kMseThreads) {
        const double diff = (double)a.a[row + j] * (double)a.inv_rows_a - (double)a.b[row + j] * (double)a.inv_rows_b;
        acc += diff * diff;
    }
    part[threadIdx.x] = acc;
    __syncthreads();
    for (int half = kMseThreads / 2; half >= 1; half >>= 1) {
        if ((int)threadIdx.x < half) part[threadIdx.x] += part[threadIdx.x + half];
        __syncthreads();
    }
    if (threadIdx.x == 0) a.mse[blockIdx.x] = (float)(part[0] / (double)L);
}

hipError_t launch_map_mse(const Plan& p, const float* scores_a, float rows_a, const float* scores_b, float rows_b,
                          float* mse, hipStream_t st) {
    MseArgs a;
    a.a = scores_a; a.b = scores_b; a.mse = mse;
    a.inv_rows_a = 1.0f / rows_a; a.inv_rows_b = 1.0f / rows_b;
    a.h_kv = p.h_kv; a.T = p.T; a.tab = p.tab;
    return launch_kernel(jq_map_mse_kernel, dim3((unsigned)(p.n_layers * p.n_seq * p.h_kv)), dim3(kMseThreads), 0, st, nullptr,
                         -1, a);
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
    a.keep_first = p.keep_first; a.keep_last = p.keep_last;
    a.inv_k = 1.0f / (float)p.pool_k;
    a.T = p.T;
    a.tab = p.tab;
    return a;
}

hipError_t launch_pool(const Plan& p, const float* scores, float* pooled, uint32_t* hist_or_null, hipStream_t st) {
    const PoolArgs a = make_args(p, scores, pooled, hist_or_null);
    dim3 grid((unsigned)((p.T + kPoolBlockPos - 1) / kPoolBlockPos), p.h_kv, p.n_layers);
    if (p.pool_k == 7) return launch_kernel(jq_pool_kernel<true, 7>, grid, dim3(kPoolThreads), 0, st, p.marks, kTrPool, a);
    return launch_kernel(jq_pool_kernel<true, 0>, grid, dim3(kPoolThreads), 0, st, p.marks, kTrPool, a);
}

hipError_t launch_hist(const Plan& p, const float* pooled, uint32_t* hist, hipStream_t st) {
    const PoolArgs a = make_args(p, pooled, nullptr, hist);
    dim3 grid((unsigned)((p.T + kPoolBlockPos - 1) / kPoolBlockPos), p.h_kv, p.n_layers);
    return launch_kernel(jq_pool_kernel<false, 0>, grid, dim3(kPoolThreads), 0, st, nullptr, -1, a);
}

hipError_t launch_fill_u32(uint32_t* dst, size_t n, uint32_t v, hipStream_t st) {
    if (n == 0) return hipSuccess;
    const size_t want = (n + 255) / 256;
    const unsigned blocks = (unsigned)(want < 1024 ? want : 1024);
    return launch_kernel(jq_fill_u32_kernel, dim3(blocks), dim3(256), 0, st, nullptr, -1, dst, n, v);
}

}  // namespace jq
