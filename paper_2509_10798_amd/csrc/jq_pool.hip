// 1-D average pooling of the importance scores (the pooling settings the paper's
// Section 5.1 shares with its baselines), fused with the first radix histogram that the top-B
// selection needs, plus two small helpers (fill, standalone histogram).
//
//   pooled[l,g,t] = (1/k) * sum_{|u| <= (k-1)/2} scores[l,g,t+u],  zero outside t's own sequence.
//
// Memory-bound and tiny next to the K passes.  A block stages its span plus halo in LDS (zeros
// where the sequence ends), so every score is fetched from global memory once; blocks never straddle
// sequences, and pooling widths beyond the staged halo read their taps straight from global memory.
// On the way the block also prepares the top-B selection: the level-1 radix histogram of its problem and
// the block's own elements sorted by level-1 bin.
#include "jq_common.h"

namespace jq {

constexpr int kPoolThreads = 256;
constexpr int kPoolPerThread = 4;                              // one run of four consecutive positions per thread
constexpr int kPoolBlockPos = kPoolThreads * kPoolPerThread;  // 1024 positions per block (2048 and 8192 were slower:
                                                              // the kernel is one latency chain per block, and more,
                                                              // shorter chains overlap better)
static_assert(kPoolBlockPos == kSegLen, "one segment of the selection's lists per pooling workgroup");
constexpr int kPoolMaxHalo = 32;                               // (pool_k - 1) / 2 up to here uses the LDS path
constexpr int kWinBins = 128;                                  // histogram window below the block's top bin
constexpr int kWinCopies = 16;
constexpr int kWinStride = kWinBins + 1;                       // +1: copies of one bin fall into different banks

struct PoolArgs {
    const float* in;   // [n_layers][h_kv][T]
    float* out;        // same shape (null for the histogram-only kernel)
    uint32_t* hist;    // [n_layers][n_seq][h_kv][kHistStride] or null
    uint2* seg;        // [n_layers][h_kv][n_seg][head] (key, position) by level-1 bin, highest first, or null
    uint4* seg_hdr;    // [n_layers][h_kv][n_seg]: (lowest bin of the block's window, elements inside it, key in the segment's last slot, -)
    int32_t head;      // entries kept per segment (a multiple of 64, at most kSegLen)
    int32_t n_layers, h_kv, pool_k;
    int32_t keep_first, keep_last;  // always-kept positions (they land in the histogram's top bin)
    float inv_k;
    int64_t T;
    int32_t one_L;                   // single-sequence calls: the sequence's length (0 otherwise), next to the other
                                     // scalars so that the first kernel-argument reads do not chain through the tables
    int32_t n_seg;                   // workgroups per layer and head
    int32_t cu_seg[JQ_MAX_SEQ + 1];  // ... per sequence
    SeqTab tab;
};

// One workgroup pools kSegLen consecutive positions of ONE sequence (workgroups never straddle sequences, so
// pooling windows stop at sequence ends and every count goes to its own problem's histogram).
//
// Histogram of the block's values: neighbouring scores crowd into a few bins, which would serialise
// LDS atomics on one word; so the 128 bins below the block's highest bin are kept in 16 interleaved
// copies (lane & 15 picks the copy) and merged into the problem's global histogram with one
// device-scope atomic per non-empty bin.  Values more than 32 octaves below the block's maximum
// (the far tail of a peaked softmax, exact zeros) are counted in a single full-width LDS histogram
// that is cleared, filled and flushed only by blocks that meet such a value.
//
// Sorted segment: the same counters, turned into running offsets, give every element inside the window a
// slot -- ordered by level-1 bin, highest first (any order inside a bin) -- and the first `head` slots are
// written out as (key, position) pairs: the block's segment of the selection's lists.  The selection reads
// a segment until it meets a bin below the threshold bin, so it needs no pass of its own over all scores; a
// block with more qualifying elements than its segment holds (or whose window ends above the threshold
// bin) is re-read from the pooled scores themselves.
template <bool POOL, int K>  // K: pool_k known at compile time (taps unrolled), or 0 for any
__global__ __launch_bounds__(kPoolThreads) void jq_pool_kernel(PoolArgs a) {
    __shared__ uint32_t win[kWinCopies * kWinStride];
    __shared__ uint32_t wave_top[kPoolThreads / 64], wave_bottom[kPoolThreads / 64];
    __shared__ uint32_t scan_tmp[kPoolThreads / 64 + 1];
    __shared__ __attribute__((aligned(16))) uint2 sorted[kSegLen];  // head of the block's segment, assembled before it is written out
    // staged inputs; once the block's values are in registers the same memory serves as the full-width
    // histogram `low` of the far tail
    __shared__ __attribute__((aligned(16))) float tile[(POOL ? kPoolBlockPos + 2 * kPoolMaxHalo + 8 : 4) > kHistBins
                                                           ? (POOL ? kPoolBlockPos + 2 * kPoolMaxHalo + 8 : 4) : kHistBins];
    uint32_t* low = (uint32_t*)tile;
    const int g = blockIdx.y, layer = blockIdx.z;
    const int s = a.one_L ? 0 : find_seq(a.cu_seg, a.tab.n_seq, blockIdx.x);
    const int64_t lo = a.one_L ? 0 : a.tab.cu_seq[s], hi = a.one_L ? a.one_L : a.tab.cu_seq[s + 1];
    const int Ls = (int)(hi - lo);
    const int jblk = ((int)blockIdx.x - (a.one_L ? 0 : a.cu_seg[s])) * kPoolBlockPos;  // first position of the block inside its sequence
    const int cnt = min(kPoolBlockPos, Ls - jblk);                     // positions of this block (>= 1)
    const int64_t row = ((int64_t)layer * a.h_kv + g) * a.T;
    const float* in_row = a.in + row;
    const int64_t p0 = lo + jblk;  // the block covers row positions p0 .. p0 + cnt - 1
    const bool do_hist = a.hist != nullptr;
    const int r = K ? (K - 1) / 2 : (a.pool_k - 1) / 2;
    const bool staged = POOL && r <= kPoolMaxHalo;  // uniform

    if (do_hist) {
        for (int b = threadIdx.x; b < kWinCopies * kWinStride; b += kPoolThreads) win[b] = 0;
    }
    if (staged) {
        const int n = cnt + 2 * r;
        for (int i = threadIdx.x; i < n; i += kPoolThreads) {
            const int64_t q = p0 - r + i;
            tile[i] = (q >= lo && q < hi) ? in_row[q] : 0.f;
        }
    }
    lds_barrier();
    // Thread t owns the run of four consecutive positions 4t ..: with the taps unrolled a run reads its 4 + 2r
    // inputs as a few 16-byte LDS loads (lanes 16 B apart: no bank conflict) instead of 2r + 1 loads per output,
    // and stores one 16-byte vector when the row allows it.
    const int j0 = threadIdx.x * 4;
    float v[4] = {0.f, 0.f, 0.f, 0.f};
    if (j0 < cnt) {
        if (!POOL) {
#pragma unroll
            for (int u = 0; u < 4; ++u)
                if (j0 + u < cnt) v[u] = in_row[p0 + j0 + u];
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
                for (int64_t q = q0; q <= q1 && j0 + u < cnt; ++q) acc += in_row[q];
                v[u] = acc * a.inv_k;
            }
        }
        if (POOL) {
            if (((row + p0) & 3) == 0 && j0 + 3 < cnt) {
                store_stream16(&a.out[row + p0 + j0], make_uint4(__float_as_uint(v[0]), __float_as_uint(v[1]), __float_as_uint(v[2]), __float_as_uint(v[3])));
            } else {
#pragma unroll
                for (int u = 0; u < 4; ++u)
                    if (j0 + u < cnt) a.out[row + p0 + j0 + u] = v[u];
            }
        }
    }
    if (!do_hist) return;  // uniform

    uint32_t key[4], bin[4];
    uint32_t top = 0, bottom = 0xFFFFFFFFu;
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const bool in = j0 + u < cnt;
        key[u] = select_key(v[u], jblk + j0 + u, Ls, a.keep_first, a.keep_last);
        bin[u] = in ? key[u] >> 21 : 0xFFFFFFFFu;  // 0xFFFFFFFF: no element
        if (in) { top = max(top, bin[u]); bottom = min(bottom, bin[u]); }
    }
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) {
        top = max(top, (uint32_t)__shfl_xor((int)top, d));
        bottom = min(bottom, (uint32_t)__shfl_xor((int)bottom, d));
    }
    if ((threadIdx.x & 63) == 0) { wave_top[threadIdx.x >> 6] = top; wave_bottom[threadIdx.x >> 6] = bottom; }
    lds_barrier();
#pragma unroll
    for (int wv = 0; wv < kPoolThreads / 64; ++wv) { top = max(top, wave_top[wv]); bottom = min(bottom, wave_bottom[wv]); }
    const uint32_t base = top >= kWinBins - 1 ? top - (kWinBins - 1) : 0u;  // window = [base, base + 127]
    uint32_t* gh = a.hist + (((int64_t)layer * a.tab.n_seq + s) * a.h_kv + g) * kHistStride;
    uint32_t* my = win + (threadIdx.x & (kWinCopies - 1)) * kWinStride;
    const bool any_below = bottom < base;  // uniform over the block: some value lies below the window
    if (any_below) {
        for (uint32_t b = threadIdx.x; b < base; b += kPoolThreads) low[b] = 0;
        lds_barrier();
    }
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        if (bin[e] == 0xFFFFFFFFu) continue;
        if (bin[e] >= base) atomicAdd(&my[bin[e] - base], 1u);
        else atomicAdd(&low[bin[e]], 1u);
    }
    lds_barrier();
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
    if (a.seg == nullptr) return;  // uniform

    // Counting sort by (bin, highest first; copy): thread t owns bin 127 - t/2 of the window and eight of its
    // sixteen copies, so thread order is slot order.  The counters become running offsets.
    const int brel = kWinBins - 1 - (int)(threadIdx.x >> 1);
    const int c0 = (int)(threadIdx.x & 1) * (kWinCopies / 2);
    lds_barrier();  // the flush above has read the counters
    uint32_t cn[kWinCopies / 2];
    uint32_t sum = 0;
#pragma unroll
    for (int k = 0; k < kWinCopies / 2; ++k) {
        cn[k] = win[(c0 + k) * kWinStride + brel];
        sum += cn[k];
    }
    uint32_t n_win;  // elements inside the window: the sorted part of the segment
    uint32_t run = block_scan_incl<kPoolThreads>(sum, scan_tmp, &n_win) - sum;
#pragma unroll
    for (int k = 0; k < kWinCopies / 2; ++k) {
        win[(c0 + k) * kWinStride + brel] = run;
        run += cn[k];
    }
    lds_barrier();
    const int64_t seg_id = ((int64_t)layer * a.h_kv + g) * a.n_seg + blockIdx.x;
    const uint32_t head = (uint32_t)a.head;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        if (bin[e] == 0xFFFFFFFFu || bin[e] < base) continue;
        const uint32_t slot = atomicAdd(&my[bin[e] - base], 1u);
        if (slot < head) sorted[slot] = make_uint2(key[e], (uint32_t)(jblk + j0 + e));
    }
    lds_barrier();
    // written out in slot order, 32 bytes per thread (slots past min(head, n_win) are never read)
    if ((uint32_t)j0 < min(head, n_win)) {
        const uint4* src = (const uint4*)&sorted[j0];
        uint4* dst = (uint4*)(a.seg + seg_id * head + j0);
        store_stream16(dst, src[0]);
        store_stream16(dst + 1, src[1]);
    }
    if (threadIdx.x == 0) store_stream16(&a.seg_hdr[seg_id], make_uint4(base, n_win, n_win >= head ? sorted[head - 1].x : 0u, 0u));
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

// The fused forward's last step: one thread per (layer, sequence, KV head) adds the partial sums that the
// sequence's workgroups of the comparing launch left, in workgroup order, and divides by the sequence length.
struct MseReduceArgs {
    const double* part;  // [n_layers][n_cgrp][h_kv]
    float* mse;          // [n_layers][n_seq][h_kv]
    int32_t n_layers, n_seq, h_kv, n_cgrp;
    int32_t cu_cgrp[JQ_MAX_SEQ + 1];
    int32_t cu_seq[JQ_MAX_SEQ + 1];
};
__global__ __launch_bounds__(64) void jq_mse_reduce_kernel(MseReduceArgs a) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= a.n_layers * a.n_seq * a.h_kv) return;
    const int g = i % a.h_kv, s = (i / a.h_kv) % a.n_seq, layer = i / (a.h_kv * a.n_seq);
    double sum = 0.0;
    for (int cg = a.cu_cgrp[s]; cg < a.cu_cgrp[s + 1]; ++cg) sum += a.part[((int64_t)layer * a.n_cgrp + cg) * a.h_kv + g];
    a.mse[i] = (float)(sum / (double)(a.cu_seq[s + 1] - a.cu_seq[s]));
}

hipError_t launch_mse_reduce(const Plan& p, const double* part, float* mse, hipStream_t st) {
    MseReduceArgs a;
    a.part = part; a.mse = mse;
    a.n_layers = p.n_layers; a.n_seq = p.n_seq; a.h_kv = p.h_kv; a.n_cgrp = p.cu_cgrp2[p.n_seq];
    for (int s = 0; s <= p.n_seq; ++s) { a.cu_cgrp[s] = p.cu_cgrp2[s]; a.cu_seq[s] = p.tab.cu_seq[s]; }
    const int n = p.n_layers * p.n_seq * p.h_kv;
    return launch_kernel(jq_mse_reduce_kernel, dim3((unsigned)((n + 63) / 64)), dim3(64), 0, st, nullptr, -1, a);
}

__global__ __launch_bounds__(256) void jq_fill_u32_kernel(uint32_t* dst, size_t n, uint32_t v) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (; i < n; i += stride) dst[i] = v;
}

template __global__ void jq_pool_kernel<true, 7>(PoolArgs);  // placement: see jq_lib.hip

static PoolArgs make_args(const Plan& p, const float* in, float* out, uint32_t* hist, char* ws) {
    PoolArgs a;
    a.in = in; a.out = out; a.hist = hist;
    const bool lists = hist && ws && select_fast_path(p);  // the streaming selection reads the scores themselves
    a.seg = lists ? (uint2*)(ws + p.off_seg) : nullptr;
    a.seg_hdr = lists ? (uint4*)(ws + p.off_seghdr) : nullptr;
    a.head = p.seg_head;
    a.n_layers = p.n_layers; a.h_kv = p.h_kv; a.pool_k = p.pool_k;
    a.keep_first = p.keep_first; a.keep_last = p.keep_last;
    a.inv_k = 1.0f / (float)p.pool_k;
    a.T = p.T;
    a.one_L = p.n_seq == 1 ? p.tab.cu_seq[1] : 0;
    a.n_seg = p.n_seg;
    for (int s = 0; s <= p.n_seq; ++s) a.cu_seg[s] = p.cu_seg[s];
    a.tab = p.tab;
    return a;
}

hipError_t launch_pool(const Plan& p, const float* scores, float* pooled, uint32_t* hist_or_null, char* ws_or_null,
                       hipStream_t st) {
    const PoolArgs a = make_args(p, scores, pooled, hist_or_null, ws_or_null);
    dim3 grid((unsigned)p.n_seg, p.h_kv, p.n_layers);
    if (p.pool_k == 7) return launch_kernel(jq_pool_kernel<true, 7>, grid, dim3(kPoolThreads), 0, st, p.marks, kTrPool, a);
    return launch_kernel(jq_pool_kernel<true, 0>, grid, dim3(kPoolThreads), 0, st, p.marks, kTrPool, a);
}

hipError_t launch_hist(const Plan& p, const float* pooled, uint32_t* hist, char* ws_or_null, hipStream_t st) {
    const PoolArgs a = make_args(p, pooled, nullptr, hist, ws_or_null);
    dim3 grid((unsigned)p.n_seg, p.h_kv, p.n_layers);
    return launch_kernel(jq_pool_kernel<false, 0>, grid, dim3(kPoolThreads), 0, st, nullptr, -1, a);
}

hipError_t launch_fill_u32(uint32_t* dst, size_t n, uint32_t v, hipStream_t st) {
    if (n == 0) return hipSuccess;
    const size_t want = (n + 255) / 256;
    const unsigned blocks = (unsigned)(want < 1024 ? want : 1024);
    return launch_kernel(jq_fill_u32_kernel, dim3(blocks), dim3(256), 0, st, nullptr, -1, dst, n, v);
}

}  // namespace jq
