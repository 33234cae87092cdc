// Importance scores of the prompt keys under the soft-token queries
// (paper Section 4.3, Eq. 3), as two K-streaming MFMA passes for gfx950.
//
//   pass 1 (stats):  per query row r, an offset m_r and Z_r = sum_j 2^(t_rj - m_r) of its base-2 logits
//                    t_rj = c * q_r.k_j, c = scale * log2(e); one (m, Z) partial per workgroup.
//   merge:           beta_r = m_r + log2 Z_r over a sequence's partials, as -beta_r / c split into three
//                    bf16 terms -- done by every pass-2 workgroup for its own head in its start-up (a
//                    separate small kernel only when a sequence leaves more than 64 partials).
//   pass 2 (score):  score_j = sum_r 2^(c * (q_r.k_j - beta_r / c)).  The -beta_r/c term enters
//                    through one extra MFMA step whose key-side operand is 1.0, so the epilogue is one
//                    multiply, one exp2 and one add per logit.
// Variants of the same kernels: supplied normalisers (pass 2 alone), the soft tokens' own keys or the prompt's
// own last tokens as causally masked tiles of pass 1, keys read out of a paged pool.
//
// One wave owns one (layer, sequence, KV head) and a strided set of that sequence's 32-key tiles, and
// keeps the head's (up to) 128 query rows in registers as MFMA operands.  The four waves of a workgroup
// work on the same head and fetch its query rows together (one row tile each, whole rows, turned into
// operand order through LDS) -- gathering them one row per lane would cost every wave 32 row-strided
// loads that touch 32 cache lines each.  Key tiles of 32 keys x 128 channels are
// fetched asynchronously, straight from global memory into a private, XOR-swizzled 8 KiB LDS slot
// (buffer loads with the LDS modifier, 16 B per lane, 16 lanes per 256-byte key row, so every 128-byte
// line is requested whole), two slots per wave used alternately, and read back in MFMA operand order without
// bank conflicts.  After the start-up waves never share LDS, so the streaming loop has no workgroup barrier;
// its only synchronisation is the wave's own s_waitcnt on its outstanding loads.
//
// MFMA 32x32x16 bf16 operand layout used here: lane l supplies row/column (l & 31) and the 8
// contraction elements selected by (l >> 5); both operands use the same element order, so any
// fixed channel permutation cancels.  Result: lane l holds column (l & 31), register v holds row
// 8*(v/4) + 4*(l>>5) + (v&3).
#include <type_traits>

#include "jq_common.h"

namespace jq {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

struct ScoreArgs {
    const uint16_t* Q;
    const uint16_t* K;
    const uint16_t* K_tail;  // [n_layers][n_seq][n_q][h_kv][d] keys of the soft tokens themselves, or null
    const float* lse;        // [n_layers][n_seq][n_q][h_q] caller-supplied natural-log normalisers, or null
    float inv_scale;         // 1 / scale
    int32_t one_L, one_waves;  // single-sequence calls: the sequence's length and its number of waves per head (0
                               // otherwise), next to the pointers, so that a wave's first kernel-argument reads
                               // do not chain through the per-sequence tables further down
    float2* stats;    // [n_layers][n_cgrp of pass 1][h_kv][RP]: (m, Z) per pass-1 workgroup
    uint2* aug;       // [n_layers][n_seq][h_kv][RP]: bf16 triple of -beta/c
    float* scores;    // [n_layers][h_kv][T]
    int32_t n_layers, n_seq, n_q, h_q, h_kv, group, rows, RP, chunk_keys, n_chunks;
    int32_t n_cgrp;       // workgroups per layer and head: sum over sequences of ceil(waves / 4)
    // pass 2 only: where pass 1 left its per-workgroup statistics (its own n_cgrp and per-sequence offsets),
    // and whether this launch merges them itself (otherwise jq_combine_kernel has filled `aug`)
    int32_t n_part, fuse_combine;
    int32_t group_shift;  // log2(group) when group is a power of two, else -1
    int32_t window;       // 1: the queries are the sequence's own last n_q tokens; query i sees keys 0 .. L - n_q + i
    int32_t depth;        // key tiles a wave keeps in flight: 1 (the default) or 2
    int32_t row_tile0;   // first query-row tile of this launch
    int32_t accumulate;  // pass 2: add to `scores` instead of overwriting
    float c;             // scale * log2(e)
    int64_t T;
    uint32_t* zero;      // combine: words to clear for the later selection stage (nullable)
    uint64_t zero_words;
    // paged K (PAGED kernels): K is [n_layers][n_pages][1 << page_shift][h_kv][d]; token t of sequence s lives in
    // page block_table[s * max_pages + (t >> page_shift)]
    const int32_t* block_table;
    int32_t page_shift, n_pages, max_pages;
    // the per-sequence tables come last: every scalar above sits in the first few hundred bytes of the kernel
    // arguments, which a wave fetches in one go
    int32_t cu_part[JQ_MAX_SEQ + 1];
    SeqTab tab;
    // DIFF kernels (training-side forward, Eq. 3-5): instead of storing its scores the launch compares them with
    // the map of the other query set and leaves one partial sum of squared differences per workgroup
    const float* diff_ref;    // [n_layers][h_kv][T]
    double* diff_part;        // [n_layers][n_cgrp][h_kv]
    float diff_inv_ref, diff_inv_own;  // 1 / summed probability rows of either map
};

constexpr int kSlotBytes = kKeyTile * kHeadDim * 2;  // 8 KiB

__device__ __forceinline__ bf16x8 as_bf16x8(u32x4 v) { return __builtin_bit_cast(bf16x8, v); }

// Key tiles arrive through loads that write LDS directly; the compiler does not track them, so the
// waits are explicit.  Loads complete in issue order, and every tile is exactly 8 loads, hence
// "at most 8 outstanding" means: everything older than the newest tile has landed.
// (s_waitcnt immediates: vmcnt in bits 3:0 and 15:14, expcnt 6:4, lgkmcnt 11:8; unused fields = no wait.)
__device__ __forceinline__ void wait_tile_landed(bool newer_tile_in_flight) {
    if (newer_tile_in_flight) __builtin_amdgcn_s_waitcnt(0x0F78);  // vmcnt(8)
    else __builtin_amdgcn_s_waitcnt(0x0F70);                        // vmcnt(0)
    __builtin_amdgcn_sched_barrier(0);
    asm volatile("" ::: "memory");
}

// The fragments just read from an LDS slot must be in registers before the slot is refilled.
__device__ __forceinline__ void wait_frags_read() {
    asm volatile("" ::: "memory");
    __builtin_amdgcn_sched_barrier(0);
    __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0)
    __builtin_amdgcn_sched_barrier(0);
    asm volatile("" ::: "memory");
}

// Which (layer, sequence, head) and which of its key tiles this wave owns.  A sequence of L keys gets
// W = ceil(L / chunk_keys) waves per head; wave w of them takes the 32-key tiles w, w + W, w + 2W, ...
// Interleaving the tiles (instead of giving each wave one contiguous range) makes all waves that run
// at the same time sweep one window of the key tensor, which DRAM serves at close to its streaming rate.
// The four waves of a workgroup are consecutive waves of ONE (layer, sequence, head), so they can share
// the head's query rows; a sequence whose W is not a multiple of four leaves the last workgroup's
// surplus waves without tiles (they only help with the query rows).
struct WaveItem {
    int layer, seq, g;
    int wave, n_waves;                // w and W
    int L;                            // keys in the sequence
    int n_tiles;                      // tiles this wave owns (0: surplus wave)
    int64_t tok0;                     // first token of the sequence in the flattened T axis
};

__device__ __forceinline__ void wave_item(const ScoreArgs& a, bool reverse, WaveItem& w) {
    uint32_t b = blockIdx.x;  // the grid is exactly n_layers * n_cgrp * h_kv workgroups (below 2^31: 32-bit arithmetic)
    if (reverse) b = gridDim.x - 1 - b;
    // readfirstlane makes the wave index (and everything derived from it) a scalar for the compiler
    const int wv = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    w.g = (int)(b % (uint32_t)a.h_kv);  // heads vary fastest: neighbouring workgroups read neighbouring 256-byte pieces of a token row
    const uint32_t rest = b / (uint32_t)a.h_kv;
    const int cg = (int)(rest % (uint32_t)a.n_cgrp);
    w.layer = (int)(rest / (uint32_t)a.n_cgrp);
    if (a.one_L) {  // one sequence: nothing to look up
        w.seq = 0;
        w.L = a.one_L;
        w.n_waves = a.one_waves;
        w.wave = cg * kScoreWaves + wv;
        w.tok0 = 0;
    } else {
        w.seq = find_seq(a.tab.cu_cgrp, a.tab.n_seq, cg);
        w.L = a.tab.cu_seq[w.seq + 1] - a.tab.cu_seq[w.seq];
        w.n_waves = a.tab.cu_chunk[w.seq + 1] - a.tab.cu_chunk[w.seq];
        w.wave = (cg - a.tab.cu_cgrp[w.seq]) * kScoreWaves + wv;
        w.tok0 = a.tab.cu_seq[w.seq];
    }
    const int seq_tiles = (w.L + kKeyTile - 1) / kKeyTile;  // >= n_waves, since a chunk is at least one tile
    w.n_tiles = w.wave < w.n_waves ? (seq_tiles - w.wave + w.n_waves - 1) / w.n_waves : 0;
}

// ---- key tiles: global -> LDS -------------------------------------------------------------------
// A tile is 32 key rows of 256 B.  Load i (0..7) of a wave moves rows 4i..4i+3: lane l fetches 16 B
// of row r = 4i + (l >> 4), and the hardware stores them at slot + 1024 i + 16 l, i.e. at row r,
// physical 16-byte chunk (l & 15).  To realise the swizzle "logical chunk c lives at physical chunk
// c ^ (r & 15)" the lane therefore fetches logical chunk (l & 15) ^ (r & 15) from global memory.
// With (r & 15) = 4 (i & 3) + (l >> 4) the lane's byte offset takes four values over the 8 loads;
// the rest of the address is wave-uniform (buffer resource + scalar offset).
struct TileLanes {
    uint32_t voff[4];  // (l >> 4) * row_bytes + 16 * (((l & 15) ^ (l >> 4)) ^ 4 j),  j = i & 3
};

__device__ __forceinline__ TileLanes tile_lanes(int lane, uint32_t row_bytes) {
    TileLanes tl;
    const uint32_t a = lane >> 4, x = (lane & 15) ^ a;
#pragma unroll
    for (int j = 0; j < 4; ++j) tl.voff[j] = a * row_bytes + ((x ^ (4u * j)) << 4);
    return tl;
}

__device__ __forceinline__ void lds_dma16(__amdgpu_buffer_rsrc_t rsrc, char* dst, uint32_t voff, uint32_t soff) {
    __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (__attribute__((address_space(3))) void*)dst, 16, (int)voff,
                                             (int)soff, 0, 0);
}

// `tile_off` = byte offset of the tile's first key row inside the buffer resource (uniform).
__device__ __forceinline__ void fetch_tile(__amdgpu_buffer_rsrc_t rsrc, char* slot, uint32_t tile_off,
                                           uint32_t row_bytes, int valid, const TileLanes& tl, int lane) {
    if (valid >= kKeyTile) {
#pragma unroll
        for (int i = 0; i < 8; ++i) lds_dma16(rsrc, slot + 1024 * i, tl.voff[i & 3], tile_off + 4 * i * row_bytes);
    } else {  // last, partial tile of a sequence: rows past the end re-read the last valid key (masked later)
        asm volatile("" : "+v"(lane));  // keep this rarely taken path's address arithmetic out of the caller's loop
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int r = 4 * i + (lane >> 4);
            const uint32_t voff = (uint32_t)min(r, valid - 1) * row_bytes + (((lane & 15) ^ (r & 15)) << 4);
            lds_dma16(rsrc, slot + 1024 * i, voff, tile_off);
        }
    }
}

// The same with the general addressing whatever `valid` (>= 1) is: no branch, for requests that have to sit in one
// basic block with other loads.
__device__ __forceinline__ void fetch_tile_any(__amdgpu_buffer_rsrc_t rsrc, char* slot, uint32_t tile_off,
                                               uint32_t row_bytes, int valid, int lane) {
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const int r = 4 * i + (lane >> 4);
        const uint32_t voff = (uint32_t)min(r, valid - 1) * row_bytes + (((lane & 15) ^ (r & 15)) << 4);
        lds_dma16(rsrc, slot + 1024 * i, voff, tile_off);
    }
}

// MFMA operand fragments of the tile in `slot`: lane l takes key row (l & 31), logical chunks
// 2 ks + (l >> 5), ks = 0..7.  The 16 lanes of a quarter wave hit 16 distinct physical chunks.
__device__ __forceinline__ void lds_get_frags(const char* slot, bf16x8 (&kf)[8], int lane) {
    const int r = lane & 31;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
        const int chunk = 2 * ks + (lane >> 5);
        kf[ks] = as_bf16x8(*(const u32x4*)(slot + r * 256 + ((chunk ^ (r & 15)) << 4)));
    }
}

// ---- start-up: the query rows as MFMA operands of every wave, with the first key tile in flight ---------
// Query rows of the workgroup's KV head (row r = i * group + hh  <->  Q[i, g*group + hh]): wave qt fetches row
// tile qt like a key tile -- every load instruction covers four whole 256-byte rows (lane l takes 16 B of row
// 4i + (l >> 4)), so each cache line is requested once -- and writes it, swizzled, into its own second LDS slot;
// after a barrier every wave reads all tiles in operand order; a second barrier frees the slots for key tiles.
// The compiler cannot tell which LDS bytes a direct-to-LDS load writes, so before any LDS access it generates
// it waits for every such load that is outstanding -- here that would be the first key tile, whose flight
// (the first sixteenth of K arriving at the rate of the memory system) is exactly what the start-up should hide
// behind.  The LDS instructions of the start-up are therefore written out, with their own waits: nothing the
// compiler generates touches LDS between the request of the first key tile and the first wait_tile_landed().
// Global loads into registers issued BEFORE the tile's request still get their exact waits from the compiler
// (loads return in issue order, so waiting for one of them never waits for the younger tile).
__device__ __forceinline__ uint32_t lds_addr(const void* p) {
    return (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const char*)p;
}
__device__ __forceinline__ void lds_wait_all() { asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); }
__device__ __forceinline__ void lds_put16(uint32_t addr, u32x4 v) { asm volatile("ds_write_b128 %0, %1" ::"v"(addr), "v"(v) : "memory"); }
__device__ __forceinline__ void lds_put8(uint32_t addr, uint2 v) {
    const uint64_t x = (uint64_t)v.x | ((uint64_t)v.y << 32);
    asm volatile("ds_write_b64 %0, %1" ::"v"(addr), "v"(x) : "memory");
}
__device__ __forceinline__ uint2 lds_get8_waited(uint32_t addr) {
    uint64_t x;
    asm volatile("ds_read_b64 %0, %1\n\ts_waitcnt lgkmcnt(0)" : "=&v"(x) : "v"(addr) : "memory");
    return make_uint2((uint32_t)x, (uint32_t)(x >> 32));
}
// lds_get_frags with explicit instructions; returns when the fragments are in registers
__device__ __forceinline__ void lds_get_frags_waited(uint32_t slot, bf16x8 (&kf)[8], int lane) {
    const uint32_t r = (uint32_t)lane & 31u, hi = (uint32_t)lane >> 5;
    uint32_t ad[8];
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) ad[ks] = slot + r * 256u + (((2u * ks + hi) ^ (r & 15u)) << 4);
    u32x4 o0, o1, o2, o3, o4, o5, o6, o7;
    asm volatile(
        "ds_read_b128 %0, %8\n\tds_read_b128 %1, %9\n\tds_read_b128 %2, %10\n\tds_read_b128 %3, %11\n\t"
        "ds_read_b128 %4, %12\n\tds_read_b128 %5, %13\n\tds_read_b128 %6, %14\n\tds_read_b128 %7, %15\n\t"
        "s_waitcnt lgkmcnt(0)"
        : "=&v"(o0), "=&v"(o1), "=&v"(o2), "=&v"(o3), "=&v"(o4), "=&v"(o5), "=&v"(o6), "=&v"(o7)
        : "v"(ad[0]), "v"(ad[1]), "v"(ad[2]), "v"(ad[3]), "v"(ad[4]), "v"(ad[5]), "v"(ad[6]), "v"(ad[7])
        : "memory");
    kf[0] = as_bf16x8(o0); kf[1] = as_bf16x8(o1); kf[2] = as_bf16x8(o2); kf[3] = as_bf16x8(o3);
    kf[4] = as_bf16x8(o4); kf[5] = as_bf16x8(o5); kf[6] = as_bf16x8(o6); kf[7] = as_bf16x8(o7);
}
// Barrier between phases that communicate through the LDS instructions above (each of which has waited for its
// own completion): no fence, hence no wait the compiler would add for loads in flight.
__device__ __forceinline__ void bare_barrier() {
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
}
// Where the query rows that this wave stages live (every wave computes addresses, so that the loads themselves
// can be issued unconditionally; waves beyond the row tiles take the last tile's and never store them).  Rows past
// the end take the address of row 0 of the head, in bounds, and are zeroed when staged -- `pad`, bit i: load i is
// such a row.
template <int NQT>
__device__ __forceinline__ void q_rows_where(const ScoreArgs& a, const WaveItem& w, int lane, const u32x4* (&src)[8], uint32_t& pad) {
    const int wv = min(__builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6)), NQT - 1);
    const char* qbase = (const char*)a.Q + ((int64_t)(w.layer * a.n_seq + w.seq) * a.n_q) * a.h_q * kHeadDim * 2;
    pad = 0;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const int r = 4 * i + (lane >> 4);
        const int row = (a.row_tile0 + wv) * kRowTile + r;
        const bool valid = row < a.rows;
        const int rowc = valid ? row : 0;
        int it, hh;
        if (a.group_shift >= 0) { it = rowc >> a.group_shift; hh = rowc & (a.group - 1); }
        else { it = rowc / a.group; hh = rowc % a.group; }
        const int c = (lane & 15) ^ (r & 15);
        src[i] = (const u32x4*)(qbase + ((int64_t)it * a.h_q + (w.g * a.group + hh)) * kHeadDim * 2 + c * 16);
        pad |= valid ? 0u : 1u << i;
    }
}
// ... and their way through LDS into operand order, with the first key tile in flight.  Every wave of the
// workgroup must call this (two barriers).
template <int NQT>
__device__ __forceinline__ void q_rows_stage(int lane, char* lds_base, const u32x4 (&raw)[8], uint32_t pad, bf16x8 (&qf)[NQT][8]) {
    static_assert(NQT <= kScoreWaves, "one wave per query-row tile");
    const int wv = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    if (wv < NQT) {
        const uint32_t slot = lds_addr(lds_base + (wv * 2 + 1) * kSlotBytes);
#pragma unroll
        for (int i = 0; i < 8; ++i) lds_put16(slot + 1024u * i + 16u * lane, (pad >> i) & 1u ? u32x4{0u, 0u, 0u, 0u} : raw[i]);
        lds_wait_all();
    }
    bare_barrier();
#pragma unroll
    for (int qt = 0; qt < NQT; ++qt) lds_get_frags_waited(lds_addr(lds_base + (qt * 2 + 1) * kSlotBytes), qf[qt], lane);
    bare_barrier();
}

struct KeyStream {
    __amdgpu_buffer_rsrc_t rsrc;  // this head's rows of the whole sequence (PAGED: of the layer's whole pool)
    uint32_t row_bytes;
    const int32_t* pages;         // PAGED: the sequence's row of the block table
    uint32_t page_shift, page_mask, last_page;
};

template <bool PAGED>
__device__ __forceinline__ KeyStream key_stream(const ScoreArgs& a, const WaveItem& w) {
    KeyStream ks;
    ks.row_bytes = (uint32_t)a.h_kv * kHeadDim * 2;
    // the resource covers exactly this head's rows of the sequence, or of the layer's pool (the host checks
    // that this is below 4 GiB); every generated offset stays inside it
    const int64_t first_row = PAGED ? ((int64_t)w.layer * a.n_pages) << a.page_shift : (int64_t)w.layer * a.T + w.tok0;
    const uint32_t n_rows = PAGED ? (uint32_t)a.n_pages << a.page_shift : (uint32_t)w.L;
    const char* kseq = (const char*)a.K + (first_row * a.h_kv + w.g) * kHeadDim * 2;
    const uint32_t bytes = (n_rows - 1) * ks.row_bytes + kHeadDim * 2;
    ks.rsrc = __builtin_amdgcn_make_buffer_rsrc((void*)kseq, 0, (int)bytes, 0x00020000);
    ks.pages = PAGED ? a.block_table + (int64_t)w.seq * a.max_pages : nullptr;
    ks.page_shift = (uint32_t)a.page_shift;
    ks.page_mask = (1u << a.page_shift) - 1u;
    ks.last_page = (uint32_t)a.n_pages - 1u;
    return ks;
}

// Byte offset of sequence tile t inside the key stream's resource.  A page holds a whole number of 32-key
// tiles, so a tile never straddles pages; `page` is the block-table entry of the tile's page (clamped here,
// so that a corrupt table cannot send a load outside the pool).
template <bool PAGED>
__device__ __forceinline__ uint32_t tile_offset(const KeyStream& ks, int t, int page) {
    const uint32_t tok = (uint32_t)t * kKeyTile;
    if (!PAGED) return tok * ks.row_bytes;
    const uint32_t p = (uint32_t)clamp_page(page, (int32_t)ks.last_page + 1);  // the same clamp as the gather's
    return ((p << ks.page_shift) + (tok & ks.page_mask)) * ks.row_bytes;
}
// One table word per tile, at a wave-uniform address.  The table is read-only for the whole launch, so it is
// read through the constant address space: that makes the load a scalar one with a wait of its own -- a
// vector load would have to be waited for together with every key tile in flight.
typedef const int32_t __attribute__((address_space(4))) * const_i32_ptr;
template <bool PAGED>
__device__ __forceinline__ int tile_page(const KeyStream& ks, int t) {
    return PAGED ? ((const_i32_ptr)ks.pages)[((uint32_t)t * kKeyTile) >> ks.page_shift] : 0;
}

// ------------------------------------------------------------------------------------------------
// pass 1: softmax statistics
// ------------------------------------------------------------------------------------------------
// One 32-key tile against the wave's query rows: rows of the MFMA result are keys, columns are
// query rows, so each lane updates the running (m, Z) of its own query column from its 16 keys.
// MASKED: key (row of the tile) number >= valid[qt] does not exist for query tile qt's column of this lane --
// used for the last, partial tile of a sequence (one uniform bound) and for the tiles of the soft tokens'
// own keys, where the bound is causal and differs per lane.
__device__ __forceinline__ f32x16 stats_chain(const bf16x8 (&kf)[8], const bf16x8 (&q)[8]) {
    f32x16 acc = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int k8 = 0; k8 < 8; ++k8) acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[k8], q[k8], acc, 0, 0, 0);
    return acc;
}

// Two instances exist.  <false, true>, the hot one: unmasked tile, offsets m kept as they are, only
// Z += sum 2^(t - m).  Any offset gives the same (m, Z) pair up to rounding as long as no term overflows; terms
// that underflow are negligible next to the contribution of the offset's own key.  `flag` there marks the wave's
// first tile, which sets each lane's offset -- to the largest of four of the lane's 16 logits, so that the first
// tile runs through the very code of all later ones.  <true, false>, the general one: masked, and `flag` says
// whether the offsets are kept (then m stays and the update below reduces to Z += sum) or follow the running
// maximum.
template <int NQT, bool MASKED, bool FIXED>
__device__ __forceinline__ void stats_tile(const bf16x8 (&kf)[8], const bf16x8 (&qf)[NQT][8], float (&m)[NQT],
                                           float (&z)[NQT], float c, const int (&valid)[NQT], int half, bool flag) {
    // software pipeline: the MFMA chain of query tile qt+1 is interleaved with the max/exp2/add work of tile qt
    f32x16 acc = stats_chain(kf, qf[0]);
#pragma unroll
    for (int qt = 0; qt < NQT; ++qt) {
        f32x16 nxt = acc;
        if (qt + 1 < NQT) nxt = stats_chain(kf, qf[qt + 1]);
        if (MASKED) {
#pragma unroll
            for (int v = 0; v < 16; ++v)
                if (8 * (v >> 2) + 4 * half + (v & 3) >= valid[qt]) acc[v] = -INFINITY;
        }
        float mnew = m[qt];
        if (FIXED) mnew = flag ? fmaxf(fmaxf(acc[0], acc[5]), fmaxf(acc[10], acc[15])) * c : mnew;
        if (!FIXED) {
            float tmax = fmaxf(acc[0], acc[1]);
#pragma unroll
            for (int v = 2; v < 16; ++v) tmax = fmaxf(tmax, acc[v]);
            mnew = flag ? mnew : fmaxf(m[qt], tmax * c);  // a fully masked column keeps m: 2^(-inf - m) = 0 either way
        }
        float s0 = __builtin_amdgcn_exp2f(fmaf(acc[0], c, -mnew));
        float s1 = __builtin_amdgcn_exp2f(fmaf(acc[1], c, -mnew));
        float s2 = __builtin_amdgcn_exp2f(fmaf(acc[2], c, -mnew));
        float s3 = __builtin_amdgcn_exp2f(fmaf(acc[3], c, -mnew));
#pragma unroll
        for (int v = 4; v < 16; v += 4) {
            s0 += __builtin_amdgcn_exp2f(fmaf(acc[v + 0], c, -mnew));
            s1 += __builtin_amdgcn_exp2f(fmaf(acc[v + 1], c, -mnew));
            s2 += __builtin_amdgcn_exp2f(fmaf(acc[v + 2], c, -mnew));
            s3 += __builtin_amdgcn_exp2f(fmaf(acc[v + 3], c, -mnew));
        }
        if (FIXED) {
            z[qt] += (s0 + s1) + (s2 + s3);
            m[qt] = mnew;
        } else {
            z[qt] = z[qt] * __builtin_amdgcn_exp2f(m[qt] - mnew) + ((s0 + s1) + (s2 + s3));
            m[qt] = mnew;
        }
        if (qt + 1 < NQT) {
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);  // one MFMA
                __builtin_amdgcn_sched_group_barrier(0x002, 8, 0);  // then a few VALU
            }
        }
        __builtin_amdgcn_sched_barrier(0);
        acc = nxt;
    }
}

template <int NQT, bool PAGED>
__global__ __launch_bounds__(kScoreWaves * 64, 2) void jq_stats_kernel(ScoreArgs a) {
    __shared__ __attribute__((aligned(1024))) char lds[kScoreWaves][2][kSlotBytes];
    WaveItem w;
    wave_item(a, false, w);
    const int lane = threadIdx.x & 63;
    const int half = lane >> 5;
    char* slots = &lds[__builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6))][0][0];

    const KeyStream ks = key_stream<PAGED>(a, w);
    const TileLanes tl = tile_lanes(lane, ks.row_bytes);
    // With the soft tokens' own keys in the softmax, the sequence's first wave takes them as further tiles
    // after its prompt tiles (same row stride, n_q rows), masked causally per query row.
    const int n_tail = (a.K_tail && w.wave == 0) ? (a.n_q + kKeyTile - 1) / kKeyTile : 0;  // wave 0 always has tiles
    const int n_all = w.n_tiles + n_tail;
    __amdgpu_buffer_rsrc_t tail_rsrc = ks.rsrc;
    if (n_tail) {
        const char* kt = (const char*)a.K_tail + ((int64_t)(w.layer * a.n_seq + w.seq) * a.n_q * a.h_kv + w.g) * kHeadDim * 2;
        tail_rsrc = __builtin_amdgcn_make_buffer_rsrc((void*)kt, 0, (int)((uint32_t)(a.n_q - 1) * ks.row_bytes + kHeadDim * 2),
                                                      0x00020000);
    }
    // the wave's k-th tile is tile w.wave + k * w.n_waves of the sequence and uses slot k & 1.  PAGED: tiles are
    // requested in the order k = 0, 1, 2, ...; the table word of the NEXT request is loaded while this one is
    // issued, so its latency never sits in front of a tile's loads (`first_page` primes the sequence).
    int page_next = 0;
    auto first_page = [&]() __attribute__((always_inline)) { if (PAGED && w.n_tiles > 0) page_next = tile_page<PAGED>(ks, w.wave); };
    auto fetch = [&](int k) __attribute__((always_inline)) {
        if (k < w.n_tiles) {
            const int t = w.wave + k * w.n_waves;
            const int page = page_next;
            if (PAGED && k + 1 < w.n_tiles) page_next = tile_page<PAGED>(ks, t + w.n_waves);
            fetch_tile(ks.rsrc, slots + (k & 1) * kSlotBytes, tile_offset<PAGED>(ks, t, page), ks.row_bytes,
                       w.L - t * kKeyTile, tl, lane);
        } else {
            const int t = k - w.n_tiles;
            fetch_tile(tail_rsrc, slots + (k & 1) * kSlotBytes, (uint32_t)t * kKeyTile * ks.row_bytes, ks.row_bytes,
                       a.n_q - t * kKeyTile, tl, lane);
        }
    };
    // The first key tile goes to slot 0 at once; the second slots first serve as the staging area that turns
    // the workgroup's query rows into operand order.  From then on the wave's tiles alternate between its two
    // slots, and the next tile is requested as soon as the current one's fragments are in registers (with
    // a.depth == 2 the tile after that one is in flight as well).
    // As in the second pass the query rows are requested first, into registers, the key tile after them, and the
    // rows pass through LDS while the tile is in flight (explicit LDS instructions, every request unconditional in
    // one basic block: see lds_addr()).  A wave without tiles requests the sequence's first tile and drops it.
    bf16x8 qf[NQT][8];
    {
        const u32x4* qsrc[8];
        uint32_t qpad;
        q_rows_where<NQT>(a, w, lane, qsrc, qpad);
        const int t_first = w.n_tiles > 0 ? w.wave : 0;
        const int page_first = PAGED ? tile_page<PAGED>(ks, t_first) : 0;
        if (PAGED && w.n_tiles > 1) page_next = tile_page<PAGED>(ks, t_first + w.n_waves);
        const uint32_t off_first = tile_offset<PAGED>(ks, t_first, page_first);
        const int valid_first = min(kKeyTile, w.L - t_first * kKeyTile);
        __builtin_amdgcn_sched_barrier(0);
        u32x4 qraw[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) qraw[i] = *qsrc[i];
        __builtin_amdgcn_sched_barrier(0);
        fetch_tile_any(ks.rsrc, slots, off_first, ks.row_bytes, valid_first, lane);
        __builtin_amdgcn_sched_barrier(0);
        q_rows_stage<NQT>(lane, &lds[0][0][0], qraw, qpad, qf);
    }
    const float c = a.c;
    float m[NQT], z[NQT];
#pragma unroll
    for (int qt = 0; qt < NQT; ++qt) { m[qt] = -1.0e30f; z[qt] = 0.0f; }
    if (n_all > 0) {  // not a surplus wave of the sequence's last workgroup
    const int D = a.depth;  // uniform
    if (D == 2 && n_all > 1) fetch(1);

    // Every load older than the second tile's eight (first tile, query rows) is covered
    // by the first wait of the sweep.  Tiles that lie entirely inside the keys every query row sees (all L
    // prompt keys, or the L - n_q keys in front of the window when the queries are the prompt's own last
    // tokens) need no mask; the others -- the sequence's partial last tile, the window's tiles -- are the
    // last of the tiles of whichever waves own them.
    const int n_common = a.window ? w.L - a.n_q : w.L;
    const int common_tiles = n_common / kKeyTile;  // sequence tiles 0 .. common_tiles - 1 are unmasked
    const int n_full = common_tiles > w.wave ? min(w.n_tiles, (common_tiles - 1 - w.wave) / w.n_waves + 1) : 0;
    // soft token of this lane's query row in each query tile (row r = i * group + hh): it sees soft tokens 0..i
    int soft_i[NQT];
#pragma unroll
    for (int qt = 0; qt < NQT; ++qt) soft_i[qt] = ((a.row_tile0 + qt) * kRowTile + (lane & 31)) / a.group;
    // The kernel holds TWO copies of the tile body, not one per case: the hot one (unmasked tile, offsets fixed
    // after the wave's first tile) and a general one whose masking and offset rule are run-time flags, used by the
    // few masked tiles (partial last tile, window, soft tokens' own keys) and by the rare repeat of a sweep.
    // (A copy per case made the kernel 45 KB of code instead of 23 KB, for no gain in time.)
    auto tile_prologue = [&](int k, bf16x8 (&kf)[8]) __attribute__((always_inline)) {
        wait_tile_landed(D == 2 && k + 1 < n_all);
        lds_get_frags(slots + (k & 1) * kSlotBytes, kf, lane);
        if (k + D < n_all) {
            wait_frags_read();
            fetch(k + D);
        }
    };
    // rows of tile k that exist for this lane's query row of each query tile (32 or more: all of them)
    auto valid_rows = [&](int k, int (&valid)[NQT]) __attribute__((always_inline)) {
        if (k < w.n_tiles) {
            const int t0 = (w.wave + k * w.n_waves) * kKeyTile;
#pragma unroll
            for (int qt = 0; qt < NQT; ++qt) valid[qt] = (a.window ? n_common + soft_i[qt] + 1 : w.L) - t0;
        } else {  // soft token t * 32 + j is visible to the row of soft token i iff it is <= i
            const int t = k - w.n_tiles;
#pragma unroll
            for (int qt = 0; qt < NQT; ++qt) valid[qt] = soft_i[qt] + 1 - t * kKeyTile;
        }
    };
    // First sweep: the wave's first tile sets each lane's offset m from its logits there, later tiles keep it --
    // no maximum to track.  A logit more than 2^7 (base 2) above that offset overflows 2^(t - m) to infinity, which
    // cannot be repaired afterwards, so such a wave (wave-uniform decision) sweeps again with the running maximum.
    int k = 0;
    for (; k < n_full; ++k) {
        bf16x8 kf[8];
        tile_prologue(k, kf);
        int valid[NQT];
#pragma unroll
        for (int qt = 0; qt < NQT; ++qt) valid[qt] = kKeyTile;
        stats_tile<NQT, false, true>(kf, qf, m, z, c, valid, half, k == 0);
    }
    bool repeat = false;  // uniform
    for (;;) {
        for (; k < n_all; ++k) {
            bf16x8 kf[8];
            tile_prologue(k, kf);
            int valid[NQT];
            valid_rows(k, valid);
            stats_tile<NQT, true, false>(kf, qf, m, z, c, valid, half, !repeat && k > 0);
        }
        bool overflow = false;
#pragma unroll
        for (int qt = 0; qt < NQT; ++qt) overflow |= !(z[qt] < INFINITY);
        if (repeat || !__builtin_expect(__any(overflow), 0)) break;
        repeat = true;
#pragma unroll
        for (int qt = 0; qt < NQT; ++qt) { m[qt] = -1.0e30f; z[qt] = 0.0f; }
        wait_frags_read();
        first_page();
        fetch(0);
        if (D == 2 && n_all > 1) fetch(1);
        k = 0;
    }

    }  // n_all > 0

    // Lanes l and l+32 hold the same query rows over complementary keys: merge them; then the four waves of
    // the workgroup merge their rows through LDS (every slot is idle by now), in wave order, into the one
    // partial the workgroup leaves per query row.
    float2* mine = (float2*)slots;  // [NQT * 32] of this wave
#pragma unroll
    for (int qt = 0; qt < NQT; ++qt) {
        const float mo = __shfl_xor(m[qt], 32), zo = __shfl_xor(z[qt], 32);
        const float mm = fmaxf(m[qt], mo);
        const float zz = z[qt] * __builtin_amdgcn_exp2f(m[qt] - mm) + zo * __builtin_amdgcn_exp2f(mo - mm);
        if (half == 0) mine[qt * kRowTile + lane] = make_float2(mm, zz);
    }
    __syncthreads();
    if (threadIdx.x < NQT * kRowTile) {
        float M = -1.0e30f, Z = 0.f;
#pragma unroll
        for (int wv = 0; wv < kScoreWaves; ++wv) {
            const float2 mz = ((const float2*)&lds[wv][0][0])[threadIdx.x];
            const float mm = fmaxf(M, mz.x);
            Z = Z * __builtin_amdgcn_exp2f(M - mm) + mz.y * __builtin_amdgcn_exp2f(mz.x - mm);
            M = mm;
        }
        const int cg = (a.one_L ? 0 : a.tab.cu_cgrp[w.seq]) + w.wave / kScoreWaves;  // this workgroup among the layer's, per head
        a.stats[(((int64_t)w.layer * a.n_cgrp + cg) * a.h_kv + w.g) * a.RP + a.row_tile0 * kRowTile + threadIdx.x] = make_float2(M, Z);
    }
}

// The instance of the headline shape (128 query rows per KV head, dense cache), emitted here so that it lies next
// to the other kernels of a step in the library's code (see jq_lib.hip).
template __global__ void jq_stats_kernel<4, false>(ScoreArgs);

// -beta/c as the three truncated bf16 terms that enter the second pass through its extra MFMA step.
__device__ __forceinline__ uint2 split_bf16x3(float x) {
    const uint32_t hi = __float_as_uint(x) & 0xFFFF0000u;
    const float r1 = x - __uint_as_float(hi);
    const uint32_t mid = __float_as_uint(r1) & 0xFFFF0000u;
    const float r2 = r1 - __uint_as_float(mid);
    const uint32_t lo = __float_as_uint(r2) & 0xFFFF0000u;
    return make_uint2((hi >> 16) | mid, lo >> 16);
}

constexpr int kCombineLanes = 32;  // partial-lanes per query row
__global__ __launch_bounds__(kRowTile * kCombineLanes) void jq_combine_kernel(ScoreArgs a) {
    // one workgroup per (layer, sequence, head, tile of 32 rows); thread = (row r, partial-lane kl)
    __shared__ float2 part[kCombineLanes][kRowTile];
    const int r = threadIdx.x & (kRowTile - 1), kl = threadIdx.x / kRowTile;
    const int tiles = a.RP / kRowTile;
    const int rt = blockIdx.x % tiles;
    int rest = blockIdx.x / tiles;
    const int g = rest % a.h_kv;
    rest /= a.h_kv;
    const int s = rest % a.n_seq;
    const int layer = rest / a.n_seq;
    const int row = rt * kRowTile + r;

    if (a.zero) {  // clear the selection histograms and counters while we are here
        const uint64_t per = (a.zero_words + gridDim.x - 1) / gridDim.x;
        const uint64_t z0 = per * blockIdx.x, z1 = z0 + per < a.zero_words ? z0 + per : a.zero_words;
        for (uint64_t i = z0 + threadIdx.x; i < z1; i += blockDim.x) a.zero[i] = 0u;
    }

    const int c0 = a.tab.cu_cgrp[s], c1 = a.tab.cu_cgrp[s + 1];
    const float2* p = a.stats + (((int64_t)layer * a.n_cgrp + c0) * a.h_kv + g) * a.RP + row;
    const int64_t step = (int64_t)a.h_kv * a.RP;
    float M = -1.0e30f, Z = 0.f;
    for (int k0 = kl; k0 < c1 - c0; k0 += 8 * kCombineLanes) {  // 8 independent loads in flight per thread
        float2 mz[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int k = k0 + u * kCombineLanes;
            mz[u] = k < c1 - c0 ? p[k * step] : make_float2(-1.0e30f, 0.f);
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const float mm = fmaxf(M, mz[u].x);
            Z = Z * __builtin_amdgcn_exp2f(M - mm) + mz[u].y * __builtin_amdgcn_exp2f(mz[u].x - mm);
            M = mm;
        }
    }
    part[kl][r] = make_float2(M, Z);
    __syncthreads();
    if (kl != 0) return;
    for (int k = 1; k < kCombineLanes; ++k) {  // fixed order: deterministic
        const float2 mz = part[k][r];
        const float mm = fmaxf(M, mz.x);
        Z = Z * __builtin_amdgcn_exp2f(M - mm) + mz.y * __builtin_amdgcn_exp2f(mz.x - mm);
        M = mm;
    }
    // padded rows (row >= rows) get 2^(c*x) = 0
    const float x = row < a.rows ? -(M + __log2f(Z)) / a.c : -1.0e30f;
    a.aug[((int64_t)(layer * a.n_seq + s) * a.h_kv + g) * a.RP + row] = split_bf16x3(x);
}

// ------------------------------------------------------------------------------------------------
// pass 2: normalised probabilities summed over the query rows
// ------------------------------------------------------------------------------------------------
// q.k - beta/c for one tile of 32 query rows against the 32 keys in `kf` (rows = query rows, columns = keys).
__device__ __forceinline__ f32x16 score_chain(const bf16x8 (&q)[8], bf16x8 qaug, const bf16x8 (&kf)[8], bf16x8 ones) {
    f32x16 acc = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int k8 = 0; k8 < 8; ++k8) acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(q[k8], kf[k8], acc, 0, 0, 0);
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(qaug, ones, acc, 0, 0, 0);  // - beta_r / c
}

// FROM_LSE: the caller supplied the normalisers and no statistics pass has run: lse becomes the -beta/c terms
// on the fly (beta = lse * log2 e, c = scale * log2 e, so -beta/c = -lse / scale), and the launch also clears
// the words the selection stage needs cleared.
// DIFF: the scores are not stored; (ref / rows_ref - score / rows_own)^2 is summed instead (Eq. 5 of the paper on
// the maps of Eq. 3 and Eq. 4), in fp64 per lane, then in a fixed order over lanes and waves.
template <int NQT, bool FROM_LSE, bool PAGED, bool DIFF = false>
__global__ __launch_bounds__(kScoreWaves * 64, 2) void jq_score_kernel(ScoreArgs a) {
    __shared__ __attribute__((aligned(1024))) char lds[kScoreWaves][2][kSlotBytes];
    __shared__ double diff_s[DIFF ? kScoreWaves : 1];
    if (DIFF && threadIdx.x < kScoreWaves) diff_s[threadIdx.x] = 0.0;  // before the start-up's barriers
    WaveItem w;
    wave_item(a, true, w);  // reversed order: the keys pass 1 read last are fetched first
    const int lane = threadIdx.x & 63;
    const int half = lane >> 5;
    char* slots = &lds[__builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6))][0][0];

    const KeyStream ks = key_stream<PAGED>(a, w);
    const TileLanes tl = tile_lanes(lane, ks.row_bytes);
    // The wave walks its tiles from the last to the first (pass 1 swept the keys front to back, so the end
    // of the sequence is what the caches still hold): its k-th tile here is sequence tile tile_of(k).
    auto tile_of = [&](int k) { return w.wave + (w.n_tiles - 1 - k) * w.n_waves; };
    // PAGED: as in the first pass, the table word of the next request (k + 1) is loaded one request ahead
    int page_next = 0;  // set by the start-up's first request
    auto fetch = [&](int k) __attribute__((always_inline)) {
        const int t = tile_of(k);
        const int page = page_next;
        if (PAGED && k + 1 < w.n_tiles) page_next = tile_page<PAGED>(ks, t - w.n_waves);
        fetch_tile(ks.rsrc, slots + (k & 1) * kSlotBytes, tile_offset<PAGED>(ks, t, page), ks.row_bytes,
                   w.L - t * kKeyTile, tl, lane);
    };
    bf16x8 qf[NQT][8];
    bf16x8 qaug[NQT];
    // Start-up.  Requested first, into registers: the query rows, the first pass's partial statistics (or the
    // normalisers themselves); then the first key tile, straight into LDS.  Everything up to the sweep works on the
    // former while the latter is in flight (see lds_addr() above for why the LDS instructions here are explicit).
    // The compiler can only count on loads that are certain to have been issued, so every request below is
    // unconditional -- addresses are clamped, values that turn out not to be needed are dropped -- and all of them
    // sit in one basic block: then each wait is exactly "everything older than this value", never the key tile.
    const bool fused = !FROM_LSE && a.fuse_combine;  // uniform
    constexpr int kFirstParts = 16;  // partials per thread requested up front: all of them for up to 32 per row
    const int p0 = (int)(threadIdx.x & 1);
    // Pass 1 left one (m, Z) partial per workgroup; unless a combine launch has merged them already, this
    // workgroup merges the partials of its head's rows itself: thread t takes row t / 2 and every second
    // partial; pairs meet by shuffle, and the rows' -beta/c terms pass through LDS.
    const int mrow = min((int)(threadIdx.x >> 1), NQT * kRowTile - 1);
    const int c0 = (a.one_L || !fused) ? 0 : a.cu_part[w.seq];
    const int n_p = !fused ? 1 : a.one_L ? a.n_part : a.cu_part[w.seq + 1] - c0;
    const float2* pp = a.stats + (((int64_t)w.layer * a.n_part + c0) * a.h_kv + w.g) * a.RP + a.row_tile0 * kRowTile + mrow;
    const int64_t pstep = (int64_t)a.h_kv * a.RP;
    const u32x4* qsrc[8];
    uint32_t qpad;
    q_rows_where<NQT>(a, w, lane, qsrc, qpad);
    const float* nsrc[NQT];  // FROM_LSE: the lane's rows' normalisers; otherwise the merged -beta/c terms of a combine launch
#pragma unroll
    for (int qt = 0; qt < NQT; ++qt) {
        const int row = min((a.row_tile0 + qt) * kRowTile + (lane & 31), a.rows - 1);
        if (FROM_LSE) {
            const int i = row / a.group, h = w.g * a.group + row % a.group;
            nsrc[qt] = a.lse + ((int64_t)(w.layer * a.n_seq + w.seq) * a.n_q + i) * a.h_q + h;
        } else {
            nsrc[qt] = (const float*)(a.aug + ((int64_t)(w.layer * a.n_seq + w.seq) * a.h_kv + w.g) * a.RP + (a.row_tile0 + qt) * kRowTile + (lane & 31));
        }
    }
    const int t_first = w.n_tiles > 0 ? tile_of(0) : 0;  // a surplus wave requests the sequence's first tile and drops it
    const int page_first = PAGED ? tile_page<PAGED>(ks, t_first) : 0;
    if (PAGED && w.n_tiles > 1) page_next = tile_page<PAGED>(ks, t_first - w.n_waves);
    const uint32_t off_first = tile_offset<PAGED>(ks, t_first, page_first);
    const int valid_first = min(kKeyTile, w.L - t_first * kKeyTile);
    __builtin_amdgcn_sched_barrier(0);
    u32x4 qraw[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) qraw[i] = *qsrc[i];
    float2 mz[kFirstParts];
#pragma unroll
    for (int u = 0; u < kFirstParts; ++u) mz[u] = pp[min(p0 + 2 * u, n_p - 1) * pstep];
    uint2 aug_direct[NQT];
#pragma unroll
    for (int qt = 0; qt < NQT; ++qt) {
        if (FROM_LSE) aug_direct[qt] = make_uint2(__float_as_uint(*nsrc[qt]), 0u);
        else aug_direct[qt] = *(const uint2*)nsrc[qt];
    }
    __builtin_amdgcn_sched_barrier(0);
    fetch_tile_any(ks.rsrc, slots, off_first, ks.row_bytes, valid_first, lane);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int u = 0; u < kFirstParts; ++u)
        if (!fused || p0 + 2 * u >= n_p) mz[u] = make_float2(-1.0e30f, 0.f);
    const bool merges = fused && (threadIdx.x >> 1) < NQT * kRowTile;
    if (FROM_LSE) {
#pragma unroll
        for (int qt = 0; qt < NQT; ++qt) {
            const int row = (a.row_tile0 + qt) * kRowTile + (lane & 31);
            // padded rows get 2^(c*x) = 0
            aug_direct[qt] = split_bf16x3(row < a.rows ? -__uint_as_float(aug_direct[qt].x) * a.inv_scale : -1.0e30f);
        }
    }
    q_rows_stage<NQT>(lane, &lds[0][0][0], qraw, qpad, qf);
    float cM = -1.0e30f, cZ = 0.f;
    auto merge_in = [&](float2 t) __attribute__((always_inline)) {
        const float mm = fmaxf(cM, t.x);
        cZ = cZ * __builtin_amdgcn_exp2f(cM - mm) + t.y * __builtin_amdgcn_exp2f(t.x - mm);
        cM = mm;
    };
    if (merges) {  // ascending partial index, the same order whatever their number
#pragma unroll
        for (int u = 0; u < kFirstParts; ++u) merge_in(mz[u]);
        for (int k0 = p0 + 2 * kFirstParts; k0 < n_p; k0 += 16) {  // a sequence that left more than 32 partials
            float2 more[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) more[u] = k0 + 2 * u < n_p ? pp[(k0 + 2 * u) * pstep] : make_float2(-1.0e30f, 0.f);
#pragma unroll
            for (int u = 0; u < 8; ++u) merge_in(more[u]);
        }
    }
    auto set_aug = [&](int qt, uint2 t) {  // the three bf16 terms sit in k-elements 0..2 of the extra MFMA step (lane half 0)
        u32x4 v = {0u, 0u, 0u, 0u};
        if (half == 0) { v[0] = t.x; v[1] = t.y; }
        qaug[qt] = as_bf16x8(v);
    };
    if (fused) {
        const float oM = __shfl_xor(cM, 1), oZ = __shfl_xor(cZ, 1);  // the odd neighbour's half; even threads finish the row
        const float mm = fmaxf(cM, oM);
        const float zz = cZ * __builtin_amdgcn_exp2f(cM - mm) + oZ * __builtin_amdgcn_exp2f(oM - mm);
        const int crow = a.row_tile0 * kRowTile + (int)(threadIdx.x >> 1);
        const uint32_t aug_s = lds_addr(&lds[0][1][0]);  // the query rows have left this slot (second barrier of q_rows_stage)
        if (!(threadIdx.x & 1) && (threadIdx.x >> 1) < NQT * kRowTile) {
            lds_put8(aug_s + 8u * (threadIdx.x >> 1), split_bf16x3(crow < a.rows ? -(mm + __log2f(zz)) / a.c : -1.0e30f));
            lds_wait_all();
        }
        bare_barrier();
#pragma unroll
        for (int qt = 0; qt < NQT; ++qt) set_aug(qt, lds_get8_waited(aug_s + 8u * (qt * kRowTile + (lane & 31))));
        bare_barrier();  // the slot is refilled with a key tile next
    } else {
#pragma unroll
        for (int qt = 0; qt < NQT; ++qt) set_aug(qt, aug_direct[qt]);
    }
    if (a.zero) {  // words the selection needs cleared (stores: they only join the loads the sweep's first wait covers)
        const uint64_t per = (a.zero_words + gridDim.x - 1) / gridDim.x;
        const uint64_t z0 = per * blockIdx.x, z1 = z0 + per < a.zero_words ? z0 + per : a.zero_words;
        for (uint64_t i = z0 + threadIdx.x; i < z1; i += blockDim.x) a.zero[i] = 0u;
    }
    if (w.n_tiles == 0) {  // surplus wave of the sequence's last workgroup
        if (DIFF) __syncthreads();  // the workgroup's final merge
        return;
    }
    const int D = a.depth;  // uniform
    if (D == 2 && w.n_tiles > 1) fetch(1);
    u32x4 ones_bits = {0u, 0u, 0u, 0u};
    if (half == 0) { ones_bits[0] = 0x3F803F80u; ones_bits[1] = 0x00003F80u; }  // 1.0 at elements 0..2
    const bf16x8 ones = as_bf16x8(ones_bits);

    float* out = a.scores + ((int64_t)w.layer * a.h_kv + w.g) * a.T + w.tok0;
    const float c = a.c;
    float pending = 0.f;  // previous tile's result, stored one iteration late so that the store has a
                          // whole tile of compute to retire before the next wait on outstanding loads
    const int n_scored = a.window ? w.L - a.n_q : w.L;  // the window's own positions report 0
    double dacc = 0.0;  // DIFF: this lane's sum of squared map differences
    auto store_tile = [&](int k, float v) {  // only the sequence's last tile can be partial
        const int t = tile_of(k);
        if (lane < 32 && t * kKeyTile + lane < w.L) {
            float* o = out + t * kKeyTile + lane;
            if (t * kKeyTile + lane >= n_scored) v = 0.f;
            if (DIFF) {
                const float own = a.accumulate ? *o + v : v;
                const double d = (double)a.diff_ref[o - a.scores] * (double)a.diff_inv_ref - (double)own * (double)a.diff_inv_own;
                dacc += d * d;
            } else {
                *o = a.accumulate ? *o + v : v;
            }
        }
    };

    // everything older than the second tile's eight loads (first tile, Q, the -beta/c terms) is in after this
    wait_tile_landed(D == 2 && w.n_tiles > 1);
    for (int k = 0; k < w.n_tiles; ++k) {
        if (k > 0) wait_tile_landed(D == 2 && k + 1 < w.n_tiles);
        bf16x8 kf[8];
        lds_get_frags(slots + (k & 1) * kSlotBytes, kf, lane);
        if (k > 0) store_tile(k - 1, pending);
        if (k + D < w.n_tiles) {  // issued after the store: only these 8 loads are newer than tile k+1
            wait_frags_read();
            fetch(k + D);
        }
        // Software pipeline over the query-row tiles: the MFMA chain of tile qt+1 is issued between the
        // exp2/add instructions of tile qt (a wave issues in order, so without interleaving its VALU work
        // would sit behind the whole dependent MFMA chain).
        float s0 = 0.f, s1 = 0.f, s2 = 0.f, s3 = 0.f;
        f32x16 acc = score_chain(qf[0], qaug[0], kf, ones);
#pragma unroll
        for (int qt = 0; qt < NQT; ++qt) {
            f32x16 nxt = acc;
            if (qt + 1 < NQT) nxt = score_chain(qf[qt + 1], qaug[qt + 1], kf, ones);
#pragma unroll
            for (int v = 0; v < 16; v += 4) {
                s0 += __builtin_amdgcn_exp2f(acc[v + 0] * c);
                s1 += __builtin_amdgcn_exp2f(acc[v + 1] * c);
                s2 += __builtin_amdgcn_exp2f(acc[v + 2] * c);
                s3 += __builtin_amdgcn_exp2f(acc[v + 3] * c);
            }
            if (qt + 1 < NQT) {
#pragma unroll
                for (int i = 0; i < 9; ++i) {
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);  // one MFMA
                    __builtin_amdgcn_sched_group_barrier(0x002, 5, 0);  // then a few VALU
                }
            }
            __builtin_amdgcn_sched_barrier(0);
            acc = nxt;
        }
        float s = (s0 + s1) + (s2 + s3);
        s += __shfl_xor(s, 32);  // the two lane halves hold complementary query rows of the same key
        pending = s;
    }
    store_tile(w.n_tiles - 1, pending);
    if (DIFF) {  // lanes 0..31 hold the sums: butterfly within the half wave, then the four waves in wave order
#pragma unroll
        for (int off = 16; off >= 1; off >>= 1) dacc += __shfl_xor(dacc, off);
        const int wv = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
        if (lane == 0) diff_s[wv] = dacc;
        __syncthreads();
        if (threadIdx.x == 0) {
            const int cg = (a.one_L ? 0 : a.tab.cu_cgrp[w.seq]) + w.wave / kScoreWaves;  // wave 0 always has tiles
            double sum = 0.0;
#pragma unroll
            for (int i = 0; i < kScoreWaves; ++i) sum += diff_s[i];
            a.diff_part[((int64_t)w.layer * a.n_cgrp + cg) * a.h_kv + w.g] = sum;
        }
    }
}

template __global__ void jq_score_kernel<4, false, false, false>(ScoreArgs);  // placement: see jq_lib.hip

// ------------------------------------------------------------------------------------------------
// host side
// ------------------------------------------------------------------------------------------------
template <bool PAGED>
static hipError_t launch_stats_n(int nqt, const ScoreArgs& a, dim3 grid, hipStream_t st, void* const* marks) {
    dim3 block(kScoreWaves * 64);
    switch (nqt) {
        case 1: return launch_kernel(jq_stats_kernel<1, PAGED>, grid, block, 0, st, marks, kTrStats, a);
        case 2: return launch_kernel(jq_stats_kernel<2, PAGED>, grid, block, 0, st, marks, kTrStats, a);
        case 3: return launch_kernel(jq_stats_kernel<3, PAGED>, grid, block, 0, st, marks, kTrStats, a);
        default: return launch_kernel(jq_stats_kernel<4, PAGED>, grid, block, 0, st, marks, kTrStats, a);
    }
}

template <bool FROM_LSE, bool PAGED>
static hipError_t launch_score_n(int nqt, const ScoreArgs& a, dim3 grid, hipStream_t st, void* const* marks) {
    dim3 block(kScoreWaves * 64);
    switch (nqt) {
        case 1: return launch_kernel(jq_score_kernel<1, FROM_LSE, PAGED>, grid, block, 0, st, marks, kTrScore, a);
        case 2: return launch_kernel(jq_score_kernel<2, FROM_LSE, PAGED>, grid, block, 0, st, marks, kTrScore, a);
        case 3: return launch_kernel(jq_score_kernel<3, FROM_LSE, PAGED>, grid, block, 0, st, marks, kTrScore, a);
        default: return launch_kernel(jq_score_kernel<4, FROM_LSE, PAGED>, grid, block, 0, st, marks, kTrScore, a);
    }
}

static hipError_t launch_score_diff_n(int nqt, const ScoreArgs& a, dim3 grid, hipStream_t st) {
    dim3 block(kScoreWaves * 64);
    switch (nqt) {
        case 1: return launch_kernel(jq_score_kernel<1, false, false, true>, grid, block, 0, st, nullptr, -1, a);
        case 2: return launch_kernel(jq_score_kernel<2, false, false, true>, grid, block, 0, st, nullptr, -1, a);
        case 3: return launch_kernel(jq_score_kernel<3, false, false, true>, grid, block, 0, st, nullptr, -1, a);
        default: return launch_kernel(jq_score_kernel<4, false, false, true>, grid, block, 0, st, nullptr, -1, a);
    }
}

hipError_t launch_score(const Plan& p, const void* Q, const void* K, float* scores, char* ws, hipStream_t st,
                        uint32_t* zero, size_t zero_words, const float* lse, const void* k_tail, const MseFuse* fuse) {
    void* const* marks = p.marks;
    ScoreArgs a;
    a.Q = (const uint16_t*)Q;
    a.K = (const uint16_t*)K;
    a.K_tail = (const uint16_t*)k_tail;
    a.stats = (float2*)(ws + p.off_stats);
    a.aug = (uint2*)(ws + p.off_aug);
    a.scores = scores;
    a.n_layers = p.n_layers; a.n_seq = p.n_seq; a.n_q = p.n_q; a.h_q = p.h_q; a.h_kv = p.h_kv;
    a.group = p.group; a.rows = p.rows; a.RP = p.row_tiles * kRowTile;
    a.window = p.window;
    // Key tiles a wave keeps in flight: one.  The next tile is requested as soon as the current one's fragments are
    // in registers and arrives while the wave computes; a second tile in flight only queues in the memory system
    // (both passes already move data at the rate a plain read of K reaches) and costs the second pass 2.5 us on
    // the 128K layer (46.7 -> 44.2 us; first pass 47.3 -> 46.8).
    const int depth_cold = knobs().depth1, depth_second = knobs().depth2;  // ablation knobs (default 1)
    a.depth = depth_cold;
    a.group_shift = -1;
    for (int sh = 0; sh < 16; ++sh)
        if (p.group == (1 << sh)) a.group_shift = sh;
    a.row_tile0 = 0; a.accumulate = 0;
    a.c = p.scale * 1.4426950408889634f;
    a.T = p.T;
    a.zero = zero; a.zero_words = zero_words;
    a.tab = p.tab;
    a.block_table = p.block_table; a.page_shift = p.page_shift; a.n_pages = p.n_pages; a.max_pages = p.max_pages;
    a.diff_ref = nullptr; a.diff_part = nullptr; a.diff_inv_ref = a.diff_inv_own = 0.0f;
    const bool paged = p.block_table != nullptr;
    if (fuse && (paged || lse)) return hipErrorInvalidValue;  // the fused comparison exists for dense two-pass calls
    a.chunk_keys = p.chunk_keys; a.n_chunks = p.n_chunks;
    a.n_cgrp = p.tab.cu_cgrp[p.n_seq];
    a.one_L = p.n_seq == 1 ? p.tab.cu_seq[1] : 0;
    a.one_waves = p.n_seq == 1 ? p.tab.cu_chunk[1] : 0;

    dim3 grid((unsigned)((int64_t)p.n_layers * a.n_cgrp * p.h_kv));
    hipError_t e;
    a.lse = lse;
    a.inv_scale = 1.0f / p.scale;
    a.n_part = 0; a.fuse_combine = 0;
    for (int s = 0; s <= p.n_seq; ++s) a.cu_part[s] = 0;
    if (!lse) {
        for (int rg = 0; rg < p.row_groups; ++rg) {
            a.row_tile0 = rg * kMaxRowTiles;
            const int nqt = min(kMaxRowTiles, p.row_tiles - a.row_tile0);
            e = paged ? launch_stats_n<true>(nqt, a, grid, st, marks) : launch_stats_n<false>(nqt, a, grid, st, marks);
            if (e != hipSuccess) return e;
        }
        // Pass 1 leaves one partial per workgroup.  With few of them per sequence every pass-2 workgroup merges
        // its head's partials itself; a very long sequence has hundreds, and then one small launch merges them
        // once (and clears the selection's words on the way).
        int max_parts = 0;
        for (int s = 0; s < p.n_seq; ++s) max_parts = max(max_parts, p.tab.cu_cgrp[s + 1] - p.tab.cu_cgrp[s]);
        a.fuse_combine = max_parts <= 64;
        if (!a.fuse_combine) {
            const int64_t n_row_tiles = (int64_t)p.n_layers * p.n_seq * p.h_kv * p.row_tiles;
            e = launch_kernel(jq_combine_kernel, dim3((unsigned)n_row_tiles), dim3(kRowTile * kCombineLanes), 0, st, nullptr, -1, a);
            if (e != hipSuccess) return e;
            a.zero = nullptr;  // done by the combine launch
        }
        // the second pass cuts the sequences into its own number of waves
        a.n_part = a.n_cgrp;
        for (int s = 0; s <= p.n_seq; ++s) a.cu_part[s] = p.tab.cu_cgrp[s];
        a.chunk_keys = p.chunk_keys2; a.n_chunks = p.n_chunks2;
        for (int s = 0; s <= p.n_seq; ++s) { a.tab.cu_chunk[s] = p.cu_chunk2[s]; a.tab.cu_cgrp[s] = p.cu_cgrp2[s]; }
        a.n_cgrp = p.cu_cgrp2[p.n_seq];
        a.one_waves = p.n_seq == 1 ? p.cu_chunk2[1] : 0;
        grid = dim3((unsigned)((int64_t)p.n_layers * a.n_cgrp * p.h_kv));
        a.depth = depth_second;
    }
    for (int rg = 0; rg < p.row_groups; ++rg) {
        a.row_tile0 = rg * kMaxRowTiles;
        a.accumulate = rg > 0;
        if (rg > 0) a.zero = nullptr;  // cleared once, by the first launch (normalisers supplied: no combine step does it)
        const int nqt = min(kMaxRowTiles, p.row_tiles - a.row_tile0);
        if (fuse && rg == p.row_groups - 1) {  // the last row group completes the scores: compare instead of storing
            a.diff_ref = fuse->ref; a.diff_part = fuse->part;
            a.diff_inv_ref = fuse->inv_rows_ref; a.diff_inv_own = fuse->inv_rows_own;
            e = launch_score_diff_n(nqt, a, grid, st);
            if (e != hipSuccess) return e;
            continue;
        }
        if (paged) e = lse ? launch_score_n<true, true>(nqt, a, grid, st, marks) : launch_score_n<false, true>(nqt, a, grid, st, marks);
        else e = lse ? launch_score_n<true, false>(nqt, a, grid, st, marks) : launch_score_n<false, false>(nqt, a, grid, st, marks);
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

}  // namespace jq
