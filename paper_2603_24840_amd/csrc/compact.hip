// arrol_compact: gather the survivors' paged KV cache, block tables and token buffers into a
// dense destination pool (Sec. 4.3 (i): pruned requests leave the pool and their capacity is
// reused; (ii) / Alg. 1: survivors are filtered and re-batched).
//
// Two launches on the caller's stream, no host round trip:
//   plan  one workgroup: pages per survivor, exclusive prefix scan (wave scan + LDS carry),
//         destination block tables / lengths / source map / page count.
//   copy  HBM streaming: one 512-lane workgroup per (layer, K|V, survivor, logical page) chunk,
//         every lane moving 16 bytes per access (non-temporal), the loads of a 16 KiB pass issued
//         before its stores; extra workgroups move the token rows.  Within a (layer, K|V) slab the
//         grid visits the destination pages as 8 interleaved ascending streams (stream_order).
#include "common.h"

namespace {

constexpr int kPlanThreads = 1024;
constexpr int kCopyThreads = 512;  // measured: 512 lanes x 2 accesses per 16 KiB chunk streams fastest
constexpr int kCopyUnroll = 2;     // 16-byte accesses per lane issued before the stores
constexpr unsigned kCopyStreams = 8;

// Visiting order of n equally sized pieces of work whose addresses ascend with their index: position k of the
// launch order takes piece stream_order(k, n).  The n pieces are cut into kCopyStreams contiguous parts (the first
// ones one piece longer when n is no multiple); consecutive positions take the next piece of
// consecutive parts, so the workgroups in flight at any time write to (and, for sorted sources, read from) 8
// regions spread over the slab instead of one.  A bijection of [0, n) for every n >= 1.  Measured on the
// benchmark pools against plain ascending order: +4 % for the out-of-place copy with 32 KiB chunks (6.0-6.1 TB/s
// on the 120 and 155 GB pools), +1 % with 16 KiB chunks, +10 % for the in-place copy with 16 KiB chunks; 2, 4,
// 16 and 32 streams were all slower than 8 on the large pools.
__device__ __forceinline__ unsigned stream_order(unsigned k, unsigned n) {
    const unsigned len = (n + kCopyStreams - 1) / kCopyStreams;     // pieces of a long part
    const unsigned n_long = n - (len - 1) * kCopyStreams;           // parts 0 .. n_long-1 hold len pieces, the rest len-1
    // round `round` takes piece `round` of every part that has one: in the last round (len - 1) only the n_long
    // long parts, and k < n leaves exactly those
    const unsigned round = k / kCopyStreams, part = k - round * kCopyStreams;
    return (part < n_long ? part * len : n_long * len + (part - n_long) * (len - 1)) + round;
}

// compute units of the current device, looked up once per device (0 on failure)
int compute_units() {
    static std::atomic<int> cached[64];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 0;
    int n = cached[dev].load(std::memory_order_acquire);
    if (n > 0) return n;
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) return 0;
    cached[dev].store(n, std::memory_order_release);
    return n;
}

__device__ __forceinline__ int pages_of(const int32_t* seq_len_src, int src, int n_src, int page_tokens, int ppr) {
    if (src < 0 || src >= n_src) return 0;
    const int len = seq_len_src[src];
    if (len <= 0) return 0;
    const int np = (len - 1) / page_tokens + 1;
    return np < ppr ? np : ppr;
}

// workspace layout: int32 base[n_keep + 1]
__global__ __launch_bounds__(kPlanThreads) void compact_plan_kernel(
    const int32_t* __restrict__ survivor_idx, const int32_t* __restrict__ seq_len_src, int n_src, int n_keep,
    int page_tokens, int ppr, int32_t* __restrict__ base, int32_t* __restrict__ block_table_dst,
    int32_t* __restrict__ seq_len_dst, int32_t* __restrict__ src_of_dst, int64_t* __restrict__ n_pages_used) {
    __shared__ int wave_tot[kPlanThreads / ARROL_WAVE];
    __shared__ int carry_s;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    if (tid == 0) carry_s = 0;
    __syncthreads();
    for (int r0 = 0; r0 < n_keep; r0 += kPlanThreads) {
        const int r = r0 + tid;
        int src = -1, np = 0;
        if (r < n_keep) {
            src = survivor_idx[r];
            np = pages_of(seq_len_src, src, n_src, page_tokens, ppr);
        }
        int incl = np;  // inclusive scan inside the wave
#pragma unroll
        for (int o = 1; o < ARROL_WAVE; o <<= 1) {
            const int v = __shfl_up(incl, o, ARROL_WAVE);
            if (lane >= o) incl += v;
        }
        if (lane == 63) wave_tot[wave] = incl;
        __syncthreads();
        int before = carry_s;
        for (int wv = 0; wv < wave; ++wv) before += wave_tot[wv];
        const int excl = before + incl - np;
        if (r < n_keep) {
            const bool valid = src >= 0 && src < n_src;
            base[r] = excl;
            seq_len_dst[r] = valid ? seq_len_src[src] : 0;
            src_of_dst[r] = valid ? src : -1;
        }
        __syncthreads();
        if (tid == kPlanThreads - 1) carry_s = excl + np;
        __syncthreads();
    }
    if (tid == 0) {
        base[n_keep] = carry_s;
        *n_pages_used = carry_s;
    }
    // block tables: base[] was written by this workgroup; make it visible, then fill rows
    __syncthreads();
    const int64_t total = static_cast<int64_t>(n_keep) * ppr;
    for (int64_t i = tid; i < total; i += kPlanThreads) {
        const int r = static_cast<int>(i / ppr), p = static_cast<int>(i % ppr);
        const int np = base[r + 1] - base[r];
        block_table_dst[i] = p < np ? base[r] + p : -1;
    }
}

// UNROLL 16-byte accesses per lane are issued before the stores: 2 for chunks below 32 KiB (one pass per 16 KiB
// chunk), 4 from 32 KiB on (a whole 32 KiB chunk in flight: +1-2 % on the 120 and 155 GB pools, nothing at 16 KiB)
template <int UNROLL>
__global__ __launch_bounds__(kCopyThreads) void compact_copy_kernel(
    const u32x4* __restrict__ kv_src, u32x4* __restrict__ kv_dst, int64_t chunk_vec, int64_t src_pages,
    int64_t dst_pages, const int32_t* __restrict__ block_table_src, const int32_t* __restrict__ survivor_idx,
    const int32_t* __restrict__ base, int n_src, int n_keep, int ppr, int64_t kv_blocks,
    const int32_t* __restrict__ tokens_src, int32_t* __restrict__ tokens_dst, int max_len) {
    const int64_t bid = blockIdx.x;
    if (bid < kv_blocks) {
        // bid = slab * (n_keep * ppr) + position; the position's slot r * ppr + p follows stream_order
        const int64_t slots = static_cast<int64_t>(n_keep) * ppr;
        const int64_t slab = bid / slots;
        const int64_t slot = stream_order(static_cast<unsigned>(bid - slab * slots), static_cast<unsigned>(slots));
        const int r = static_cast<int>(slot / ppr), p = static_cast<int>(slot - static_cast<int64_t>(r) * ppr);
        const int b0 = base[r];
        if (p >= base[r + 1] - b0) return;
        const int src = survivor_idx[r];  // valid: the plan gave this survivor pages
        const int64_t sp = block_table_src[static_cast<int64_t>(src) * ppr + p];
        const int64_t dp = static_cast<int64_t>(b0) + p;
        if (sp < 0 || sp >= src_pages || dp >= dst_pages) return;
        const u32x4* s = kv_src + (slab * src_pages + sp) * chunk_vec;
        u32x4* d = kv_dst + (slab * dst_pages + dp) * chunk_vec;
        for (int64_t v0 = 0; v0 < chunk_vec; v0 += kCopyThreads * UNROLL) {
            u32x4 x[UNROLL];
#pragma unroll
            for (int u = 0; u < UNROLL; ++u) {
                const int64_t v = v0 + u * kCopyThreads + threadIdx.x;
                if (v < chunk_vec) x[u] = __builtin_nontemporal_load(s + v);
            }
#pragma unroll
            for (int u = 0; u < UNROLL; ++u) {
                const int64_t v = v0 + u * kCopyThreads + threadIdx.x;
                if (v < chunk_vec) __builtin_nontemporal_store(x[u], d + v);
            }
        }
    } else {
        const int r = static_cast<int>(bid - kv_blocks);
        const int src = survivor_idx[r];
        const bool valid = src >= 0 && src < n_src;
        const int32_t* s = tokens_src + static_cast<int64_t>(valid ? src : 0) * max_len;
        int32_t* d = tokens_dst + static_cast<int64_t>(r) * max_len;
        for (int i = threadIdx.x; i < max_len; i += kCopyThreads) d[i] = valid ? s[i] : 0;
    }
}

__global__ void compact_empty_kernel(int64_t* n_pages_used) { *n_pages_used = 0; }

// ---- in-place variant: fill the holes below the live-page count with the live pages above it ----------
// workspace layout (int32): live[P] | new_page[P] | hole_list[P] | mover_list[P] | counters[2] = {n_live, m}

__global__ void inplace_clear_kernel(int32_t* live, int64_t P) {
    const int64_t i = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
    if (i < P) live[i] = 0;
}

// one thread per (survivor rank, logical page): flag the physical page as live; thread p == 0 writes the
// per-survivor outputs
__global__ void inplace_mark_kernel(const int32_t* __restrict__ survivor_idx, const int32_t* __restrict__ seq_len_src,
                                    const int32_t* __restrict__ block_table_src, int n_src, int n_keep,
                                    int page_tokens, int ppr, int64_t P, int32_t* __restrict__ live,
                                    int32_t* __restrict__ seq_len_dst, int32_t* __restrict__ src_of_dst) {
    const int64_t i = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
    if (i >= static_cast<int64_t>(n_keep) * ppr) return;
    const int r = static_cast<int>(i / ppr), p = static_cast<int>(i % ppr);
    const int src = survivor_idx[r];
    const bool valid = src >= 0 && src < n_src;
    if (p == 0) {
        seq_len_dst[r] = valid ? seq_len_src[src] : 0;
        src_of_dst[r] = valid ? src : -1;
    }
    if (p < pages_of(seq_len_src, src, n_src, page_tokens, ppr)) {
        const int64_t page = block_table_src[static_cast<int64_t>(src) * ppr + p];
        if (page >= 0 && page < P) live[page] = 1;
    }
}

// one workgroup: n_live = number of live pages; holes = dead pages below n_live, movers = live pages at or
// above it, both ascending (ballot + popcount ranks, LDS carries); new_page[] maps every live page to its
// final position
__global__ __launch_bounds__(kPlanThreads) void inplace_plan_kernel(
    const int32_t* __restrict__ live, int64_t P, int32_t* __restrict__ new_page, int32_t* __restrict__ hole_list,
    int32_t* __restrict__ mover_list, int32_t* __restrict__ counters, int64_t* __restrict__ n_pages_used,
    int64_t* __restrict__ n_moved) {
    __shared__ int wave_h[kPlanThreads / ARROL_WAVE], wave_m[kPlanThreads / ARROL_WAVE];
    __shared__ int carry_h, carry_m, total_s;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    int cnt = 0;
    for (int64_t p = tid; p < P; p += kPlanThreads) cnt += live[p];
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) cnt += __shfl_xor(cnt, m, ARROL_WAVE);
    if (lane == 0) wave_h[wave] = cnt;
    if (tid == 0) { carry_h = 0; carry_m = 0; }
    __syncthreads();
    if (tid == 0) {
        int t = 0;
        for (int w = 0; w < kPlanThreads / ARROL_WAVE; ++w) t += wave_h[w];
        total_s = t;
    }
    __syncthreads();
    const int64_t n_live = total_s;
    for (int64_t p0 = 0; p0 < P; p0 += kPlanThreads) {
        const int64_t p = p0 + tid;
        const bool is_live = p < P && live[p] != 0;
        const bool hole = p < n_live && !is_live;
        const bool mover = p < P && p >= n_live && is_live;
        const uint64_t bh = __ballot(hole), bm = __ballot(mover);
        __syncthreads();   // previous chunk's carries have been read
        if (lane == 0) { wave_h[wave] = __popcll(bh); wave_m[wave] = __popcll(bm); }
        __syncthreads();
        int before_h = carry_h, before_m = carry_m;
        for (int w = 0; w < wave; ++w) { before_h += wave_h[w]; before_m += wave_m[w]; }
        const uint64_t below = (1ull << lane) - 1ull;
        if (hole) hole_list[before_h + __popcll(bh & below)] = static_cast<int32_t>(p);
        if (mover) mover_list[before_m + __popcll(bm & below)] = static_cast<int32_t>(p);
        if (p < P) new_page[p] = (is_live && p < n_live) ? static_cast<int32_t>(p) : -1;
        __syncthreads();
        if (tid == kPlanThreads - 1) { carry_h = before_h + __popcll(bh); carry_m = before_m + __popcll(bm); }
    }
    __syncthreads();
    const int m = carry_m;   // == carry_h: as many holes as movers
    for (int k = tid; k < m; k += kPlanThreads) new_page[mover_list[k]] = hole_list[k];
    if (tid == 0) {
        counters[0] = static_cast<int32_t>(n_live);
        counters[1] = m;
        *n_pages_used = n_live;
        if (n_moved) *n_moved = m;
    }
}

// copy blocks: (slab, k) moves page mover_list[k] onto hole_list[k]; table blocks: remapped block tables
__global__ __launch_bounds__(kCopyThreads) void inplace_copy_kernel(
    u32x4* __restrict__ kv, int64_t chunk_vec, int64_t P, const int32_t* __restrict__ hole_list,
    const int32_t* __restrict__ mover_list, const int32_t* __restrict__ counters, int64_t m_bound, int64_t kv_blocks,
    const int32_t* __restrict__ new_page, const int32_t* __restrict__ survivor_idx,
    const int32_t* __restrict__ seq_len_src, const int32_t* __restrict__ block_table_src, int n_src, int page_tokens,
    int ppr, int32_t* __restrict__ block_table_dst) {
    const int64_t bid = blockIdx.x;
    if (bid < kv_blocks) {
        const int64_t slab = bid / m_bound, k = bid - slab * m_bound;
        if (k >= counters[1]) return;
        const u32x4* s = kv + (slab * P + mover_list[k]) * chunk_vec;
        u32x4* d = kv + (slab * P + hole_list[k]) * chunk_vec;
        for (int64_t v0 = 0; v0 < chunk_vec; v0 += kCopyThreads * kCopyUnroll) {
            u32x4 x[kCopyUnroll];
#pragma unroll
            for (int u = 0; u < kCopyUnroll; ++u) {
                const int64_t v = v0 + u * kCopyThreads + threadIdx.x;
                if (v < chunk_vec) x[u] = __builtin_nontemporal_load(s + v);
            }
#pragma unroll
            for (int u = 0; u < kCopyUnroll; ++u) {
                const int64_t v = v0 + u * kCopyThreads + threadIdx.x;
                if (v < chunk_vec) __builtin_nontemporal_store(x[u], d + v);
            }
        }
    } else {
        const int r = static_cast<int>(bid - kv_blocks);
        const int src = survivor_idx[r];
        const int np = pages_of(seq_len_src, src, n_src, page_tokens, ppr);
        for (int p = threadIdx.x; p < ppr; p += kCopyThreads) {
            int32_t out = -1;
            if (p < np) {
                const int64_t page = block_table_src[static_cast<int64_t>(src) * ppr + p];
                if (page >= 0 && page < P) out = new_page[page];
            }
            block_table_dst[static_cast<int64_t>(r) * ppr + p] = out;
        }
    }
}

// ---- in-place variant, planning in ONE launch (pools of up to kFusedMaxPages pages) --------------------
// One workgroup keeps the live-page bitmap and its per-word prefix counts in LDS:
//   clear bitmap -> mark the survivors' pages (LDS atomic OR) -> prefix counts (n_live = total) ->
//   hole / mover lists (rank of a page = prefix of its word + popcount below its bit) ->
//   remapped block tables, lengths, source map, counters.
// LDS: 2 x 4 bytes per 32 pages, i.e. P / 4 bytes.
constexpr int64_t kFusedMaxPages = 512 * 1024;   // 128 KiB of LDS

__global__ __launch_bounds__(kPlanThreads) void inplace_fused_plan_kernel(
    const int32_t* __restrict__ survivor_idx, const int32_t* __restrict__ seq_len_src,
    const int32_t* __restrict__ block_table_src, int n_src, int n_keep, int page_tokens, int ppr, int P,
    int32_t* __restrict__ hole_list, int32_t* __restrict__ mover_list, int32_t* __restrict__ counters,
    int32_t* __restrict__ block_table_dst, int32_t* __restrict__ seq_len_dst, int32_t* __restrict__ src_of_dst,
    int64_t* __restrict__ n_pages_used, int64_t* __restrict__ n_moved) {
    extern __shared__ uint32_t plan_lds[];
    __shared__ int wave_tot[kPlanThreads / ARROL_WAVE];
    __shared__ int live_below_s;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n_words = (P + 31) >> 5;
    uint32_t* bitmap = plan_lds;               // [n_words]
    uint32_t* prefix = plan_lds + n_words;     // [n_words] live pages in earlier words
    for (int w = tid; w < n_words; w += kPlanThreads) bitmap[w] = 0u;
    __syncthreads();
    const int64_t slots = static_cast<int64_t>(n_keep) * ppr;
    for (int64_t i = tid; i < slots; i += kPlanThreads) {
        const int r = static_cast<int>(i / ppr), p = static_cast<int>(i - static_cast<int64_t>(r) * ppr);
        const int src = survivor_idx[r];
        const bool valid = src >= 0 && src < n_src;
        if (p == 0) {
            seq_len_dst[r] = valid ? seq_len_src[src] : 0;
            src_of_dst[r] = valid ? src : -1;
        }
        if (p < pages_of(seq_len_src, src, n_src, page_tokens, ppr)) {
            const int page = block_table_src[static_cast<int64_t>(src) * ppr + p];
            if (page >= 0 && page < P) atomicOr(&bitmap[page >> 5], 1u << (page & 31));
        }
    }
    __syncthreads();
    // exclusive prefix of the per-word popcounts: each thread owns a contiguous run of words
    const int per = (n_words + kPlanThreads - 1) / kPlanThreads;
    const int w0 = tid * per, w1 = w0 + per < n_words ? w0 + per : n_words;
    int mine = 0;
    for (int w = w0; w < w1; ++w) mine += __popc(bitmap[w]);
    int incl = mine;
#pragma unroll
    for (int o = 1; o < ARROL_WAVE; o <<= 1) {
        const int v = __shfl_up(incl, o, ARROL_WAVE);
        if (lane >= o) incl += v;
    }
    if (lane == 63) wave_tot[wave] = incl;
    __syncthreads();
    int before = 0, total = 0;
    for (int wv = 0; wv < kPlanThreads / ARROL_WAVE; ++wv) {
        if (wv < wave) before += wave_tot[wv];
        total += wave_tot[wv];
    }
    int run = before + incl - mine;
    for (int w = w0; w < w1; ++w) {
        prefix[w] = static_cast<uint32_t>(run);
        run += __popc(bitmap[w]);
    }
    const int n_live = total;
    __syncthreads();
    // live pages below n_live (= n_live minus the holes)
    if (tid == 0) {
        int lb = n_live;   // n_live == P: every page is live
        if (n_live < P) {
            const int w = n_live >> 5, b = n_live & 31;
            lb = static_cast<int>(prefix[w]) + __popc(bitmap[w] & ((1u << b) - 1u));
        }
        live_below_s = lb;
    }
    __syncthreads();
    const int live_below = live_below_s;
    const int m = n_live - live_below;         // holes below n_live == live pages at or above it
    // hole and mover lists, both ascending by construction of the ranks
    for (int w = w0; w < w1; ++w) {
        const uint32_t bits = bitmap[w];
        const int base = w << 5;
        int rank = static_cast<int>(prefix[w]);                 // live pages before page base + b
        for (int b = 0; b < 32; ++b) {
            const int page = base + b;
            if (page >= P) break;
            const bool is_live = (bits >> b) & 1u;
            if (is_live) {
                if (page >= n_live) mover_list[rank - live_below] = page;
                ++rank;
            } else if (page < n_live) {
                hole_list[page - rank] = page;
            }
        }
    }
    __syncthreads();   // the lists, written by this workgroup to global memory, are read back below
    for (int64_t i = tid; i < slots; i += kPlanThreads) {
        const int r = static_cast<int>(i / ppr), p = static_cast<int>(i - static_cast<int64_t>(r) * ppr);
        const int src = survivor_idx[r];
        int32_t out = -1;
        if (p < pages_of(seq_len_src, src, n_src, page_tokens, ppr)) {
            const int page = block_table_src[static_cast<int64_t>(src) * ppr + p];
            if (page >= 0 && page < P) {
                if (page < n_live) {
                    out = page;
                } else {
                    const int rank = static_cast<int>(prefix[page >> 5]) + __popc(bitmap[page >> 5] & ((1u << (page & 31)) - 1u));
                    out = hole_list[rank - live_below];
                }
            }
        }
        block_table_dst[i] = out;
    }
    if (tid == 0) {
        counters[0] = n_live;
        counters[1] = m;
        *n_pages_used = n_live;
        if (n_moved) *n_moved = m;
    }
}

// Copy of the mover -> hole pairs (both lists ascend), every (layer, K|V) slab.  The host knows only a bound on the
// pair count (the exact one is in counters[1] on the device), and which form is fastest depends on the chunk size;
// both forms were measured on the pools of the benchmark configurations.
//
// Chunks below 32 KiB: one workgroup per (slab, position), slab by slab, position < the host-side bound; positions
// beyond the device-side count exit at once, the others take pair stream_order(position, count) - 5.8-5.9 TB/s on
// the 8.6 GB pool of 16 KiB chunks against 5.1-5.4 in ascending pair order (a persistent grid: 5.0-5.3).
__global__ __launch_bounds__(kCopyThreads) void inplace_copy_pairs_kernel(
    u32x4* __restrict__ kv, int64_t chunk_vec, int64_t P, const int32_t* __restrict__ hole_list,
    const int32_t* __restrict__ mover_list, const int32_t* __restrict__ counters, unsigned m_bound) {
    const unsigned slab = blockIdx.x / m_bound;
    const unsigned pos = blockIdx.x - slab * m_bound;
    const unsigned n_pairs = static_cast<unsigned>(counters[1]);
    if (pos >= n_pairs) return;
    const unsigned k = stream_order(pos, n_pairs);
    const u32x4* s = kv + (static_cast<int64_t>(slab) * P + mover_list[k]) * chunk_vec;
    u32x4* d = kv + (static_cast<int64_t>(slab) * P + hole_list[k]) * chunk_vec;
    for (int64_t v0 = 0; v0 < chunk_vec; v0 += kCopyThreads * kCopyUnroll) {
        u32x4 x[kCopyUnroll];
#pragma unroll
        for (int u = 0; u < kCopyUnroll; ++u) {
            const int64_t v = v0 + u * kCopyThreads + threadIdx.x;
            if (v < chunk_vec) x[u] = __builtin_nontemporal_load(s + v);
        }
#pragma unroll
        for (int u = 0; u < kCopyUnroll; ++u) {
            const int64_t v = v0 + u * kCopyThreads + threadIdx.x;
            if (v < chunk_vec) __builtin_nontemporal_store(x[u], d + v);
        }
    }
}

// Chunks of 32 KiB and more: a persistent grid (4 workgroups per compute unit) walks the count * n_slabs copies
// with the slab as the fast index, workgroup b taking copies b, b + grid, b + 2 grid, ...: no workgroup is launched
// only to exit (with one workgroup per copy, half of a bound-sized grid is idle on the benchmark pools and the
// dispatch of those idle workgroups alone costs 7 %).  6.15-6.3 TB/s on the 120 and 155 GB pools against 5.8-5.9
// for one workgroup per copy in its best order; walking pair-fast instead: 5.2.  The loop ends for every workgroup
// after at most ceil(count * n_slabs / grid) copies.
__global__ __launch_bounds__(kCopyThreads) void inplace_copy_walk_kernel(
    u32x4* __restrict__ kv, int64_t chunk_vec, int64_t P, const int32_t* __restrict__ hole_list,
    const int32_t* __restrict__ mover_list, const int32_t* __restrict__ counters, unsigned n_slabs) {
    const unsigned n_pairs = static_cast<unsigned>(counters[1]);
    // copy = k * n_slabs + slab, advanced by gridDim.x per step without a division in the loop
    const unsigned step_k = gridDim.x / n_slabs, step_slab = gridDim.x - step_k * n_slabs;
    unsigned k = blockIdx.x / n_slabs, slab = blockIdx.x - k * n_slabs;
    while (k < n_pairs) {
        const u32x4* s = kv + (static_cast<int64_t>(slab) * P + mover_list[k]) * chunk_vec;
        u32x4* d = kv + (static_cast<int64_t>(slab) * P + hole_list[k]) * chunk_vec;
        for (int64_t v0 = 0; v0 < chunk_vec; v0 += kCopyThreads * kCopyUnroll) {
            u32x4 x[kCopyUnroll];
#pragma unroll
            for (int u = 0; u < kCopyUnroll; ++u) {
                const int64_t v = v0 + u * kCopyThreads + threadIdx.x;
                if (v < chunk_vec) x[u] = __builtin_nontemporal_load(s + v);
            }
#pragma unroll
            for (int u = 0; u < kCopyUnroll; ++u) {
                const int64_t v = v0 + u * kCopyThreads + threadIdx.x;
                if (v < chunk_vec) __builtin_nontemporal_store(x[u], d + v);
            }
        }
        k += step_k;
        slab += step_slab;
        if (slab >= n_slabs) { slab -= n_slabs; ++k; }
    }
}

bool same_geometry(const arrol_kv_layout& a, const arrol_kv_layout& b) {
    return a.n_layers == b.n_layers && a.page_tokens == b.page_tokens && a.n_kv_heads == b.n_kv_heads &&
           a.head_dim == b.head_dim;
}

}  // namespace

extern "C" size_t arrol_compact_workspace_bytes(int32_t n_keep) {
    if (n_keep < 0) return 0;
    return ((static_cast<size_t>(n_keep) + 1) * sizeof(int32_t) + 255) & ~static_cast<size_t>(255);
}

// ---- scratch of arrol_compact_static: one base offset per survivor plus the total, in device memory that
// is part of the loaded code object (nothing is allocated at run time).  Every GPU the library runs on holds
// its own copy at its own address; the address is looked up once per device and kept.
static __device__ __align__(256) int32_t scratch[ARROL_COMPACT_STATIC_MAX_KEEP + 1];
static std::atomic<int32_t*> g_scratch_ptr[64];

static int32_t* static_scratch_of_current_device() {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return nullptr;
    int32_t* p = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (p) return p;
    void* sym = nullptr;
    if (hipGetSymbolAddress(&sym, HIP_SYMBOL(scratch)) != hipSuccess || !sym) return nullptr;
    p = static_cast<int32_t*>(sym);
    g_scratch_ptr[dev].store(p, std::memory_order_release);
    return p;
}

namespace {

// Argument checks and the two launches shared by arrol_compact and arrol_compact_static; `base` is the
// int32 [n_keep + 1] scratch (caller's workspace or the library's static array), already validated.
int compact_validate(const void* kv_src, const arrol_kv_layout& src, const void* kv_dst, const arrol_kv_layout& dst,
                     const int32_t* block_table_src, const int32_t* seq_len_src, int32_t max_pages_per_seq,
                     const int32_t* tokens_src, int32_t max_len, const int32_t* survivor_idx,
                     const int32_t* block_table_dst, const int32_t* seq_len_dst, const int32_t* tokens_dst,
                     const int32_t* src_of_dst) {
    if (!same_geometry(src, dst) || src.n_layers < 1 || src.page_tokens < 1 || src.n_kv_heads < 1 ||
        src.head_dim < 1 || src.n_pages < 0 || dst.n_pages < 0 || max_pages_per_seq < 1)
        return ARROL_EINVAL;
    const int64_t chunk_bytes = static_cast<int64_t>(src.page_tokens) * src.n_kv_heads * src.head_dim * 2;
    if (chunk_bytes % 16) return ARROL_EINVAL;
    if (!kv_src || !kv_dst || !block_table_src || !seq_len_src || !survivor_idx || !block_table_dst ||
        !seq_len_dst || !src_of_dst || !arrol_aligned16(kv_src) || !arrol_aligned16(kv_dst))
        return ARROL_EINVAL;
    const bool with_tokens = tokens_src != nullptr || tokens_dst != nullptr;
    if (with_tokens && (!tokens_src || !tokens_dst || max_len < 0)) return ARROL_EINVAL;
    // the pools may not overlap
    const char* a0 = static_cast<const char*>(kv_src);
    const char* b0 = static_cast<const char*>(kv_dst);
    const int64_t a_len = chunk_bytes * src.n_pages * src.n_layers * 2, b_len = chunk_bytes * dst.n_pages * dst.n_layers * 2;
    if (a0 < b0 + b_len && b0 < a0 + a_len) return ARROL_EINVAL;
    return ARROL_OK;
}

int compact_enqueue(const void* kv_src, const arrol_kv_layout& src, void* kv_dst, const arrol_kv_layout& dst,
                    const int32_t* block_table_src, const int32_t* seq_len_src, int32_t max_pages_per_seq,
                    const int32_t* tokens_src, int32_t max_len, const int32_t* survivor_idx, int32_t n_src,
                    int32_t n_keep, int32_t* block_table_dst, int32_t* seq_len_dst, int32_t* tokens_dst,
                    int32_t* src_of_dst, int64_t* n_pages_used, int32_t* base, hipStream_t st) {
    const int64_t chunk_bytes = static_cast<int64_t>(src.page_tokens) * src.n_kv_heads * src.head_dim * 2;
    const bool with_tokens = tokens_src != nullptr;
    const int64_t slots = static_cast<int64_t>(n_keep) * max_pages_per_seq;
    if (slots > INT32_MAX) return ARROL_EINVAL;  // page ids are int32
    const int64_t kv_blocks = slots * src.n_layers * 2;
    const int64_t blocks = kv_blocks + (with_tokens && max_len > 0 ? n_keep : 0);
    if (blocks > INT32_MAX) return ARROL_EINVAL;
    arrol_launch(compact_plan_kernel, dim3(1), dim3(kPlanThreads), 0, st, survivor_idx, seq_len_src, n_src,
                 n_keep, src.page_tokens, max_pages_per_seq, base, block_table_dst, seq_len_dst, src_of_dst,
                 n_pages_used);
    if (arrol_launch_failed()) return arrol_launch_status();
    arrol_launch(chunk_bytes >= 32768 ? compact_copy_kernel<4> : compact_copy_kernel<kCopyUnroll>, dim3(static_cast<unsigned>(blocks)), dim3(kCopyThreads), 0, st,
                 static_cast<const u32x4*>(kv_src), static_cast<u32x4*>(kv_dst), chunk_bytes / 16,
                 src.n_pages, dst.n_pages, block_table_src, survivor_idx, base, n_src, n_keep,
                 max_pages_per_seq, kv_blocks, tokens_src, tokens_dst, max_len);
    return arrol_launch_status();
}

}  // namespace

extern "C" int arrol_compact(const void* kv_src, arrol_kv_layout src, void* kv_dst, arrol_kv_layout dst,
                             const int32_t* block_table_src, const int32_t* seq_len_src,
                             int32_t max_pages_per_seq, const int32_t* tokens_src, int32_t max_len,
                             const int32_t* survivor_idx, int32_t n_src, int32_t n_keep,
                             int32_t* block_table_dst, int32_t* seq_len_dst, int32_t* tokens_dst,
                             int32_t* src_of_dst, int64_t* n_pages_used,
                             void* workspace, size_t workspace_bytes, void* stream) {
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (n_keep < 0 || n_src < 0 || !n_pages_used) return ARROL_EINVAL;
    if (n_keep == 0) {
        arrol_launch(compact_empty_kernel, dim3(1), dim3(1), 0, st, n_pages_used);
        return arrol_launch_status();
    }
    const int rc = compact_validate(kv_src, src, kv_dst, dst, block_table_src, seq_len_src, max_pages_per_seq,
                                    tokens_src, max_len, survivor_idx, block_table_dst, seq_len_dst, tokens_dst,
                                    src_of_dst);
    if (rc != ARROL_OK) return rc;
    if (!workspace || !arrol_aligned16(workspace) || workspace_bytes < arrol_compact_workspace_bytes(n_keep))
        return ARROL_EWORKSPACE;
    return compact_enqueue(kv_src, src, kv_dst, dst, block_table_src, seq_len_src, max_pages_per_seq, tokens_src,
                           max_len, survivor_idx, n_src, n_keep, block_table_dst, seq_len_dst, tokens_dst,
                           src_of_dst, n_pages_used, static_cast<int32_t*>(workspace), st);
}

extern "C" int arrol_compact_static(const void* kv_src, arrol_kv_layout src, void* kv_dst, arrol_kv_layout dst,
                                    const int32_t* block_table_src, const int32_t* seq_len_src,
                                    int32_t max_pages_per_seq, const int32_t* tokens_src, int32_t max_len,
                                    const int32_t* survivor_idx, int32_t n_src, int32_t n_keep,
                                    int32_t* block_table_dst, int32_t* seq_len_dst, int32_t* tokens_dst,
                                    int32_t* src_of_dst, int64_t* n_pages_used, void* stream) {
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (n_keep < 0 || n_src < 0 || !n_pages_used) return ARROL_EINVAL;
    if (n_keep > ARROL_COMPACT_STATIC_MAX_KEEP) return ARROL_EWORKSPACE;   // the fixed scratch holds no more
    if (n_keep == 0) {
        arrol_launch(compact_empty_kernel, dim3(1), dim3(1), 0, st, n_pages_used);
        return arrol_launch_status();
    }
    const int rc = compact_validate(kv_src, src, kv_dst, dst, block_table_src, seq_len_src, max_pages_per_seq,
                                    tokens_src, max_len, survivor_idx, block_table_dst, seq_len_dst, tokens_dst,
                                    src_of_dst);
    if (rc != ARROL_OK) return rc;
    int32_t* base = static_scratch_of_current_device();
    if (!base) return ARROL_EHIP;
    // base[0 .. n_keep] is rewritten in full by the plan kernel, so nothing has to be cleared between calls
    return compact_enqueue(kv_src, src, kv_dst, dst, block_table_src, seq_len_src, max_pages_per_seq, tokens_src,
                           max_len, survivor_idx, n_src, n_keep, block_table_dst, seq_len_dst, tokens_dst,
                           src_of_dst, n_pages_used, base, st);
}

extern "C" size_t arrol_compact_inplace_workspace_bytes(int64_t n_pages) {
    if (n_pages < 0) return 0;
    return ((4 * static_cast<size_t>(n_pages) + 2) * sizeof(int32_t) + 255) & ~static_cast<size_t>(255);
}

extern "C" int arrol_compact_inplace(void* kv, arrol_kv_layout layout, const int32_t* block_table_src,
                                     const int32_t* seq_len_src, int32_t max_pages_per_seq,
                                     const int32_t* survivor_idx, int32_t n_src, int32_t n_keep,
                                     int32_t* block_table_dst, int32_t* seq_len_dst, int32_t* src_of_dst,
                                     int64_t* n_pages_used, int64_t* n_moved, void* workspace,
                                     size_t workspace_bytes, void* stream) {
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (n_keep < 0 || n_src < 0 || !n_pages_used) return ARROL_EINVAL;
    if (layout.n_layers < 1 || layout.page_tokens < 1 || layout.n_kv_heads < 1 || layout.head_dim < 1 ||
        layout.n_pages < 0 || layout.n_pages > INT32_MAX || max_pages_per_seq < 1)
        return ARROL_EINVAL;
    const int64_t chunk_bytes = static_cast<int64_t>(layout.page_tokens) * layout.n_kv_heads * layout.head_dim * 2;
    if (chunk_bytes % 16) return ARROL_EINVAL;
    if (n_keep > 0 && (!kv || !block_table_src || !seq_len_src || !survivor_idx || !block_table_dst || !seq_len_dst ||
                       !src_of_dst || !arrol_aligned16(kv)))
        return ARROL_EINVAL;
    if (!workspace || !arrol_aligned16(workspace) ||
        workspace_bytes < arrol_compact_inplace_workspace_bytes(layout.n_pages))
        return ARROL_EWORKSPACE;
    const int64_t P = layout.n_pages;
    const int64_t slots = static_cast<int64_t>(n_keep) * max_pages_per_seq;
    if (slots > INT32_MAX) return ARROL_EINVAL;
    int32_t* live = static_cast<int32_t*>(workspace);
    int32_t* new_page = live + P;
    int32_t* hole_list = new_page + P;
    int32_t* mover_list = hole_list + P;
    int32_t* counters = mover_list + P;
    if (P <= kFusedMaxPages) {
        // planning in one launch (bitmap in LDS), then the copy over the pairs alone
        const int n_words = static_cast<int>((P + 31) >> 5);
        const int lds_bytes = 2 * n_words * static_cast<int>(sizeof(uint32_t));
        static arrol_device_flags fused_ok;
        if (!arrol_allow_lds(&inplace_fused_plan_kernel, static_cast<int>(kFusedMaxPages / 4), fused_ok)) return ARROL_EHIP;
        arrol_launch(inplace_fused_plan_kernel, dim3(1), dim3(kPlanThreads), lds_bytes, st, survivor_idx, seq_len_src,
                     block_table_src, n_src, n_keep, layout.page_tokens, max_pages_per_seq, static_cast<int>(P),
                     hole_list, mover_list, counters, block_table_dst, seq_len_dst, src_of_dst, n_pages_used, n_moved);
        if (arrol_launch_failed()) return arrol_launch_status();
        // no more pairs than survivor pages, than dead pages (P - live >= holes), or than half the pool
        const int64_t m_bound = slots < P / 2 ? slots : P / 2;
        const int n_slabs = layout.n_layers * 2;
        if (m_bound == 0) return arrol_launch_status();
        if (chunk_bytes >= 32768) {
            const int n_cu = compute_units();
            if (n_cu <= 0) return ARROL_EHIP;
            arrol_launch(inplace_copy_walk_kernel, dim3(static_cast<unsigned>(n_cu) * 4u), dim3(kCopyThreads), 0, st,
                         static_cast<u32x4*>(kv), chunk_bytes / 16, P, hole_list, mover_list, counters,
                         static_cast<unsigned>(n_slabs));
        } else {
            const int64_t blocks = m_bound * n_slabs;
            if (blocks > INT32_MAX) return ARROL_EINVAL;
            arrol_launch(inplace_copy_pairs_kernel, dim3(static_cast<unsigned>(blocks)), dim3(kCopyThreads), 0, st,
                         static_cast<u32x4*>(kv), chunk_bytes / 16, P, hole_list, mover_list, counters,
                         static_cast<unsigned>(m_bound));
        }
        return arrol_launch_status();
    }
    if (P > 0) {
        arrol_launch(inplace_clear_kernel, dim3(static_cast<unsigned>((P + 255) / 256)), dim3(256), 0, st, live, P);
        if (arrol_launch_failed()) return arrol_launch_status();
    }
    if (slots > 0) {
        arrol_launch(inplace_mark_kernel, dim3(static_cast<unsigned>((slots + 255) / 256)), dim3(256), 0, st,
                           survivor_idx, seq_len_src, block_table_src, n_src, n_keep, layout.page_tokens,
                           max_pages_per_seq, P, live, seq_len_dst, src_of_dst);
        if (arrol_launch_failed()) return arrol_launch_status();
    }
    arrol_launch(inplace_plan_kernel, dim3(1), dim3(kPlanThreads), 0, st, live, P, new_page, hole_list,
                       mover_list, counters, n_pages_used, n_moved);
    if (arrol_launch_failed()) return arrol_launch_status();
    const int64_t m_bound = slots < P ? slots : P;   // no more movers than survivor pages or pool pages
    const int64_t kv_blocks = m_bound * layout.n_layers * 2;
    const int64_t blocks = kv_blocks + n_keep;
    if (blocks > INT32_MAX) return ARROL_EINVAL;
    if (blocks == 0) return ARROL_OK;
    arrol_launch(inplace_copy_kernel, dim3(static_cast<unsigned>(blocks)), dim3(kCopyThreads), 0, st,
                       static_cast<u32x4*>(kv), chunk_bytes / 16, P, hole_list, mover_list, counters,
                       m_bound > 0 ? m_bound : 1, kv_blocks, new_page, survivor_idx, seq_len_src, block_table_src,
                       n_src, layout.page_tokens, max_pages_per_seq, block_table_dst);
    return arrol_launch_status();
}
