// Shared "NT" contraction pipeline of the fused log-prob kernel and the MLP quality head (gfx950, wave64):
// a workgroup of 8 wavefronts multiplies A rows by B rows over a K extent that is contiguous in both,
//     acc[a][b] += sum_k A[a][k] * B[b][k]        (bf16 operands, fp32 accumulation, v_mfma_f32_32x32x16_bf16)
// for one 256-row block of B and a run of 256-row tiles of A, and hands every finished 256 x 256 accumulator
// tile to a caller-supplied epilogue while it is still in registers.  In the MFMA result layout a lane's 16
// values of a 32 x 32 block share the B row (column = lane % 32) and lie on 16 different A rows, so a
// reduction over A rows per B row (logsumexp over the vocabulary, sum over hidden units) is lane-local.
//
// Operands go global -> LDS directly (no staging registers) into a ring of RING K32 slots (32 k-values =
// 64 bytes of each of the BM + BN tile rows).  Loads always fetch whole 128-byte lines of a row, i.e. the
// two K32 halves that go to two consecutive slots (a "pair").  The L1 path moves 64 bytes per clock, so a
// pair costs as many L1 cycles as half of its MFMA time; to keep that evenly spread, the A lines of a pair
// are requested during one K32 iteration and its B lines during the next.  The pipeline per iteration i
// (chunk i lives in slot i % RING):
//   K16 step 0: MFMAs on fragments already in registers; between them the step-1 fragment reads of
//               slot i and two of this iteration's four load instructions;
//   K16 step 1: MFMAs; between them the step-0 reads of the A fragments of slot i+1 (certified one
//               barrier earlier), then - four MFMAs before the end - the wait for this wave's older
//               loads and the workgroup barrier, then the step-0 reads of the B fragments of slot i+1
//               and the remaining loads.  The last MFMAs cover the latency of those reads, so the
//               matrix pipe never waits for an LDS round trip behind a barrier.
// The barrier inside iteration i certifies the A part of slot i+2 and the B part of slot i+1 and
// releases slot i-1 (A lines) / slot i-2.. for refilling; see the table in the loop for who loads what.
//
// B_KMAJOR = true is the "TN" form: B is given K-major, B[k][b] with the b index contiguous (row k starts
// k * b_stride bytes after the base), so an operand that is stored rollout-major can be contracted over the
// rollouts without a transposed copy.  A K32 slot then holds 32 k-rows of 256 b-values (512 bytes each, the
// same 16 KiB), a load instruction moves two whole k-rows, and the B fragments come out of LDS through the
// transposing read ds_read_b64_tr_b16: in each block of 16 lanes, lane 4e + q supplies the address of four
// consecutive b-values of k-row e, and lane j receives the four k-values of b-value j (layout measured on
// the device).  16-byte chunk c of k-row r sits at chunk position c ^ 4 (r % 4) of its row, so the four rows
// that 32 lanes read together fall on different banks.
#pragma once
#include <type_traits>

#include "common.h"

namespace ring_nt {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

template <int BM_, int BN_, int WM_, int WN_>
struct RingTile {
    static constexpr int BM = BM_, BN = BN_, WM = WM_, WN = WN_;
    static constexpr int NT = WM * WN * ARROL_WAVE;
    static constexpr int NW = WM * WN;
    static constexpr int TM = BM / WM / 32, TN = BN / WN / 32;
    static constexpr int RING = 5;
    static constexpr int SLOT_BYTES = (BM + BN) * 64;
    static constexpr int LDS_BYTES = RING * SLOT_BYTES;
    static constexpr int G = BM / 16 / NW;                  // 16-row load groups per wave and operand
    static constexpr int LOADS = 2 * G;                     // load instructions per wave and iteration
    static_assert(BM == BN, "A and B tiles are loaded by the same code in alternate iterations");
    static_assert(BM % (16 * NW) == 0, "whole 16-row load groups per wave");
    static_assert(LOADS == 4 && TM * TN == 8 && TM + TN <= 8, "the hand-placed schedule below");
};

template <int N>
__device__ __forceinline__ void wait_vmcnt() {  // s_waitcnt vmcnt(N) only (gfx9 encoding), N <= 15
    __builtin_amdgcn_s_waitcnt(0x0F70 | N);
}

// What one workgroup walks.  Row r of an operand starts r * stride bytes after its base; every row holds the
// K extent [0, n_k64 * 64) contiguously from the base (a K split passes bases already advanced to its first
// k).  a_rows / b_rows are the numbers of rows that exist from the base on: tile rows beyond them are clamped
// to the last row, so every load stays inside the operands (the epilogue masks what those rows produce).
struct Walk {
    const char* a_base;       // A row 0 of tile vt_lo ... the tiles are BM rows apart
    const char* b_base;       // B row 0 of this workgroup's block
    unsigned a_stride, b_stride;  // bytes between consecutive rows (< 16 MiB: a lane's row offset is 32-bit)
    int a_rows;               // A rows from a_base on: rows [0, a_rows) exist
    int b_rows;               // B rows of this block that exist (1 .. BN)
    int n_tiles;              // A tiles to walk
    int n_k64;                // K extent / 64
    int b_k_rows;             // B_KMAJOR only: k-rows of B that exist from b_base on (> 64 * (n_k64 - 1));
                              // b_rows is then the number of valid b-values (a multiple of 8), b_stride the
                              // bytes between k-rows
};

// Walks the tiles, accumulating into the caller's `acc` (cleared here first); `epilogue(acc, tile_index)` is
// called once per finished tile (tile_index counts from 0) and must leave the accumulators cleared if more
// tiles follow.  A caller that walks ONE tile can pass an empty epilogue and work on `acc` after the call:
// on return every load into LDS and every fragment read has finished and the workgroup has passed a barrier,
// so LDS is free for the caller too.
template <class C, bool B_KMAJOR = false, class Epilogue>
__device__ __forceinline__ void walk(const Walk& w, unsigned char* lds, f32x16 (&acc)[C::TM][C::TN], Epilogue&& epilogue) {
    constexpr int BM = C::BM, BN = C::BN, TM = C::TM, TN = C::TN, RING = C::RING;
    typedef __attribute__((address_space(3))) void* lds_ptr_t;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / C::WN, wn = wave % C::WN;
    const int l31 = lane & 31, lh = lane >> 5;
    const int n_k64 = w.n_k64;
    // (readfirstlane: wave-uniform by construction; it keeps the loop control in scalar registers)
    const int n_pairs = __builtin_amdgcn_readfirstlane(w.n_tiles * n_k64);   // pair = two K32 slots = one 128-byte line per row
    const int n_chunks = 2 * n_pairs;

    // ---- loader geometry: one instruction moves 16 rows x 64 bytes; lane -> (row lane/4, physical
    //      16-byte position lane%4), which holds logical chunk (lane%4) ^ ((row/4)%4) -----------
    const int ld_row = lane >> 2;
    const int ld_kb = ((lane & 3) ^ ((lane >> 4) & 3)) * 16;   // byte offset inside the K32 half
    // Addresses are (wave-uniform 64-bit base in SGPRs) + (per-lane 32-bit byte offset): the base
    // carries tile and K position, the lane offset the row inside the tile (clamped at the end of the
    // operand, so every load stays inside A and B) and the swizzled chunk.
    unsigned a_voff[C::G], b_voff[C::G];
    int b_lrow[C::G];   // B_KMAJOR: this lane's k-row inside a K32 slot, per load group
    if constexpr (B_KMAJOR) {
        // one instruction = 2 k-rows x 512 bytes: lane -> (k-row lane/32, chunk position lane%32)
        const int chunks_valid = w.b_rows >> 3;
#pragma unroll
        for (int g = 0; g < C::G; ++g) {
            b_lrow[g] = (wave * C::G + g) * 2 + (lane >> 5);
            int c = (lane & 31) ^ ((b_lrow[g] & 3) << 2);
            c = c < chunks_valid ? c : chunks_valid - 1;
            b_voff[g] = static_cast<unsigned>(c) * 16;
        }
    } else {
        const int rows_valid = w.b_rows;
#pragma unroll
        for (int g = 0; g < C::G; ++g) {
            int r = (wave * C::G + g) * 16 + ld_row;
            r = r < rows_valid ? r : rows_valid - 1;
            b_voff[g] = static_cast<unsigned>(r) * w.b_stride + ld_kb;
        }
    }
    auto point_at_tile = [&](int t) {
        const int left = w.a_rows - t * BM;
        const int rows_valid = left < BM ? (left > 0 ? left : 1) : BM;   // left <= 0 only past the last pair
#pragma unroll
        for (int g = 0; g < C::G; ++g) {
            int r = (wave * C::G + g) * 16 + ld_row;
            r = r < rows_valid ? r : rows_valid - 1;
            a_voff[g] = static_cast<unsigned>(r) * w.a_stride + ld_kb;
        }
    };
    // two load streams, each walking the pairs 0 .. n_pairs-1: A lines and B lines
    int a_t = 0, a_k64 = 0, a_slot = 0, a_issued = 0;
    int b_k64 = 0, b_slot = 0, b_issued = 0;
    const char* a_base = w.a_base;
    const char* b_base = w.b_base;
    point_at_tile(a_t);
    const unsigned lds0 = static_cast<unsigned>(reinterpret_cast<size_t>((lds_ptr_t)lds));
    // The q-th (q = 2*g + h) of the LOADS load instructions of a group: 16-row group g of this wave, K32
    // half h (-> first / second slot of the pair).  `stream` picks A lines or B lines at compile time.  Written as asm
    // so that the compiler keeps its own LDS wait counters exact; completion is tracked by hand with
    // s_waitcnt vmcnt + the workgroup barrier.
    auto issue_one = [&](auto stream, int q) {
        constexpr bool is_b = decltype(stream)::value;
        const int g = q >> 1, h = q & 1;
        const int slot0 = is_b ? b_slot : a_slot;
        const int s_h = h == 0 ? slot0 : (slot0 + 1 == RING ? 0 : slot0 + 1);
        const int r0 = (wave * C::G + g) * 16;
        const unsigned dst = lds0 + s_h * C::SLOT_BYTES + (is_b ? BM * 64 : 0) + r0 * 64;
        const char* base = (is_b ? b_base : a_base) + h * 64;
        unsigned voff = is_b ? b_voff[g] : a_voff[g];
        if constexpr (B_KMAJOR && is_b) {
            // k-row of the pair, clamped to the last row that exists (the A operand is zero there)
            const int left = w.b_k_rows - b_k64 * 64;                     // >= 1, wave-uniform
            int r = h * 32 + b_lrow[g];
            r = r < left ? r : left - 1;
            voff += static_cast<unsigned>(r) * w.b_stride;
            base = b_base;
        }
        asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(voff), "s"(base), "s"(dst) : "memory");
    };
    auto advance = [&](auto stream) {
        constexpr bool is_b = decltype(stream)::value;
        if (is_b) {
            const int64_t pair_bytes = B_KMAJOR ? static_cast<int64_t>(64) * w.b_stride : 128;
            b_base += pair_bytes;
            if (++b_k64 == n_k64) { b_k64 = 0; b_base -= n_k64 * pair_bytes; }   // next A tile: B rewinds
            b_slot = b_slot + 2 >= RING ? b_slot + 2 - RING : b_slot + 2;
            ++b_issued;
        } else {
            a_base += 128;
            if (++a_k64 == n_k64) {   // next A tile: on by a tile minus the K extent just walked
                a_k64 = 0;
                ++a_t;
                a_base += static_cast<int64_t>(BM) * w.a_stride - static_cast<int64_t>(n_k64) * 128;
                point_at_tile(a_t);
            }
            a_slot = a_slot + 2 >= RING ? a_slot + 2 - RING : a_slot + 2;
            ++a_issued;
        }
    };
    auto issue_group = [&](auto stream) {
#pragma unroll
        for (int q = 0; q < C::LOADS; ++q) issue_one(stream, q);
        advance(stream);
    };
    constexpr std::false_type kA{};   // A lines
    constexpr std::true_type kB{};    // B lines

#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    // fragment reads: row (wave base + i*32 + l31) of a slot, 16-byte chunk kk*2 + lh, swizzled
    const int swz = (l31 >> 2) & 3;
    const int a_off0 = (wm * (BM / C::WM) + l31) * 64 + ((lh ^ swz) << 4);          // K16 step 0
    const int a_off1 = (wm * (BM / C::WM) + l31) * 64 + (((2 + lh) ^ swz) << 4);    // K16 step 1
    const int b_off0 = BM * 64 + (wn * (BN / C::WN) + l31) * 64 + ((lh ^ swz) << 4);
    const int b_off1 = BM * 64 + (wn * (BN / C::WN) + l31) * 64 + (((2 + lh) ^ swz) << 4);
    bf16x8 fa0[TM], fb0[TN], fa1[TM], fb1[TN];   // fragments of K16 step 0 / step 1
    auto read_a = [&](bf16x8 (&fa)[TM], const unsigned char* base, int off, int m) {
        fa[m] = *reinterpret_cast<const bf16x8*>(base + off + m * 32 * 64);
    };
    // B_KMAJOR: lane 16 b + 4 e + q of a wavefront addresses k-row 8 lh + 4 h2 + e (+ 16 per K16 step),
    // b-values wn*64 + j*32 + 16 (b % 2) + 4 q .. + 3; block j = 1 is 4 chunks on, which the swizzle turns into ^ 64
    int bt_off[2] = {0, 0};
    if constexpr (B_KMAJOR) {
        const int e = (lane & 15) >> 2, q = lane & 3;
        const int chunk = wn * (BN / C::WN / 8) + 2 * ((lane >> 4) & 1) + (q >> 1);
#pragma unroll
        for (int h2 = 0; h2 < 2; ++h2)
            bt_off[h2] = BM * 64 + (8 * lh + 4 * h2 + e) * 512 + ((chunk ^ (e << 2)) << 4) + (q & 1) * 8;
    }
    auto read_b = [&](bf16x8 (&fb)[TN], const unsigned char* base, int k16, int j) {   // k16: K16 step 0 / 1 of the slot
        if constexpr (B_KMAJOR) {
            typedef short s16x4 __attribute__((ext_vector_type(4)));
            typedef __attribute__((address_space(3))) s16x4* lds_s16x4_t;
            const int step = k16 * 16 * 512;
            const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_t)(base + ((bt_off[0] ^ (j << 6)) + step)));
            const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_t)(base + ((bt_off[1] ^ (j << 6)) + step)));
            fb[j] = __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
        } else {
            fb[j] = *reinterpret_cast<const bf16x8*>(base + (k16 ? b_off1 : b_off0) + j * 32 * 64);
        }
    };
    auto mma = [&](bf16x8 (&fa)[TM], bf16x8 (&fb)[TN], int x) {
        acc[x / TN][x % TN] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[x / TN], fb[x % TN], acc[x / TN][x % TN], 0, 0, 0);
    };

    // Load schedule (pair p = chunks 2p, 2p+1 -> slots 2p % RING, (2p+1) % RING):
    //   up front           A(0), B(0), A(1)
    //   iteration 2p-2     B(p)   (even iterations, p >= 1)
    //   iteration 2p-3     A(p)   (odd iterations,  p >= 2)
    // The barrier inside iteration i needs every group requested before iteration i to have landed
    // (A part of slot i+2, B part of slot i+1), i.e. only this iteration's own loads may be in flight.
    if (n_pairs > 0) { issue_group(kA); issue_group(kB); }
    if (n_pairs > 1) issue_group(kA);
    if (n_pairs > 0) {
        if (n_pairs > 1) wait_vmcnt<C::LOADS>(); else wait_vmcnt<0>();
        __syncthreads();
#pragma unroll
        for (int j = 0; j < TN; ++j) read_b(fb0, lds, 0, j);
#pragma unroll
        for (int m = 0; m < TM; ++m) read_a(fa0, lds, a_off0, m);
    }
    int tile = 0, kc = 0, slot = 0;
    const int n_kc = 2 * n_k64;
    // `always` = std::true_type: steady state, the iteration's four loads are unconditional (no branches
    // between the MFMAs); std::false_type: drain, loads only while the stream still has pairs to request.
    auto iteration = [&](auto stream, auto always) {
        constexpr bool is_b = decltype(stream)::value;
        const unsigned char* cur = lds + slot * C::SLOT_BYTES;
        slot = slot + 1 == RING ? 0 : slot + 1;
        const unsigned char* nxt = lds + slot * C::SLOT_BYTES;
        const bool loads = decltype(always)::value || (is_b ? b_issued : a_issued) < n_pairs;   // wave-uniform
        // ---- K16 step 0 -------------------------------------------------------------------------
        mma(fa0, fb0, 0); mma(fa0, fb0, 1);
        __builtin_amdgcn_sched_barrier(0);
        read_b(fb1, cur, 1, 0); read_b(fb1, cur, 1, 1);
        if (loads) issue_one(stream, 0);
        __builtin_amdgcn_sched_barrier(0);
        mma(fa0, fb0, 2); mma(fa0, fb0, 3);
        __builtin_amdgcn_sched_barrier(0);
        read_a(fa1, cur, a_off1, 0); read_a(fa1, cur, a_off1, 1);
        __builtin_amdgcn_sched_barrier(0);
        mma(fa0, fb0, 4); mma(fa0, fb0, 5);
        __builtin_amdgcn_sched_barrier(0);
        read_a(fa1, cur, a_off1, 2); read_a(fa1, cur, a_off1, 3);
        if (loads) issue_one(stream, 1);
        __builtin_amdgcn_sched_barrier(0);
        mma(fa0, fb0, 6); mma(fa0, fb0, 7);
        __builtin_amdgcn_sched_barrier(0);
        // ---- K16 step 1 -------------------------------------------------------------------------
        mma(fa1, fb1, 0); mma(fa1, fb1, 1);
        __builtin_amdgcn_sched_barrier(0);
        read_a(fa0, nxt, a_off0, 0); read_a(fa0, nxt, a_off0, 1);           // A part of slot i+1: certified already
        if (loads) issue_one(stream, 2);
        __builtin_amdgcn_sched_barrier(0);
        mma(fa1, fb1, 2); mma(fa1, fb1, 3);
        __builtin_amdgcn_sched_barrier(0);
        // everything this wave requested before this iteration has landed (3 younger loads may fly);
        // its own LDS reads are complete; then all waves agree
        if (loads) wait_vmcnt<3>(); else wait_vmcnt<0>();
        __builtin_amdgcn_s_waitcnt(0xC07F);   // lgkmcnt(0) only
        __syncthreads();
        read_b(fb0, nxt, 0, 0); read_b(fb0, nxt, 0, 1);           // B part of slot i+1: certified just now
        read_a(fa0, nxt, a_off0, 2); read_a(fa0, nxt, a_off0, 3);
        __builtin_amdgcn_sched_barrier(0);
        mma(fa1, fb1, 4); mma(fa1, fb1, 5);
        __builtin_amdgcn_sched_barrier(0);
        if (loads) { issue_one(stream, 3); advance(stream); }
        __builtin_amdgcn_sched_barrier(0);
        mma(fa1, fb1, 6); mma(fa1, fb1, 7);
    };
    auto end_of_pair = [&]() {
        kc += 2;
        if (kc == n_kc) {   // a tile ends on an odd chunk (the K extent is a multiple of 64)
            epilogue(acc, tile);
            kc = 0;
            ++tile;
        }
    };
    // even iteration i requests the B lines of pair i/2 + 1, odd iteration i+1 the A lines of pair i/2 + 2
    int i = 0;
    for (; i < n_chunks && a_issued < n_pairs; i += 2) {   // steady state (the A stream runs one pair ahead)
        iteration(kB, std::true_type{});
        iteration(kA, std::true_type{});
        end_of_pair();
    }
    for (; i < n_chunks; i += 2) {                          // drain: the last two pairs
        iteration(kB, std::false_type{});
        iteration(kA, std::false_type{});
        end_of_pair();
    }
    wait_vmcnt<0>();
    __builtin_amdgcn_s_waitcnt(0xC07F);
    __syncthreads();   // every fragment read and every load into LDS has finished
}

}  // namespace ring_nt
