// "NT" contraction pipeline of the MLP quality head's large-batch kernels (gfx950, wave64), the single-tile
// form of the pipeline of the fused log-prob kernel: a workgroup of 8 wavefronts multiplies 256 A rows by 256
// B rows over a K extent that is contiguous in both,
//     acc[a][b] = sum_k A[a][k] * B[b][k]        (bf16 operands, fp32 accumulation, v_mfma_f32_16x16x32_bf16)
// and leaves the 256 x 256 accumulator tile in registers for the caller's epilogue.  In the MFMA result layout
// a lane's 4 values of a 16 x 16 block share the B row (column = lane % 16) and lie on 4 consecutive A rows
// (4 * (lane / 16) + v), so a reduction over A rows per B row (the sum over hidden units) is lane-local.
//
// Operands go global -> LDS directly (no staging registers) into a ring of RING K32 slots (32 k-values =
// 64 bytes of each of the BM + BN tile rows); one MFMA consumes a whole slot.  Loads always fetch whole
// 128-byte lines of a row, i.e. the two K32 halves that go to two consecutive slots (a "pair"); the A lines
// of a pair are requested during one K32 iteration and its B lines during the next.  Per iteration i (chunk i
// lives in slot i % RING, its fragments are in registers when the iteration starts):
//   rows 0-3 of MFMAs (a row = one 16-row A block x the 4 B blocks, B blocks in snake order so that
//               consecutive MFMAs share an operand); A fragment r of slot i+1 is read into the registers of
//               A fragment r once row r has been issued (its A part was certified one barrier earlier; the
//               last two fragments only at the start of the next iteration); the four loads of the iteration;
//   the wait for this wave's older loads, the workgroup barrier;
//   the B fragments of slot i+1 (certified just now) into the second B fragment set, then rows 4-7 with the
//               remaining A fragment reads between them.
// The barrier inside iteration i certifies the A part of slot i+2 and the B part of slot i+1; every read of
// slot i has completed by then, so slot i is free for refilling from there on.  Past its last pair a stream
// keeps requesting that pair's lines (they exist) into slots nobody reads, so the loop has no variant
// without loads.
//
// LDS layout: 16-byte chunk c of tile row r sits at chunk position c ^ 2 * ((r / 4) % 2) of its 64-byte row.
// A 128-bit LDS read serves per cycle the 16 lanes that share lane bit 5 and the parity of lane bits 2, 3, 4
// (measured); with this position two lanes of a half-wave that fall on the same 16-byte bank group differ in
// lane bit 3 alone, and the fragment reads (lane -> row lane % 16, K chunk lane / 16) run without conflicts.
//
// B_KMAJOR = true is the "TN" form: B is given K-major, B[k][b] with the b index contiguous (row k starts
// k * b_stride bytes after the base), so an operand that is stored rollout-major can be contracted over the
// rollouts without a transposed copy.  A K32 slot then holds 32 k-rows of 256 b-values (512 bytes each, the
// same 16 KiB), a load instruction moves two whole k-rows, and the B fragments come out of LDS through the
// transposing read ds_read_b64_tr_b16: in each block of 16 lanes, lane 4e + q supplies the address of four
// consecutive b-values of k-row e, and lane j receives the four k-values of b-value j (layout measured on
// the device).  16-byte chunk c of k-row r sits at chunk position c ^ 4 (r % 4) ^ 2 ((r / 8) % 2) of its row: the 32
// lanes of a half-wave, which a 64-bit read serves together, then fall on 32 different 8-byte bank pairs.
#pragma once
#include <type_traits>

#include "common.h"

namespace ring_nt {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

template <int BM_, int BN_, int WM_, int WN_>
struct RingTile {
    static constexpr int BM = BM_, BN = BN_, WM = WM_, WN = WN_;
    static constexpr int NT = WM * WN * ARROL_WAVE;
    static constexpr int NW = WM * WN;
    static constexpr int TI = BM / WM / 16, TJ = BN / WN / 16;   // 16 x 16 blocks per wave: A rows x B rows
    static constexpr int RING = 5;
    static constexpr int SLOT_BYTES = (BM + BN) * 64;
    static constexpr int LDS_BYTES = RING * SLOT_BYTES;
    static constexpr int G = BM / 16 / NW;                  // 16-row load groups per wave and operand
    static constexpr int LOADS = 2 * G;                     // load instructions per wave and iteration
    static_assert(BM == BN, "A and B tiles are loaded by the same code in alternate iterations");
    static_assert(BM % (16 * NW) == 0, "whole 16-row load groups per wave");
    static_assert(LOADS == 4 && TI == 8 && TJ == 4, "the hand-placed schedule below");
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
    const char* a_base;       // A row 0 of the tile
    const char* b_base;       // B row 0 of this workgroup's block
    unsigned a_stride, b_stride;  // bytes between consecutive rows (< 16 MiB: a lane's row offset is 32-bit)
    int a_rows;               // A rows from a_base on: rows [0, a_rows) exist (>= 1)
    int b_rows;               // B rows of this block that exist (1 .. BN)
    int n_k64;                // K extent / 64 (0: nothing to do, the accumulators come back cleared)
    int b_k_rows;             // B_KMAJOR only: k-rows of B that exist from b_base on (> 64 * (n_k64 - 1));
                              // b_rows is then the number of valid b-values (a multiple of 8), b_stride the
                              // bytes between k-rows
};

// Accumulates one tile into the caller's `acc` (cleared here first): acc[i][j][v] belongs to A row
// wm * (BM / WM) + 16 i + 4 (lane / 16) + v and B row wn * (BN / WN) + 16 j + lane % 16 of the tile, with
// wm = wave / WN, wn = wave % WN.  On return every load into LDS and every fragment read has finished and the
// workgroup has passed a barrier, so LDS is free for the caller.
template <class C, bool B_KMAJOR = false>
__device__ __forceinline__ void walk(const Walk& w, unsigned char* lds, f32x4 (&acc)[C::TI][C::TJ]) {
    constexpr int BM = C::BM, BN = C::BN, TI = C::TI, TJ = C::TJ, RING = C::RING;
    typedef __attribute__((address_space(3))) void* lds_ptr_t;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / C::WN, wn = wave % C::WN;
    const int l15 = lane & 15, lq = lane >> 4;
    // (readfirstlane: wave-uniform by construction; it keeps the loop control in scalar registers)
    const int n_k64 = __builtin_amdgcn_readfirstlane(w.n_k64);   // pairs: two K32 slots = one 128-byte line per row

#pragma unroll
    for (int i = 0; i < TI; ++i)
#pragma unroll
        for (int j = 0; j < TJ; ++j)
#pragma unroll
            for (int v = 0; v < 4; ++v) acc[i][j][v] = 0.f;
    if (n_k64 <= 0) return;   // wave-uniform, the same for the whole workgroup

    // ---- loader geometry: one instruction moves 16 rows x 64 bytes; lane -> (row lane/4, physical
    //      16-byte position lane%4), which holds logical chunk (lane%4) ^ 2*((row/4)%2) -----------
    const int ld_row = lane >> 2;
    const int ld_kb = ((lane & 3) ^ (((lane >> 4) & 1) << 1)) * 16;   // byte offset inside the K32 half
    // Addresses are (wave-uniform 64-bit base in SGPRs) + (per-lane 32-bit byte offset): the base
    // carries the K position, the lane offset the row inside the tile (clamped at the end of the
    // operand, so every load stays inside A and B) and the swizzled chunk.
    unsigned a_voff[C::G], b_voff[C::G];
    int b_lrow[C::G];   // B_KMAJOR: this lane's k-row inside a K32 slot, per load group
    if constexpr (B_KMAJOR) {
        // one instruction = 2 k-rows x 512 bytes: lane -> (k-row lane/32, chunk position lane%32)
        const int chunks_valid = w.b_rows >> 3;
#pragma unroll
        for (int g = 0; g < C::G; ++g) {
            b_lrow[g] = (wave * C::G + g) * 2 + (lane >> 5);
            int c = (lane & 31) ^ ((b_lrow[g] & 3) << 2) ^ (((b_lrow[g] >> 3) & 1) << 1);
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
    {
        const int rows_valid = w.a_rows < BM ? w.a_rows : BM;
#pragma unroll
        for (int g = 0; g < C::G; ++g) {
            int r = (wave * C::G + g) * 16 + ld_row;
            r = r < rows_valid ? r : rows_valid - 1;
            a_voff[g] = static_cast<unsigned>(r) * w.a_stride + ld_kb;
        }
    }
    // two load streams, each walking the pairs 0 .. n_k64-1 and then staying on the last one
    int a_k64 = 0, a_slot = 0;
    int b_k64 = 0, b_slot = 0;
    const char* a_base = w.a_base;
    const char* b_base = w.b_base;
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
            if (b_k64 + 1 < n_k64) {    // past the last pair: stay on it
                ++b_k64;
                b_base += B_KMAJOR ? static_cast<int64_t>(64) * w.b_stride : 128;
            }
            b_slot = b_slot + 2 >= RING ? b_slot + 2 - RING : b_slot + 2;
        } else {
            if (a_k64 + 1 < n_k64) {
                ++a_k64;
                a_base += 128;
            }
            a_slot = a_slot + 2 >= RING ? a_slot + 2 - RING : a_slot + 2;
        }
    };
    auto issue_group = [&](auto stream) {
#pragma unroll
        for (int q = 0; q < C::LOADS; ++q) issue_one(stream, q);
        advance(stream);
    };
    constexpr std::false_type kA{};   // A lines
    constexpr std::true_type kB{};    // B lines

    // fragment reads: one MFMA takes the whole K32 of a slot: row (wave base + i*16 + lane%16), 16-byte chunk
    // lane/16 at position chunk ^ 2*((row/4)%2)
    const int swz = ((l15 >> 2) & 1) << 1;
    const int a_off = (wm * (BM / C::WM) + l15) * 64 + ((lq ^ swz) << 4);
    const int b_off = BM * 64 + (wn * (BN / C::WN) + l15) * 64 + ((lq ^ swz) << 4);
    // B_KMAJOR: lane 16 lq + 4 e + q addresses k-row 8 lq + 4 h2 + e, b-values wn*64 + 16 j + 4 q .. + 3; block j
    // is 2 j chunks on: an XOR with j << 5 (XORs commute with the swizzle)
    int bt_off[2] = {0, 0};
    if constexpr (B_KMAJOR) {
        const int e = l15 >> 2, q = l15 & 3;
        const int chunk = wn * (BN / C::WN / 8) + (q >> 1);
#pragma unroll
        for (int h2 = 0; h2 < 2; ++h2)
            bt_off[h2] = BM * 64 + (8 * lq + 4 * h2 + e) * 512 + ((chunk ^ (e << 2) ^ ((lq & 1) << 1)) << 4) + (q & 1) * 8;
    }
    bf16x8 fa[TI], fbe[TJ], fbo[TJ];   // A fragments (reloaded row by row), B fragments of even / odd iterations
    auto read_a = [&](const unsigned char* base, int i) {
        fa[i] = *reinterpret_cast<const bf16x8*>(base + a_off + i * 16 * 64);
    };
    auto read_b = [&](bf16x8 (&fb)[TJ], const unsigned char* base, int j) {
        if constexpr (B_KMAJOR) {
            typedef short s16x4 __attribute__((ext_vector_type(4)));
            typedef __attribute__((address_space(3))) s16x4* lds_s16x4_t;
            const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_t)(base + (bt_off[0] ^ (j << 5))));
            const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_t)(base + (bt_off[1] ^ (j << 5))));
            fb[j] = __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
        } else {
            fb[j] = *reinterpret_cast<const bf16x8*>(base + b_off + j * 16 * 64);
        }
    };

    // Load schedule (pair p = chunks 2p, 2p+1 -> slots 2p % RING, (2p+1) % RING):
    //   up front           A(0), B(0), A(1)
    //   iteration 2p-2     B(p)   (even iterations, p >= 1)
    //   iteration 2p-3     A(p)   (odd iterations,  p >= 2)
    // The barrier inside iteration i needs every group requested before iteration i to have landed
    // (A part of slot i+2, B part of slot i+1), i.e. only this iteration's own loads may be in flight.
    issue_group(kA); issue_group(kB); issue_group(kA);
    wait_vmcnt<C::LOADS>();
    __syncthreads();
#pragma unroll
    for (int j = 0; j < TJ; ++j) read_b(fbe, lds, j);
#pragma unroll
    for (int i = 0; i < TI - 2; ++i) read_a(lds, i);
    int slot = 0;
    auto iteration = [&](auto stream) {
        constexpr bool is_b = decltype(stream)::value;
        const unsigned char* cur = lds + slot * C::SLOT_BYTES;
        slot = slot + 1 == RING ? 0 : slot + 1;
        const unsigned char* nxt = lds + slot * C::SLOT_BYTES;
        bf16x8 (&fb)[TJ] = is_b ? fbe : fbo;
        bf16x8 (&fbn)[TJ] = is_b ? fbo : fbe;
        // (scheduling fences around every row: without them the compiler lets LDS reads drift between the MFMAs)
        auto row = [&](int i) {
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int jj = 0; jj < TJ; ++jj) {
                const int j = (i & 1) ? TJ - 1 - jj : jj;
                acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
            }
            __builtin_amdgcn_sched_barrier(0);
        };
        read_a(cur, 6); read_a(cur, 7);
        row(0);
        read_a(nxt, 0);
        issue_one(stream, 0);
        issue_one(stream, 1);
        row(1);
        read_a(nxt, 1);
        issue_one(stream, 2);
        issue_one(stream, 3); advance(stream);
        row(2);
        row(3);
        // everything this wave requested before this iteration has landed (its own 4 loads may fly); its own
        // LDS reads are complete (the last one was issued two rows of MFMAs ago); then all waves agree
        wait_vmcnt<4>();
        __builtin_amdgcn_s_waitcnt(0xC07F);   // lgkmcnt(0) only
        __syncthreads();
#pragma unroll
        for (int j = 0; j < TJ; ++j) read_b(fbn, nxt, j);                    // B part of slot i+1: certified just now
        row(4);
        read_a(nxt, 2); read_a(nxt, 3);
        row(5);
        read_a(nxt, 4); read_a(nxt, 5);
        row(6);
        row(7);
    };
    // even iteration i requests the B lines of pair i/2 + 1, odd iteration i+1 the A lines of pair i/2 + 2
    for (int p = 0; p < n_k64; ++p) {
        iteration(kB);
        iteration(kA);
    }
    wait_vmcnt<0>();
    __builtin_amdgcn_s_waitcnt(0xC07F);
    __syncthreads();   // every fragment read and every load into LDS has finished
}

}  // namespace ring_nt
