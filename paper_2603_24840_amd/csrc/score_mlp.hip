// arrol_score_mlp: quality head as a 2-layer MLP (Sec. 4.2 allows a small two-layer MLP as the
// rollout quality head), followed by the sigmoid normalisation (App. A.4):
//     a = relu(W1 h + b1),  s = <w2, a> + b2,  q = sigmoid(s)
// One fused kernel: bf16 MFMA for W1 h (transposed, A^T = W1 H^T, so that a lane's accumulator values
// belong to one rollout and the reduction over hidden units is lane-local), bias + ReLU + the dot with w2
// on the accumulators in registers; the [N, m] activations never reach memory.
// Tile: 256 hidden units x 128 rollouts per workgroup pass, 4 wavefronts, each 2 x (32 units) x 128
// rollouts; K chunks of 64 in XOR-swizzled 16-byte chunks, loaded global -> LDS directly into three stages
// when d is a multiple of 64, else staged global -> registers -> LDS (two stages).
//
// arrol_score_mlp_grad: cross-entropy training gradient of the same head (Sec. 4.2, Sec. 4.3 (iii)).  The same
// tile loop runs in two more modes:
//   delta   recomputes the pre-activations and, instead of the w2 dot, writes delta^T[u][i] =
//           r_i * w2[u] * [pre > 0] (bf16, unit-major) and the per-workgroup sums for dL/dw2 and dL/db1;
//   wgrad   the contraction over rollouts dL/dW1 = delta^T . H as the same "A rows x B rows over a shared
//           contiguous K" product, with A = delta^T [m, N] and B = H^T [d, N] (transposed once into the
//           workspace), fp32 tile stores, optionally split over K with partial slabs added in a fixed order.
#include "common.h"
#include "ring_nt.h"

namespace {

using ring_nt::bf16x8;
typedef float f32x16 __attribute__((ext_vector_type(16)));   // 32x32x16 accumulators of the tile and small-batch kernels

constexpr int kThreads = 256;
constexpr int BU = 256;   // hidden units per pass
constexpr int BR = 128;   // rollouts per workgroup
constexpr int BK = 64;
constexpr int TU = 2;     // 32-unit blocks per wave (unit rows c*128 + wave*32 + ...)
constexpr int TR = 4;     // 32-rollout blocks per wave
constexpr int kStageBytes = (BU + BR) * BK * 2;
constexpr int kLdsBytes = 2 * kStageBytes;          // register-staged path: two stages
constexpr int kRingStages = 3;                      // direct-to-LDS path: three stages, two of them in flight
constexpr int kRingLdsBytes = kRingStages * kStageBytes;
constexpr int kRingLoadsA = BU / 8 / 4;             // load instructions (8 rows x 128 bytes) per wave and stage
constexpr int kRingLoadsB = BR / 8 / 4;
constexpr int kRingLoads = kRingLoadsA + kRingLoadsB;
constexpr int kPassA = BU * (BK / 8) / kThreads;   // 16-byte loads per thread for the W1 tile
constexpr int kPassB = BR * (BK / 8) / kThreads;

__device__ __forceinline__ int chunk_offset(int r, int c) { return r * 128 + ((c ^ ((r >> 1) & 7)) << 4); }

enum MlpMode { kForward = 0, kDelta = 1, kWgrad = 2, kForwardKeep = 3 };   // kForwardKeep: ring kernel only

// The tile loop multiplies A rows (w1, a_stride elements apart, m of them) with B rows (hidden, n_rows of
// them) over a contiguous K extent of d elements.
struct MlpArgs {
    const uint16_t* hidden; int64_t row_stride; const int64_t* row_index;
    const uint16_t* w1; int64_t a_stride; const float* b1; const float* w2; float b2;
    int n_rows, d, m;
    float* score_out; float* prob_out;
    // delta mode
    const float* resid;          // [n_rows] r_i = (q_i - y_i) / N
    uint16_t* delta_t;           // [m][delta_stride] bf16
    uint16_t* delta_lo;          // NULL, or [m][delta_stride] bf16: bf16(delta - float(delta_t)), the second term
    int64_t delta_stride;
    float* unit_partial;         // [gridDim.x][2][m]: sums over the workgroup's rollouts for dL/dw2, dL/db1
    // wgrad mode: blockIdx.y = K split, blockIdx.z = group of 256 A rows
    float* c_out;                // [gridDim.y][m][c_stride] fp32
    int64_t c_stride;
    int kc_per_split;            // K chunks (of 64) per split
};

template <int N>
__device__ __forceinline__ void mlp_wait_vmcnt() {  // s_waitcnt vmcnt(N) only (gfx9 encoding), N <= 15
    __builtin_amdgcn_s_waitcnt(0x0F70 | N);
}

// RING = false: any d (multiple of 8), K chunks staged global -> registers -> LDS, one chunk ahead.
// RING = true (d a multiple of 64): K chunks go global -> LDS directly (no staging registers) into three
// stages, two chunks ahead, so that a workgroup that is alone on its CU (few rollouts) still hides the
// memory latency.  One instruction moves 8 tile rows x 128 bytes; lane l writes physical chunk l%8 of row
// l/8, and fetches the logical chunk that the XOR swizzle stores there.
template <int MODE, bool RING>
__global__ __launch_bounds__(kThreads) void score_mlp_kernel(MlpArgs a) {
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    typedef __attribute__((address_space(3))) void* lds_ptr_t;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l31 = lane & 31, lh = lane >> 5;
    const int row0 = blockIdx.x * BR;

    // staging geometry: thread -> (tile row tid/8 (+32 per pass), 16-byte chunk tid%8)
    const int ld_c = tid & 7, ld_r = tid >> 3;
    const int ld_lds = chunk_offset(ld_r, ld_c);
    const uint16_t* h_row[kPassB];
#pragma unroll
    for (int p = 0; p < kPassB; ++p) {
        int r = row0 + ld_r + p * 32;
        r = r < a.n_rows ? r : a.n_rows - 1;
        const int64_t src = a.row_index ? a.row_index[r] : r;
        h_row[p] = a.hidden + src * a.row_stride;
    }
    const int n_kc_all = (a.d + BK - 1) / BK;
    // forward / delta: every K chunk, every group of 256 units in turn; wgrad: one K split, one group
    const int kc0 = MODE == kWgrad ? static_cast<int>(blockIdx.y) * a.kc_per_split : 0;
    const int kc1 = MODE == kWgrad ? (kc0 + a.kc_per_split < n_kc_all ? kc0 + a.kc_per_split : n_kc_all) : n_kc_all;
    const int n_kc = kc1 - kc0;
    const int g0 = MODE == kWgrad ? static_cast<int>(blockIdx.z) : 0;
    const int n_groups = MODE == kWgrad ? 1 : (a.m + BU - 1) / BU;
    const int total_it = n_groups * n_kc;

    float resid[TR] = {0.f, 0.f, 0.f, 0.f};
    if (MODE == kDelta) {
#pragma unroll
        for (int j = 0; j < TR; ++j) {
            const int r = row0 + j * 32 + l31;
            resid[j] = r < a.n_rows ? a.resid[r] : 0.f;
        }
    }

    constexpr int NSTAGE_REGS = RING ? 1 : kPassA + kPassB;
    uint4 stage[NSTAGE_REGS];
    int ld_g = g0, ld_kc = 0;
    auto issue_loads = [&]() {
        const int k = (kc0 + ld_kc) * BK + ld_c * 8;
        const bool k_ok = k < a.d;
#pragma unroll
        for (int p = 0; p < kPassA; ++p) {
            int u = ld_g * BU + ld_r + p * 32;
            u = u < a.m ? u : a.m - 1;
            stage[p] = k_ok ? *reinterpret_cast<const uint4*>(a.w1 + static_cast<int64_t>(u) * a.a_stride + k) : make_uint4(0, 0, 0, 0);
        }
#pragma unroll
        for (int p = 0; p < kPassB; ++p)
            stage[kPassA + p] = k_ok ? *reinterpret_cast<const uint4*>(h_row[p] + k) : make_uint4(0, 0, 0, 0);
        if (++ld_kc == n_kc) { ld_kc = 0; ++ld_g; }
    };
    auto store_stage = [&](int buf) {
        unsigned char* sa = lds + buf * kStageBytes + ld_lds;
        unsigned char* sb = sa + BU * BK * 2;
#pragma unroll
        for (int p = 0; p < kPassA; ++p) *reinterpret_cast<uint4*>(sa + p * 32 * 128) = stage[p];
#pragma unroll
        for (int p = 0; p < kPassB; ++p) *reinterpret_cast<uint4*>(sb + p * 32 * 128) = stage[kPassA + p];
    };

    // ---- direct-to-LDS loader (RING) ---------------------------------------------------------------------
    // wave w fetches A groups w*8 .. w*8+7 and B groups w*4 .. w*4+3 of every stage (a group = 8 tile rows)
    const int rl_row = lane >> 3;                                     // row inside the group
    constexpr int NPTR_A = RING ? kRingLoadsA : 1, NPTR_B = RING ? kRingLoadsB : 1;
    const uint16_t* ring_a[NPTR_A];                                   // per lane: row base + logical chunk, k = 0
    const uint16_t* ring_b[NPTR_B];
    const unsigned lds0 = static_cast<unsigned>(reinterpret_cast<size_t>((lds_ptr_t)lds));
    auto ring_point_a = [&](int grp) {                                // A rows of unit group `grp`
#pragma unroll
        for (int q = 0; q < NPTR_A; ++q) {
            const int r = (wave * kRingLoadsA + q) * 8 + rl_row;      // tile row 0 .. 255
            int u = grp * BU + r;
            u = u < a.m ? u : a.m - 1;
            const int logical = (lane & 7) ^ ((r >> 1) & 7);
            ring_a[q] = a.w1 + static_cast<int64_t>(u) * a.a_stride + logical * 8;
        }
    };
    if (RING) {
#pragma unroll
        for (int q = 0; q < NPTR_B; ++q) {
            const int r = (wave * kRingLoadsB + q) * 8 + rl_row;      // tile row 0 .. 127
            int row = row0 + r;
            row = row < a.n_rows ? row : a.n_rows - 1;
            const int64_t src = a.row_index ? a.row_index[row] : row;
            const int logical = (lane & 7) ^ ((r >> 1) & 7);
            ring_b[q] = a.hidden + src * a.row_stride + logical * 8;
        }
        ring_point_a(g0);
    }
    int ring_g = g0, ring_kc = 0, ring_buf = 0;
    auto ring_issue = [&]() {                                         // the next chunk -> stage ring_buf
        const int64_t k = static_cast<int64_t>(kc0 + ring_kc) * BK;
        const unsigned dst_a = lds0 + ring_buf * kStageBytes + wave * kRingLoadsA * 1024;
        const unsigned dst_b = lds0 + ring_buf * kStageBytes + BU * BK * 2 + wave * kRingLoadsB * 1024;
#pragma unroll
        for (int q = 0; q < NPTR_A; ++q) {
            const uint16_t* src = ring_a[q] + k;
            asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(src), "s"(dst_a + q * 1024) : "memory");
        }
#pragma unroll
        for (int q = 0; q < NPTR_B; ++q) {
            const uint16_t* src = ring_b[q] + k;
            asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(src), "s"(dst_b + q * 1024) : "memory");
        }
        ring_buf = ring_buf + 1 == kRingStages ? 0 : ring_buf + 1;
        if (++ring_kc == n_kc) {
            ring_kc = 0;
            ++ring_g;
            ring_point_a(ring_g);        // rows of the next unit group (clamped: harmless past the last group)
        }
    };

    f32x16 acc[TU][TR];
#pragma unroll
    for (int c = 0; c < TU; ++c)
#pragma unroll
        for (int j = 0; j < TR; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[c][j][v] = 0.f;
    float part[TR] = {0.f, 0.f, 0.f, 0.f};   // this lane's share of s for rollout row0 + j*32 + l31

    const int swz = (l31 >> 1) & 7;
    if (RING) {
        ring_issue();
        if (total_it > 1) ring_issue();
    } else {
        issue_loads();
        store_stage(0);
        __syncthreads();
    }
    int g = g0, kc = 0, buf = 0;
    for (int it = 0; it < total_it; ++it) {
        const bool more = it + 1 < total_it;
        if (RING) {
            // this wave's share of chunk `it` has landed (only the chunk after it may still be in flight) ...
            if (more) mlp_wait_vmcnt<kRingLoads>(); else mlp_wait_vmcnt<0>();
            // ... then so has everybody's, and nobody still reads the stage of chunk it-1, which chunk it+2 refills
            __syncthreads();
            if (it + 2 < total_it) ring_issue();
        } else if (more) {
            issue_loads();
        }
        const unsigned char* sa = lds + buf * kStageBytes;
        const unsigned char* sb = sa + BU * BK * 2;
        buf = buf + 1 == (RING ? kRingStages : 2) ? 0 : buf + 1;
#pragma unroll
        for (int kk = 0; kk < BK / 16; ++kk) {
            const int coff = ((kk * 2 + lh) ^ swz) << 4;
            bf16x8 fa[TU], fb[TR];
#pragma unroll
            for (int c = 0; c < TU; ++c)
                fa[c] = *reinterpret_cast<const bf16x8*>(sa + (c * 128 + wave * 32 + l31) * 128 + coff);
#pragma unroll
            for (int j = 0; j < TR; ++j)
                fb[j] = *reinterpret_cast<const bf16x8*>(sb + (j * 32 + l31) * 128 + coff);
#pragma unroll
            for (int c = 0; c < TU; ++c)
#pragma unroll
                for (int j = 0; j < TR; ++j)
                    acc[c][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[c], fb[j], acc[c][j], 0, 0, 0);
        }
        if (!RING) {
            if (more) store_stage(buf);
            __syncthreads();
        }
        if (++kc == n_kc) {
            // acc[c][j][v] belongs to A row (unit) g*BU + c*128 + wave*32 + (v/4)*8 + lh*4 + v%4 and B row
            // (rollout) row0 + j*32 + l31
#pragma unroll
            for (int c = 0; c < TU; ++c)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int u = g * BU + c * 128 + wave * 32 + (v >> 2) * 8 + lh * 4 + (v & 3);
                    const bool live = u < a.m;
                    if (MODE == kWgrad) {
                        float* crow = a.c_out + (static_cast<int64_t>(blockIdx.y) * a.m + u) * a.c_stride;
#pragma unroll
                        for (int j = 0; j < TR; ++j) {
                            const int col = row0 + j * 32 + l31;
                            if (live && col < a.n_rows) crow[col] = acc[c][j][v];
                            acc[c][j][v] = 0.f;
                        }
                    } else {
                        const float bias = (live && a.b1) ? a.b1[u] : 0.f;
                        const float w = live ? a.w2[u] : 0.f;
                        if (MODE == kForward) {
#pragma unroll
                            for (int j = 0; j < TR; ++j) {
                                part[j] = fmaf(fmaxf(acc[c][j][v] + bias, 0.f), w, part[j]);
                                acc[c][j][v] = 0.f;
                            }
                        } else {
                            float gw = 0.f, gb = 0.f;
                            uint16_t* drow = a.delta_t + static_cast<int64_t>(live ? u : 0) * a.delta_stride + row0 + l31;
#pragma unroll
                            for (int j = 0; j < TR; ++j) {
                                const float pre = acc[c][j][v] + bias;
                                const float dl = pre > 0.f ? resid[j] * w : 0.f;
                                gw = fmaf(resid[j], fmaxf(pre, 0.f), gw);
                                gb += dl;
                                if (live) {
                                    const uint16_t hi = f32_to_bf16_rne(dl);
                                    drow[j * 32] = hi;
                                    if (a.delta_lo) (a.delta_lo + (drow - a.delta_t))[j * 32] = f32_to_bf16_rne(dl - bf16_lo(hi));
                                }
                                acc[c][j][v] = 0.f;
                            }
                            // sum over the 32 rollout lanes of this half-wave (both halves run the same steps)
#pragma unroll
                            for (int msk = 16; msk >= 1; msk >>= 1) {
                                gw += __shfl_xor(gw, msk, ARROL_WAVE);
                                gb += __shfl_xor(gb, msk, ARROL_WAVE);
                            }
                            if (live && l31 == 0) {
                                float* up = a.unit_partial + static_cast<int64_t>(blockIdx.x) * 2 * a.m;
                                up[u] = gw;
                                up[a.m + u] = gb;
                            }
                        }
                    }
                }
            kc = 0;
            ++g;
        }
    }
    if (MODE != kForward) return;
    // lane halves hold different units of the same rollout; then the four waves
#pragma unroll
    for (int j = 0; j < TR; ++j) part[j] += __shfl_xor(part[j], 32, ARROL_WAVE);
    if (RING) __syncthreads();                    // every wave has finished reading the last stage
    float* red = reinterpret_cast<float*>(lds);   // [4 waves][BR]
    if (lh == 0) {
#pragma unroll
        for (int j = 0; j < TR; ++j) red[wave * BR + j * 32 + l31] = part[j];
    }
    __syncthreads();
    if (tid < BR && row0 + tid < a.n_rows) {
        const float s = red[tid] + red[BR + tid] + red[2 * BR + tid] + red[3 * BR + tid] + a.b2;
        float q;
        if (s >= 0.f) {
            q = 1.f / (1.f + expf(-s));
        } else {
            const float e = expf(s);
            q = e / (1.f + e);
        }
        if (a.score_out) a.score_out[row0 + tid] = s;
        a.prob_out[row0 + tid] = q;
    }
}

// ---------------------------------------------------------------------------------------------------------
// Small batches (a few hundred rollouts): the tile kernel above would run on n_rows / 128 compute units and
// each of them would walk all of K behind a three-stage ring (bytes in flight over memory latency: ~90 us
// for 512 x 2048 x 512).  Here every wavefront owns one 32-unit x 32-rollout block of the pre-activations
// over the whole K, n_rows/32 x m/32 wavefronts in all, and takes its MFMA fragments straight from global
// memory: no LDS, no barrier, kSmallDepth K64 blocks (2 x 4 x 16 bytes per lane each) in flight per lane,
// one wavefront per workgroup.
// The contraction does not care in which order K is visited, so a lane loads 64 CONTIGUOUS bytes of its row
// per K64 block (lane half lh takes k in [32 lh, 32 lh + 32)) and the q-th 16 bytes feed the q-th MFMA of
// the block, the same assignment on both operands.  Each wavefront writes sum_u w2[u] relu(pre[u] + b1[u])
// over its 32 units to partial[unit block][rollout]; a second kernel adds the unit blocks in index order.
constexpr int kSmallMaxRows = 4096;     // beyond this the tile kernel has enough workgroups of its own
constexpr int kSmallDepth = 4;          // K64 blocks in flight
constexpr int kSmallThreads = 64;       // one wavefront per workgroup: its lanes address 64 different cache lines per
                                        // load, so the texture addresser of a compute unit is the resource to spread over

__global__ __launch_bounds__(kSmallThreads) void score_mlp_small_kernel(
    const uint16_t* __restrict__ hidden, int64_t row_stride, const int64_t* __restrict__ row_index,
    const uint16_t* __restrict__ w1, const float* __restrict__ b1, const float* __restrict__ w2, int n_rows, int d, int m,
    int n_ub, float* __restrict__ partial, float* __restrict__ act_t, int64_t act_stride) {
    const int lane = threadIdx.x & 63;
    const int l31 = lane & 31, lh = lane >> 5;
    const int ub = blockIdx.y;                      // unit block
    const int r0 = blockIdx.x * 32, u0 = ub * 32;
    int row = r0 + l31;
    row = row < n_rows ? row : n_rows - 1;
    int unit = u0 + l31;
    unit = unit < m ? unit : m - 1;
    const int64_t src = row_index ? row_index[row] : row;
    const uint4* hp = reinterpret_cast<const uint4*>(hidden + src * row_stride + lh * 32);
    const uint4* wp = reinterpret_cast<const uint4*>(w1 + static_cast<int64_t>(unit) * d + lh * 32);
    const int n_kb = d / 64;                        // host: d is a multiple of 64
    uint4 fa[kSmallDepth][4], fb[kSmallDepth][4];
    auto load_block = [&](int slot, int kb) {       // 8 uint4 = one K64 block of this lane's two rows
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            fa[slot][q] = wp[kb * 8 + q];
            fb[slot][q] = hp[kb * 8 + q];
        }
    };
#pragma unroll
    for (int s = 0; s < kSmallDepth; ++s)
        if (s < n_kb) load_block(s, s);
    f32x16 acc;
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[v] = 0.f;
    for (int kb0 = 0; kb0 < n_kb; kb0 += kSmallDepth) {
#pragma unroll
        for (int s = 0; s < kSmallDepth; ++s) {
            const int kb = kb0 + s;
            if (kb < n_kb) {                        // wave-uniform
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, fa[s][q]),
                                                                  __builtin_bit_cast(bf16x8, fb[s][q]), acc, 0, 0, 0);
                if (kb + kSmallDepth < n_kb) load_block(s, kb + kSmallDepth);
            }
        }
    }
    // acc[v] = pre-activation of unit u0 + (v/4)*8 + lh*4 + v%4 for rollout r0 + l31
    float part = 0.f;
#pragma unroll
    for (int v = 0; v < 16; ++v) {
        const int u = u0 + (v >> 2) * 8 + lh * 4 + (v & 3);
        const bool live = u < m;
        const float bias = (live && b1) ? b1[u] : 0.f;
        const float w = live ? w2[u] : 0.f;
        const float act = fmaxf(acc[v] + bias, 0.f);
        part = fmaf(act, w, part);
        // the gradient call keeps relu(pre), unit-major (see mlp_delta_kernel)
        if (act_t && live && r0 + l31 < n_rows) act_t[static_cast<int64_t>(u) * act_stride + r0 + l31] = act;
    }
    part += __shfl_xor(part, 32, ARROL_WAVE);       // the two lane halves hold different units of one rollout
    if (lh == 0 && r0 + l31 < n_rows) partial[static_cast<int64_t>(ub) * n_rows + r0 + l31] = part;
}

__global__ __launch_bounds__(256) void score_mlp_small_finish_kernel(const float* __restrict__ partial, int n_ub,
                                                                     int n_rows, float b2, float* __restrict__ score_out,
                                                                     float* __restrict__ prob_out) {
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i >= n_rows) return;
    float s = 0.f;
    for (int ub = 0; ub < n_ub; ++ub) s += partial[static_cast<int64_t>(ub) * n_rows + i];
    s += b2;
    float q;
    if (s >= 0.f) {
        q = 1.f / (1.f + expf(-s));
    } else {
        const float e = expf(s);
        q = e / (1.f + e);
    }
    if (score_out) score_out[i] = s;
    prob_out[i] = q;
}

// ---------------------------------------------------------------------------------------------------------
// Large batches (more than kSmallMaxRows rollouts, d a multiple of 64, rows addressed without row_index):
// the contractions on the 8-wavefront direct-to-LDS ring pipeline of ring_nt.h (v_mfma_f32_16x16x32_bf16), one
// 256 x 256 accumulator tile per workgroup: grid = (blocks of 256 B rows, tiles of 256 A rows, K splits).
//   forward  A = W1 [m, d], B = hidden [N, d]: bias + ReLU + w2 dot per rollout (lane-local over the
//            units), partial scores [unit tile][rollout] to the workspace, summed by the finish kernel;
//            for the gradient call the same pass also keeps the activations a = relu(pre) in fp32, unit-major
//            (the accumulator's own layout: 16 lanes = 16 consecutive rollouts), so that nothing is recomputed:
//            delta^T = r w2 [a > 0] and the per-unit sums are then one streaming pass (mlp_delta_kernel);
//   wgrad    A = delta^T [m, n_pad], B = the hidden states themselves, [N, d] = K-major (ring_nt's TN form, no
//            transposed copy), over K = rollouts (split): fp32 tile stores.
using RingCfg = ring_nt::RingTile<256, 256, 2, 4>;

struct MlpRingArgs {
    const uint16_t* a; unsigned a_stride;   // A rows (bytes between rows), a_rows of them
    const uint16_t* b; unsigned b_stride;   // B rows, b_rows of them; wgrad: k-rows of b_rows values, b_k_rows of them
    int a_rows, b_rows, b_k_rows, n_k64, k64_per_split;
    const float* b1; const float* w2;
    float* partial;              // forward: [gridDim.y][b_rows]
    float* act_t; int64_t act_stride;       // forward for the gradient: relu(pre), [a_rows][act_stride] fp32
    float* c_out; int64_t c_stride;         // wgrad: [gridDim.z][a_rows][c_stride]
};

template <int MODE>
__global__ __launch_bounds__(RingCfg::NT) void mlp_ring_kernel(MlpRingArgs a) {
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    using C = RingCfg;
    constexpr int BM = C::BM, BN = C::BN, TI = C::TI, TJ = C::TJ;
    const int tb = blockIdx.x, vt = blockIdx.y;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / C::WN, wn = wave % C::WN;
    const int l15 = lane & 15, lq = lane >> 4;
    const int k64_lo = MODE == kWgrad ? static_cast<int>(blockIdx.z) * a.k64_per_split : 0;
    const int k64_hi = MODE == kWgrad ? (k64_lo + a.k64_per_split < a.n_k64 ? k64_lo + a.k64_per_split : a.n_k64) : a.n_k64;

    ring_nt::Walk w;
    w.a_base = reinterpret_cast<const char*>(a.a) + static_cast<int64_t>(vt) * BM * a.a_stride + static_cast<int64_t>(k64_lo) * 128;
    w.b_base = MODE == kWgrad
                   ? reinterpret_cast<const char*>(a.b) + static_cast<int64_t>(k64_lo) * 64 * a.b_stride + static_cast<int64_t>(tb) * BN * 2
                   : reinterpret_cast<const char*>(a.b) + static_cast<int64_t>(tb) * BN * a.b_stride + static_cast<int64_t>(k64_lo) * 128;
    w.a_stride = a.a_stride;
    w.b_stride = a.b_stride;
    w.a_rows = a.a_rows - vt * BM;
    w.b_rows = a.b_rows - tb * BN < BN ? a.b_rows - tb * BN : BN;
    w.n_k64 = k64_hi > k64_lo ? k64_hi - k64_lo : 0;
    w.b_k_rows = a.b_k_rows - k64_lo * 64;

    const int unit0 = vt * BM + wm * (BM / C::WM);           // first A row of this wavefront
    const int row0 = tb * BN + wn * (BN / C::WN);            // first B row of this wavefront
    float part[TJ] = {0.f, 0.f, 0.f, 0.f};
    ring_nt::f32x4 acc[TI][TJ];
    ring_nt::walk<C, MODE == kWgrad>(w, lds, acc);
    {
        // acc[i][j][v]: A row unit0 + i*16 + lq*4 + v, B row row0 + j*16 + l15
#pragma unroll
        for (int i = 0; i < TI; ++i)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int u = unit0 + i * 16 + lq * 4 + v;
                const bool live = u < a.a_rows;
                if (MODE == kWgrad) {
                    float* crow = a.c_out + (static_cast<int64_t>(blockIdx.z) * a.a_rows + u) * a.c_stride;
#pragma unroll
                    for (int j = 0; j < TJ; ++j) {
                        const int col = row0 + j * 16 + l15;
                        if (live && col < a.b_rows) crow[col] = acc[i][j][v];
                    }
                } else {
                    const float bias = (live && a.b1) ? a.b1[u] : 0.f;
                    const float wu = live ? a.w2[u] : 0.f;
                    float* arow = MODE == kForwardKeep ? a.act_t + static_cast<int64_t>(live ? u : 0) * a.act_stride : nullptr;
#pragma unroll
                    for (int j = 0; j < TJ; ++j) {
                        const float act = fmaxf(acc[i][j][v] + bias, 0.f);
                        part[j] = fmaf(act, wu, part[j]);
                        if (MODE == kForwardKeep) {
                            const int col = row0 + j * 16 + l15;
                            if (live && col < a.b_rows) arow[col] = act;
                        }
                    }
                }
            }
    }
    if (MODE == kWgrad) return;
    // the four lane quarters and the two wavefront rows hold different units of the same rollouts
    float* red = reinterpret_cast<float*>(lds);   // [WM][BN]
#pragma unroll
    for (int j = 0; j < TJ; ++j) {
        part[j] += __shfl_xor(part[j], 16, ARROL_WAVE);
        part[j] += __shfl_xor(part[j], 32, ARROL_WAVE);
    }
    if (lq == 0) {
#pragma unroll
        for (int j = 0; j < TJ; ++j) red[wm * BN + wn * (BN / C::WN) + j * 16 + l15] = part[j];
    }
    __syncthreads();
    for (int col = tid; col < BN; col += C::NT) {
        const int r = tb * BN + col;
        if (r < a.b_rows) a.partial[static_cast<int64_t>(vt) * a.b_rows + r] = red[col] + red[BN + col];
    }
}

template <int MODE>
int launch_mlp_ring(const MlpRingArgs& a, dim3 grid, hipStream_t st) {
    static arrol_device_flags ok;
    if (!arrol_allow_lds(&mlp_ring_kernel<MODE>, RingCfg::LDS_BYTES, ok)) return ARROL_EHIP;
    arrol_launch(mlp_ring_kernel<MODE>, grid, dim3(RingCfg::NT), RingCfg::LDS_BYTES, st, a);
    return ARROL_OK;
}

// the ring kernels address a lane's row with a 32-bit byte offset inside a 256-row tile
bool ring_applies(int n_rows, int d, int64_t row_stride_elems, const int64_t* row_index) {
    return n_rows > kSmallMaxRows && d % 64 == 0 && row_index == nullptr && row_stride_elems * 2 * 256 < (1ll << 31);
}

// dL/dW1 on the ring pipeline's K-major B form: any batch size, rows addressed in place
bool ring_wgrad_applies(int d, int64_t row_stride_elems, const int64_t* row_index) {
    return d % 64 == 0 && row_index == nullptr && row_stride_elems * 2 * 256 < (1ll << 31);
}

// r_i = (q_i - y_i) / N and the loss: one workgroup per 1024 rows writes its two partial sums, the second
// kernel adds them in block order (fixed summation order, bit-reproducible)
__global__ __launch_bounds__(1024) void mlp_residual_kernel(const float* __restrict__ score,
                                                            const float* __restrict__ prob,
                                                            const float* __restrict__ labels, int n_rows,
                                                            float* __restrict__ resid, float* __restrict__ block_sums) {
    __shared__ float red[2][16];
    const float inv_n = 1.f / static_cast<float>(n_rows);
    float loss = 0.f, rs = 0.f;
    const int i = blockIdx.x * 1024 + threadIdx.x;
    if (i < n_rows) {
        const float s = score[i], y = labels[i];
        const float r = (prob[i] - y) * inv_n;
        resid[i] = r;
        rs = r;
        loss = fmaxf(s, 0.f) - y * s + log1pf(expf(-fabsf(s)));
    }
    loss = wave_sum_f32(loss);
    rs = wave_sum_f32(rs);
    const int lane = threadIdx.x & (ARROL_WAVE - 1), wave = threadIdx.x / ARROL_WAVE;
    if (lane == 0) { red[0][wave] = loss; red[1][wave] = rs; }
    __syncthreads();
    if (threadIdx.x == 0) {
        float a = 0.f, b = 0.f;
        for (int w = 0; w < 16; ++w) { a += red[0][w]; b += red[1][w]; }
        block_sums[blockIdx.x] = a;
        block_sums[gridDim.x + blockIdx.x] = b;
    }
}

// The gradient call after a forward pass that leaves partial scores (partial[unit block][rollout]):
// score_mlp_small_finish_kernel and mlp_residual_kernel in one launch - score = sum over the unit blocks in index
// order + b2, then r_i and the loss terms as above; neither scores nor probabilities go to memory.
__global__ __launch_bounds__(1024) void mlp_finish_residual_kernel(const float* __restrict__ partial, int n_ub,
                                                                   float b2, const float* __restrict__ labels,
                                                                   int n_rows, float* __restrict__ resid,
                                                                   float* __restrict__ block_sums) {
    __shared__ float red[2][16];
    const float inv_n = 1.f / static_cast<float>(n_rows);
    float loss = 0.f, rs = 0.f;
    const int i = blockIdx.x * 1024 + threadIdx.x;
    if (i < n_rows) {
        float s = 0.f;
        for (int ub = 0; ub < n_ub; ++ub) s += partial[static_cast<int64_t>(ub) * n_rows + i];
        s += b2;
        float q;
        if (s >= 0.f) {
            q = 1.f / (1.f + expf(-s));
        } else {
            const float e = expf(s);
            q = e / (1.f + e);
        }
        const float y = labels[i];
        const float r = (q - y) * inv_n;
        resid[i] = r;
        rs = r;
        loss = fmaxf(s, 0.f) - y * s + log1pf(expf(-fabsf(s)));
    }
    loss = wave_sum_f32(loss);
    rs = wave_sum_f32(rs);
    const int lane = threadIdx.x & (ARROL_WAVE - 1), wave = threadIdx.x / ARROL_WAVE;
    if (lane == 0) { red[0][wave] = loss; red[1][wave] = rs; }
    __syncthreads();
    if (threadIdx.x == 0) {
        float a = 0.f, b = 0.f;
        for (int w = 0; w < 16; ++w) { a += red[0][w]; b += red[1][w]; }
        block_sums[blockIdx.x] = a;
        block_sums[gridDim.x + blockIdx.x] = b;
    }
}

__global__ void mlp_residual_finish_kernel(const float* __restrict__ block_sums, int n_blocks, int n_rows,
                                           float* __restrict__ loss_out, float* __restrict__ grad_b2) {
    float a = 0.f, b = 0.f;
    for (int k = 0; k < n_blocks; ++k) { a += block_sums[k]; b += block_sums[n_blocks + k]; }
    if (loss_out) *loss_out = a / static_cast<float>(n_rows);
    if (grad_b2) *grad_b2 = b;
}

// delta^T and the per-unit sums from the kept activations: one workgroup per unit u streams its row
//   delta^T[u][i] = r_i w2_u [a_ui > 0] (bf16, 0 for n_rows <= i < n_pad; optionally the bf16 remainder too),
//   dL/dw2_u = sum_i r_i a_ui,  dL/db1_u = sum_i r_i w2_u [a_ui > 0],
// each lane over its own columns in ascending order, then lanes, then wavefronts: a fixed summation order.
// Workgroup 0 also finishes the loss and dL/db2 from the residual pass's block sums.
constexpr int kDeltaThreads = 1024;
__global__ __launch_bounds__(kDeltaThreads) void mlp_delta_kernel(const float* __restrict__ act_t, int64_t act_stride,
                                                                  const float* __restrict__ resid,
                                                                  const float* __restrict__ w2, int n_rows, int n_pad,
                                                                  uint16_t* __restrict__ delta_t,
                                                                  uint16_t* __restrict__ delta_lo,
                                                                  float* __restrict__ grad_w2,
                                                                  float* __restrict__ grad_b1,
                                                                  const float* __restrict__ block_sums, int n_blocks,
                                                                  float* __restrict__ loss_out,
                                                                  float* __restrict__ grad_b2) {
    __shared__ float red[2][kDeltaThreads / ARROL_WAVE];
    const int u = blockIdx.x;
    if (u == 0 && threadIdx.x == 0) {   // loss and dL/db2: the residual pass's block sums, added in block order
        float a = 0.f, b = 0.f;
        for (int k = 0; k < n_blocks; ++k) { a += block_sums[k]; b += block_sums[n_blocks + k]; }
        if (loss_out) *loss_out = a / static_cast<float>(n_rows);
        if (grad_b2) *grad_b2 = b;
    }
    const float wu = w2[u];
    const float* arow = act_t + static_cast<int64_t>(u) * act_stride;
    uint16_t* drow = delta_t + static_cast<int64_t>(u) * n_pad;
    float gw = 0.f, gb = 0.f;
    for (int i = threadIdx.x * 4; i < n_pad; i += kDeltaThreads * 4) {   // n_pad is a multiple of 4
        float av[4] = {0.f, 0.f, 0.f, 0.f}, rv[4] = {0.f, 0.f, 0.f, 0.f};
        if (i + 3 < n_rows) {
            const float4 a4 = *reinterpret_cast<const float4*>(arow + i);
            const float4 r4 = *reinterpret_cast<const float4*>(resid + i);
            av[0] = a4.x; av[1] = a4.y; av[2] = a4.z; av[3] = a4.w;
            rv[0] = r4.x; rv[1] = r4.y; rv[2] = r4.z; rv[3] = r4.w;
        } else {
#pragma unroll
            for (int q = 0; q < 4; ++q)
                if (i + q < n_rows) { av[q] = arow[i + q]; rv[q] = resid[i + q]; }
        }
        uint16_t dq[4], lq[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const float dl = av[q] > 0.f ? rv[q] * wu : 0.f;
            gw = fmaf(rv[q], av[q], gw);
            gb += dl;
            dq[q] = f32_to_bf16_rne(dl);
            lq[q] = f32_to_bf16_rne(dl - bf16_lo(dq[q]));
        }
        uint2 o;
        o.x = static_cast<uint32_t>(dq[0]) | (static_cast<uint32_t>(dq[1]) << 16);
        o.y = static_cast<uint32_t>(dq[2]) | (static_cast<uint32_t>(dq[3]) << 16);
        *reinterpret_cast<uint2*>(drow + i) = o;
        if (delta_lo) {     // second term of the two-term form: what bf16 rounding left of delta
            o.x = static_cast<uint32_t>(lq[0]) | (static_cast<uint32_t>(lq[1]) << 16);
            o.y = static_cast<uint32_t>(lq[2]) | (static_cast<uint32_t>(lq[3]) << 16);
            *reinterpret_cast<uint2*>(delta_lo + static_cast<int64_t>(u) * n_pad + i) = o;
        }
    }
    gw = wave_sum_f32(gw);
    gb = wave_sum_f32(gb);
    const int lane = threadIdx.x & (ARROL_WAVE - 1), wave = threadIdx.x / ARROL_WAVE;
    if (lane == 0) { red[0][wave] = gw; red[1][wave] = gb; }
    __syncthreads();
    if (threadIdx.x == 0) {
        float a = 0.f, b = 0.f;
        for (int w = 0; w < kDeltaThreads / ARROL_WAVE; ++w) { a += red[0][w]; b += red[1][w]; }
        grad_w2[u] = a;
        grad_b1[u] = b;
    }
}

// out[c][i] = hidden[row(i)][c] for i < n_rows, 0 for n_rows <= i < n_pad: 64 x 64 tiles through LDS, 16 bytes
// per lane on both sides (8 lanes cover the 128 bytes a tile row has in the source and in the destination)
__global__ __launch_bounds__(256) void mlp_transpose_kernel(const uint16_t* __restrict__ hidden, int64_t row_stride,
                                                            const int64_t* __restrict__ row_index, int n_rows,
                                                            int d, int n_pad, uint16_t* __restrict__ out) {
    __shared__ __attribute__((aligned(16))) uint16_t tile_t[64][72];   // [column][rollout], 144-byte pitch
    const int i0 = blockIdx.x * 64, c0 = blockIdx.y * 64;
    const int chunk = threadIdx.x & 7, r8 = threadIdx.x >> 3;           // 32 rows x 8 chunks per pass
#pragma unroll
    for (int p = 0; p < 2; ++p) {
        const int r = r8 + p * 32, i = i0 + r, c = c0 + chunk * 8;
        uint4 v = make_uint4(0, 0, 0, 0);
        if (i < n_rows && c < d) {      // d is a multiple of 8: a chunk is inside the row or outside it
            const int64_t src = row_index ? row_index[i] : i;
            v = *reinterpret_cast<const uint4*>(hidden + src * row_stride + c);
        }
        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            tile_t[chunk * 8 + 2 * q][r] = static_cast<uint16_t>(w[q] & 0xffffu);
            tile_t[chunk * 8 + 2 * q + 1][r] = static_cast<uint16_t>(w[q] >> 16);
        }
    }
    __syncthreads();
#pragma unroll
    for (int p = 0; p < 2; ++p) {
        const int cr = r8 + p * 32, c = c0 + cr, i = i0 + chunk * 8;
        if (c < d && i < n_pad)          // n_pad is a multiple of 64: whole chunks
            *reinterpret_cast<uint4*>(out + static_cast<int64_t>(c) * n_pad + i) =
                *reinterpret_cast<const uint4*>(&tile_t[cr][chunk * 8]);
    }
}

struct GradPlan {
    int n_rb, n_pad, n_cb, n_groups, n_kc, splits, kc_per_split;
    int r_cb, r_vt, r_gt, r_splits, r_k64_per_split;
    size_t off_score, off_prob, off_resid, off_bsum, off_ht, off_dt, off_unit, off_slab, off_small, off_rslab, off_act, total;
};

size_t align256(size_t x) { return (x + 255) & ~static_cast<size_t>(255); }

GradPlan make_grad_plan(int n_rows, int d, int m, int terms) {
    GradPlan p;
    p.n_rb = (n_rows + BR - 1) / BR;
    p.n_pad = p.n_rb * BR;
    p.n_cb = (d + BR - 1) / BR;              // wgrad: 128 columns of dL/dW1 per workgroup
    // dL/dW1 contracts [hi; lo] (terms * m rows) with H and leaves one partial per term and K split
    const int mt = terms * m;
    p.n_groups = (mt + BU - 1) / BU;
    p.n_kc = p.n_pad / BK;
    // split K so that about 256 workgroups run, each with at least 8 chunks; at most 8 partial slabs
    int s = 256 / (p.n_cb * p.n_groups);
    if (s > p.n_kc / 8) s = p.n_kc / 8;
    if (s > 8) s = 8;
    if (s < 1) s = 1;
    p.kc_per_split = (p.n_kc + s - 1) / s;
    p.splits = (p.n_kc + p.kc_per_split - 1) / p.kc_per_split;
    size_t o = 0;
    p.off_score = o; o = align256(o + sizeof(float) * n_rows);
    p.off_prob = o;  o = align256(o + sizeof(float) * n_rows);
    p.off_resid = o; o = align256(o + sizeof(float) * n_rows);
    p.off_bsum = o;  o = align256(o + sizeof(float) * 2 * ((n_rows + 1023) / 1024));
    p.off_ht = o;    o = align256(o + sizeof(uint16_t) * static_cast<size_t>(d) * p.n_pad);
    p.off_dt = o;    o = align256(o + sizeof(uint16_t) * static_cast<size_t>(mt) * p.n_pad);
    // per-unit partial sums of the tile kernel: one row per 128 rollouts
    p.off_unit = o;  o = align256(o + sizeof(float) * static_cast<size_t>(p.n_rb) * 2 * m);
    p.off_slab = o;
    if (p.splits * terms > 1) o = align256(o + sizeof(float) * static_cast<size_t>(p.splits) * mt * d);
    p.off_small = o;                      // partial scores of the small-batch / ring forward pass
    if (d % 64 == 0) {
        const size_t blocks = n_rows <= kSmallMaxRows ? (m + 31) / 32 : (m + 255) / 256;
        o = align256(o + sizeof(float) * blocks * n_rows);
    }
    // ring wgrad: 256-column blocks; K split so that about 256 workgroups run, at most 8 partial slabs
    p.r_cb = (d + 255) / 256;
    p.r_vt = (m + 255) / 256;          // forward pass
    p.r_gt = (mt + 255) / 256;         // dL/dW1
    int rs = 256 / (p.r_cb * p.r_gt);
    if (rs > p.n_kc / 8) rs = p.n_kc / 8;
    if (rs > 8) rs = 8;
    if (rs < 1) rs = 1;
    p.r_k64_per_split = (p.n_kc + rs - 1) / rs;
    p.r_splits = (p.n_kc + p.r_k64_per_split - 1) / p.r_k64_per_split;
    p.off_rslab = o;
    if (d % 64 == 0 && p.r_splits * terms > 1) o = align256(o + sizeof(float) * static_cast<size_t>(p.r_splits) * mt * d);
    p.off_act = o;                        // small-batch / ring forward pass: kept activations, fp32 [m][n_pad]
    if (d % 64 == 0) o = align256(o + sizeof(float) * static_cast<size_t>(m) * p.n_pad);
    p.total = o;
    return p;
}

template <int MODE>
int launch_mlp(const MlpArgs& a, dim3 grid, hipStream_t st) {
    static arrol_device_flags lds_ok, ring_ok;
    if (a.d % BK == 0) {   // direct-to-LDS path
        if (!arrol_allow_lds(&score_mlp_kernel<MODE, true>, kRingLdsBytes, ring_ok)) return ARROL_EHIP;
        arrol_launch((score_mlp_kernel<MODE, true>), grid, dim3(kThreads), kRingLdsBytes, st, a);
    } else {
        if (!arrol_allow_lds(&score_mlp_kernel<MODE, false>, kLdsBytes, lds_ok)) return ARROL_EHIP;
        arrol_launch((score_mlp_kernel<MODE, false>), grid, dim3(kThreads), kLdsBytes, st, a);
    }
    return arrol_launch_status();
}

}  // namespace

extern "C" size_t arrol_score_mlp_workspace_bytes(int32_t n_rows, int32_t d, int32_t m) {
    if (n_rows < 1 || d < 8 || m < 1) return 0;
    if (d % 64) return 0;   // the one-launch tile kernel needs no scratch
    const size_t blocks = n_rows <= kSmallMaxRows ? (m + 31) / 32 : (m + 255) / 256;   // unit blocks of the two paths
    return align256(sizeof(float) * blocks * n_rows);
}

extern "C" int arrol_score_mlp(const void* hidden, int64_t row_stride_elems, const int64_t* row_index,
                               const void* w1, const float* b1, const float* w2, float b2, int32_t n_rows,
                               int32_t d, int32_t m, float* score_out, float* prob_out, void* workspace,
                               size_t workspace_bytes, void* stream) {
    if (n_rows < 0 || d < 8 || (d & 7) || m < 1 || row_stride_elems < d || (row_stride_elems & 7)) return ARROL_EINVAL;
    if (n_rows == 0) return ARROL_OK;
    if (!hidden || !w1 || !w2 || !prob_out || !arrol_aligned16(hidden) || !arrol_aligned16(w1)) return ARROL_EINVAL;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const size_t need = arrol_score_mlp_workspace_bytes(n_rows, d, m);
    if (need > 0 && workspace && arrol_aligned16(workspace) && workspace_bytes >= need &&
        ring_applies(n_rows, d, row_stride_elems, row_index)) {
        // large batch: one 256 x 256 tile per workgroup on the ring pipeline, then the sum over the unit tiles
        const int n_vt = (m + 255) / 256;
        MlpRingArgs r = {};
        r.a = static_cast<const uint16_t*>(w1); r.a_stride = static_cast<unsigned>(d) * 2; r.a_rows = m;
        r.b = static_cast<const uint16_t*>(hidden); r.b_stride = static_cast<unsigned>(row_stride_elems * 2); r.b_rows = n_rows;
        r.n_k64 = d / 64; r.b1 = b1; r.w2 = w2; r.partial = static_cast<float*>(workspace);
        const int rc = launch_mlp_ring<kForward>(r, dim3((n_rows + 255) / 256, n_vt), st);
        if (rc != ARROL_OK) return rc;
        if (arrol_launch_failed()) return arrol_launch_status();
        arrol_launch(score_mlp_small_finish_kernel, dim3((n_rows + 255) / 256), dim3(256), 0, st, r.partial, n_vt,
                     n_rows, b2, score_out, prob_out);
        return arrol_launch_status();
    }
    if (need > 0 && n_rows <= kSmallMaxRows && workspace && arrol_aligned16(workspace) && workspace_bytes >= need) {
        // small batch: one wavefront per 32 x 32 block of pre-activations, then the sum over the unit blocks
        const int n_ub = (m + 31) / 32;
        float* partial = static_cast<float*>(workspace);
        arrol_launch(score_mlp_small_kernel, dim3((n_rows + 31) / 32, n_ub), dim3(kSmallThreads), 0, st,
                     static_cast<const uint16_t*>(hidden), row_stride_elems, row_index, static_cast<const uint16_t*>(w1),
                     b1, w2, n_rows, d, m, n_ub, partial, static_cast<float*>(nullptr), static_cast<int64_t>(0));
        if (arrol_launch_failed()) return arrol_launch_status();
        arrol_launch(score_mlp_small_finish_kernel, dim3((n_rows + 255) / 256), dim3(256), 0, st, partial, n_ub,
                     n_rows, b2, score_out, prob_out);
        return arrol_launch_status();
    }
    MlpArgs a = {};
    a.hidden = static_cast<const uint16_t*>(hidden); a.row_stride = row_stride_elems; a.row_index = row_index;
    a.w1 = static_cast<const uint16_t*>(w1); a.a_stride = d; a.b1 = b1; a.w2 = w2; a.b2 = b2;
    a.n_rows = n_rows; a.d = d; a.m = m; a.score_out = score_out; a.prob_out = prob_out;
    return launch_mlp<kForward>(a, dim3((n_rows + BR - 1) / BR), st);
}

extern "C" size_t arrol_score_mlp_grad_workspace_bytes(int32_t n_rows, int32_t d, int32_t m, int32_t delta_terms) {
    if (n_rows < 1 || d < 8 || m < 1 || delta_terms < 1 || delta_terms > 2) return 0;
    return make_grad_plan(n_rows, d, m, delta_terms).total;
}

extern "C" int arrol_score_mlp_grad(const void* hidden, int64_t row_stride_elems, const int64_t* row_index,
                                    const void* w1, const float* b1, const float* w2, float b2,
                                    const float* labels, int32_t n_rows, int32_t d, int32_t m, float* loss_out,
                                    float* grad_w1, float* grad_b1, float* grad_w2, float* grad_b2,
                                    int32_t delta_terms, void* workspace, size_t workspace_bytes, void* stream) {
    if (n_rows < 0 || d < 8 || (d & 7) || m < 1 || row_stride_elems < d || (row_stride_elems & 7)) return ARROL_EINVAL;
    if (delta_terms < 1 || delta_terms > 2 || m > INT32_MAX / 2) return ARROL_EINVAL;
    if (!grad_w1 || !grad_b1 || !grad_w2) return ARROL_EINVAL;
    if (n_rows == 0) {   // empty batch: zero loss and gradients
        hipStream_t s0 = static_cast<hipStream_t>(stream);
        const int64_t width = static_cast<int64_t>(m) * d;
        arrol_launch(reduce_rows_f32_kernel<0>, dim3(static_cast<unsigned>((width + 31) / 32)), dim3(256), 0, s0,
                           nullptr, 0, width, width, 0.f, grad_w1);
        arrol_launch(reduce_rows_f32_kernel<0>, dim3((m + 31) / 32), dim3(256), 0, s0, nullptr, 0,
                           static_cast<int64_t>(m), static_cast<int64_t>(m), 0.f, grad_b1);
        arrol_launch(reduce_rows_f32_kernel<0>, dim3((m + 31) / 32), dim3(256), 0, s0, nullptr, 0,
                           static_cast<int64_t>(m), static_cast<int64_t>(m), 0.f, grad_w2);
        if (loss_out) arrol_launch(reduce_rows_f32_kernel<0>, dim3(1), dim3(256), 0, s0, nullptr, 0, 1, 1, 0.f, loss_out);
        if (grad_b2) arrol_launch(reduce_rows_f32_kernel<0>, dim3(1), dim3(256), 0, s0, nullptr, 0, 1, 1, 0.f, grad_b2);
        return arrol_launch_status();
    }
    if (!hidden || !w1 || !w2 || !labels || !arrol_aligned16(hidden) || !arrol_aligned16(w1)) return ARROL_EINVAL;
    const GradPlan p = make_grad_plan(n_rows, d, m, delta_terms);
    const int mt = delta_terms * m;
    if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255u) || workspace_bytes < p.total) return ARROL_EWORKSPACE;
    hipStream_t st = static_cast<hipStream_t>(stream);
    unsigned char* ws = static_cast<unsigned char*>(workspace);
    float* score = reinterpret_cast<float*>(ws + p.off_score);
    float* prob = reinterpret_cast<float*>(ws + p.off_prob);
    float* resid = reinterpret_cast<float*>(ws + p.off_resid);
    float* bsum = reinterpret_cast<float*>(ws + p.off_bsum);
    const int n_rblocks = (n_rows + 1023) / 1024;
    uint16_t* ht = reinterpret_cast<uint16_t*>(ws + p.off_ht);
    uint16_t* dt = reinterpret_cast<uint16_t*>(ws + p.off_dt);                       // [hi; lo]: delta_terms * m rows
    uint16_t* dt_lo = delta_terms == 2 ? dt + static_cast<int64_t>(m) * p.n_pad : nullptr;
    float* unit = reinterpret_cast<float*>(ws + p.off_unit);
    float* slab = reinterpret_cast<float*>(ws + p.off_slab);

    // forward pass.  Batches beyond kSmallMaxRows rows: the ring pipeline; smaller ones: one wavefront per block;
    // both keep relu(pre) for the backward pass.  Otherwise (d not a multiple of 64, or gathered rows of a large
    // batch) the one-launch tile kernel, whose pre-activations are recomputed below.
    MlpArgs a = {};
    a.hidden = static_cast<const uint16_t*>(hidden); a.row_stride = row_stride_elems; a.row_index = row_index;
    a.w1 = static_cast<const uint16_t*>(w1); a.a_stride = d; a.b1 = b1; a.w2 = w2; a.b2 = b2;
    a.n_rows = n_rows; a.d = d; a.m = m; a.score_out = score; a.prob_out = prob;
    float* act = reinterpret_cast<float*>(ws + p.off_act);
    float* partial = reinterpret_cast<float*>(ws + p.off_small);
    bool kept = true;
    int rc = ARROL_OK, n_ub = 0;
    if (ring_applies(n_rows, d, row_stride_elems, row_index)) {
        MlpRingArgs r = {};
        r.a = a.w1; r.a_stride = static_cast<unsigned>(d) * 2; r.a_rows = m;
        r.b = a.hidden; r.b_stride = static_cast<unsigned>(row_stride_elems * 2); r.b_rows = n_rows;
        r.n_k64 = d / 64; r.b1 = b1; r.w2 = w2; r.partial = partial;
        r.act_t = act; r.act_stride = p.n_pad;
        rc = launch_mlp_ring<kForwardKeep>(r, dim3((n_rows + 255) / 256, p.r_vt), st);
        if (rc != ARROL_OK) return rc;
        n_ub = p.r_vt;
    } else if (d % 64 == 0 && n_rows <= kSmallMaxRows) {
        n_ub = (m + 31) / 32;
        arrol_launch(score_mlp_small_kernel, dim3((n_rows + 31) / 32, n_ub), dim3(kSmallThreads), 0, st,
                     a.hidden, row_stride_elems, row_index, a.w1, b1, w2, n_rows, d, m, n_ub, partial, act,
                     static_cast<int64_t>(p.n_pad));
    } else {
        kept = false;
        rc = launch_mlp<kForward>(a, dim3(p.n_rb), st);
        if (rc != ARROL_OK) return rc;
    }
    if (arrol_launch_failed()) return arrol_launch_status();
    if (kept) {
        // scores from the partials, residuals and loss terms in one launch; delta^T, the per-unit sums, the loss
        // and dL/db2 in the next
        arrol_launch(mlp_finish_residual_kernel, dim3(n_rblocks), dim3(1024), 0, st, partial, n_ub, b2, labels, n_rows,
                     resid, bsum);
        arrol_launch(mlp_delta_kernel, dim3(m), dim3(kDeltaThreads), 0, st, act, static_cast<int64_t>(p.n_pad), resid, w2,
                     n_rows, p.n_pad, dt, dt_lo, grad_w2, grad_b1, bsum, n_rblocks, loss_out, grad_b2);
    } else {
        arrol_launch(mlp_residual_kernel, dim3(n_rblocks), dim3(1024), 0, st, score, prob, labels, n_rows, resid, bsum);
        arrol_launch(mlp_residual_finish_kernel, dim3(1), dim3(1), 0, st, bsum, n_rblocks, n_rows, loss_out, grad_b2);
        a.resid = resid; a.delta_t = dt; a.delta_lo = dt_lo; a.delta_stride = p.n_pad; a.unit_partial = unit;
        rc = launch_mlp<kDelta>(a, dim3(p.n_rb), st);
        if (rc != ARROL_OK) return rc;
        arrol_launch(reduce_rows_f32_kernel<0>, dim3((m + 31) / 32), dim3(256), 0, st, unit, p.n_rb,
                     static_cast<int64_t>(2) * m, static_cast<int64_t>(m), 1.f, grad_w2);
        arrol_launch(reduce_rows_f32_kernel<0>, dim3((m + 31) / 32), dim3(256), 0, st, unit + m, p.n_rb,
                     static_cast<int64_t>(2) * m, static_cast<int64_t>(m), 1.f, grad_b1);
    }
    if (arrol_launch_failed()) return arrol_launch_status();
    const int64_t width = static_cast<int64_t>(m) * d;
    if (ring_wgrad_applies(d, row_stride_elems, row_index)) {
        // dL/dW1 = delta^T . H over the rollouts, the hidden states read in place
        float* rslab = reinterpret_cast<float*>(ws + p.off_rslab);
        MlpRingArgs g = {};
        // the partials [K split][term][m][d] are delta_terms * r_splits slabs of m * d values
        const int n_slabs = p.r_splits * delta_terms;
        g.a = dt; g.a_stride = static_cast<unsigned>(p.n_pad) * 2; g.a_rows = mt;
        g.b = a.hidden; g.b_stride = static_cast<unsigned>(row_stride_elems * 2);
        g.b_rows = d; g.b_k_rows = n_rows;
        g.n_k64 = (n_rows + 63) / 64; g.k64_per_split = p.r_k64_per_split;
        g.c_out = n_slabs > 1 ? rslab : grad_w1; g.c_stride = d;
        rc = launch_mlp_ring<kWgrad>(g, dim3(p.r_cb, p.r_gt, p.r_splits), st);
        if (rc != ARROL_OK) return rc;
        if (n_slabs > 1)
            arrol_launch(reduce_rows_f32_kernel<0>, dim3(static_cast<unsigned>((width + 31) / 32)), dim3(256), 0, st,
                         rslab, n_slabs, width, width, 1.f, grad_w1);
        return arrol_launch_status();
    }
    // gathered rows or d not a multiple of 64: H^T, then the tile kernel
    arrol_launch(mlp_transpose_kernel, dim3(p.n_pad / 64, (d + 63) / 64), dim3(256), 0, st,
                 a.hidden, row_stride_elems, row_index, n_rows, d, p.n_pad, ht);
    MlpArgs g = {};
    g.hidden = ht; g.row_stride = p.n_pad; g.row_index = nullptr;
    g.w1 = dt; g.a_stride = p.n_pad;
    const int n_slabs = p.splits * delta_terms;
    g.n_rows = d; g.d = p.n_pad; g.m = mt;
    g.c_out = n_slabs > 1 ? slab : grad_w1; g.c_stride = d; g.kc_per_split = p.kc_per_split;
    rc = launch_mlp<kWgrad>(g, dim3(p.n_cb, p.splits, p.n_groups), st);
    if (rc != ARROL_OK) return rc;
    if (n_slabs > 1)
        arrol_launch(reduce_rows_f32_kernel<0>, dim3(static_cast<unsigned>((width + 31) / 32)), dim3(256), 0, st,
                     slab, n_slabs, width, width, 1.f, grad_w1);
    return arrol_launch_status();
}
