// arrol_logprob: per-token log pi(o_t | o_<t) on the re-batched survivors
// (policy term of GRPO's importance ratio, Sec. 3; computed by the frontend on the
// survivors, Sec. 4.3 (ii), Alg. 1).
//
//   logprob_t = z_t[y_t] - logsumexp_v z_t[v],   z_t = W h_t
//
// One fused kernel: bf16 MFMA (v_mfma_f32_32x32x16_bf16) LM-head contraction with the
// vocabulary tiled, an online (running max / running sum) logsumexp and the target-logit
// capture applied to each accumulator tile while it is still in registers.  The [T, V]
// logits never reach memory.  The product is computed transposed, Z^T = W H^T, so that in
// the MFMA result layout a lane's 16 accumulator values of a 32x32 block belong to ONE token
// (column = lane % 32) and 16 different vocabulary rows: the softmax reduction over the
// vocabulary is then lane-local, and the only cross-lane work is one merge at the very end.
//
// Work decomposition: grid = token blocks (BN tokens) x vocabulary splits; a workgroup walks
// the vocabulary tiles (BM rows) of its split and, inside each, the K chunks (BK) of d.
// Every (split, token) writes a partial (max, sumexp, target logit); a small second kernel
// merges the splits.  Workgroup ids are mapped so that the workgroups resident on one XCD
// (ids congruent mod 8) form a (few token blocks) x (all splits) patch and share their
// H and W tiles through that XCD's L2.
#include <type_traits>

#include "common.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kNegBig = -1.0e30f;  // finite stand-in for "no logit seen yet"
constexpr int kXcds = 8;

template <int BM_, int BN_, int BK_, int WM_, int WN_>
struct Tile {
    static constexpr int BM = BM_, BN = BN_, BK = BK_, WM = WM_, WN = WN_;
    static constexpr int NT = WM * WN * ARROL_WAVE;       // threads per workgroup
    static constexpr int TM = BM / WM / 32;               // 32-row vocab blocks per wave
    static constexpr int TN = BN / WN / 32;               // 32-token blocks per wave
    static constexpr int CPR = BK / 8;                    // 16-byte chunks per tile row
    static constexpr int ROWS_PER_PASS = NT / CPR;
    static constexpr int PA = BM / ROWS_PER_PASS;         // load passes for the W tile
    static constexpr int PB = BN / ROWS_PER_PASS;         // load passes for the H tile
    static constexpr int STAGE_BYTES = (BM + BN) * BK * 2;
    static constexpr int LDS_BYTES = 2 * STAGE_BYTES;
    static_assert(BK == 64, "the LDS swizzle below assumes 128-byte tile rows");
    static_assert(BM % (WM * 32) == 0 && BN % (WN * 32) == 0, "wave tiles are made of 32x32 blocks");
    static_assert(BM % ROWS_PER_PASS == 0 && BN % ROWS_PER_PASS == 0 && ROWS_PER_PASS % 16 == 0, "load passes");
};

// Position of 16-byte chunk c of tile row r inside a [rows][64] bf16 LDS tile.  The XOR
// spreads the 16 rows that one quarter-wave reads at the same k over all 64 banks.
__device__ __forceinline__ int lds_chunk_offset(int r, int c) { return r * 128 + ((c ^ ((r >> 1) & 7)) << 4); }

struct LogprobArgs {
    const uint16_t* H;      // [T, d]
    const uint16_t* W;      // [V, d]
    const int32_t* targets; // [T]
    float* part;            // [n_sp][3][T]  (max, sumexp, target logit)
    int64_t T;
    int V, d;
    int n_tb, n_sp, n_vt;
};

// Per-lane online-softmax state: the lane owns token (wave token base + j*32 + lane%32), j < TN.
template <int TN>
struct LaneState {
    float run_m[TN], run_s[TN], tgt_z[TN];
    int tgt[TN];
};

// Folds one finished accumulator tile into the running (max, sumexp, target logit) and clears it.
// acc[i][j][v] is the logit of vocab row vrow0 + i*32 + (v/4)*8 + lh*4 + v%4 for the lane's token of
// block j (MFMA 32x32 result layout); WROWS = vocab rows per wave tile.
template <int TM, int TN, int WROWS>
__device__ __forceinline__ void tile_epilogue(f32x16 (&acc)[TM][TN], LaneState<TN>& st, int vrow0, int V, int lh) {
    if (vrow0 + WROWS > V) {  // tile hangs over the end of the vocabulary
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const bool dead = vrow0 + i * 32 + (v >> 2) * 8 + lh * 4 + (v & 3) >= V;
#pragma unroll
                for (int j = 0; j < TN; ++j) acc[i][j][v] = dead ? -INFINITY : acc[i][j][v];
            }
    }
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        const int rel = st.tgt[j] - vrow0;
        const bool mine = rel >= 0 && rel < WROWS && ((rel >> 2) & 1) == lh;
        if (__any(mine)) {
            const int code = mine ? ((rel >> 5) * 16 + ((rel & 31) >> 3) * 4 + (rel & 3)) : -1;
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int v = 0; v < 16; ++v)
                    if (code == i * 16 + v) st.tgt_z[j] = acc[i][j][v];
        }
        float mx = acc[0][j][0];
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int v = 0; v < 16; ++v) mx = fmaxf(mx, acc[i][j][v]);
        const float m_new = fmaxf(st.run_m[j], mx);
        const float neg = -m_new * kLog2e;
        float sum = 0.f;
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                sum += __builtin_amdgcn_exp2f(fmaf(acc[i][j][v], kLog2e, neg));
                acc[i][j][v] = 0.f;
            }
        // difference first: exactly 0 when the maximum did not move (also for the -1e30 sentinel)
        st.run_s[j] = st.run_s[j] * __builtin_amdgcn_exp2f((st.run_m[j] - m_new) * kLog2e) + sum;
        st.run_m[j] = m_new;
    }
}

// End of a workgroup's vocabulary range: merge the two lane halves (same token, different vocab
// rows), then the WM waves that share a token range (through LDS, `red` = [WM][3][BN] floats, the
// staging memory being idle by now), and write the (max, sumexp, target logit) partial of split sp.
template <int TN, int WM, int WN, int BN, int NT>
__device__ __forceinline__ void write_partials(LaneState<TN>& st, float* red, int wm, int wn, int l31, int lh,
                                               int tid, int64_t tok0, int64_t T, int sp, float* part) {
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        const float om = __shfl_xor(st.run_m[j], 32, ARROL_WAVE);
        const float os = __shfl_xor(st.run_s[j], 32, ARROL_WAVE);
        const float oz = __shfl_xor(st.tgt_z[j], 32, ARROL_WAVE);
        const float m = fmaxf(st.run_m[j], om);
        st.run_s[j] = st.run_s[j] * __builtin_amdgcn_exp2f((st.run_m[j] - m) * kLog2e) +
                      os * __builtin_amdgcn_exp2f((om - m) * kLog2e);
        st.run_m[j] = m;
        st.tgt_z[j] += oz;
    }
    if (lh == 0) {
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int col = wn * (BN / WN) + j * 32 + l31;
            red[(wm * 3 + 0) * BN + col] = st.run_m[j];
            red[(wm * 3 + 1) * BN + col] = st.run_s[j];
            red[(wm * 3 + 2) * BN + col] = st.tgt_z[j];
        }
    }
    __syncthreads();
    for (int col = tid; col < BN; col += NT) {
        const int64_t t = tok0 + col;
        if (t >= T) continue;
        float m = red[col], s = red[BN + col], z = red[2 * BN + col];
#pragma unroll
        for (int w = 1; w < WM; ++w) {
            const float om = red[(w * 3 + 0) * BN + col], os = red[(w * 3 + 1) * BN + col];
            const float mm = fmaxf(m, om);
            s = s * __builtin_amdgcn_exp2f((m - mm) * kLog2e) + os * __builtin_amdgcn_exp2f((om - mm) * kLog2e);
            m = mm;
            z += red[(w * 3 + 2) * BN + col];
        }
        float* p = part + static_cast<int64_t>(sp) * 3 * T + t;
        p[0] = m;
        p[T] = s;
        p[2 * T] = z;
    }
}

// The same for the 16x16x32 MFMA result layout: acc[i][j][v] is the logit of vocab row vrow0 + i*16 + lq*4 + v
// (lq = lane / 16) for the lane's token of block j (token j*16 + lane%16 of the wave's range).  The accumulators
// are left as they are (the next tile's first MFMAs take 0 as their addend).
template <int TI, int TJ, int WROWS>
__device__ __forceinline__ void tile_epilogue16(f32x4 (&acc)[TI][TJ], LaneState<TJ>& st, int vrow0, int V, int lq,
                                                const int32_t* tgt_wave, int tgt_valid, int l15) {
    // the lane's targets are fetched again for every tile (from cache) instead of living in registers through
    // the K loop: tgt_wave (wave-uniform) points at the wave's first token, of which tgt_valid exist
    int tgt[TJ];
#pragma unroll
    for (int j = 0; j < TJ; ++j) tgt[j] = j * 16 + l15 < tgt_valid ? tgt_wave[j * 16 + l15] : -1;
    if (vrow0 + WROWS > V) {  // tile hangs over the end of the vocabulary
        const int lim = V - vrow0 - lq * 4;   // rows of this lane from here on are past the end: one value per tile,
#pragma unroll                                // compared with constants (nothing per (i, v) to keep in registers)
        for (int i = 0; i < TI; ++i)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const bool dead = i * 16 + v >= lim;
#pragma unroll
                for (int j = 0; j < TJ; ++j) acc[i][j][v] = dead ? -INFINITY : acc[i][j][v];
            }
    }
#pragma unroll
    for (int j = 0; j < TJ; ++j) {
        const int rel = tgt[j] - vrow0;
        const bool mine = rel >= 0 && rel < WROWS && ((rel >> 2) & 3) == lq;
        if (__any(mine)) {
            const int code = mine ? ((rel >> 4) * 4 + (rel & 3)) : -1;
#pragma unroll
            for (int i = 0; i < TI; ++i)
#pragma unroll
                for (int v = 0; v < 4; ++v)
                    if (code == i * 4 + v) st.tgt_z[j] = acc[i][j][v];
        }
        float mx = acc[0][j][0];
#pragma unroll
        for (int i = 0; i < TI; ++i)
#pragma unroll
            for (int v = 0; v < 4; ++v) mx = fmaxf(mx, acc[i][j][v]);
        const float m_new = fmaxf(st.run_m[j], mx);
        const float neg = -m_new * kLog2e;
        float sum = 0.f;
#pragma unroll
        for (int i = 0; i < TI; ++i)
#pragma unroll
            for (int v = 0; v < 4; ++v) sum += __builtin_amdgcn_exp2f(fmaf(acc[i][j][v], kLog2e, neg));
        // difference first: exactly 0 when the maximum did not move (also for the -1e30 sentinel)
        st.run_s[j] = st.run_s[j] * __builtin_amdgcn_exp2f((st.run_m[j] - m_new) * kLog2e) + sum;
        st.run_m[j] = m_new;
        __builtin_amdgcn_sched_barrier(0);   // one token column at a time: keeps the temporaries of the exp chains few
    }
}

// End of a workgroup's vocabulary range, 16x16 layout: merge the four lane quarters (same token, different
// vocab rows), then the WM waves that share a token range through LDS, and write the partial of split sp.
template <int TJ, int WM, int WN, int BN, int NT>
__device__ __forceinline__ void write_partials16(LaneState<TJ>& st, float* red, int wm, int wn, int l15, int lq,
                                                 int tid, int64_t tok0, int64_t T, int sp, float* part) {
#pragma unroll
    for (int j = 0; j < TJ; ++j) {
#pragma unroll
        for (int msk = 16; msk <= 32; msk <<= 1) {
            const float om = __shfl_xor(st.run_m[j], msk, ARROL_WAVE);
            const float os = __shfl_xor(st.run_s[j], msk, ARROL_WAVE);
            const float oz = __shfl_xor(st.tgt_z[j], msk, ARROL_WAVE);
            const float m = fmaxf(st.run_m[j], om);
            st.run_s[j] = st.run_s[j] * __builtin_amdgcn_exp2f((st.run_m[j] - m) * kLog2e) +
                          os * __builtin_amdgcn_exp2f((om - m) * kLog2e);
            st.run_m[j] = m;
            st.tgt_z[j] += oz;
        }
    }
    if (lq == 0) {
#pragma unroll
        for (int j = 0; j < TJ; ++j) {
            const int col = wn * (BN / WN) + j * 16 + l15;
            red[(wm * 3 + 0) * BN + col] = st.run_m[j];
            red[(wm * 3 + 1) * BN + col] = st.run_s[j];
            red[(wm * 3 + 2) * BN + col] = st.tgt_z[j];
        }
    }
    __syncthreads();
    for (int col = tid; col < BN; col += NT) {
        const int64_t t = tok0 + col;
        if (t >= T) continue;
        float m = red[col], s = red[BN + col], z = red[2 * BN + col];
#pragma unroll
        for (int w = 1; w < WM; ++w) {
            const float om = red[(w * 3 + 0) * BN + col], os = red[(w * 3 + 1) * BN + col];
            const float mm = fmaxf(m, om);
            s = s * __builtin_amdgcn_exp2f((m - mm) * kLog2e) + os * __builtin_amdgcn_exp2f((om - mm) * kLog2e);
            m = mm;
            z += red[(w * 3 + 2) * BN + col];
        }
        float* p = part + static_cast<int64_t>(sp) * 3 * T + t;
        p[0] = m;
        p[T] = s;
        p[2 * T] = z;
    }
}

// workgroup id -> (token block, vocab split): ids congruent mod 8 land on the same XCD, so an XCD
// works on token blocks xcd, xcd+8, ... and, for each, on all splits back to back.
__device__ __forceinline__ bool map_workgroup(const LogprobArgs& a, int& tb, int& sp, int& vt_lo, int& vt_hi) {
    const int bid = blockIdx.x;
    const int xcd = bid % kXcds, idx = bid / kXcds;
    sp = idx % a.n_sp;
    tb = (idx / a.n_sp) * kXcds + xcd;
    if (tb >= a.n_tb) return false;
    vt_lo = static_cast<int>(static_cast<int64_t>(a.n_vt) * sp / a.n_sp);
    vt_hi = static_cast<int>(static_cast<int64_t>(a.n_vt) * (sp + 1) / a.n_sp);
    return true;
}

// ---------------------------------------------------------------------------------------------
// General kernel (any d that is a multiple of 8): global -> registers -> LDS, two LDS stages.
// ---------------------------------------------------------------------------------------------
template <class C>
__global__ __launch_bounds__(C::NT) void logprob_kernel(LogprobArgs a) {
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    constexpr int BM = C::BM, BN = C::BN, BK = C::BK, TM = C::TM, TN = C::TN;

    int tb, sp, vt_lo, vt_hi;
    if (!map_workgroup(a, tb, sp, vt_lo, vt_hi)) return;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / C::WN, wn = wave % C::WN;
    const int l31 = lane & 31, lh = lane >> 5;

    // ---- global -> register -> LDS staging geometry ---------------------------------------
    const int ld_c = tid % C::CPR;             // 16-byte chunk inside the 128-byte row segment
    const int ld_r = tid / C::CPR;             // tile row of pass 0
    const int ld_lds = lds_chunk_offset(ld_r, ld_c);  // rows of later passes differ by multiples of 16
    const int64_t tok0 = static_cast<int64_t>(tb) * BN;
    const int n_kc = (a.d + BK - 1) / BK;
    const int total_it = (vt_hi - vt_lo) * n_kc;

    uint4 stage[C::PA + C::PB];
    int ld_vt = vt_lo, ld_kc = 0;              // chunk the next issue_loads() fetches
    auto issue_loads = [&]() {
        const int k = ld_kc * BK + ld_c * 8;
        const bool k_ok = k < a.d;
        const int64_t v0 = static_cast<int64_t>(ld_vt) * BM;
#pragma unroll
        for (int p = 0; p < C::PA; ++p) {
            int64_t row = v0 + ld_r + p * C::ROWS_PER_PASS;
            row = row < a.V ? row : a.V - 1;
            stage[p] = k_ok ? *reinterpret_cast<const uint4*>(a.W + row * a.d + k) : make_uint4(0, 0, 0, 0);
        }
#pragma unroll
        for (int p = 0; p < C::PB; ++p) {
            int64_t row = tok0 + ld_r + p * C::ROWS_PER_PASS;
            row = row < a.T ? row : a.T - 1;
            stage[C::PA + p] = k_ok ? *reinterpret_cast<const uint4*>(a.H + row * a.d + k) : make_uint4(0, 0, 0, 0);
        }
        if (++ld_kc == n_kc) { ld_kc = 0; ++ld_vt; }
    };
    auto store_stage = [&](int buf) {
        unsigned char* sa = lds + buf * C::STAGE_BYTES + ld_lds;
        unsigned char* sb = sa + BM * BK * 2;
#pragma unroll
        for (int p = 0; p < C::PA; ++p) *reinterpret_cast<uint4*>(sa + p * C::ROWS_PER_PASS * 128) = stage[p];
#pragma unroll
        for (int p = 0; p < C::PB; ++p) *reinterpret_cast<uint4*>(sb + p * C::ROWS_PER_PASS * 128) = stage[C::PA + p];
    };

    LaneState<TN> st;
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        st.run_m[j] = kNegBig; st.run_s[j] = 0.f; st.tgt_z[j] = 0.f;
        const int64_t t = tok0 + wn * (BN / C::WN) + j * 32 + l31;
        st.tgt[j] = t < a.T ? a.targets[t] : -1;
    }

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    // fragment read offsets: row (wave base + i*32 + l31), chunk kk*2 + lh
    const int a_row0 = wm * (BM / C::WM) + l31;
    const int b_row0 = wn * (BN / C::WN) + l31;
    const int swz = (l31 >> 1) & 7;            // same for every 32-row block of the wave

    if (total_it > 0) {
        issue_loads();
        store_stage(0);
        __syncthreads();
    }
    int vt = vt_lo, kc = 0;
    for (int it = 0; it < total_it; ++it) {
        const bool more = it + 1 < total_it;
        if (more) issue_loads();
        const unsigned char* sa = lds + (it & 1) * C::STAGE_BYTES;
        const unsigned char* sb = sa + BM * BK * 2;
#pragma unroll
        for (int kk = 0; kk < BK / 16; ++kk) {
            const int coff = ((kk * 2 + lh) ^ swz) << 4;
            bf16x8 fa[TM], fb[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i)
                fa[i] = *reinterpret_cast<const bf16x8*>(sa + (a_row0 + i * 32) * 128 + coff);
#pragma unroll
            for (int j = 0; j < TN; ++j)
                fb[j] = *reinterpret_cast<const bf16x8*>(sb + (b_row0 + j * 32) * 128 + coff);
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
        }
        if (more) store_stage((it + 1) & 1);
        __syncthreads();

        if (++kc == n_kc) {
            tile_epilogue<TM, TN, BM / C::WM>(acc, st, vt * BM + wm * (BM / C::WM), a.V, lh);
            kc = 0;
            ++vt;
        }
    }
    write_partials<TN, C::WM, C::WN, BN, C::NT>(st, reinterpret_cast<float*>(lds), wm, wn, l31, lh, tid, tok0,
                                                 a.T, sp, a.part);
}

// ---------------------------------------------------------------------------------------------
// Fast kernel (d a multiple of 64): global -> LDS directly (no staging registers) into a ring of
// RING K32 slots (32 k-values = 64 bytes of each of the BM + BN tile rows); the contraction runs on
// v_mfma_f32_16x16x32_bf16, one whole K32 slot per instruction: 8 x 4 blocks of 16 vocabulary rows x 16 tokens
// per wave.  (In a register-only loop on random operands this shape sustains 2.0 PFLOP/s under the part's
// power limit, the 32x32x16 shape 1.8; the kernel as a whole gains 2-3 % on the workloads' data.)
//
// Loads always fetch whole 128-byte lines of a row, i.e. the two K32 halves that go to two
// consecutive slots (a "pair").  The L1 path moves 64 bytes per clock, so a pair costs as many L1
// cycles as half of its MFMA time; to keep that evenly spread, the W lines ("A") of a pair are
// requested during one K32 iteration and its H lines ("B") during the next, two load instructions before the
// iteration's barrier and two right behind it.  The pipeline per iteration i (chunk i lives in slot i % RING, its
// fragments are in registers when the iteration starts):
//   rows 0-2 of MFMAs (a row = one vocabulary block x the 4 token blocks); W fragment r of slot i+1 is read
//               into the registers of W fragment r as soon as row r has been issued (the W part of slot i+1
//               was certified one barrier earlier);
//   the wait for this wave's older loads, the workgroup barrier;
//   the H fragments of slot i+1 (certified just now) into the second H fragment set, then rows 3-7 with the
//               remaining W fragment reads between them: five rows of MFMAs cover the eight waves' reads
//               queueing on the LDS, so the matrix pipe never waits for an LDS round trip behind a barrier.
// The barrier inside iteration i certifies the W part of slot i+2 and the H part of slot i+1; every read of
// slot i has completed by then (they were issued during iteration i-1 and at the start of iteration i), so
// slot i is free for refilling from there on.
// The first chunk of every vocabulary tile takes the constant 0 as its MFMA addend, so the epilogue never
// clears the accumulators.
// (ring_nt.h holds the 32x32x16 form of this pipeline in a general form - row strides, K ranges, an epilogue
// after the walk - for the MLP head's kernels, which walk one tile per workgroup.)
// ---------------------------------------------------------------------------------------------
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
    static_assert(BM == BN, "W and H tiles are loaded by the same code in alternate iterations");
    static_assert(BM % (16 * NW) == 0, "whole 16-row load groups per wave");
    static_assert(LOADS == 4, "the hand-placed schedule below");
};

template <int N>
__device__ __forceinline__ void wait_vmcnt() {  // s_waitcnt vmcnt(N) only (gfx9 encoding), N <= 15
    __builtin_amdgcn_s_waitcnt(0x0F70 | N);
}

template <class C>
__global__ __launch_bounds__(C::NT) void logprob_ring_kernel(LogprobArgs a) {
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    constexpr int BM = C::BM, BN = C::BN, RING = C::RING;
    constexpr int TI = BM / C::WM / 16, TJ = BN / C::WN / 16;   // 16 x 16 blocks per wave: vocabulary x tokens
    typedef __attribute__((address_space(3))) void* lds_ptr_t;

    int tb, sp, vt_lo, vt_hi;
    if (!map_workgroup(a, tb, sp, vt_lo, vt_hi)) return;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / C::WN, wn = wave % C::WN;
    const int l15 = lane & 15, lq = lane >> 4;
    const int64_t tok0 = static_cast<int64_t>(tb) * BN;
    const int n_k64 = a.d / 64;

    // ---- loader geometry: one instruction moves 16 rows x 64 bytes; lane -> (row lane/4, physical
    //      16-byte position lane%4), which holds logical chunk (lane%4) ^ g(row), g(row) = 2 * ((row/4)%2)
    //      (see the fragment reads) -----------
    const int ld_row = lane >> 2;
    const int ld_kb = ((lane & 3) ^ (((lane >> 4) & 1) << 1)) * 16;   // byte offset inside the K32 half
    // Addresses are (wave-uniform 64-bit base in SGPRs) + (per-lane 32-bit byte offset): the base
    // carries tile and K position, the lane offset the row inside the tile (clamped at the end of the
    // vocabulary / token range, so every load stays inside W and H) and the swizzled chunk.
    const int64_t row_bytes = static_cast<int64_t>(a.d) * 2;
    const int64_t tile_bytes = BM * row_bytes;
    unsigned a_voff[C::G], b_voff[C::G];
    {
        const int rows_valid = static_cast<int>(a.T - tok0 < BN ? a.T - tok0 : BN);
#pragma unroll
        for (int g = 0; g < C::G; ++g) {
            int r = (wave * C::G + g) * 16 + ld_row;
            r = r < rows_valid ? r : rows_valid - 1;
            b_voff[g] = static_cast<unsigned>(r) * static_cast<unsigned>(row_bytes) + ld_kb;   // < 256 rows x 16 KiB
        }
    }
    auto point_at_tile = [&](int vt) {
        const int left = a.V - vt * BM;                                      // vt * BM < V + BM: no overflow
        const int rows_valid = left < BM ? (left > 0 ? left : 1) : BM;       // left <= 0 only past the last pair
#pragma unroll
        for (int g = 0; g < C::G; ++g) {
            int r = (wave * C::G + g) * 16 + ld_row;
            r = r < rows_valid ? r : rows_valid - 1;
            a_voff[g] = static_cast<unsigned>(r) * static_cast<unsigned>(row_bytes) + ld_kb;
        }
    };
    // two load streams, each walking the pairs (pair = two K32 slots = one 128-byte line per row) of the
    // workgroup's vocabulary range: W lines (A) and H lines (B).  Past the last pair both keep requesting lines
    // that exist (W: the last line again; H: its tile from the start) into ring slots nobody reads any more,
    // so the loop below needs no variant without loads.
    int a_vt = vt_lo, a_k64 = 0, a_slot = 0;
    int b_k64 = 0, b_slot = 0;
    const char* a_base = reinterpret_cast<const char*>(a.W) + a_vt * tile_bytes;
    const char* b_base = reinterpret_cast<const char*>(a.H) + tok0 * row_bytes;
    point_at_tile(a_vt);
    const unsigned lds0 = static_cast<unsigned>(reinterpret_cast<size_t>((lds_ptr_t)lds));
    // The q-th (q = 2*g + h) of the LOADS load instructions of a group: 16-row group g of this wave, K32
    // half h (-> first / second slot of the pair).  `stream` picks W lines or H lines at compile time.  Written as asm
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
        const unsigned voff = is_b ? b_voff[g] : a_voff[g];
        asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(voff), "s"(base), "s"(dst) : "memory");
    };
    auto advance = [&](auto stream) {
        constexpr bool is_b = decltype(stream)::value;
        if (is_b) {
            b_base += 128;
            if (++b_k64 == n_k64) { b_k64 = 0; b_base -= row_bytes; }   // next vocabulary tile: H rewinds
            b_slot = b_slot + 2 >= RING ? b_slot + 2 - RING : b_slot + 2;
        } else {
            if (a_vt < vt_hi) {
                a_base += 128;
                if (++a_k64 == n_k64) {   // next vocabulary tile: W moves on by a tile minus the row just walked
                    a_k64 = 0;
                    ++a_vt;
                    if (a_vt < vt_hi) {
                        a_base += tile_bytes - row_bytes;
                        point_at_tile(a_vt);
                    } else {
                        a_base -= 128;   // past the last pair: keep requesting the last line (nobody reads that slot any more)
                    }
                }
            }
            a_slot = a_slot + 2 >= RING ? a_slot + 2 - RING : a_slot + 2;
        }
    };
    auto issue_group = [&](auto stream) {
#pragma unroll
        for (int q = 0; q < C::LOADS; ++q) issue_one(stream, q);
        advance(stream);
    };
    constexpr std::false_type kA{};   // W lines
    constexpr std::true_type kB{};    // H lines

    LaneState<TJ> st;
#pragma unroll
    for (int j = 0; j < TJ; ++j) {
        st.run_m[j] = kNegBig; st.run_s[j] = 0.f; st.tgt_z[j] = 0.f;
    }
    // tokens of this wave: tok_wave + 0 .. 63; the first tgt_valid of them exist (both wave-uniform)
    const int64_t tok_wave = tok0 + wn * (BN / C::WN);
    const int32_t* tgt_wave = a.targets + (tok_wave < a.T ? tok_wave : 0);
    const int tgt_valid = tok_wave < a.T ? static_cast<int>(a.T - tok_wave < BN / C::WN ? a.T - tok_wave : BN / C::WN) : 0;
    f32x4 acc[TI][TJ];
#pragma unroll
    for (int i = 0; i < TI; ++i)
#pragma unroll
        for (int j = 0; j < TJ; ++j)
#pragma unroll
            for (int v = 0; v < 4; ++v) acc[i][j][v] = 0.f;

    // fragment reads: one MFMA takes the whole K32 of a slot: row (wave base + i*16 + lane%16), 16-byte chunk
    // lane/16 at position chunk ^ g(row).  Measured on the device: a 128-bit LDS read serves per cycle the 16
    // lanes that share lane bit 5 and the parity of lane bits 2, 3, 4, so two lanes of a half-wave that fall on
    // the same 16-byte bank group must differ in an odd number of those bits.  Here the bank group is
    // (row%4, position) = (l1 l0, l5 ^ l2, l4): the two lanes of a half-wave that share one differ in l3 alone.
    // (The 32x32 kernel's swizzle (row/4)%4 makes them differ in l2 and l4: two-way conflicts on every read.)
    const int swz = ((l15 >> 2) & 1) << 1;
    const int a_off = (wm * (BM / C::WM) + l15) * 64 + ((lq ^ swz) << 4);
    const int b_off = BM * 64 + (wn * (BN / C::WN) + l15) * 64 + ((lq ^ swz) << 4);
    bf16x8 fa[TI], fbe[TJ], fbo[TJ];   // W fragments (reloaded row by row), H fragments of even / odd iterations
    auto read_a = [&](const unsigned char* base, int i) {
        fa[i] = *reinterpret_cast<const bf16x8*>(base + a_off + i * 16 * 64);
    };
    auto read_b = [&](bf16x8 (&fb)[TJ], const unsigned char* base, int j) {
        fb[j] = *reinterpret_cast<const bf16x8*>(base + b_off + j * 16 * 64);
    };

    // Load schedule (pair p = chunks 2p, 2p+1 -> slots 2p % RING, (2p+1) % RING):
    //   up front           A(0), B(0), A(1)
    //   iteration 2p-2     B(p)   (even iterations, p >= 1)
    //   iteration 2p-3     A(p)   (odd iterations,  p >= 2)
    // The barrier inside iteration i needs every group requested before iteration i to have landed
    // (W part of slot i+2, H part of slot i+1), i.e. only this iteration's own loads may be in flight.
    issue_group(kA); issue_group(kB); issue_group(kA);
    wait_vmcnt<C::LOADS>();
    __syncthreads();
#pragma unroll
    for (int j = 0; j < TJ; ++j) read_b(fbe, lds, j);
#pragma unroll
    for (int i = 0; i < TI - 2; ++i) read_a(lds, i);
    int slot = 0;
    // One K32 chunk: 32 MFMAs, vocabulary block by vocabulary block.  W fragment i of the next slot (its W part
    // was certified one barrier earlier) is read into fa[i] once row i of MFMAs has been issued - the last two
    // only at the start of the next iteration, long before their rows.  The workgroup barrier sits after the third
    // row; the H fragments of the next slot are read right after it into the other fragment set, with five rows of
    // MFMAs to cover the 8 waves' reads queueing on the LDS.  Two of the four loads go out before the barrier and
    // two right behind it: of the placements tried at the benchmark sizes (all four before it, barrier after row
    // 1 ... 5, loads spread over the rows) this one was the fastest on the workloads' data (+4-6 % over all four
    // before a barrier after row 3) and fetched the fewest bytes from beyond the L2; on all-zero operands it is 8 %
    // slower than that one.  Even iterations (stream = H lines) compute on fbe, odd ones on fbo.
    // `first`: first chunk of a vocabulary tile - the addend is the constant 0, so the accumulators are never cleared.
    auto iteration = [&](auto stream, auto first) {
        constexpr bool is_b = decltype(stream)::value;
        constexpr bool is_first = decltype(first)::value;
        const unsigned char* cur = lds + slot * C::SLOT_BYTES;
        slot = slot + 1 == RING ? 0 : slot + 1;
        const unsigned char* nxt = lds + slot * C::SLOT_BYTES;
        bf16x8 (&fb)[TJ] = is_b ? fbe : fbo;
        bf16x8 (&fbn)[TJ] = is_b ? fbo : fbe;
        // consecutive MFMAs always share an operand: token blocks ascend on even rows and descend on odd ones
        // (in a register-only loop under the power limit this order sustained 4 % more than plain row-major)
        auto row = [&](int i) {
#pragma unroll
            for (int jj = 0; jj < TJ; ++jj) {
                const int j = (i & 1) ? TJ - 1 - jj : jj;
                if constexpr (is_first) {
                    const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
                    acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fa[i], fb[j], zero, 0, 0, 0);
                } else {
                    acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
                }
            }
        };
        read_a(cur, 6); read_a(cur, 7);
        __builtin_amdgcn_sched_barrier(0);
        row(0);
        __builtin_amdgcn_sched_barrier(0);
        read_a(nxt, 0);
        issue_one(stream, 0);
        issue_one(stream, 1);
        __builtin_amdgcn_sched_barrier(0);
        row(1);
        __builtin_amdgcn_sched_barrier(0);
        read_a(nxt, 1);
        __builtin_amdgcn_sched_barrier(0);
        row(2);
        __builtin_amdgcn_sched_barrier(0);
        // everything this wave requested before this iteration has landed (vmcnt counts in order: its two loads of
        // this iteration may fly, the two it issued behind the previous barrier may not); its own LDS reads are
        // complete (the last one was issued a row of MFMAs ago); then all waves agree
        wait_vmcnt<2>();
        __builtin_amdgcn_s_waitcnt(0xC07F);   // lgkmcnt(0) only
        __syncthreads();
#pragma unroll
        for (int j = 0; j < TJ; ++j) read_b(fbn, nxt, j);                    // H part of slot i+1: certified just now
        __builtin_amdgcn_sched_barrier(0);
        row(3);
        __builtin_amdgcn_sched_barrier(0);
        read_a(nxt, 2);                                                      // behind every wave's H reads in the LDS queue
        issue_one(stream, 2);
        issue_one(stream, 3); advance(stream);
        __builtin_amdgcn_sched_barrier(0);
        row(4);
        __builtin_amdgcn_sched_barrier(0);
        read_a(nxt, 3);
        __builtin_amdgcn_sched_barrier(0);
        row(5);
        __builtin_amdgcn_sched_barrier(0);
        read_a(nxt, 4); read_a(nxt, 5);
        __builtin_amdgcn_sched_barrier(0);
        row(6);
        __builtin_amdgcn_sched_barrier(0);
        __builtin_amdgcn_sched_barrier(0);
        row(7);
        __builtin_amdgcn_sched_barrier(0);
        // (the scheduling fence after the last row matters: without it the compiler lets the next iteration's first
        // reads drift up into this one and the kernel loses 10 %)
    };
    static_assert(TI == 8 && TJ == 4, "the hand-placed schedule above");
    for (int vt = vt_lo; vt < vt_hi; ++vt) {
        iteration(kB, std::true_type{});
        iteration(kA, std::false_type{});
        for (int k = 1; k < n_k64; ++k) {
            iteration(kB, std::false_type{});
            iteration(kA, std::false_type{});
        }
        tile_epilogue16<TI, TJ, BM / C::WM>(acc, st, vt * BM + wm * (BM / C::WM), a.V, lq, tgt_wave, tgt_valid, l15);
        // The fragments of the next chunk are read again here rather than kept across the epilogue: held, their
        // 64 registers pushed the epilogue into scratch memory, whose latency nothing hides (every wave of the
        // workgroup is in its epilogue at the same time).  The slot is certified and not yet released.
        asm volatile("" ::: "memory");
        __builtin_amdgcn_sched_barrier(0);
        {
            const unsigned char* nxt = lds + slot * C::SLOT_BYTES;
#pragma unroll
            for (int j = 0; j < TJ; ++j) read_b(fbe, nxt, j);
#pragma unroll
            for (int i = 0; i < TI - 2; ++i) read_a(nxt, i);   // the last two: at the start of the iteration
        }
    }
    wait_vmcnt<0>();
    __builtin_amdgcn_s_waitcnt(0xC07F);
    __syncthreads();   // every fragment read and every load into LDS has finished
    write_partials16<TJ, C::WM, C::WN, BN, C::NT>(st, reinterpret_cast<float*>(lds), wm, wn, l15, lq, tid, tok0,
                                                   a.T, sp, a.part);
}

__global__ __launch_bounds__(256) void logprob_finalize_kernel(
    const float* __restrict__ part, const int32_t* __restrict__ targets, int64_t T, int V, int n_sp,
    float* __restrict__ logprob_out, float* __restrict__ lse_out) {
    const int64_t t = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    if (t >= T) return;
    float m = kNegBig, s = 0.f, z = 0.f;
    for (int sp = 0; sp < n_sp; ++sp) {
        const float* p = part + static_cast<int64_t>(sp) * 3 * T + t;
        const float om = p[0], os = p[T];
        const float mm = fmaxf(m, om);
        s = s * exp2f((m - mm) * kLog2e) + os * exp2f((om - mm) * kLog2e);
        m = mm;
        z += p[2 * T];
    }
    const float lse = m + logf(s);
    const int y = targets[t];
    logprob_out[t] = (y >= 0 && y < V) ? z - lse : __builtin_nanf("");
    if (lse_out) lse_out[t] = lse;
}

using MainTile = Tile<256, 256, 64, 2, 4>;
using FastTile = RingTile<256, 256, 2, 4>;
static_assert(MainTile::BM == FastTile::BM && MainTile::BN == FastTile::BN, "one plan serves both kernels");

struct Plan { int n_tb, n_vt, n_sp; };

Plan make_plan(int64_t T, int V, int n_splits) {
    Plan p;
    p.n_tb = static_cast<int>((T + MainTile::BN - 1) / MainTile::BN);
    p.n_vt = (V + MainTile::BM - 1) / MainTile::BM;
    int sp = n_splits;
    if (sp <= 0) {
        // enough workgroups to fill 256 CUs several times over.  The 32 workgroups resident on an XCD are then
        // 5 1/3 token blocks x 6 splits: measured at the four benchmark shapes, 6 splits are 0.4-2.1 % faster
        // than 8 and than 4, 5 or 7
        sp = 6;
        while (static_cast<int64_t>(p.n_tb) * sp < 1024 && sp < 64) sp *= 2;
    }
    if (sp > p.n_vt) sp = p.n_vt;
    if (sp < 1) sp = 1;
    p.n_sp = sp;
    return p;
}

}  // namespace

extern "C" size_t arrol_logprob_workspace_bytes(int64_t T, int32_t V, int32_t d, int32_t n_splits) {
    (void)d;
    if (T <= 0 || V < 1 || n_splits < 0) return 0;
    const Plan p = make_plan(T, V, n_splits);
    return (static_cast<size_t>(p.n_sp) * 3 * static_cast<size_t>(T) * sizeof(float) + 255) & ~static_cast<size_t>(255);
}

extern "C" int arrol_logprob(const void* hidden, const void* lm_head, const int32_t* targets,
                             int64_t T, int32_t V, int32_t d, float* logprob_out, float* lse_out,
                             int32_t n_splits, void* workspace, size_t workspace_bytes, void* stream) {
    if (T < 0 || V < 1 || d < 8 || (d & 7) || n_splits < 0) return ARROL_EINVAL;
    if (T == 0) return ARROL_OK;
    if (!hidden || !lm_head || !targets || !logprob_out || !arrol_aligned16(hidden) || !arrol_aligned16(lm_head))
        return ARROL_EINVAL;
    const Plan p = make_plan(T, V, n_splits);
    if (static_cast<int64_t>(p.n_tb) + kXcds > INT32_MAX / p.n_sp) return ARROL_EINVAL;
    if (!workspace || !arrol_aligned16(workspace) || workspace_bytes < arrol_logprob_workspace_bytes(T, V, d, n_splits))
        return ARROL_EWORKSPACE;
    hipStream_t st = static_cast<hipStream_t>(stream);
    static arrol_device_flags general_ok, fast_ok;
    if (!arrol_allow_lds(&logprob_kernel<MainTile>, MainTile::LDS_BYTES, general_ok) ||
        !arrol_allow_lds(&logprob_ring_kernel<FastTile>, FastTile::LDS_BYTES, fast_ok))
        return ARROL_EHIP;
    LogprobArgs a;
    a.H = static_cast<const uint16_t*>(hidden);
    a.W = static_cast<const uint16_t*>(lm_head);
    a.targets = targets;
    a.part = static_cast<float*>(workspace);
    a.T = T; a.V = V; a.d = d;
    a.n_tb = p.n_tb; a.n_sp = p.n_sp; a.n_vt = p.n_vt;
    const int tb_pad = (p.n_tb + kXcds - 1) / kXcds * kXcds;
    if (d % 64 == 0)
        arrol_launch(logprob_ring_kernel<FastTile>, dim3(tb_pad * p.n_sp), dim3(FastTile::NT), FastTile::LDS_BYTES, st, a);
    else
        arrol_launch(logprob_kernel<MainTile>, dim3(tb_pad * p.n_sp), dim3(MainTile::NT), MainTile::LDS_BYTES, st, a);
    if (arrol_launch_failed()) return arrol_launch_status();
    arrol_launch(logprob_finalize_kernel, dim3(static_cast<unsigned>((T + 255) / 256)), dim3(256), 0, st,
                       static_cast<const float*>(workspace), targets, T, V, p.n_sp, logprob_out, lse_out);
    return arrol_launch_status();
}
