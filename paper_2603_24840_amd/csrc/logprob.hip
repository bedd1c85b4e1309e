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
#include "common.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

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

template <class C>
__global__ __launch_bounds__(C::NT) void logprob_kernel(LogprobArgs a) {
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    constexpr int BM = C::BM, BN = C::BN, BK = C::BK, TM = C::TM, TN = C::TN;

    // ---- workgroup -> (token block, vocab split), XCD-aware ------------------------------
    const int bid = blockIdx.x;
    const int xcd = bid % kXcds, idx = bid / kXcds;
    const int sp = idx % a.n_sp;
    const int tb = (idx / a.n_sp) * kXcds + xcd;
    if (tb >= a.n_tb) return;
    const int vt_lo = static_cast<int>(static_cast<int64_t>(a.n_vt) * sp / a.n_sp);
    const int vt_hi = static_cast<int>(static_cast<int64_t>(a.n_vt) * (sp + 1) / a.n_sp);

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

    // ---- per-lane softmax state: lane owns token wn*(BN/WN) + j*32 + l31 for j < TN --------
    float run_m[TN], run_s[TN], tgt_z[TN];
    int tgt[TN];
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        run_m[j] = kNegBig; run_s[j] = 0.f; tgt_z[j] = 0.f;
        const int64_t t = tok0 + wn * (BN / C::WN) + j * 32 + l31;
        tgt[j] = t < a.T ? a.targets[t] : -1;
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
            // ---- tile epilogue: acc[i][j][v] is the logit of vocab row
            //      vrow0 + i*32 + (v/4)*8 + lh*4 + v%4 for this lane's token of block j ----------
            const int vrow0 = vt * BM + wm * (BM / C::WM);
            if (vrow0 + BM / C::WM > a.V) {  // tile hangs over the end of the vocabulary
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        const bool dead = vrow0 + i * 32 + (v >> 2) * 8 + lh * 4 + (v & 3) >= a.V;
#pragma unroll
                        for (int j = 0; j < TN; ++j) acc[i][j][v] = dead ? -INFINITY : acc[i][j][v];
                    }
            }
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const int rel = tgt[j] - vrow0;
                const bool mine = rel >= 0 && rel < BM / C::WM && ((rel >> 2) & 1) == lh;
                if (__any(mine)) {
                    const int code = mine ? ((rel >> 5) * 16 + ((rel & 31) >> 3) * 4 + (rel & 3)) : -1;
#pragma unroll
                    for (int i = 0; i < TM; ++i)
#pragma unroll
                        for (int v = 0; v < 16; ++v)
                            if (code == i * 16 + v) tgt_z[j] = acc[i][j][v];
                }
                float mx = acc[0][j][0];
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int v = 0; v < 16; ++v) mx = fmaxf(mx, acc[i][j][v]);
                const float m_new = fmaxf(run_m[j], mx);
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
                run_s[j] = run_s[j] * __builtin_amdgcn_exp2f((run_m[j] - m_new) * kLog2e) + sum;
                run_m[j] = m_new;
            }
            kc = 0;
            ++vt;
        }
    }

    // ---- merge the two lane halves (same token, different vocab rows) -------------------------
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        const float om = __shfl_xor(run_m[j], 32, ARROL_WAVE);
        const float os = __shfl_xor(run_s[j], 32, ARROL_WAVE);
        const float oz = __shfl_xor(tgt_z[j], 32, ARROL_WAVE);
        const float m = fmaxf(run_m[j], om);
        run_s[j] = run_s[j] * __builtin_amdgcn_exp2f((run_m[j] - m) * kLog2e) +
                   os * __builtin_amdgcn_exp2f((om - m) * kLog2e);
        run_m[j] = m;
        tgt_z[j] += oz;
    }
    // ---- merge the WM waves that share a token range, through LDS ---------------------------
    float* red = reinterpret_cast<float*>(lds);  // [WM][3][BN]; the staging buffers are idle now
    if (lh == 0) {
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int col = wn * (BN / C::WN) + j * 32 + l31;
            red[(wm * 3 + 0) * BN + col] = run_m[j];
            red[(wm * 3 + 1) * BN + col] = run_s[j];
            red[(wm * 3 + 2) * BN + col] = tgt_z[j];
        }
    }
    __syncthreads();
    for (int col = tid; col < BN; col += C::NT) {
        const int64_t t = tok0 + col;
        if (t >= a.T) continue;
        float m = red[col], s = red[BN + col], z = red[2 * BN + col];
#pragma unroll
        for (int w = 1; w < C::WM; ++w) {
            const float om = red[(w * 3 + 0) * BN + col], os = red[(w * 3 + 1) * BN + col];
            const float mm = fmaxf(m, om);
            s = s * __builtin_amdgcn_exp2f((m - mm) * kLog2e) + os * __builtin_amdgcn_exp2f((om - mm) * kLog2e);
            m = mm;
            z += red[(w * 3 + 2) * BN + col];
        }
        float* p = a.part + static_cast<int64_t>(sp) * 3 * a.T + t;
        p[0] = m;
        p[a.T] = s;
        p[2 * a.T] = z;
    }
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

int g_force_splits = 0;  // 0 = heuristic

struct Plan { int n_tb, n_vt, n_sp; };

Plan make_plan(int64_t T, int V) {
    Plan p;
    p.n_tb = static_cast<int>((T + MainTile::BN - 1) / MainTile::BN);
    p.n_vt = (V + MainTile::BM - 1) / MainTile::BM;
    int sp = g_force_splits;
    if (sp <= 0) {
        // enough workgroups to fill 256 CUs several times over; 8 splits make the
        // 32 workgroups resident on an XCD a 4-token-block x 8-split patch
        sp = 8;
        while (static_cast<int64_t>(p.n_tb) * sp < 1024 && sp < 64) sp *= 2;
    }
    if (sp > p.n_vt) sp = p.n_vt;
    if (sp < 1) sp = 1;
    p.n_sp = sp;
    return p;
}

}  // namespace

extern "C" int arrol_set_tuning(const char* key, int value) {
    if (!key) return ARROL_EINVAL;
    if (!__builtin_strcmp(key, "logprob_splits")) { g_force_splits = value; return ARROL_OK; }
    return ARROL_EINVAL;
}

extern "C" size_t arrol_logprob_workspace_bytes(int64_t T, int32_t V, int32_t d) {
    (void)d;
    if (T <= 0 || V < 1) return 0;
    const Plan p = make_plan(T, V);
    return (static_cast<size_t>(p.n_sp) * 3 * static_cast<size_t>(T) * sizeof(float) + 255) & ~static_cast<size_t>(255);
}

extern "C" int arrol_logprob(const void* hidden, const void* lm_head, const int32_t* targets,
                             int64_t T, int32_t V, int32_t d, float* logprob_out, float* lse_out,
                             void* workspace, size_t workspace_bytes, void* stream) {
    if (T < 0 || V < 1 || d < 8 || (d & 7)) return ARROL_EINVAL;
    if (T == 0) return ARROL_OK;
    if (!hidden || !lm_head || !targets || !logprob_out || !arrol_aligned16(hidden) || !arrol_aligned16(lm_head))
        return ARROL_EINVAL;
    const Plan p = make_plan(T, V);
    if (static_cast<int64_t>(p.n_tb) + kXcds > INT32_MAX / p.n_sp) return ARROL_EINVAL;
    if (!workspace || !arrol_aligned16(workspace) || workspace_bytes < arrol_logprob_workspace_bytes(T, V, d))
        return ARROL_EWORKSPACE;
    hipStream_t st = static_cast<hipStream_t>(stream);
    static bool attr_done = false;
    if (!attr_done) {
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(&logprob_kernel<MainTile>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, MainTile::LDS_BYTES) != hipSuccess)
            return ARROL_EHIP;
        attr_done = true;
    }
    LogprobArgs a;
    a.H = static_cast<const uint16_t*>(hidden);
    a.W = static_cast<const uint16_t*>(lm_head);
    a.targets = targets;
    a.part = static_cast<float*>(workspace);
    a.T = T; a.V = V; a.d = d;
    a.n_tb = p.n_tb; a.n_sp = p.n_sp; a.n_vt = p.n_vt;
    const int tb_pad = (p.n_tb + kXcds - 1) / kXcds * kXcds;
    hipLaunchKernelGGL(logprob_kernel<MainTile>, dim3(tb_pad * p.n_sp), dim3(MainTile::NT), MainTile::LDS_BYTES, st, a);
    if (hipGetLastError() != hipSuccess) return ARROL_EHIP;
    hipLaunchKernelGGL(logprob_finalize_kernel, dim3(static_cast<unsigned>((T + 255) / 256)), dim3(256), 0, st,
                       static_cast<const float*>(workspace), targets, T, V, p.n_sp, logprob_out, lse_out);
    return arrol_launch_status();
}
