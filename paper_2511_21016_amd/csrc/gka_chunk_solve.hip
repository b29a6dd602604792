// Per-chunk solve: chunk-wise Frobenius norms (Section 4.2.1), the fused Chebyshev driver
// (Algorithm 1 on all tokens of the chunk at once) and the readout y_c = U_c xhat_c of Eq. (CH).
//
// One workgroup = one chunk of one (batch, head) pair = four waves. Wave w owns the token block tw = w & 1
// (tokens 32 tw .. 32 tw + 31) and the feature half fh = w >> 1 (rows 32 mt .., mt in its half of the D / 32
// row blocks). Two such workgroups fit a CU, so every SIMD holds two waves of different chunks and one
// chunk's memory and barrier waits are covered by the other's arithmetic.
//
// All products are computed transposed, tokens along the MFMA N dimension: lane (n, g) holds token
// c = 32 tw + n, and an accumulator tile holds rows kidx(r, g) of that token's feature vector. Consequences:
// every per-token scalar (zeta_c, lambda_c, L, rho, omega_i) is a per-lane scalar, the iterate never leaves
// registers, and an accumulator tile converts in place into the B operand of the next contraction. The chunk's
// initial state H_[n] and the keys sit in LDS in fragment order as the A operands. With
// H_c = zeta_c H_[n] + sum_{j<=c} M[j,c] k_j k_j^T (Section 4.2.1):
//
//   (H_c x_c) = zeta_c * (H_[n] x_c)  +  sum_{j<=c} M[j,c] k_j (k_j . x_c)
//               `-- state product --'     `-- P = K X^T, mask, K^T (P o M) --'
//
// Both contractions run over all D features of x_c, so the two waves of a token block exchange their halves
// of the operand through LDS once per pass.
//
// The Chebyshev recurrence is run in its residual form (same iterates in exact arithmetic):
//   delta_i = (omega_i - 1) delta_{i-1} + (2 omega_i / (L + mu)) r_{i-1},  xi_i = xi_{i-1} + delta_i,
//   r_i = q - (H_c + lambda_c I) xi_i,
// with g_i = H_c xi_i - q accumulated over the passes inside the MFMA accumulators (the operand of each pass
// is the shrinking update delta_i, not the iterate), split as g = zeta * gS + gI.
#include "gka_device.hpp"
#include "gka_kernels.hpp"

namespace gka {

constexpr int kSolveThreads = 256;

template <class MMA, int D>
struct SolveShape {
    typedef typename MMA::frag frag;
    typedef typename MMA::elem_t elem_t;
    static constexpr int NB = D / 32;
    static constexpr int NBH = NB / 2;              // row blocks per feature half
    static constexpr int HS = MMA::HS;
    static constexpr int JB = kChunk / 32;
    static constexpr int H_FRAGS = NB * NB * HS;
    static constexpr int K_FRAGS = JB * NB * HS;
    static constexpr int KT_FRAGS = NB * JB * HS;
    static constexpr int X_FRAGS = 2 * NB * HS;     // operand exchange: [token block][blk][h]
    static constexpr size_t h_bytes = (size_t)H_FRAGS * 64 * sizeof(frag);
    static constexpr size_t k_bytes = (size_t)K_FRAGS * 64 * sizeof(frag);
    static constexpr size_t kt_bytes = (size_t)KT_FRAGS * 64 * sizeof(frag);
    static constexpr size_t x_bytes = (size_t)X_FRAGS * 64 * sizeof(frag);
    // Row-major staging tile of one chunk of k or v rows: unpadded and swizzled, exactly the size of the
    // operand-exchange region, which it shares (the two are never live together).
    typedef SwizzledRows<D * (int)sizeof(elem_t), (int)sizeof(elem_t)> Rows;
    static_assert((size_t)kChunk * D * sizeof(elem_t) == x_bytes, "staging tile and exchange region coincide");
    static constexpr size_t lds_bytes = h_bytes + k_bytes + kt_bytes + x_bytes;
};

// Calls fill(std::integral_constant<int, s>) for the (unrolled, hence constant) step s of N.
template <int N, class Fill, int S = 0>
__device__ __forceinline__ void fill_step(Fill &fill, int s)
{
    if constexpr (S < N) {
        if (s == S) fill(std::integral_constant<int, S>{});
        else fill_step<N, Fill, S + 1>(fill, s);
    }
}

// acc[a] += sum_s A[a][s] * B[s] over NSTEPS contraction steps; all operands are LDS fragment arrays
// (fragment s of a set at [s * 64 + lane]). The fragments of step s + 1 are requested before the MFMAs of
// step s are issued, so LDS latency is paid once per call, not once per MFMA. `fill(step)` is called once per
// step with the step as a compile-time constant: independent vector-ALU work of the caller that is issued between
// the MFMAs, where the wave would otherwise wait for the matrix pipe.
struct NoFill {
    template <class S>
    __device__ __forceinline__ void operator()(S) const {}
};
// N_FROM_ZERO: the first N_FROM_ZERO accumulators start from zero (their incoming values are ignored): the first MFMA of each
// takes a constant zero as its C operand, which costs no instruction, instead of sixteen register moves.
template <class MMA, int NSTEPS, int NA, class Fill = NoFill, int N_FROM_ZERO = 0>
__device__ __forceinline__ void fused_gemm(const typename MMA::frag *const (&A)[NA], const typename MMA::frag *B,
                                           f32x16 (&acc)[NA], int lane, Fill fill = Fill())
{
    typename MMA::frag abuf[2][NA], bbuf[2];
#pragma unroll
    for (int x = 0; x < NA; ++x) abuf[0][x] = A[x][lane];
    bbuf[0] = B[lane];
#pragma unroll
    for (int s = 0; s < NSTEPS; ++s) {
        const int cur = s & 1, nxt = cur ^ 1;
        if (s + 1 < NSTEPS) {
#pragma unroll
            for (int x = 0; x < NA; ++x) abuf[nxt][x] = A[x][(s + 1) * 64 + lane];
            bbuf[nxt] = B[(s + 1) * 64 + lane];
        }
        __builtin_amdgcn_sched_barrier(0);     // keep the requests for step s + 1 ahead of the MFMAs of step s
#pragma unroll
        for (int x = 0; x < NA; ++x)
            acc[x] = MMA::mma(abuf[cur][x], bbuf[cur], (s == 0 && x < N_FROM_ZERO) ? zero16() : acc[x]);
        fill_step<NSTEPS>(fill, s);
        __builtin_amdgcn_sched_barrier(0);
    }
}

// The two products of a pass that share the B operand (the published delta), in one sweep over its NSTEPS fragments:
// pacc[j] = sum_s K[j][s] * B[s] (from zero) and gS[i] += sum_s Hs[i][s] * B[s]. Every B fragment is read from LDS
// once. The A fragments are staggered instead of double-buffered as a whole: those of the state product are
// requested at the start of their own step and arrive while the key MFMAs run; the keys and B of the next step are
// requested before the state MFMAs. `fill(step)` as in fused_gemm.
template <class MMA, int NSTEPS, int NJ, int NBH, class Fill>
__device__ __forceinline__ void fused_pass_sweep(const typename MMA::frag *const (&K)[NJ],
                                                 const typename MMA::frag *const (&Hs)[NBH],
                                                 const typename MMA::frag *B, f32x16 (&pacc)[NJ], f32x16 (&gS)[NBH],
                                                 int lane, Fill fill)
{
    typename MMA::frag kb[2][NJ], bb[2], hb[NBH];
#pragma unroll
    for (int j = 0; j < NJ; ++j) kb[0][j] = K[j][lane];
    bb[0] = B[lane];
#pragma unroll
    for (int s = 0; s < NSTEPS; ++s) {
        const int cur = s & 1, nxt = cur ^ 1;
#pragma unroll
        for (int i = 0; i < NBH; ++i) hb[i] = Hs[i][s * 64 + lane];
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int j = 0; j < NJ; ++j) pacc[j] = MMA::mma(kb[cur][j], bb[cur], s == 0 ? zero16() : pacc[j]);
        __builtin_amdgcn_sched_barrier(0);
        if (s + 1 < NSTEPS) {
#pragma unroll
            for (int j = 0; j < NJ; ++j) kb[nxt][j] = K[j][(s + 1) * 64 + lane];
            bb[nxt] = B[(s + 1) * 64 + lane];
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int i = 0; i < NBH; ++i) gS[i] = MMA::mma(hb[i], bb[cur], gS[i]);
        fill_step<NSTEPS>(fill, s);
        __builtin_amdgcn_sched_barrier(0);
    }
}

// (P o M) as B-operand fragments, key blocks jt <= TW
template <class MMA, int TW>
__device__ __forceinline__ void mask_p(const f32x16 (&pacc)[TW + 1], const f32x16 (&mreg)[TW + 1],
                                       typename MMA::frag (&pm)[TW + 1][MMA::HS])
{
    constexpr int VEC = MMA::VEC, HS = MMA::HS;
#pragma unroll
    for (int jt = 0; jt <= TW; ++jt)
#pragma unroll
        for (int hh = 0; hh < HS; ++hh) {
            float t[VEC];
#pragma unroll
            for (int p = 0; p < VEC; ++p) t[p] = pacc[jt][hh * VEC + p] * mreg[jt][hh * VEC + p];
            pm[jt][hh] = MMA::pack(t);
        }
}

// acc[i] += sum_{jt<=TW,h} AT[mt0 + i][jt][h] * pm[jt][h]     (AT = K^T or V^T fragments in LDS). With a filler the MFMAs
// are issued in the order (jt, h, i), so that consecutive ones use different accumulators, and `fill(step)` is called
// after each of the NBH * (TW + 1) * HS of them with its index as a compile-time constant (see fused_gemm).
template <class MMA, int NBH, int TW, class Fill = NoFill>
__device__ __forceinline__ void gemm_intra(const typename MMA::frag *sAT, int mt0,
                                           const typename MMA::frag (&pm)[TW + 1][MMA::HS], f32x16 (&acc)[NBH],
                                           int lane, Fill fill = Fill())
{
    constexpr int HS = MMA::HS, NM = NBH * (TW + 1) * HS;
    typename MMA::frag af[NBH][TW + 1][HS];
#pragma unroll
    for (int i = 0; i < NBH; ++i)
#pragma unroll
        for (int jt = 0; jt <= TW; ++jt)
#pragma unroll
            for (int hh = 0; hh < HS; ++hh) af[i][jt][hh] = sAT[(((mt0 + i) * 2 + jt) * HS + hh) * 64 + lane];
    if constexpr (std::is_same<Fill, NoFill>::value) {
#pragma unroll
        for (int i = 0; i < NBH; ++i)
#pragma unroll
            for (int jt = 0; jt <= TW; ++jt)
#pragma unroll
                for (int hh = 0; hh < HS; ++hh) acc[i] = MMA::mma(af[i][jt][hh], pm[jt][hh], acc[i]);
    } else {
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int jt = 0; jt <= TW; ++jt)
#pragma unroll
            for (int hh = 0; hh < HS; ++hh)
#pragma unroll
                for (int i = 0; i < NBH; ++i) {
                    acc[i] = MMA::mma(af[i][jt][hh], pm[jt][hh], acc[i]);
                    fill_step<NM>(fill, (jt * HS + hh) * NBH + i);
                    __builtin_amdgcn_sched_barrier(0);
                }
    }
}

// A block of N16 * kSolveThreads 16-byte units copied global -> LDS by the workgroup, asynchronously and without
// staging registers (w = wave index, wave-uniform).
template <int N16>
__device__ __forceinline__ void async_block_copy(void *lds_dst, const void *gsrc, int w, int lane)
{
    const buffer_rsrc src = make_raw_buffer(gsrc);
#pragma unroll
    for (int i = 0; i < N16; ++i) {
        const int unit0 = (i * (kSolveThreads / 64) + w) * 64;
        async_copy16_to_lds((char *)lds_dst + (size_t)unit0 * 16, src, lane * 16, unit0 * 16);
    }
}

// One chunk of rows of x (k or v): global -> registers (load), registers -> row-major LDS tile of operand
// elements (store).
template <class MMA, class IO, int D>
struct RowStage {
    typedef typename SolveShape<MMA, D>::Rows Rows;
    static constexpr int P4 = D / 4;
    static constexpr int NP = kChunk * P4 / kSolveThreads;
    typename IO::raw4 r[NP];
    // Rows past the end of the sequence are read from the last valid row (no divergent branch around the
    // loads, which would force a wait on each) and zeroed when stored.
    __device__ __forceinline__ void load(const void *x, int64_t base, int64_t stride_t, int tok0, int T, int tid)
    {
#pragma unroll
        for (int i = 0; i < NP; ++i) {
            const int piece = i * kSolveThreads + tid;
            const int row = piece / P4, c4 = piece % P4;
            const int tok = min(tok0 + row, T - 1);
            r[i] = IO::load_raw4(x, base + (int64_t)tok * stride_t + 4 * c4);
        }
    }
    __device__ __forceinline__ void store(typename MMA::elem_t *sRow, int tok0, int T, int tid) const
    {
#pragma unroll
        for (int i = 0; i < NP; ++i) {
            const int piece = i * kSolveThreads + tid;
            f32x4 v = IO::cvt4(r[i]);
            if (tok0 + piece / P4 >= T) v = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
            MMA::store4(sRow + Rows()(piece / P4, 4 * (piece % P4)), v);
        }
    }
};

// Fragments K[jt][blk][h]: rows = tokens of block jt, contraction index = features in kidx order.
template <class MMA, int D>
__device__ __forceinline__ void build_row_frags(typename MMA::frag *sK, const typename MMA::elem_t *sRow, int w,
                                                int lane)
{
    typedef SolveShape<MMA, D> SH;
    constexpr int VEC = MMA::VEC, HS = MMA::HS, NB = SH::NB;
    const typename SH::Rows at;
    const int n = lane & 31, g = lane >> 5;
    for (int f = w; f < SH::K_FRAGS; f += 4) {
        const int hh = f % HS, blk = (f / HS) % NB, jt = f / (HS * NB);
        if constexpr (VEC == 8) {
            // kidx(8*hh + p, g) = 16*hh + 8*(p/4) + 4*g + p%4: two runs of four consecutive features
            const int col = 32 * blk + 16 * hh + 4 * g;
            u16x4 lo = *(const u16x4 *)(sRow + at(32 * jt + n, col)), hi = *(const u16x4 *)(sRow + at(32 * jt + n, col + 8));
            u16x8 u = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
            sK[f * 64 + lane] = __builtin_bit_cast(typename MMA::frag, u);
        } else {
            typename MMA::elem_t e[VEC];
#pragma unroll
            for (int p = 0; p < VEC; ++p) e[p] = sRow[at(32 * jt + n, 32 * blk + kidx(hh * VEC + p, g))];
            sK[f * 64 + lane] = MMA::pack_elems(e);
        }
    }
}

// Fragments AT[mt][jt][h]: row 32*mt + n of X^T, contraction index = tokens j = 32*jt + kidx(h*VEC + p, g).
// UNTRACKED: the tile is read with gather_transposed_bf16_untracked (a copy into another part of LDS is in flight).
template <class MMA, int D, bool UNTRACKED = false>
__device__ __forceinline__ void build_transposed_frags(typename MMA::frag *sAT, const typename MMA::elem_t *sRow,
                                                       int w, int lane)
{
    typedef SolveShape<MMA, D> SH;
    constexpr int VEC = MMA::VEC, HS = MMA::HS;
    const typename SH::Rows at;
    const int n = lane & 31, g = lane >> 5;
    for (int f = w; f < SH::KT_FRAGS; f += 4) {
        const int hh = f % HS, jt = (f / HS) % 2, mt = f / (2 * HS);
        if constexpr (VEC == 8) {
            const int t0 = 32 * jt + 16 * hh + 4 * g;       // kidx(8*hh + p, g) = 16*hh + 8*(p/4) + 4*g + p%4
            const int col16 = 32 * mt + 16 * ((lane >> 4) & 1);
            sAT[f * 64 + lane] = UNTRACKED ? gather_transposed_bf16_untracked(sRow, at, col16, lane, t0, t0 + 8)
                                           : gather_transposed_bf16(sRow, at, col16, lane, t0, t0 + 8);
        } else {
            auto tok_of = [&](int p) { return 32 * jt + kidx(hh * VEC + p, g); };
            sAT[f * 64 + lane] = gather_transposed<MMA>(sRow, at, 32 * mt + n, tok_of);
        }
    }
}

// This wave's halves of an operand go to the exchange region: fragments [token block][row block][h].
template <class MMA, int NB>
__device__ __forceinline__ void publish_operand(typename MMA::frag *sX, const typename MMA::frag (&own)[NB / 2][MMA::HS],
                                                int tw, int mt0, int lane)
{
#pragma unroll
    for (int i = 0; i < NB / 2; ++i)
#pragma unroll
        for (int hh = 0; hh < MMA::HS; ++hh) sX[((tw * NB + mt0 + i) * MMA::HS + hh) * 64 + lane] = own[i][hh];
}

// The work of one wave. TW (token block) is a template parameter so that the causal structure (key blocks
// jt <= TW) is resolved at compile time; fh (feature half) only enters through mt0.
// GATED: the layer's variants (write gate, alpha-connection, lambda_t = a ||H_t||_F) are compiled in; the plain
// kernel carries none of their loads, registers or branches.
template <class MMA, class IO, int D, int TW, bool GATED>
__device__ __forceinline__ void chunk_solve_wave(const SolveArgs &a, unsigned char *smem, int w)
{
    typedef SolveShape<MMA, D> SH;
    constexpr int NB = SH::NB, NBH = SH::NBH;
    constexpr int VEC = MMA::VEC, HS = MMA::HS;
    constexpr int NSTEPS = NB * HS;            // MFMA steps of a contraction over all D features
    constexpr int NJ = TW + 1;                 // key blocks visible to this token block
    typedef typename MMA::frag frag;
    typedef typename MMA::elem_t elem_t;

    frag *sH = (frag *)smem;
    frag *sK = (frag *)(smem + SH::h_bytes);
    frag *sKT = (frag *)(smem + SH::h_bytes + SH::k_bytes);
    frag *sX = (frag *)(smem + SH::h_bytes + SH::k_bytes + SH::kt_bytes);
    elem_t *sRow = (elem_t *)sX;               // staging tile of k (then v) rows shares the exchange region
    float *sW = (float *)sX;                   // so do the per-token scalars of the Frobenius phase
    float *sA = sW + kChunk;                   // [2][kChunk]

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int fh = w >> 1;                     // w: wave index, wave-uniform
    const int mt0 = fh * NBH;
    const int n = lane & 31, g = lane >> 5;
    // Consecutive workgroups take the same chunk index of consecutive (batch, head) pairs: in the [B,T,H,d]
    // layout the heads of a token are adjacent, so workgroups that run together read adjacent memory.
    const int pair = blockIdx.x % a.n_pairs;
    const int chunk_local = blockIdx.x / a.n_pairs;
    const int chunk = a.chunk0 + chunk_local;
    const int b = (a.pair0 + pair) / a.H, h = (a.pair0 + pair) % a.H;
    const int64_t chunk_id = (int64_t)chunk_local * a.n_pairs + pair;     // workspace index within this launch
    const int64_t base_bh = (int64_t)b * a.stride_b + (int64_t)h * a.stride_h;
    const int64_t gate_base = (int64_t)b * a.T * a.H + h;
    const int tok0 = chunk * kChunk;
    const int c_local = 32 * TW + n;
    const int tok = tok0 + c_local;
    const bool valid = tok < a.T;

    // ---------------- staging ----------------
    constexpr int H16 = (int)(SH::h_bytes / 16 / kSolveThreads);   // 16-byte units of a state block per thread
    const int64_t tok_off = base_bh + (int64_t)min(tok, a.T - 1) * a.stride_t;
    float lam, hn2 = 0.0f;
    float Gall;                                // lane j: G_j = sum_{i<=j} log2 gamma_i over the chunk
    typename IO::raw4 qraw[NBH][4];            // q of this lane's token, rows of this wave's feature half
    // every global read of the prologue is issued here, before the first wait; the gates first: loads return in
    // issue order, and the decay mask below needs nothing else, so it is built while the k rows are on their way
    const float gm = a.gate[gate_base + (int64_t)min(tok0 + lane, a.T - 1) * a.H];
    // optional inputs: without them a valid array is read instead and the value replaced (no branch around a load)
    float ball = 1.0f;                          // lane j: write gate beta_j of token j (Remark in Section 4.1)
    if constexpr (GATED) {
        const float bm_raw = (a.beta ? a.beta : a.gate)[gate_base + (int64_t)min(tok0 + lane, a.T - 1) * a.H];
        ball = a.beta ? bm_raw : 1.0f;
    }
    // plain readout (variants' kernel only): no solve, so neither H_[n] nor its norm is read
    const bool solve = !(GATED && a.readout_only);
    if (solve) async_block_copy<H16>(sH, (const frag *)a.ws_H + chunk_id * (SH::H_FRAGS * 64), w, lane);   // H_[n] -> LDS
    RowStage<MMA, IO, D> krows;
    krows.load(a.k, base_bh, a.stride_t, tok0, a.T, tid);
#pragma unroll
    for (int i = 0; i < NBH; ++i)
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4)
            qraw[i][q4] = IO::load_raw4(a.q, tok_off + 32 * (mt0 + i) + 8 * q4 + 4 * g);
    typename IO::raw4 qlo[GATED ? NBH : 1][4];   // remainder of the right-hand side (variants' kernel), if given
    bool has_qlo = false;
    if constexpr (GATED) {
        has_qlo = a.q_lo != nullptr;
        if (has_qlo) {
#pragma unroll
            for (int i = 0; i < NBH; ++i)
#pragma unroll
                for (int q4 = 0; q4 < 4; ++q4)
                    qlo[i][q4] = IO::load_raw4(a.q_lo, tok_off + 32 * (mt0 + i) + 8 * q4 + 4 * g);
        }
    }
    lam = ((!GATED || a.lambda) ? a.lambda : a.gate)[gate_base + (int64_t)min(tok, a.T - 1) * a.H];
    float hn[NB * NB];
#pragma unroll
    for (int i = 0; i < NB * NB; ++i) hn[i] = solve ? a.ws_hn[chunk_id * (NB * NB) + i] : 0.0f;

    // ---------------- decay mask (Section 4.2.1; log-space form of Appendix B.2, base 2) ----------------
    // With the write gate, H_c = zeta_c H_[n] + sum_{j<=c} M[j,c] beta_j k_j k_j^T (the same for U): beta_j is folded
    // into the mask, m[j,c] = M[j,c] beta_j, which every product below uses.
    // every wave scans the chunk's gates itself: no LDS round trip for the per-token decays
    Gall = wave_inclusive_scan((tok0 + lane < a.T) ? log2_gate(gm) : 0.0f, lane);
    const float Gc = __shfl(Gall, c_local, 64);
    const float zeta = exp2f(Gc);
    f32x16 mreg[NJ];
#pragma unroll
    for (int jt = 0; jt < NJ; ++jt)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int j = 32 * jt + kidx(r, g);
            // (one LDS-crossbar shuffle per value; as pairs of lane reads and a select they took twice the instructions)
            const float Gj = __shfl(Gall, j, 64);
            float bj = 1.0f;
            if constexpr (GATED) bj = __shfl(ball, j, 64);
            // hardware exp2: results below the normal range (decays under 2^-126) are flushed to zero
            const float decay = __builtin_amdgcn_exp2f(Gc - Gj);
            mreg[jt][r] = (j <= c_local) ? (GATED ? bj * decay : decay) : 0.0f;
        }
    const float bc = GATED ? __shfl(ball, c_local, 64) : 1.0f;   // write gate of this lane's token
    __builtin_amdgcn_sched_barrier(0);         // the mask is not scheduled behind the wait for the k rows
    krows.store(sRow, tok0, a.T, tid);
    lds_barrier();
    build_row_frags<MMA, D>(sK, sRow, w, lane);
    build_transposed_frags<MMA, D>(sKT, sRow, w, lane);
    if (!valid) lam = 1.0f;
#pragma unroll
    for (int i = 0; i < NB * NB; ++i) hn2 += hn[i];
    wait_all_memory();                         // H_[n] has landed in LDS
    lds_barrier();                           // fragments and H_[n] visible; the staging tile is free

    // ---------------- chunk-wise Frobenius norm ----------------
    // ||H_c||^2 = zeta_c^2 ||H_[n]||^2 + sum_{j<=c} m[j,c]^2 w_j,
    // w_j = 2 (zeta_j k_j^T H_[n] k_j + sum_{i<j} m[i,j] G_ij^2) / beta_j + G_jj^2,  G = K K^T:
    // the three-term expansion of Section 4.2.1 with its double sum over (i, j) folded by
    // M[i,c] M[j,c] = M[j,c]^2 M[i,j] (i < j), written with the gated mask m (a token with beta_j = 0 has m[j,.] = 0
    // and contributes nothing: its w_j is set to 0).
    // Operand sets of the fused contractions: key blocks jt <= TW first, then this wave's row blocks of the state.
    const frag *Aset[NJ + NBH];
#pragma unroll
    for (int jt = 0; jt < NJ; ++jt) Aset[jt] = sK + (jt * NSTEPS) * 64;
#pragma unroll
    for (int i = 0; i < NBH; ++i) Aset[NJ + i] = sH + ((mt0 + i) * NSTEPS) * 64;
    const frag *Kset[NJ], *Hset[NBH];
#pragma unroll
    for (int jt = 0; jt < NJ; ++jt) Kset[jt] = Aset[jt];
#pragma unroll
    for (int i = 0; i < NBH; ++i) Hset[i] = Aset[NJ + i];
    const frag *myK = sK + (TW * NSTEPS) * 64;         // this token block's keys as a B operand
    if (solve) {
        f32x16 acc[NJ + NBH];
        fused_gemm<MMA, NSTEPS, NJ + NBH, NoFill, NJ + NBH>(Aset, myK, acc, lane);
        // k_c^T H_[n] k_c: this wave's rows of H_[n] k_c, then summed over the two feature halves
        float a_part = 0.0f;
#pragma unroll
        for (int i = 0; i < NBH; ++i)
#pragma unroll
            for (int hh = 0; hh < HS; ++hh) {
                const frag kf = myK[((mt0 + i) * HS + hh) * 64 + lane];   // rows kidx(hh*VEC + p, g) of block mt0 + i
#pragma unroll
                for (int p = 0; p < VEC; ++p) a_part += acc[NJ + i][hh * VEC + p] * MMA::elem(kf, p);
            }
        a_part += __shfl_xor(a_part, 32, 64);
        if (g == 0) sA[fh * kChunk + c_local] = a_part;
        // sum_{i<c} m[i,c] G_ic^2: the mask is zero above the diagonal, so the sum runs over the whole column and the
        // diagonal term m[c,c] G_cc^2 (m[c,c] = beta_c) is taken out again; G_cc^2 sits in the diagonal key block
        float b_part = 0.0f, d_part = 0.0f;
#pragma unroll
        for (int jt = 0; jt < NJ; ++jt)
#pragma unroll
            for (int r = 0; r < 16; ++r) b_part += mreg[jt][r] * (acc[jt][r] * acc[jt][r]);
#pragma unroll
        for (int r = 0; r < 16; ++r)
            if (32 * TW + kidx(r, g) == c_local) d_part = acc[TW][r] * acc[TW][r];
        b_part -= bc * d_part;
        b_part += __shfl_xor(b_part, 32, 64);
        d_part += __shfl_xor(d_part, 32, 64);
        lds_barrier();
        if (fh == 0 && g == 0) {
            const float cross = 2.0f * (zeta * (sA[c_local] + sA[kChunk + c_local]) + b_part);
            sW[c_local] = GATED ? (bc > 0.0f ? cross / bc + d_part : 0.0f) : cross + d_part;
        }
    }
    lds_barrier();
    float fro;
    {
        float f_part = 0.0f;
#pragma unroll
        for (int jt = 0; jt < NJ; ++jt)
#pragma unroll
            for (int r = 0; r < 16; ++r) f_part += mreg[jt][r] * mreg[jt][r] * sW[32 * jt + kidx(r, g)];
        f_part += __shfl_xor(f_part, 32, 64);
        fro = solve ? sqrtf(fmaxf(zeta * zeta * hn2 + f_part, 0.0f)) : 0.0f;   // (no solve: sW was not written)
    }
    if (a.fro_out && valid && fh == 0 && g == 0) a.fro_out[gate_base + (int64_t)tok * a.H] = fro;
    if (GATED && !a.lambda) lam = valid ? a.lambda_scale * fro : 1.0f;      // Section 4.1: lambda_t = a ||H_t||_F
    if (!solve) lam = 1.0f;                    // plain readout: the discarded starting point stays finite

    // ---------------- Chebyshev iteration (Algorithm 1), residual form ----------------
    const float L = fro + lam, mu = lam;       // Section 4.1: L = ||H_t||_F + lambda_t, mu = lambda_t
    const float s0 = 2.0f / (L + mu);
    const float rho = (L - mu) / (L + mu);
    const float rho2 = rho * rho;
    float xi[NBH][16], dl[NBH][16];
    f32x16 gS[NBH], gI[NBH];
    frag own[NBH][HS];
#pragma unroll
    for (int i = 0; i < NBH; ++i) {
        gS[i] = zero16();
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
            f32x4 qv4 = IO::cvt4(qraw[i][q4]);
            if constexpr (GATED) {
                if (has_qlo) qv4 += IO::cvt4(qlo[i][q4]);
            }
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float qv = valid ? qv4[e] : 0.0f;
                gI[i][4 * q4 + e] = -qv;
                dl[i][4 * q4 + e] = s0 * qv;      // delta_0 = xi_0 - xi_{-1} = xi_0 = 2 q / (L + mu)
            }
        }
#pragma unroll
        for (int hh = 0; hh < HS; ++hh) own[i][hh] = MMA::pack(&dl[i][hh * VEC]);
    }
    const frag *myX = sX + (TW * NSTEPS) * 64;         // this token block's operand in the exchange region
    float omega = 2.0f;
    // xi lags one update behind: xi += delta is applied while the next pass's first sweep runs (and once after the
    // last pass), so it starts from xi_{-1} = 0
#pragma unroll
    for (int i = 0; i < NBH; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) xi[i][r] = 0.0f;
    lds_barrier();                           // sW, sA are dead: the region becomes the operand exchange
    for (int it = 0; it < a.n_iter; ++it) {
        // operands are re-read from LDS in every pass (they are not kept in registers across passes)
        asm volatile("" ::: "memory");
        publish_operand<MMA, NB>(sX, own, TW, mt0, lane);
        lds_barrier();
        // One sweep over the D features of delta for both products that take it as B operand: P = K delta^T (key
        // blocks jt <= TW) and the state product. xi += delta is issued between its MFMAs.
        f32x16 pacc[NJ];
        auto add_delta = [&](auto step) {
            constexpr int S = decltype(step)::value;
            constexpr int TOTAL = NBH * 16, PER = (TOTAL + NSTEPS - 1) / NSTEPS;
#pragma unroll
            for (int e = 0; e < PER; ++e) {
                const int idx = S * PER + e;
                if (idx < TOTAL) xi[idx / 16][idx % 16] += dl[idx / 16][idx % 16];
            }
        };
        if constexpr (MMA::kFusedPassSweep) {
            fused_pass_sweep<MMA, NSTEPS, NJ, NBH>(Kset, Hset, myX, pacc, gS, lane, add_delta);
        } else {
            fused_gemm<MMA, NSTEPS, NJ, decltype(add_delta), NJ>(Kset, myX, pacc, lane, add_delta);
            fused_gemm<MMA, NSTEPS, NBH>(Hset, myX, gS, lane);
        }
        frag pm[NJ][HS];
        mask_p<MMA, TW>(pacc, mreg, pm);
        lds_barrier();                       // the exchange region may be overwritten from here on
        omega = 4.0f / (4.0f - rho2 * omega);                      // weight schedule
        const float cm = omega - 1.0f, ncs = -omega * s0;
        // -r_{i-1} = zeta gS + gI + lam xi; delta_i = cm delta_{i-1} - omega s0 r_{i-1}: the gS term is formed while the
        // MFMAs that finish gI are in flight
        constexpr int TOTAL = NBH * 16, NM = NBH * (TW + 1) * HS, PERM = (TOTAL + NM - 1) / NM;
        if constexpr (MMA::kFusedPassSweep) {
            gemm_intra<MMA, NBH, TW>(sKT, mt0, pm, gI, lane, [&](auto step) {
                constexpr int S = decltype(step)::value;
                const float ncz = ncs * zeta;
#pragma unroll
                for (int e = 0; e < PERM; ++e) {
                    const int idx = S * PERM + e;
                    if (idx < TOTAL)
                        dl[idx / 16][idx % 16] = cm * dl[idx / 16][idx % 16] + ncz * gS[idx / 16][idx % 16];
                }
            });
        } else {
            // many short MFMAs per product: the compiler's own schedule is better than a pinned interleaving
            gemm_intra<MMA, NBH, TW>(sKT, mt0, pm, gI, lane);
            const float ncz = ncs * zeta;
#pragma unroll
            for (int i = 0; i < NBH; ++i)
#pragma unroll
                for (int r = 0; r < 16; ++r) dl[i][r] = cm * dl[i][r] + ncz * gS[i][r];
        }
        const float ncl = ncs * lam;
#pragma unroll
        for (int i = 0; i < NBH; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) dl[i][r] += ncl * xi[i][r];
#pragma unroll
        for (int i = 0; i < NBH; ++i) {
            // The last term is written as inline assembly (below). The compiler does not track the matrix pipe's
            // result hazard for inline assembly: a vector instruction may read an MFMA result only some wait states
            // after the MFMA was issued, and only for its own instructions does the compiler insert the idle cycles.
            // So the first read of gI[i] is one of its own: the coefficient of the assembly statements is routed
            // through an instruction that reads gI[i] (0 * gI + ncs), which orders them behind it and behind the wait.
            // (The converse also holds: no MFMA may take a register that inline assembly has just written. The
            // results below go to LDS and to vector instructions only.)
            const float ncs_i = __builtin_fmaf(gI[i][0], 0.0f, ncs);
#pragma unroll
            for (int r = 0; r < 16; ++r) {                                               // delta_i
                // three-address form: the result goes straight into the loop-carried register instead of a
                // temporary that is copied there at the end of the pass
                float t = dl[i][r];
                asm("v_fma_f32 %0, %1, %2, %3" : "=v"(dl[i][r]) : "v"(ncs_i), "v"(gI[i][r]), "v"(t));
            }
#pragma unroll
            for (int hh = 0; hh < HS; ++hh) own[i][hh] = MMA::pack(&dl[i][hh * VEC]);
        }
    }
#pragma unroll
    for (int i = 0; i < NBH; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) xi[i][r] += dl[i][r];                               // xi_r

    // ---------------- readout y_c = zeta_c U_[n] xhat_c + sum_{j<=c} M[j,c] v_j (k_j . xhat_c) ----------------
    constexpr int NSPL = MMA::kSplitReadout ? 2 : 1;
    const frag *Uw = (const frag *)a.ws_U + chunk_id * (NSPL * SH::H_FRAGS * 64);
    RowStage<MMA, IO, D> vrows;
    // The addresses of the readout's loads and staging stores are formed here, from a copy of the thread index that
    // the compiler cannot trace back past this point: formed before the passes (where it would hoist them, or keep
    // those of the k rows) they would occupy registers across the loop.
    int tid_late = tid;
    asm volatile("" : "+v"(tid_late));
    const int lane_late = tid_late & 63;
    if (!(GATED && a.solve_only)) vrows.load(a.v, base_bh, a.stride_t, tok0, a.T, tid_late);
    // optional output of the solve's result (the variants' kernel only, so that the plain kernel carries no trace of it)
    if (GATED && a.xhat_out && valid) {
        float *xo = a.xhat_out + (gate_base + (int64_t)tok * a.H) * D;
#pragma unroll
        for (int i = 0; i < NBH; ++i)
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4)
                *(f32x4 *)(xo + 32 * (mt0 + i) + 8 * q4 + 4 * g) =
                    f32x4{xi[i][4 * q4], xi[i][4 * q4 + 1], xi[i][4 * q4 + 2], xi[i][4 * q4 + 3]};
    }
    if (GATED && a.solve_only) return;         // (whole workgroup) the caller wants xhat only: no U_[n], no readout
    // alpha-connection (Section 4.3): the readout is applied to alpha xhat + (1 - alpha) q
    if (GATED && a.alpha) {
        const float al = valid ? a.alpha[gate_base + (int64_t)tok * a.H] : 1.0f;
#pragma unroll
        for (int i = 0; i < NBH; ++i)
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
                const f32x4 qv4 = IO::load4(a.q, tok_off + 32 * (mt0 + i) + 8 * q4 + 4 * g);
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    xi[i][4 * q4 + e] = al * xi[i][4 * q4 + e] + (1.0f - al) * (valid ? qv4[e] : 0.0f);
            }
    }
    // the operand of the readout as B operand: the rounded value and, on the bf16 path, the rounding remainder as a
    // second operand
    frag ownlo[NBH][HS];
#pragma unroll
    for (int i = 0; i < NBH; ++i)
#pragma unroll
        for (int hh = 0; hh < HS; ++hh) {
            own[i][hh] = MMA::pack(&xi[i][hh * VEC]);
            if (NSPL == 2) {
                float lo[VEC], back[VEC];
                MMA::unpack(own[i][hh], back);
#pragma unroll
                for (int p = 0; p < VEC; ++p) lo[p] = xi[i][hh * VEC + p] - back[p];
                ownlo[i][hh] = MMA::pack(lo);
            }
        }
    // The rounding remainder of U_[n] is used once, against the rounded xhat: its fragments go from global memory
    // straight into registers (the passes' registers are free by now) and never pass through LDS.
    frag ulo[NBH][NSTEPS];
    if (NSPL == 2) {
        const frag *Ulo = Uw + SH::H_FRAGS * 64;
#pragma unroll
        for (int i = 0; i < NBH; ++i)
#pragma unroll
            for (int st = 0; st < NSTEPS; ++st) ulo[i][st] = Ulo[((mt0 + i) * NSTEPS + st) * 64 + lane_late];
    }
    lds_barrier();                           // every wave is done with H_[n], K^T and the exchange region
    async_block_copy<H16>(sH, Uw, w, lane_late);    // U_[n] (rounded part) replaces H_[n]
    vrows.store(sRow, tok0, a.T, tid_late);
    lds_barrier();
    build_transposed_frags<MMA, D, true>(sKT, sRow, w, lane_late);      // V^T replaces K^T
    lds_barrier();                           // the staging tile becomes the exchange region again
    publish_operand<MMA, NB>(sX, own, TW, mt0, lane);
    wait_all_memory();
    lds_barrier();
    f32x16 acc[NJ + NBH];
    fused_gemm<MMA, NSTEPS, NJ + NBH, NoFill, NJ + NBH>(Aset, myX, acc, lane);   // K xhat^T and U xhat
    if (NSPL == 2) {
        // remainder of U_[n] (registers) times the rounded xhat (still published)
#pragma unroll
        for (int st = 0; st < NSTEPS; ++st) {
            const frag bx = myX[st * 64 + lane];
#pragma unroll
            for (int i = 0; i < NBH; ++i) acc[NJ + i] = MMA::mma(ulo[i][st], bx, acc[NJ + i]);
        }
        lds_barrier();
        publish_operand<MMA, NB>(sX, ownlo, TW, mt0, lane);
        lds_barrier();
        fused_gemm<MMA, NSTEPS, NJ + NBH>(Aset, myX, acc, lane);      // K and rounded U on the remainder of xhat
    }
    frag pm[NJ][HS];
    f32x16 y[NBH];
    {
        f32x16 pacc[NJ];
#pragma unroll
        for (int jt = 0; jt < NJ; ++jt) pacc[jt] = acc[jt];
        mask_p<MMA, TW>(pacc, mreg, pm);
    }
#pragma unroll
    for (int i = 0; i < NBH; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) y[i][r] = acc[NJ + i][r] * zeta;
    gemm_intra<MMA, NBH, TW>(sKT, mt0, pm, y, lane);
    if (valid) {
#pragma unroll
        for (int i = 0; i < NBH; ++i)
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4)
                IO::store4(a.o, tok_off + 32 * (mt0 + i) + 8 * q4 + 4 * g, y[i][4 * q4], y[i][4 * q4 + 1],
                           y[i][4 * q4 + 2], y[i][4 * q4 + 3]);
    }
}

template <class MMA, class IO, int D, bool GATED>
__device__ __forceinline__ void chunk_solve_body(const SolveArgs &a)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    // wave-uniform: token block and feature half of this wave
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    if (w & 1)
        chunk_solve_wave<MMA, IO, D, 1, GATED>(a, smem, w);
    else
        chunk_solve_wave<MMA, IO, D, 0, GATED>(a, smem, w);
}

// bf16 path: capped at 256 registers so that two workgroups (two waves per SIMD) share a CU.
template <class IO, int D, bool GATED>
__global__ __launch_bounds__(kSolveThreads) __attribute__((amdgpu_waves_per_eu(2, 2))) void chunk_solve_kernel_bf16(
    SolveArgs a)
{
    chunk_solve_body<MmaBF16, IO, D, GATED>(a);
}

// fp32 path: its fragments are twice as large, one workgroup per CU.
template <class IO, int D, bool GATED>
__global__ __launch_bounds__(kSolveThreads) void chunk_solve_kernel_f32(SolveArgs a)
{
    chunk_solve_body<MmaF32, IO, D, GATED>(a);
}

template <class MMA, class IO, int D, bool GATED>
struct SolveKernel;
template <class IO, int D, bool GATED>
struct SolveKernel<MmaBF16, IO, D, GATED> {
    static constexpr auto fn = chunk_solve_kernel_bf16<IO, D, GATED>;
};
template <class IO, int D, bool GATED>
struct SolveKernel<MmaF32, IO, D, GATED> {
    static constexpr auto fn = chunk_solve_kernel_f32<IO, D, GATED>;
};

template <class MMA, class IO, int D, bool GATED>
static hipError_t launch_chunk_solve_g(const SolveArgs &a, int n_pairs, hipStream_t stream)
{
    typedef SolveShape<MMA, D> SH;
    auto kern = SolveKernel<MMA, IO, D, GATED>::fn;
    // (set once per kernel instantiation and device, not per launch)
    static bool attr_set_on[64] = {};
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= 64 || !attr_set_on[dev]) {
        e = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)SH::lds_bytes);
        if (e != hipSuccess) return e;
        if (dev >= 0 && dev < 64) attr_set_on[dev] = true;
    }
    SolveArgs args = a;
    args.n_pairs = n_pairs;
    dim3 grid((unsigned)(n_pairs * a.n_chunks)), block(kSolveThreads);
    const size_t lds = SH::lds_bytes;
    hipLaunchKernelGGL(kern, grid, block, lds, stream, args);
    return hipGetLastError();
}

template <class MMA, class IO, int D>
static hipError_t launch_chunk_solve_t(const SolveArgs &a, int n_pairs, hipStream_t stream)
{
    if (a.beta || a.alpha || !a.lambda || a.xhat_out) return launch_chunk_solve_g<MMA, IO, D, true>(a, n_pairs, stream);
    return launch_chunk_solve_g<MMA, IO, D, false>(a, n_pairs, stream);
}

hipError_t launch_chunk_solve(const SolveArgs &a, int n_pairs, int d, bool io_bf16, bool compute_bf16,
                              hipStream_t stream)
{
    if (compute_bf16) {
        if (d == 128) return launch_chunk_solve_t<MmaBF16, IOBF16, 128>(a, n_pairs, stream);
        return launch_chunk_solve_t<MmaBF16, IOBF16, 64>(a, n_pairs, stream);
    }
    if (io_bf16) {
        if (d == 128) return launch_chunk_solve_t<MmaF32, IOBF16, 128>(a, n_pairs, stream);
        return launch_chunk_solve_t<MmaF32, IOBF16, 64>(a, n_pairs, stream);
    }
    if (d == 128) return launch_chunk_solve_t<MmaF32, IOF32, 128>(a, n_pairs, stream);
    return launch_chunk_solve_t<MmaF32, IOF32, 64>(a, n_pairs, stream);
}

size_t ws_H_bytes_per_chunk(int d, bool compute_bf16) { return (size_t)d * d * (compute_bf16 ? 2 : 4); }
size_t ws_U_bytes_per_chunk(int d, bool compute_bf16) { return (size_t)d * d * (compute_bf16 ? 4 : 4); }
size_t ws_hn_bytes_per_chunk(int d) { return (size_t)(d / 32) * (d / 32) * sizeof(float); }

}  // namespace gka
