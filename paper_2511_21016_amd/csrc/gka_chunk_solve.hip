// Per-chunk solve: chunk-wise Frobenius norms (Section 4.2.1), the fused Chebyshev driver
// (Algorithm 1 on all tokens of the chunk at once) and the readout y_c = U_c xhat_c of Eq. (CH).
//
// One workgroup = one chunk of one (batch, head) pair = two waves; wave w owns tokens 32w .. 32w+31.
// All products are computed transposed, tokens along the MFMA N dimension: lane (n, g) of wave w holds
// token c = 32w + n, and an accumulator tile holds rows kidx(r, g) of that token's feature vector.
// Consequences: every per-token scalar (zeta_c, lambda_c, L, rho, omega_i) is a per-lane scalar, the
// iterate / residual never leave registers, and an accumulator tile converts in place into the B operand
// of the next contraction. The chunk's initial state H_[n] and the keys sit in LDS in fragment order as
// the A operands. With H_c = zeta_c H_[n] + sum_{j<=c} M[j,c] k_j k_j^T (Section 4.2.1):
//
//   (H_c x_c) = zeta_c * (H_[n] x_c)  +  sum_{j<=c} M[j,c] k_j (k_j . x_c)
//               `-- state product --'     `-- P = K X^T, mask, K^T (P o M) --'
//
// The Chebyshev recurrence is run in its residual form (same iterates in exact arithmetic):
//   delta_i = (omega_i - 1) delta_{i-1} + (2 omega_i / (L + mu)) r_{i-1},  xi_i = xi_{i-1} + delta_i,
//   r_i = r_{i-1} - (H_c + lambda_c I) delta_i,
// so that the low-precision operand of each product is the shrinking update delta_i, not the iterate.
#include "gka_device.hpp"
#include "gka_kernels.hpp"

namespace gka {

#ifdef GKA_DEBUG_TIMERS
__device__ unsigned long long g_dbg_timers[64 * 16];
#define GKA_TSTAMP(i)                                                                   \
    do {                                                                                \
        if (threadIdx.x == 0 && blockIdx.x >= 2048 && blockIdx.x < 2112) g_dbg_timers[(blockIdx.x - 2048) * 16 + (i)] = __builtin_amdgcn_s_memtime(); \
    } while (0)
#else
#define GKA_TSTAMP(i) do {} while (0)
#endif

template <class MMA, int D>
struct SolveShape {
    typedef typename MMA::frag frag;
    typedef typename MMA::elem_t elem_t;
    static constexpr int NB = D / 32;
    static constexpr int HS = MMA::HS;
    static constexpr int JB = kChunk / 32;
    static constexpr int H_FRAGS = NB * NB * HS;
    static constexpr int K_FRAGS = JB * NB * HS;
    static constexpr int KT_FRAGS = NB * JB * HS;
    // row-major staging tile of one chunk of k or v rows, padded against bank conflicts
    static constexpr int RS = D + 16 / (int)sizeof(elem_t);
    static constexpr size_t row_bytes = (size_t)kChunk * RS * sizeof(elem_t);
    static constexpr size_t h_bytes = (size_t)H_FRAGS * 64 * sizeof(frag);
    static constexpr size_t k_bytes = (size_t)K_FRAGS * 64 * sizeof(frag);
    static constexpr size_t kt_bytes = (size_t)KT_FRAGS * 64 * sizeof(frag);
    static constexpr bool row_aliases_h = row_bytes <= h_bytes;   // staging tile reuses the state region
    static constexpr size_t lds_bytes =
        h_bytes + k_bytes + kt_bytes + (row_aliases_h ? 0 : row_bytes) + 2 * kChunk * sizeof(float);
};

// pacc[jt] += sum_{blk,h} K[jt][blk][h] * X[blk][h] for the key blocks jt <= w (causal)
template <class MMA, int NB>
__device__ __forceinline__ void gemm_p(const typename MMA::frag *sK, const typename MMA::frag (&X)[NB][MMA::HS],
                                       f32x16 (&pacc)[2], int w, int lane)
{
#pragma unroll
    for (int blk = 0; blk < NB; ++blk)
#pragma unroll
        for (int hh = 0; hh < MMA::HS; ++hh)
            pacc[0] = MMA::mma(sK[((0 * NB + blk) * MMA::HS + hh) * 64 + lane], X[blk][hh], pacc[0]);
    if (w == 1) {
#pragma unroll
        for (int blk = 0; blk < NB; ++blk)
#pragma unroll
            for (int hh = 0; hh < MMA::HS; ++hh)
                pacc[1] = MMA::mma(sK[((1 * NB + blk) * MMA::HS + hh) * 64 + lane], X[blk][hh], pacc[1]);
    }
}

// (P o M) as B-operand fragments
template <class MMA>
__device__ __forceinline__ void mask_p(const f32x16 (&pacc)[2], const f32x16 (&mreg)[2],
                                       typename MMA::frag (&pm)[2][MMA::HS], int w)
{
    constexpr int VEC = MMA::VEC, HS = MMA::HS;
#pragma unroll
    for (int hh = 0; hh < HS; ++hh) {
        float t[VEC];
#pragma unroll
        for (int p = 0; p < VEC; ++p) t[p] = pacc[0][hh * VEC + p] * mreg[0][hh * VEC + p];
        pm[0][hh] = MMA::pack(t);
    }
    if (w == 1) {
#pragma unroll
        for (int hh = 0; hh < HS; ++hh) {
            float t[VEC];
#pragma unroll
            for (int p = 0; p < VEC; ++p) t[p] = pacc[1][hh * VEC + p] * mreg[1][hh * VEC + p];
            pm[1][hh] = MMA::pack(t);
        }
    }
}

// acc += sum_{blk,h} A[mt][blk][h] * X[blk][h]      (A = H_[n] or U_[n] fragments in LDS)
template <class MMA, int NB>
__device__ __forceinline__ f32x16 gemm_state_mt(const typename MMA::frag *sA, int mt,
                                                const typename MMA::frag (&X)[NB][MMA::HS], f32x16 acc, int lane)
{
#pragma unroll
    for (int blk = 0; blk < NB; ++blk)
#pragma unroll
        for (int hh = 0; hh < MMA::HS; ++hh)
            acc = MMA::mma(sA[((mt * NB + blk) * MMA::HS + hh) * 64 + lane], X[blk][hh], acc);
    return acc;
}

// acc += sum_{jt<=w,h} AT[mt][jt][h] * pm[jt][h]     (AT = K^T or V^T fragments)
template <class MMA>
__device__ __forceinline__ f32x16 gemm_intra_mt(const typename MMA::frag *sAT, int mt,
                                                const typename MMA::frag (&pm)[2][MMA::HS], f32x16 acc, int w,
                                                int lane)
{
    constexpr int HS = MMA::HS;
#pragma unroll
    for (int hh = 0; hh < HS; ++hh) acc = MMA::mma(sAT[((mt * 2 + 0) * HS + hh) * 64 + lane], pm[0][hh], acc);
    if (w == 1) {
#pragma unroll
        for (int hh = 0; hh < HS; ++hh) acc = MMA::mma(sAT[((mt * 2 + 1) * HS + hh) * 64 + lane], pm[1][hh], acc);
    }
    return acc;
}

// A block of N16 * 128 16-byte units copied global -> registers -> LDS by the 128 threads of the workgroup.
// The two halves are separate calls so that the global loads can be issued long before the LDS region is free.
template <int N16>
struct BlockCopy {
    uint4 r[N16];
    __device__ __forceinline__ void load(const void *src, int tid)
    {
        const uint4 *s = (const uint4 *)src;
#pragma unroll
        for (int i = 0; i < N16; ++i) r[i] = s[i * 128 + tid];
    }
    __device__ __forceinline__ void store(void *dst, int tid) const
    {
        uint4 *d = (uint4 *)dst;
#pragma unroll
        for (int i = 0; i < N16; ++i) d[i * 128 + tid] = r[i];
    }
};

// One chunk of rows of x (k or v): global -> registers (load), registers -> row-major LDS tile of operand
// elements (store); rows past T are zero.
template <class MMA, class IO, int D>
struct RowStage {
    static constexpr int RS = SolveShape<MMA, D>::RS;
    static constexpr int P4 = D / 4;
    static constexpr int NP = kChunk * P4 / 128;
    typename IO::raw4 r[NP];
    // Rows past the end of the sequence are read from the last valid row (no divergent branch around the
    // loads, which would force a wait on each) and zeroed when stored.
    __device__ __forceinline__ void load(const void *x, int64_t base, int64_t stride_t, int tok0, int T, int tid)
    {
#pragma unroll
        for (int i = 0; i < NP; ++i) {
            const int piece = i * 128 + tid;
            const int row = piece / P4, c4 = piece % P4;
            const int tok = min(tok0 + row, T - 1);
            r[i] = IO::load_raw4(x, base + (int64_t)tok * stride_t + 4 * c4);
        }
    }
    __device__ __forceinline__ void store(typename MMA::elem_t *sRow, int tok0, int T, int tid) const
    {
#pragma unroll
        for (int i = 0; i < NP; ++i) {
            const int piece = i * 128 + tid;
            f32x4 v = IO::cvt4(r[i]);
            if (tok0 + piece / P4 >= T) v = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
            MMA::store4(sRow + (piece / P4) * RS + 4 * (piece % P4), v);
        }
    }
};

// Fragments K[jt][blk][h]: rows = tokens of block jt, contraction index = features in kidx order.
template <class MMA, int D>
__device__ __forceinline__ void build_row_frags(typename MMA::frag *sK, const typename MMA::elem_t *sRow, int w,
                                                int lane)
{
    typedef SolveShape<MMA, D> SH;
    constexpr int VEC = MMA::VEC, HS = MMA::HS, NB = SH::NB, RS = SH::RS;
    const int n = lane & 31, g = lane >> 5;
#pragma unroll 4
    for (int f = w; f < SH::K_FRAGS; f += 2) {
        const int hh = f % HS, blk = (f / HS) % NB, jt = f / (HS * NB);
        if constexpr (VEC == 8) {
            // kidx(8*hh + p, g) = 16*hh + 8*(p/4) + 4*g + p%4: two runs of four consecutive features
            const typename MMA::elem_t *src = sRow + (32 * jt + n) * RS + 32 * blk + 16 * hh + 4 * g;
            u16x4 lo = *(const u16x4 *)src, hi = *(const u16x4 *)(src + 8);
            u16x8 u = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
            sK[f * 64 + lane] = __builtin_bit_cast(typename MMA::frag, u);
        } else {
            typename MMA::elem_t e[VEC];
#pragma unroll
            for (int p = 0; p < VEC; ++p) e[p] = sRow[(32 * jt + n) * RS + 32 * blk + kidx(hh * VEC + p, g)];
            sK[f * 64 + lane] = MMA::pack_elems(e);
        }
    }
}

// Fragments AT[mt][jt][h]: row 32*mt + n of X^T, contraction index = tokens j = 32*jt + kidx(h*VEC + p, g).
template <class MMA, int D>
__device__ __forceinline__ void build_transposed_frags(typename MMA::frag *sAT, const typename MMA::elem_t *sRow,
                                                       int w, int lane)
{
    typedef SolveShape<MMA, D> SH;
    constexpr int VEC = MMA::VEC, HS = MMA::HS, RS = SH::RS;
    const int n = lane & 31, g = lane >> 5;
#pragma unroll 4
    for (int f = w; f < SH::KT_FRAGS; f += 2) {
        const int hh = f % HS, jt = (f / HS) % 2, mt = f / (2 * HS);
        if constexpr (VEC == 8) {
            const int t0 = 32 * jt + 16 * hh + 4 * g;       // kidx(8*hh + p, g) = 16*hh + 8*(p/4) + 4*g + p%4
            sAT[f * 64 + lane] =
                gather_transposed_bf16(sRow, RS, 32 * mt + 16 * ((lane >> 4) & 1), lane, t0, t0 + 8);
        } else {
            auto tok_of = [&](int p) { return 32 * jt + kidx(hh * VEC + p, g); };
            sAT[f * 64 + lane] = gather_transposed<MMA>(sRow, RS, 32 * mt + n, tok_of);
        }
    }
}

template <class MMA, class IO, int D>
__global__ __launch_bounds__(128) void chunk_solve_kernel(SolveArgs a)
{
    typedef SolveShape<MMA, D> SH;
    constexpr int NB = SH::NB;
    constexpr int VEC = MMA::VEC, HS = MMA::HS;
    typedef typename MMA::frag frag;
    typedef typename MMA::elem_t elem_t;

    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    frag *sH = (frag *)smem;
    frag *sK = (frag *)(smem + SH::h_bytes);
    frag *sKT = (frag *)(smem + SH::h_bytes + SH::k_bytes);
    unsigned char *tail = smem + SH::h_bytes + SH::k_bytes + SH::kt_bytes;
    elem_t *sRow = SH::row_aliases_h ? (elem_t *)smem : (elem_t *)tail;
    float *sG = (float *)(tail + (SH::row_aliases_h ? 0 : SH::row_bytes));
    float *sW = sG + kChunk;

    const int tid = threadIdx.x;
    const int lane = tid & 63, w = tid >> 6;
    const int n = lane & 31, g = lane >> 5;
    const int chunk = blockIdx.x % a.n_chunks_total;
    const int pair = blockIdx.x / a.n_chunks_total;
    const int b = pair / a.H, h = pair % a.H;
    const int64_t chunk_id = (int64_t)pair * a.n_chunks_total + chunk;
    const int64_t base_bh = (int64_t)b * a.stride_b + (int64_t)h * a.stride_h;
    const int64_t gate_base = (int64_t)b * a.T * a.H + h;
    const int tok0 = chunk * kChunk;
    const int c_local = 32 * w + n;
    const int tok = tok0 + c_local;
    const bool valid = tok < a.T;

    GKA_TSTAMP(0);
    // ---------------- staging ----------------
    constexpr int H16 = (int)(SH::h_bytes / 16 / 128);     // 16-byte units of a state block per thread
    const int64_t tok_off = base_bh + (int64_t)min(tok, a.T - 1) * a.stride_t;
    float lam, hn2 = 0.0f;
    typename IO::raw4 qraw[NB][4];
    {
        // every global read of the prologue is issued here, before the first wait
        RowStage<MMA, IO, D> krows;
        BlockCopy<H16> hcopy;
        krows.load(a.k, base_bh, a.stride_t, tok0, a.T, tid);
        hcopy.load((const frag *)a.ws_H + chunk_id * (SH::H_FRAGS * 64), tid);
#pragma unroll
        for (int blk = 0; blk < NB; ++blk)
#pragma unroll
            for (int i = 0; i < 4; ++i) qraw[blk][i] = IO::load_raw4(a.q, tok_off + 32 * blk + 8 * i + 4 * g);
        const int64_t gl_idx = gate_base + (int64_t)min(tok, a.T - 1) * a.H;
        lam = a.lambda[gl_idx];
        float hn[NB * NB];
#pragma unroll
        for (int i = 0; i < NB * NB; ++i) hn[i] = a.ws_hn[chunk_id * (NB * NB) + i];
        if (w == 0) {
            const int t = tok0 + lane;
            const float gm = a.gate[gate_base + (int64_t)min(t, a.T - 1) * a.H];
            const float lg = (t < a.T) ? log_gate(gm) : 0.0f;
            sG[lane] = wave_inclusive_scan(lg, lane);
        }
        if (!valid) lam = 1.0f;
#pragma unroll
        for (int i = 0; i < NB * NB; ++i) hn2 += hn[i];
        GKA_TSTAMP(1);
        krows.store(sRow, tok0, a.T, tid);
        __syncthreads();
        GKA_TSTAMP(2);
        build_row_frags<MMA, D>(sK, sRow, w, lane);
        build_transposed_frags<MMA, D>(sKT, sRow, w, lane);
        __syncthreads();                       // the staging tile may alias the state region
        GKA_TSTAMP(3);
        hcopy.store(sH, tid);
    }
    __syncthreads();
    GKA_TSTAMP(4);

    // ---------------- decay mask (Section 4.2.1; log-space form of Appendix B.2) ----------------
    const float Gc = sG[c_local];
    const float zeta = expf(Gc);
    f32x16 mreg[2];
#pragma unroll
    for (int jt = 0; jt < 2; ++jt)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int j = 32 * jt + kidx(r, g);
            mreg[jt][r] = (j <= c_local) ? expf(Gc - sG[j]) : 0.0f;
        }

    GKA_TSTAMP(5);
    // ---------------- chunk-wise Frobenius norm ----------------
    // ||H_c||^2 = zeta_c^2 ||H_[n]||^2 + sum_{j<=c} M[j,c]^2 w_j,
    // w_j = 2 (zeta_j k_j^T H_[n] k_j + sum_{i<j} M[i,j] G_ij^2) + G_jj^2,  G = K K^T:
    // the three-term expansion of Section 4.2.1 with its double sum over (i, j) folded by
    // M[i,c] M[j,c] = M[j,c]^2 M[i,j] (i < j).
    f32x16 pacc[2];
    frag X[NB][HS];
    {
#pragma unroll
        for (int blk = 0; blk < NB; ++blk)
#pragma unroll
            for (int hh = 0; hh < HS; ++hh) X[blk][hh] = sK[((w * NB + blk) * HS + hh) * 64 + lane];
        float a_part = 0.0f;
#pragma unroll
        for (int mt = 0; mt < NB; ++mt) {
            f32x16 acc = gemm_state_mt<MMA, NB>(sH, mt, X, zero16(), lane);
#pragma unroll
            for (int r = 0; r < 16; ++r) a_part += acc[r] * MMA::elem(X[mt][r / VEC], r % VEC);
        }
        pacc[0] = zero16();
        pacc[1] = zero16();
        gemm_p<MMA, NB>(sK, X, pacc, w, lane);
        float b_part = 0.0f, d_part = 0.0f;
#pragma unroll
        for (int jt = 0; jt < 2; ++jt)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int j = 32 * jt + kidx(r, g);
                const float g2 = pacc[jt][r] * pacc[jt][r];
                if (j < c_local) b_part += mreg[jt][r] * g2;
                if (j == c_local) d_part += g2;
            }
        a_part += __shfl_xor(a_part, 32, 64);
        b_part += __shfl_xor(b_part, 32, 64);
        d_part += __shfl_xor(d_part, 32, 64);
        if (g == 0) sW[c_local] = 2.0f * (zeta * a_part + b_part) + d_part;
    }
    __syncthreads();
    float fro;
    {
        float f_part = 0.0f;
#pragma unroll
        for (int jt = 0; jt < 2; ++jt)
#pragma unroll
            for (int r = 0; r < 16; ++r) f_part += mreg[jt][r] * mreg[jt][r] * sW[32 * jt + kidx(r, g)];
        f_part += __shfl_xor(f_part, 32, 64);
        fro = sqrtf(fmaxf(zeta * zeta * hn2 + f_part, 0.0f));
    }
    if (a.fro_out && valid && g == 0) a.fro_out[gate_base + (int64_t)tok * a.H] = fro;

    GKA_TSTAMP(6);
    // ---------------- Chebyshev iteration (Algorithm 1), residual form ----------------
    const float L = fro + lam, mu = lam;       // Section 4.1: L = ||H_t||_F + lambda_t, mu = lambda_t
    const float s0 = 2.0f / (L + mu);
    const float rho = (L - mu) / (L + mu);
    const float rho2 = rho * rho;
    // Registers: xi (iterate) and dl (last update) per token; the product g_i = H_c xi_i - q is accumulated
    // over the passes inside the MFMA accumulators, split as g = zeta * gS + gI (state part, intra-chunk
    // part), so that r_i = q - (H_c + lambda) xi_i = -(zeta gS + gI + lambda xi_i) needs no storage.
    float xi[NB][16], dl[NB][16];
    f32x16 gS[NB], gI[NB];
#pragma unroll
    for (int blk = 0; blk < NB; ++blk) {
        gS[blk] = zero16();
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float qv = valid ? IO::cvt4(qraw[blk][i])[e] : 0.0f;
                gI[blk][4 * i + e] = -qv;
                xi[blk][4 * i + e] = s0 * qv;     // xi_0 = 2 q / (L + mu); delta_0 = xi_0 - xi_{-1} = xi_0
                dl[blk][4 * i + e] = s0 * qv;
            }
#pragma unroll
        for (int hh = 0; hh < HS; ++hh) X[blk][hh] = MMA::pack(&dl[blk][hh * VEC]);
    }
    float omega = 2.0f;
    for (int it = 0; it < a.n_iter; ++it) {
        // the A operands are re-read from LDS in every pass: keeping them in registers across passes costs
        // more register moves than the LDS reads it saves
        asm volatile("" ::: "memory");
        pacc[0] = zero16();
        pacc[1] = zero16();
        gemm_p<MMA, NB>(sK, X, pacc, w, lane);
        frag pm[2][HS];
        mask_p<MMA>(pacc, mreg, pm, w);
        omega = 4.0f / (4.0f - rho2 * omega);                      // weight schedule
        const float cm = omega - 1.0f, ncs = -omega * s0;
        frag Xn[NB][HS];
#pragma unroll
        for (int mt = 0; mt < NB; ++mt) {
            gS[mt] = gemm_state_mt<MMA, NB>(sH, mt, X, gS[mt], lane);
            gI[mt] = gemm_intra_mt<MMA>(sKT, mt, pm, gI[mt], w, lane);
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const float nres = zeta * gS[mt][r] + gI[mt][r] + lam * xi[mt][r];   // -r_{i-1}
                dl[mt][r] = cm * dl[mt][r] + ncs * nres;                             // delta_i
                xi[mt][r] += dl[mt][r];                                              // xi_i
            }
#pragma unroll
            for (int hh = 0; hh < HS; ++hh) Xn[mt][hh] = MMA::pack(&dl[mt][hh * VEC]);
        }
#pragma unroll
        for (int blk = 0; blk < NB; ++blk)
#pragma unroll
            for (int hh = 0; hh < HS; ++hh) X[blk][hh] = Xn[blk][hh];
    }

    GKA_TSTAMP(7);
    // ---------------- readout y_c = zeta_c U_[n] xhat_c + sum_{j<=c} M[j,c] v_j (k_j . xhat_c) ----------------
    constexpr int NSPL = MMA::kSplitReadout ? 2 : 1;
    const frag *Uw = (const frag *)a.ws_U + chunk_id * (NSPL * SH::H_FRAGS * 64);
    RowStage<MMA, IO, D> vrows;
    BlockCopy<H16> ucopy, ulocopy;
    vrows.load(a.v, base_bh, a.stride_t, tok0, a.T, tid);
    ucopy.load(Uw, tid);
    if (NSPL == 2) ulocopy.load(Uw + SH::H_FRAGS * 64, tid);
    GKA_TSTAMP(8);
    __syncthreads();                           // both waves are done with sH and sKT
    vrows.store(sRow, tok0, a.T, tid);
    __syncthreads();
    build_transposed_frags<MMA, D>(sKT, sRow, w, lane);
    __syncthreads();
    GKA_TSTAMP(9);
    ucopy.store(sH, tid);
    frag Xlo[NB][HS];
#pragma unroll
    for (int blk = 0; blk < NB; ++blk)
#pragma unroll
        for (int hh = 0; hh < HS; ++hh) {
            X[blk][hh] = MMA::pack(&xi[blk][hh * VEC]);
            if (NSPL == 2) {
                float lo[VEC];
#pragma unroll
                for (int p = 0; p < VEC; ++p) lo[p] = xi[blk][hh * VEC + p] - MMA::elem(X[blk][hh], p);
                Xlo[blk][hh] = MMA::pack(lo);
            }
        }
    pacc[0] = zero16();
    pacc[1] = zero16();
    gemm_p<MMA, NB>(sK, X, pacc, w, lane);
    if (NSPL == 2) gemm_p<MMA, NB>(sK, Xlo, pacc, w, lane);
    frag pm[2][HS];
    mask_p<MMA>(pacc, mreg, pm, w);
    __syncthreads();
    f32x16 acc[NB];
#pragma unroll
    for (int mt = 0; mt < NB; ++mt) {
        acc[mt] = gemm_state_mt<MMA, NB>(sH, mt, X, zero16(), lane);
        if (NSPL == 2) acc[mt] = gemm_state_mt<MMA, NB>(sH, mt, Xlo, acc[mt], lane);
    }
    if (NSPL == 2) {
        __syncthreads();
        ulocopy.store(sH, tid);
        __syncthreads();
#pragma unroll
        for (int mt = 0; mt < NB; ++mt) acc[mt] = gemm_state_mt<MMA, NB>(sH, mt, X, acc[mt], lane);
    }
#pragma unroll
    for (int mt = 0; mt < NB; ++mt) {
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[mt][r] *= zeta;
        acc[mt] = gemm_intra_mt<MMA>(sKT, mt, pm, acc[mt], w, lane);
    }
    GKA_TSTAMP(10);
    if (valid) {
#pragma unroll
        for (int mt = 0; mt < NB; ++mt)
#pragma unroll
            for (int i = 0; i < 4; ++i)
                IO::store4(a.o, tok_off + 32 * mt + 8 * i + 4 * g, acc[mt][4 * i], acc[mt][4 * i + 1],
                           acc[mt][4 * i + 2], acc[mt][4 * i + 3]);
    }
    GKA_TSTAMP(11);
}

#ifdef GKA_DEBUG_TIMERS
extern "C" int gka_debug_read_timers(unsigned long long *host)
{
    return (int)hipMemcpyFromSymbol(host, HIP_SYMBOL(g_dbg_timers), sizeof(g_dbg_timers));
}
#endif

template <class MMA, class IO, int D>
static hipError_t launch_chunk_solve_t(const SolveArgs &a, int n_pairs, hipStream_t stream)
{
    typedef SolveShape<MMA, D> SH;
    auto kern = chunk_solve_kernel<MMA, IO, D>;
    hipError_t e = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize,
                                       (int)SH::lds_bytes);
    if (e != hipSuccess) return e;
    dim3 grid((unsigned)(n_pairs * a.n_chunks_total)), block(128);
    hipLaunchKernelGGL(kern, grid, block, SH::lds_bytes, stream, a);
    return hipGetLastError();
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
