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
    // row-major staging tile of one chunk of k or v rows, padded against bank conflicts
    static constexpr int RS = D + 16 / (int)sizeof(elem_t);
    static constexpr size_t row_bytes = (size_t)kChunk * RS * sizeof(elem_t);
    static constexpr size_t h_bytes = (size_t)H_FRAGS * 64 * sizeof(frag);
    static constexpr size_t k_bytes = (size_t)K_FRAGS * 64 * sizeof(frag);
    static constexpr size_t kt_bytes = (size_t)KT_FRAGS * 64 * sizeof(frag);
    static constexpr size_t x_bytes = (size_t)X_FRAGS * 64 * sizeof(frag);
    static constexpr bool row_aliases_h = row_bytes <= h_bytes;   // staging tile reuses the state region
    static constexpr size_t misc_bytes = 4 * kChunk * sizeof(float);   // sG, sW, sA[2]; aliases the exchange region
    static_assert(misc_bytes <= x_bytes, "per-token scalars must fit the exchange region");
    static constexpr size_t lds_bytes = h_bytes + k_bytes + kt_bytes + x_bytes + (row_aliases_h ? 0 : row_bytes);
};

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

// pacc[jt] += sum_{blk,h} K[jt][blk][h] * X[blk][h] for the key blocks jt <= tw (causal)
template <class MMA, int NB>
__device__ __forceinline__ void gemm_p(const typename MMA::frag *sK, const typename MMA::frag (&X)[NB][MMA::HS],
                                       f32x16 (&pacc)[2], int tw, int lane)
{
#pragma unroll
    for (int blk = 0; blk < NB; ++blk)
#pragma unroll
        for (int hh = 0; hh < MMA::HS; ++hh)
            pacc[0] = MMA::mma(sK[((0 * NB + blk) * MMA::HS + hh) * 64 + lane], X[blk][hh], pacc[0]);
    if (tw == 1) {
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
                                       typename MMA::frag (&pm)[2][MMA::HS], int tw)
{
    constexpr int VEC = MMA::VEC, HS = MMA::HS;
#pragma unroll
    for (int hh = 0; hh < HS; ++hh) {
        float t[VEC];
#pragma unroll
        for (int p = 0; p < VEC; ++p) t[p] = pacc[0][hh * VEC + p] * mreg[0][hh * VEC + p];
        pm[0][hh] = MMA::pack(t);
    }
    if (tw == 1) {
#pragma unroll
        for (int hh = 0; hh < HS; ++hh) {
            float t[VEC];
#pragma unroll
            for (int p = 0; p < VEC; ++p) t[p] = pacc[1][hh * VEC + p] * mreg[1][hh * VEC + p];
            pm[1][hh] = MMA::pack(t);
        }
    }
}

// acc += sum_{jt<=tw,h} AT[mt][jt][h] * pm[jt][h]     (AT = K^T or V^T fragments)
template <class MMA>
__device__ __forceinline__ f32x16 gemm_intra_mt(const typename MMA::frag *sAT, int mt,
                                                const typename MMA::frag (&pm)[2][MMA::HS], f32x16 acc, int tw,
                                                int lane)
{
    constexpr int HS = MMA::HS;
#pragma unroll
    for (int hh = 0; hh < HS; ++hh) acc = MMA::mma(sAT[((mt * 2 + 0) * HS + hh) * 64 + lane], pm[0][hh], acc);
    if (tw == 1) {
#pragma unroll
        for (int hh = 0; hh < HS; ++hh) acc = MMA::mma(sAT[((mt * 2 + 1) * HS + hh) * 64 + lane], pm[1][hh], acc);
    }
    return acc;
}

// A block of N16 * kSolveThreads 16-byte units copied global -> registers -> LDS by the workgroup. The two
// halves are separate calls so that the global loads can be issued long before the LDS region is free.
template <int N16>
struct BlockCopy {
    uint4 r[N16];
    __device__ __forceinline__ void load(const void *src, int tid)
    {
        const uint4 *s = (const uint4 *)src;
#pragma unroll
        for (int i = 0; i < N16; ++i) r[i] = s[i * kSolveThreads + tid];
    }
    __device__ __forceinline__ void store(void *dst, int tid) const
    {
        uint4 *d = (uint4 *)dst;
#pragma unroll
        for (int i = 0; i < N16; ++i) d[i * kSolveThreads + tid] = r[i];
    }
};

// One chunk of rows of x (k or v): global -> registers (load), registers -> row-major LDS tile of operand
// elements (store).
template <class MMA, class IO, int D>
struct RowStage {
    static constexpr int RS = SolveShape<MMA, D>::RS;
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
    for (int f = w; f < SH::K_FRAGS; f += 4) {
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
    for (int f = w; f < SH::KT_FRAGS; f += 4) {
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

// The two waves of a token block swap the halves of an operand: each writes the fragments of its own row
// blocks, and after the barrier reads all of them. The second barrier frees the region for the next write.
template <class MMA, int NB>
__device__ __forceinline__ void exchange_operand(typename MMA::frag *sX, const typename MMA::frag (&own)[NB / 2][MMA::HS],
                                                 typename MMA::frag (&X)[NB][MMA::HS], int tw, int fh, int lane)
{
    constexpr int HS = MMA::HS, NBH = NB / 2;
#pragma unroll
    for (int i = 0; i < NBH; ++i)
#pragma unroll
        for (int hh = 0; hh < HS; ++hh) sX[((tw * NB + fh * NBH + i) * HS + hh) * 64 + lane] = own[i][hh];
    __syncthreads();
#pragma unroll
    for (int blk = 0; blk < NB; ++blk)
#pragma unroll
        for (int hh = 0; hh < HS; ++hh) X[blk][hh] = sX[((tw * NB + blk) * HS + hh) * 64 + lane];
    __syncthreads();
}

template <class MMA, class IO, int D>
__device__ __forceinline__ void chunk_solve_body(const SolveArgs &a)
{
    typedef SolveShape<MMA, D> SH;
    constexpr int NB = SH::NB, NBH = SH::NBH;
    constexpr int VEC = MMA::VEC, HS = MMA::HS;
    typedef typename MMA::frag frag;
    typedef typename MMA::elem_t elem_t;

    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    frag *sH = (frag *)smem;
    frag *sK = (frag *)(smem + SH::h_bytes);
    frag *sKT = (frag *)(smem + SH::h_bytes + SH::k_bytes);
    frag *sX = (frag *)(smem + SH::h_bytes + SH::k_bytes + SH::kt_bytes);
    elem_t *sRow = SH::row_aliases_h ? (elem_t *)smem : (elem_t *)(smem + SH::h_bytes + SH::k_bytes + SH::kt_bytes + SH::x_bytes);
    float *sG = (float *)sX;                   // per-token scalars live in the exchange region before the passes
    float *sW = sG + kChunk;
    float *sA = sW + kChunk;                   // [2][kChunk]

    const int tid = threadIdx.x;
    const int lane = tid & 63, w = tid >> 6;
    const int tw = w & 1, fh = w >> 1;
    const int mt0 = fh * NBH;
    const int n = lane & 31, g = lane >> 5;
    const int chunk = blockIdx.x % a.n_chunks_total;
    const int pair = blockIdx.x / a.n_chunks_total;
    const int b = (a.pair0 + pair) / a.H, h = (a.pair0 + pair) % a.H;
    const int64_t chunk_id = (int64_t)pair * a.n_chunks_total + chunk;    // workspace index within this launch
    const int64_t base_bh = (int64_t)b * a.stride_b + (int64_t)h * a.stride_h;
    const int64_t gate_base = (int64_t)b * a.T * a.H + h;
    const int tok0 = chunk * kChunk;
    const int c_local = 32 * tw + n;
    const int tok = tok0 + c_local;
    const bool valid = tok < a.T;

    // ---------------- staging ----------------
    constexpr int H16 = (int)(SH::h_bytes / 16 / kSolveThreads);   // 16-byte units of a state block per thread
    const int64_t tok_off = base_bh + (int64_t)min(tok, a.T - 1) * a.stride_t;
    float lam, hn2 = 0.0f;
    typename IO::raw4 qraw[NBH][4];            // q of this lane's token, rows of this wave's feature half
    {
        // every global read of the prologue is issued here, before the first wait
        RowStage<MMA, IO, D> krows;
        BlockCopy<H16> hcopy;
        krows.load(a.k, base_bh, a.stride_t, tok0, a.T, tid);
        hcopy.load((const frag *)a.ws_H + chunk_id * (SH::H_FRAGS * 64), tid);
#pragma unroll
        for (int i = 0; i < NBH; ++i)
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4)
                qraw[i][q4] = IO::load_raw4(a.q, tok_off + 32 * (mt0 + i) + 8 * q4 + 4 * g);
        lam = a.lambda[gate_base + (int64_t)min(tok, a.T - 1) * a.H];
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
        krows.store(sRow, tok0, a.T, tid);
        __syncthreads();
        build_row_frags<MMA, D>(sK, sRow, w, lane);
        build_transposed_frags<MMA, D>(sKT, sRow, w, lane);
        __syncthreads();                       // the staging tile may alias the state region
        hcopy.store(sH, tid);
    }
    __syncthreads();

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
            for (int hh = 0; hh < HS; ++hh) X[blk][hh] = sK[((tw * NB + blk) * HS + hh) * 64 + lane];
        // k_c^T H_[n] k_c: this wave's rows of H_[n] k_c, then summed over the two feature halves
        float a_part = 0.0f;
#pragma unroll
        for (int i = 0; i < NBH; ++i) {
            f32x16 acc = gemm_state_mt<MMA, NB>(sH, mt0 + i, X, zero16(), lane);
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                // same row of the same token: element (mt0 + i, r) of the B operand
                float kv = 0.0f;
#pragma unroll
                for (int blk = 0; blk < NB; ++blk)
                    if (blk == mt0 + i) kv = MMA::elem(X[blk][r / VEC], r % VEC);
                a_part += acc[r] * kv;
            }
        }
        a_part += __shfl_xor(a_part, 32, 64);
        if (g == 0) sA[fh * kChunk + c_local] = a_part;
        pacc[0] = zero16();
        pacc[1] = zero16();
        gemm_p<MMA, NB>(sK, X, pacc, tw, lane);
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
        b_part += __shfl_xor(b_part, 32, 64);
        d_part += __shfl_xor(d_part, 32, 64);
        __syncthreads();
        if (fh == 0 && g == 0)
            sW[c_local] = 2.0f * (zeta * (sA[c_local] + sA[kChunk + c_local]) + b_part) + d_part;
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
    if (a.fro_out && valid && fh == 0 && g == 0) a.fro_out[gate_base + (int64_t)tok * a.H] = fro;
    __syncthreads();                           // sG, sW, sA are dead: the region becomes the operand exchange

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
            const f32x4 qv4 = IO::cvt4(qraw[i][q4]);
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float qv = valid ? qv4[e] : 0.0f;
                gI[i][4 * q4 + e] = -qv;
                xi[i][4 * q4 + e] = s0 * qv;      // xi_0 = 2 q / (L + mu); delta_0 = xi_0 - xi_{-1} = xi_0
                dl[i][4 * q4 + e] = s0 * qv;
            }
        }
#pragma unroll
        for (int hh = 0; hh < HS; ++hh) own[i][hh] = MMA::pack(&dl[i][hh * VEC]);
    }
    float omega = 2.0f;
    for (int it = 0; it < a.n_iter; ++it) {
        // A operands are re-read from LDS in every pass (they are not kept in registers across passes)
        asm volatile("" ::: "memory");
        exchange_operand<MMA, NB>(sX, own, X, tw, fh, lane);
        pacc[0] = zero16();
        pacc[1] = zero16();
        gemm_p<MMA, NB>(sK, X, pacc, tw, lane);
        frag pm[2][HS];
        mask_p<MMA>(pacc, mreg, pm, tw);
        omega = 4.0f / (4.0f - rho2 * omega);                      // weight schedule
        const float cm = omega - 1.0f, ncs = -omega * s0;
#pragma unroll
        for (int i = 0; i < NBH; ++i) {
            gS[i] = gemm_state_mt<MMA, NB>(sH, mt0 + i, X, gS[i], lane);
            gI[i] = gemm_intra_mt<MMA>(sKT, mt0 + i, pm, gI[i], tw, lane);
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const float nres = zeta * gS[i][r] + gI[i][r] + lam * xi[i][r];   // -r_{i-1}
                dl[i][r] = cm * dl[i][r] + ncs * nres;                            // delta_i
                xi[i][r] += dl[i][r];                                             // xi_i
            }
#pragma unroll
            for (int hh = 0; hh < HS; ++hh) own[i][hh] = MMA::pack(&dl[i][hh * VEC]);
        }
    }

    // ---------------- readout y_c = zeta_c U_[n] xhat_c + sum_{j<=c} M[j,c] v_j (k_j . xhat_c) ----------------
    constexpr int NSPL = MMA::kSplitReadout ? 2 : 1;
    const frag *Uw = (const frag *)a.ws_U + chunk_id * (NSPL * SH::H_FRAGS * 64);
    RowStage<MMA, IO, D> vrows;
    BlockCopy<H16> ucopy, ulocopy;
    vrows.load(a.v, base_bh, a.stride_t, tok0, a.T, tid);
    ucopy.load(Uw, tid);
    if (NSPL == 2) ulocopy.load(Uw + SH::H_FRAGS * 64, tid);
    // xhat as B operand: hi part, and for the bf16 path the rounding remainder as a second operand
    frag Xlo[NB][HS];
    {
        frag ownlo[NBH][HS];
#pragma unroll
        for (int i = 0; i < NBH; ++i)
#pragma unroll
            for (int hh = 0; hh < HS; ++hh) {
                own[i][hh] = MMA::pack(&xi[i][hh * VEC]);
                if (NSPL == 2) {
                    float lo[VEC];
#pragma unroll
                    for (int p = 0; p < VEC; ++p) lo[p] = xi[i][hh * VEC + p] - MMA::elem(own[i][hh], p);
                    ownlo[i][hh] = MMA::pack(lo);
                }
            }
        exchange_operand<MMA, NB>(sX, own, X, tw, fh, lane);      // its first barrier also ends all use of sH, sKT
        if (NSPL == 2) exchange_operand<MMA, NB>(sX, ownlo, Xlo, tw, fh, lane);
    }
    vrows.store(sRow, tok0, a.T, tid);
    pacc[0] = zero16();
    pacc[1] = zero16();
    gemm_p<MMA, NB>(sK, X, pacc, tw, lane);
    if (NSPL == 2) gemm_p<MMA, NB>(sK, Xlo, pacc, tw, lane);
    frag pm[2][HS];
    mask_p<MMA>(pacc, mreg, pm, tw);
    __syncthreads();
    build_transposed_frags<MMA, D>(sKT, sRow, w, lane);
    __syncthreads();
    ucopy.store(sH, tid);
    __syncthreads();
    f32x16 acc[NBH];
#pragma unroll
    for (int i = 0; i < NBH; ++i) {
        acc[i] = gemm_state_mt<MMA, NB>(sH, mt0 + i, X, zero16(), lane);
        if (NSPL == 2) acc[i] = gemm_state_mt<MMA, NB>(sH, mt0 + i, Xlo, acc[i], lane);
    }
    if (NSPL == 2) {
        __syncthreads();
        ulocopy.store(sH, tid);
        __syncthreads();
#pragma unroll
        for (int i = 0; i < NBH; ++i) acc[i] = gemm_state_mt<MMA, NB>(sH, mt0 + i, X, acc[i], lane);
    }
#pragma unroll
    for (int i = 0; i < NBH; ++i) {
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][r] *= zeta;
        acc[i] = gemm_intra_mt<MMA>(sKT, mt0 + i, pm, acc[i], tw, lane);
    }
    if (valid) {
#pragma unroll
        for (int i = 0; i < NBH; ++i)
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4)
                IO::store4(a.o, tok_off + 32 * (mt0 + i) + 8 * q4 + 4 * g, acc[i][4 * q4], acc[i][4 * q4 + 1],
                           acc[i][4 * q4 + 2], acc[i][4 * q4 + 3]);
    }
}

// bf16 path: capped at 256 registers so that two workgroups (two waves per SIMD) share a CU.
template <class IO, int D>
__global__ __launch_bounds__(kSolveThreads) __attribute__((amdgpu_waves_per_eu(2, 2))) void chunk_solve_kernel_bf16(
    SolveArgs a)
{
    chunk_solve_body<MmaBF16, IO, D>(a);
}

// fp32 path: its fragments are twice as large, one workgroup per CU.
template <class IO, int D>
__global__ __launch_bounds__(kSolveThreads) void chunk_solve_kernel_f32(SolveArgs a)
{
    chunk_solve_body<MmaF32, IO, D>(a);
}

template <class MMA, class IO, int D>
struct SolveKernel;
template <class IO, int D>
struct SolveKernel<MmaBF16, IO, D> {
    static constexpr auto fn = chunk_solve_kernel_bf16<IO, D>;
};
template <class IO, int D>
struct SolveKernel<MmaF32, IO, D> {
    static constexpr auto fn = chunk_solve_kernel_f32<IO, D>;
};

template <class MMA, class IO, int D>
static hipError_t launch_chunk_solve_t(const SolveArgs &a, int n_pairs, hipStream_t stream)
{
    typedef SolveShape<MMA, D> SH;
    auto kern = SolveKernel<MMA, IO, D>::fn;
    hipError_t e = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize,
                                       (int)SH::lds_bytes);
    if (e != hipSuccess) return e;
    dim3 grid((unsigned)(n_pairs * a.n_chunks_total)), block(kSolveThreads);
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
