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

template <class MMA, int NB>
struct SolveShape {
    static constexpr int HS = MMA::HS;
    static constexpr int JB = kChunk / 32;
    static constexpr int H_FRAGS = NB * NB * HS;
    static constexpr int K_FRAGS = JB * NB * HS;
    static constexpr int KT_FRAGS = NB * JB * HS;
    static constexpr size_t lds_bytes =
        (size_t)(H_FRAGS + K_FRAGS + KT_FRAGS) * 64 * sizeof(typename MMA::frag) + 2 * kChunk * sizeof(float);
};

// acc[mt] += sum_{blk,h} A[mt][blk][h] * X[blk][h]      (A = H_[n] or U_[n] fragments in LDS)
template <class MMA, int NB>
__device__ __forceinline__ void gemm_state(const typename MMA::frag *sA, const typename MMA::frag (&X)[NB][MMA::HS],
                                           f32x16 (&acc)[NB], int lane)
{
#pragma unroll
    for (int mt = 0; mt < NB; ++mt)
#pragma unroll
        for (int blk = 0; blk < NB; ++blk)
#pragma unroll
            for (int hh = 0; hh < MMA::HS; ++hh)
                acc[mt] = MMA::mma(sA[((mt * NB + blk) * MMA::HS + hh) * 64 + lane], X[blk][hh], acc[mt]);
}

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

// acc[mt] += sum_{jt<=w,h} AT[mt][jt][h] * (pacc o mreg)[jt][h]     (AT = K^T or V^T fragments)
template <class MMA, int NB>
__device__ __forceinline__ void gemm_intra(const typename MMA::frag *sAT, const f32x16 (&pacc)[2],
                                           const f32x16 (&mreg)[2], f32x16 (&acc)[NB], int w, int lane)
{
    constexpr int VEC = MMA::VEC, HS = MMA::HS;
    typename MMA::frag pm[2][HS];
#pragma unroll
    for (int jt = 0; jt < 2; ++jt)
#pragma unroll
        for (int hh = 0; hh < HS; ++hh) {
            float t[VEC];
#pragma unroll
            for (int p = 0; p < VEC; ++p) t[p] = pacc[jt][hh * VEC + p] * mreg[jt][hh * VEC + p];
            pm[jt][hh] = MMA::pack(t);
        }
#pragma unroll
    for (int mt = 0; mt < NB; ++mt) {
#pragma unroll
        for (int hh = 0; hh < HS; ++hh)
            acc[mt] = MMA::mma(sAT[((mt * 2 + 0) * HS + hh) * 64 + lane], pm[0][hh], acc[mt]);
    }
    if (w == 1) {
#pragma unroll
        for (int mt = 0; mt < NB; ++mt) {
#pragma unroll
            for (int hh = 0; hh < HS; ++hh)
                acc[mt] = MMA::mma(sAT[((mt * 2 + 1) * HS + hh) * 64 + lane], pm[1][hh], acc[mt]);
        }
    }
}

// Copy n16 16-byte units from global to LDS with the whole workgroup.
__device__ __forceinline__ void copy_to_lds(void *dst, const void *src, int n16, int tid, int nthreads)
{
    const uint4 *s = (const uint4 *)src;
    uint4 *d = (uint4 *)dst;
    for (int i = tid; i < n16; i += nthreads) d[i] = s[i];
}

// Stage the transposed fragments AT[mt][jt][h]: row 32*mt + n of X^T, contraction index the chunk's
// tokens j = 32*jt + kidx(h*VEC + p, g).   X = K (for the iterations) or V (for the readout).
template <class MMA, class IO, int NB>
__device__ __forceinline__ void stage_transposed(typename MMA::frag *sAT, const void *x, int64_t base, int64_t stride_t,
                                                 int tok0, int T, int w, int lane)
{
    constexpr int VEC = MMA::VEC, HS = MMA::HS;
    const int n = lane & 31, g = lane >> 5;
    for (int f = w; f < NB * 2 * HS; f += 2) {
        const int hh = f % HS, jt = (f / HS) % 2, mt = f / (2 * HS);
        float t[VEC];
#pragma unroll
        for (int p = 0; p < VEC; ++p) {
            const int tok = tok0 + 32 * jt + kidx(hh * VEC + p, g);
            t[p] = (tok < T) ? IO::load(x, base + (int64_t)tok * stride_t + 32 * mt + n) : 0.0f;
        }
        sAT[f * 64 + lane] = MMA::pack(t);
    }
}

template <class MMA, class IO, int D>
__global__ __launch_bounds__(128) void chunk_solve_kernel(SolveArgs a)
{
    constexpr int NB = D / 32;
    constexpr int VEC = MMA::VEC, HS = MMA::HS;
    typedef typename MMA::frag frag;
    typedef SolveShape<MMA, NB> SH;

    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    frag *sH = (frag *)smem;
    frag *sK = sH + SH::H_FRAGS * 64;
    frag *sKT = sK + SH::K_FRAGS * 64;
    float *sG = (float *)(sKT + SH::KT_FRAGS * 64);
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

    // ---------------- staging ----------------
    if (w == 0) {
        const int t = tok0 + lane;
        float lg = (t < a.T) ? log_gate(a.gate[gate_base + (int64_t)t * a.H]) : 0.0f;
        sG[lane] = wave_inclusive_scan(lg, lane);
    }
    copy_to_lds(sH, (const frag *)a.ws_H + chunk_id * (SH::H_FRAGS * 64),
                (int)(SH::H_FRAGS * 64 * sizeof(frag) / 16), tid, 128);
    // K fragments: rows = tokens of block jt, contraction index = features
    for (int f = w; f < SH::K_FRAGS; f += 2) {
        const int hh = f % HS, blk = (f / HS) % NB, jt = f / (HS * NB);
        const int t = tok0 + 32 * jt + n;
        float x[VEC];
#pragma unroll
        for (int p = 0; p < VEC; ++p)
            x[p] = (t < a.T) ? IO::load(a.k, base_bh + (int64_t)t * a.stride_t + 32 * blk + kidx(hh * VEC + p, g)) : 0.0f;
        sK[f * 64 + lane] = MMA::pack(x);
    }
    stage_transposed<MMA, IO, NB>(sKT, a.k, base_bh, a.stride_t, tok0, a.T, w, lane);

    // q of this lane's token, rows kidx(r, g) of each 32-block
    float qf[NB][16];
#pragma unroll
    for (int blk = 0; blk < NB; ++blk)
#pragma unroll
        for (int r = 0; r < 16; ++r)
            qf[blk][r] = valid ? IO::load(a.q, base_bh + (int64_t)tok * a.stride_t + 32 * blk + kidx(r, g)) : 0.0f;
    const float lam = valid ? a.lambda[gate_base + (int64_t)tok * a.H] : 1.0f;
    float hn2 = 0.0f;
#pragma unroll
    for (int i = 0; i < NB * NB; ++i) hn2 += a.ws_hn[chunk_id * (NB * NB) + i];
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
    f32x16 acc[NB];
    f32x16 pacc[2];
    frag X[NB][HS];
    {
#pragma unroll
        for (int blk = 0; blk < NB; ++blk)
#pragma unroll
            for (int hh = 0; hh < HS; ++hh) X[blk][hh] = sK[((w * NB + blk) * HS + hh) * 64 + lane];
#pragma unroll
        for (int mt = 0; mt < NB; ++mt) acc[mt] = zero16();
        gemm_state<MMA, NB>(sH, X, acc, lane);
        float a_part = 0.0f;
#pragma unroll
        for (int mt = 0; mt < NB; ++mt)
#pragma unroll
            for (int r = 0; r < 16; ++r) a_part += acc[mt][r] * MMA::elem(X[mt][r / VEC], r % VEC);
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

    // ---------------- Chebyshev iteration (Algorithm 1), residual form ----------------
    const float L = fro + lam, mu = lam;       // Section 4.1: L = ||H_t||_F + lambda_t, mu = lambda_t
    const float s0 = 2.0f / (L + mu);
    const float rho = (L - mu) / (L + mu);
    const float rho2 = rho * rho;
    float xi[NB][16], dl[NB][16], rs[NB][16];
#pragma unroll
    for (int blk = 0; blk < NB; ++blk) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            xi[blk][r] = s0 * qf[blk][r];      // xi_0 = 2 q / (L + mu); delta_0 = xi_0 - xi_{-1} = xi_0
            dl[blk][r] = xi[blk][r];
            rs[blk][r] = qf[blk][r];           // becomes r_0 = q - (H + lambda) xi_0 in the first pass
        }
#pragma unroll
        for (int hh = 0; hh < HS; ++hh) X[blk][hh] = MMA::pack(&qf[blk][hh * VEC]);
    }
    float omega = 2.0f;
    float sc = s0;                             // first product is taken on q itself (exact operand), then scaled
    for (int it = 0; it < a.n_iter; ++it) {
#pragma unroll
        for (int mt = 0; mt < NB; ++mt) acc[mt] = zero16();
        gemm_state<MMA, NB>(sH, X, acc, lane);
#pragma unroll
        for (int mt = 0; mt < NB; ++mt)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[mt][r] *= zeta;
        pacc[0] = zero16();
        pacc[1] = zero16();
        gemm_p<MMA, NB>(sK, X, pacc, w, lane);
        gemm_intra<MMA, NB>(sKT, pacc, mreg, acc, w, lane);
        omega = 4.0f / (4.0f - rho2 * omega);                      // weight schedule
        const float cm = omega - 1.0f, cs = omega * s0;
#pragma unroll
        for (int blk = 0; blk < NB; ++blk) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                rs[blk][r] -= sc * acc[blk][r] + lam * dl[blk][r];  // r_{i-1}
                dl[blk][r] = cm * dl[blk][r] + cs * rs[blk][r];     // delta_i
                xi[blk][r] += dl[blk][r];                           // xi_i
            }
#pragma unroll
            for (int hh = 0; hh < HS; ++hh) X[blk][hh] = MMA::pack(&dl[blk][hh * VEC]);
        }
        sc = 1.0f;
    }

    // ---------------- readout y_c = zeta_c U_[n] xhat_c + sum_{j<=c} M[j,c] v_j (k_j . xhat_c) ----------------
    __syncthreads();                           // both waves are done with sH and sKT
    constexpr int NSPL = MMA::kSplitReadout ? 2 : 1;
    const frag *Uw = (const frag *)a.ws_U + chunk_id * (NSPL * SH::H_FRAGS * 64);
    copy_to_lds(sH, Uw, (int)(SH::H_FRAGS * 64 * sizeof(frag) / 16), tid, 128);
    stage_transposed<MMA, IO, NB>(sKT, a.v, base_bh, a.stride_t, tok0, a.T, w, lane);
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
    __syncthreads();
#pragma unroll
    for (int mt = 0; mt < NB; ++mt) acc[mt] = zero16();
    pacc[0] = zero16();
    pacc[1] = zero16();
    gemm_state<MMA, NB>(sH, X, acc, lane);
    gemm_p<MMA, NB>(sK, X, pacc, w, lane);
    if (NSPL == 2) {
        gemm_state<MMA, NB>(sH, Xlo, acc, lane);
        gemm_p<MMA, NB>(sK, Xlo, pacc, w, lane);
        __syncthreads();
        copy_to_lds(sH, Uw + SH::H_FRAGS * 64, (int)(SH::H_FRAGS * 64 * sizeof(frag) / 16), tid, 128);
        __syncthreads();
        gemm_state<MMA, NB>(sH, X, acc, lane);
    }
#pragma unroll
    for (int mt = 0; mt < NB; ++mt)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[mt][r] *= zeta;
    gemm_intra<MMA, NB>(sKT, pacc, mreg, acc, w, lane);
    if (valid) {
        const int64_t obase = base_bh + (int64_t)tok * a.stride_t;
#pragma unroll
        for (int mt = 0; mt < NB; ++mt)
#pragma unroll
            for (int i = 0; i < 4; ++i)
                IO::store4(a.o, obase + 32 * mt + 8 * i + 4 * g, acc[mt][4 * i], acc[mt][4 * i + 1],
                           acc[mt][4 * i + 2], acc[mt][4 * i + 3]);
    }
}

template <class MMA, class IO, int D>
static hipError_t launch_chunk_solve_t(const SolveArgs &a, int n_pairs, hipStream_t stream)
{
    typedef SolveShape<MMA, D / 32> SH;
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
