// Chunk initial states of Section 4.2.1: H_[n], U_[n] for every chunk of every (batch, head) pair.
//
// One workgroup owns a 32-wide slab of both states of one pair: H0[32*rb .. +32][:] and
// U0[32*rb .. +32][:], held as fp32 MFMA accumulators (wave w owns columns 32*w .. +32 of the slab),
// and walks the pair's chunks in order. Per chunk it
//   1. writes the slab, as it stands before the chunk, to the workspace in the fragment order the
//      solve kernel consumes (plus the slab's contribution to ||H_[n]||_F^2),
//   2. applies the chunk: S <- zeta_C S + sum_j (zeta_C / zeta_j) a_j k_j^T  (a = k for H, a = v for U),
//      the decay weights built in log space (Appendix B.2), as one MFMA contraction over the
//      chunk's tokens.
// The final slab is written to H_final / U_final in row-major fp32 when requested.
#include "gka_device.hpp"
#include "gka_kernels.hpp"

namespace gka {

template <class MMA, class IO, int D>
__global__ __launch_bounds__(D * 2) void state_pass_kernel(StatePassArgs a)
{
    constexpr int NB = D / 32;
    constexpr int VEC = MMA::VEC;
    constexpr int HS = MMA::HS;
    constexpr int STEPS = kChunk / (2 * VEC);     // MFMA steps over the chunk's tokens
    typedef typename MMA::frag frag;

    const int lane = threadIdx.x & 63;
    const int w = threadIdx.x >> 6;               // column block of the slab owned by this wave
    const int n = lane & 31, g = lane >> 5;
    const int rb = blockIdx.x % NB;               // slab index (row block of H0 / U0)
    const int pair = blockIdx.x / NB;
    const int b = pair / a.H, h = pair % a.H;

    __shared__ float s_wd[kChunk];                // zeta_C / zeta_j of the current chunk

    const int64_t base_bh = (int64_t)b * a.stride_b + (int64_t)h * a.stride_h;
    const int64_t gate_base = (int64_t)b * a.T * a.H + h;

    // accumulators: element (row = 32*w + kidx(r,g), col n) = S0[32*rb + n][32*w + kidx(r,g)]
    f32x16 accH = zero16(), accU = zero16();
    if (a.H_init) {
        const float *Hi = a.H_init + (int64_t)pair * D * D;
        const float *Ui = a.U_init + (int64_t)pair * D * D;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            int col = 32 * w + kidx(r, g);
            accH[r] = Hi[(int64_t)(32 * rb + n) * D + col];
            accU[r] = Ui[(int64_t)(32 * rb + n) * D + col];
        }
    }

    for (int c = 0; c < a.n_chunks; ++c) {
        // ---- gates of the chunk: G_j = sum_{i<=j} log gamma_i, weights exp(G_C - G_j)
        const int tok = c * kChunk + lane;
        float lg = 0.0f;
        if (tok < a.T) lg = log_gate(a.gate[gate_base + (int64_t)tok * a.H]);
        float G = wave_inclusive_scan(lg, lane);
        float Gtot = __shfl(G, 63, 64);
        __syncthreads();                          // previous chunk's readers of s_wd are done
        if (w == 0) s_wd[lane] = expf(Gtot - G);
        const float zetaC = expf(Gtot);

        // ---- write the state before the chunk, fragment order
        const int64_t chunk_id = (int64_t)pair * a.n_chunks_total + (a.chunk0 + c);
        {
            frag *Hw = (frag *)a.ws_H + chunk_id * (NB * NB * HS * 64);
            float vals[16];
            float ss = 0.0f;
#pragma unroll
            for (int r = 0; r < 16; ++r) { vals[r] = accH[r]; ss += accH[r] * accH[r]; }
#pragma unroll
            for (int hh = 0; hh < HS; ++hh)
                Hw[((rb * NB + w) * HS + hh) * 64 + lane] = MMA::pack(vals + hh * VEC);
            ss = wave_sum(ss);
            if (lane == 0) a.ws_hn[chunk_id * (NB * NB) + rb * NB + w] = ss;

            constexpr int NSPL = MMA::kSplitReadout ? 2 : 1;
            frag *Uw = (frag *)a.ws_U + chunk_id * (NSPL * NB * NB * HS * 64);
            float lo[16];
#pragma unroll
            for (int r = 0; r < 16; ++r) vals[r] = accU[r];
#pragma unroll
            for (int hh = 0; hh < HS; ++hh) {
                frag f = MMA::pack(vals + hh * VEC);
                Uw[((rb * NB + w) * HS + hh) * 64 + lane] = f;
                if (NSPL == 2) {
#pragma unroll
                    for (int p = 0; p < VEC; ++p) lo[hh * VEC + p] = vals[hh * VEC + p] - MMA::elem(f, p);
                }
            }
            if (NSPL == 2) {
#pragma unroll
                for (int hh = 0; hh < HS; ++hh)
                    Uw[(NB * NB * HS + (rb * NB + w) * HS + hh) * 64 + lane] = MMA::pack(lo + hh * VEC);
            }
        }
        __syncthreads();                          // s_wd visible

        // ---- S <- zeta_C S + sum_j w_j a_j k_j^T
#pragma unroll
        for (int r = 0; r < 16; ++r) { accH[r] *= zetaC; accU[r] *= zetaC; }
#pragma unroll
        for (int s = 0; s < STEPS; ++s) {
            float ka[VEC], kb[VEC], vb[VEC];
#pragma unroll
            for (int p = 0; p < VEC; ++p) {
                const int j = s * 2 * VEC + g * VEC + p;
                const int t = c * kChunk + j;
                float kA = 0.0f, kB = 0.0f, vB = 0.0f;
                if (t < a.T) {
                    const int64_t off = base_bh + (int64_t)t * a.stride_t;
                    kA = IO::load(a.k, off + 32 * w + n);
                    kB = IO::load(a.k, off + 32 * rb + n);
                    vB = IO::load(a.v, off + 32 * rb + n);
                }
                ka[p] = kA * s_wd[j];
                kb[p] = kB;
                vb[p] = vB;
            }
            frag fa = MMA::pack(ka);
            accH = MMA::mma(fa, MMA::pack(kb), accH);
            accU = MMA::mma(fa, MMA::pack(vb), accU);
        }
    }

    if (a.H_final) {
        float *Hf = a.H_final + (int64_t)pair * D * D;
        float *Uf = a.U_final + (int64_t)pair * D * D;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            int col = 32 * w + kidx(r, g);
            Hf[(int64_t)(32 * rb + n) * D + col] = accH[r];
            Uf[(int64_t)(32 * rb + n) * D + col] = accU[r];
        }
    }
}

template <class MMA, class IO, int D>
static hipError_t launch_state_pass_t(const StatePassArgs &a, int n_pairs, hipStream_t stream)
{
    constexpr int NB = D / 32;
    dim3 grid(n_pairs * NB), block(D * 2);
    hipLaunchKernelGGL((state_pass_kernel<MMA, IO, D>), grid, block, 0, stream, a);
    return hipGetLastError();
}

hipError_t launch_state_pass(const StatePassArgs &a, int n_pairs, int d, bool io_bf16, bool compute_bf16,
                             hipStream_t stream)
{
    if (compute_bf16) {
        if (d == 128) return launch_state_pass_t<MmaBF16, IOBF16, 128>(a, n_pairs, stream);
        return launch_state_pass_t<MmaBF16, IOBF16, 64>(a, n_pairs, stream);
    }
    if (io_bf16) {
        if (d == 128) return launch_state_pass_t<MmaF32, IOBF16, 128>(a, n_pairs, stream);
        return launch_state_pass_t<MmaF32, IOBF16, 64>(a, n_pairs, stream);
    }
    if (d == 128) return launch_state_pass_t<MmaF32, IOF32, 128>(a, n_pairs, stream);
    return launch_state_pass_t<MmaF32, IOF32, 64>(a, n_pairs, stream);
}

}  // namespace gka
