// Recurrent steps of Eq. (CH) per (sequence, head) pair: state update (with the optional write gate), ||H_t||_F,
// Algorithm 1 with the matrix held in registers, readout (with the optional alpha-connection). One workgroup of 256
// threads per pair; all arithmetic fp32. The states are read once, advanced by a.T tokens in registers and written
// once, so the state traffic of a call does not grow with the number of tokens.
//
// The d x d states are distributed as float4 pieces in flat row-major order, piece (it*256 + t) on thread
// t, so that state reads and writes are fully coalesced: thread t holds, for each of its ITS pieces, row
// i = it*RPI + t / C4 and columns 4*(t % C4) .. +3 (C4 = d/4 pieces per row, RPI = 256/C4 rows per sweep).
// H is symmetric, so H x is evaluated column-wise, (H x)_j = sum_i H[i][j] x_i: every thread accumulates
// its rows into its four columns, and the 256/C4 partial sums per column are combined through LDS.
#include "gka_device.hpp"
#include "gka_kernels.hpp"

namespace gka {

// MULTI = false: the single-step kernel, a.T == 1 known at compile time.
// LOWER: of H_state only the 32 x 32 blocks on and below the block diagonal are read and written; the blocks above
// are rebuilt in registers from their mirror images (through LDS, once per call), so the arithmetic is the same.
template <class IO, int D, bool MULTI, bool LOWER>
__global__ __launch_bounds__(256) void decode_step_kernel(DecodeArgs a)
{
    const int T = MULTI ? a.T : 1;
    constexpr int C4 = D / 4;
    constexpr int RPI = 256 / C4;
    constexpr int ITS = D / RPI;
    const int t = threadIdx.x;
    const int pair = blockIdx.x;
    const int col4 = t % C4, rgrp = t / C4;

    __shared__ float s_q[D], s_k[D], s_v[D];
    __shared__ float s_x[D];                 // operand of the current product (delta_i or xhat)
    __shared__ float s_part[RPI][D];         // per row-group partial column sums
    __shared__ float s_red[4];

    float *Hs = a.H_state + (int64_t)pair * D * D;
    float *Us = a.U_state + (int64_t)pair * D * D;
    const int b = pair / a.H, h = pair - b * a.H;
    f32x4 hreg[ITS], ureg[ITS];
    // piece `it` of this thread lies in block row (it * RPI) / 32 (RPI divides 32) and block column bj
    const int bj = col4 / 8;
    auto held = [&](int it) { return !LOWER || bj <= (it * RPI) / 32; };
#pragma unroll
    for (int it = 0; it < ITS; ++it) {
        if (held(it)) hreg[it] = __builtin_nontemporal_load((const f32x4 *)(Hs + (int64_t)(it * 256 + t) * 4));
        ureg[it] = __builtin_nontemporal_load((const f32x4 *)(Us + (int64_t)(it * 256 + t) * 4));
    }
    if constexpr (LOWER) {
        constexpr int NBLK = D / 32, NOFF = NBLK * (NBLK - 1) / 2;
        __shared__ float s_tr[NOFF][32][33];         // the blocks below the diagonal, block (bi, bj) at bi (bi - 1) / 2 + bj
#pragma unroll
        for (int it = 0; it < ITS; ++it) {
            const int bi = (it * RPI) / 32, row = it * RPI + rgrp;
            if (bj < bi) {
#pragma unroll
                for (int e = 0; e < 4; ++e) s_tr[bi * (bi - 1) / 2 + bj][row % 32][(4 * col4) % 32 + e] = hreg[it][e];
            }
        }
        __syncthreads();
#pragma unroll
        for (int it = 0; it < ITS; ++it) {
            const int bi = (it * RPI) / 32, row = it * RPI + rgrp;
            if (bj > bi) {
#pragma unroll
                for (int e = 0; e < 4; ++e) hreg[it][e] = s_tr[bj * (bj - 1) / 2 + bi][(4 * col4 + e) % 32][row % 32];
            }
        }
    }
    for (int tok = 0; tok < T; ++tok) {
        const int64_t bth = ((int64_t)b * T + tok) * a.H + h;      // [B,T,H] index of this token
        if (t < D) {
            s_q[t] = IO::load(a.q, bth * D + t);
            s_k[t] = IO::load(a.k, bth * D + t);
            s_v[t] = IO::load(a.v, bth * D + t);
        }
        const float gamma = a.gate[bth];
        const float beta = a.beta ? a.beta[bth] : 1.0f;        // write gate (Remark in Section 4.1)
        const float alpha = a.alpha ? a.alpha[bth] : 1.0f;     // alpha-connection (Section 4.3)
        __syncthreads();

        // ---- state update (Eq. (CH)) and ||H_t||_F^2
        float kc[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) kc[e] = s_k[4 * col4 + e];
        float ss = 0.0f;
#pragma unroll
        for (int it = 0; it < ITS; ++it) {
            const int row = it * RPI + rgrp;
            const float kr = s_k[row], vr = beta * s_v[row];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                // beta (k_i k_j): the product of the two k components first, so that both mirror images of an
                // element get the same bits
                hreg[it][e] = gamma * hreg[it][e] + beta * (kr * kc[e]);
                ureg[it][e] = gamma * ureg[it][e] + vr * kc[e];
                ss += hreg[it][e] * hreg[it][e];
            }
            if (tok == T - 1) {              // the stores drain while the last token is solved
                if (held(it)) __builtin_nontemporal_store(hreg[it], (f32x4 *)(Hs + (int64_t)(it * 256 + t) * 4));
                __builtin_nontemporal_store(ureg[it], (f32x4 *)(Us + (int64_t)(it * 256 + t) * 4));
            }
        }
        ss = wave_sum(ss);
        if ((t & 63) == 0) s_red[t >> 6] = ss;
        __syncthreads();
        const float fro = sqrtf(s_red[0] + s_red[1] + s_red[2] + s_red[3]);
        const float lam = a.lambda ? a.lambda[bth] : a.lambda_scale * fro;   // Section 4.1: lambda_t = a ||H_t||_F

        // ---- Algorithm 1 in residual form; thread j < D owns component j of xi, delta, r
        const float L = fro + lam, mu = lam;
        const float s0 = 2.0f / (L + mu);
        const float rho = (L - mu) / (L + mu);
        const float rho2 = rho * rho;
        float xi = 0.0f, dl = 0.0f, rs = 0.0f;
        if (t < D) {
            xi = s0 * s_q[t];
            dl = xi;
            rs = s_q[t];
            s_x[t] = dl;
        }
        float omega = 2.0f;
        __syncthreads();
        for (int i = 0; i < a.n_iter; ++i) {
            float p[4] = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
            for (int it = 0; it < ITS; ++it) {
                const float xr = s_x[it * RPI + rgrp];
#pragma unroll
                for (int e = 0; e < 4; ++e) p[e] += hreg[it][e] * xr;
            }
            *(f32x4 *)&s_part[rgrp][4 * col4] = f32x4{p[0], p[1], p[2], p[3]};
            __syncthreads();
            omega = 4.0f / (4.0f - rho2 * omega);
            if (t < D) {
                float hx = 0.0f;
#pragma unroll
                for (int rg = 0; rg < RPI; ++rg) hx += s_part[rg][t];
                rs -= hx + lam * dl;
                dl = (omega - 1.0f) * dl + omega * s0 * rs;
                xi += dl;
                s_x[t] = dl;
            }
            __syncthreads();
        }

        // ---- readout y = U (alpha xhat + (1 - alpha) q) (rows of U are not symmetric: reduce each row over its
        // C4 lanes)
        if (t < D) s_x[t] = alpha * xi + (1.0f - alpha) * s_q[t];
        __syncthreads();
        float xc[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) xc[e] = s_x[4 * col4 + e];
#pragma unroll
        for (int it = 0; it < ITS; ++it) {
            float y = ureg[it][0] * xc[0] + ureg[it][1] * xc[1] + ureg[it][2] * xc[2] + ureg[it][3] * xc[3];
#pragma unroll
            for (int off = C4 / 2; off > 0; off >>= 1) y += __shfl_xor(y, off, 64);
            if (col4 == 0) IO::store1(a.o, bth * D + it * RPI + rgrp, y);
        }
        // the next token overwrites s_q, s_k, s_v and (two barriers later) s_x: every thread must be done with xc
        __syncthreads();
    }
}

template <bool MULTI, bool LOWER>
static void launch_decode(const DecodeArgs &a, int n_pairs, int d, bool io_bf16, hipStream_t stream)
{
    dim3 grid((unsigned)n_pairs), block(256);
    if (io_bf16) {
        if (d == 128) hipLaunchKernelGGL((decode_step_kernel<IOBF16, 128, MULTI, LOWER>), grid, block, 0, stream, a);
        else hipLaunchKernelGGL((decode_step_kernel<IOBF16, 64, MULTI, LOWER>), grid, block, 0, stream, a);
    } else {
        if (d == 128) hipLaunchKernelGGL((decode_step_kernel<IOF32, 128, MULTI, LOWER>), grid, block, 0, stream, a);
        else hipLaunchKernelGGL((decode_step_kernel<IOF32, 64, MULTI, LOWER>), grid, block, 0, stream, a);
    }
}

hipError_t launch_decode_step(const DecodeArgs &a, int n_pairs, int d, bool io_bf16, hipStream_t stream)
{
    if (a.h_lower_blocks) {
        if (a.T == 1) launch_decode<false, true>(a, n_pairs, d, io_bf16, stream);
        else launch_decode<true, true>(a, n_pairs, d, io_bf16, stream);
    } else {
        if (a.T == 1) launch_decode<false, false>(a, n_pairs, d, io_bf16, stream);
        else launch_decode<true, false>(a, n_pairs, d, io_bf16, stream);
    }
    return hipGetLastError();
}

}  // namespace gka
