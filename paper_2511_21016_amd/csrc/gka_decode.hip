// Recurrent steps of Eq. (CH) per (sequence, head) pair: state update (with the optional write gate), ||H_t||_F,
// Algorithm 1 with the matrix held in registers, readout (with the optional alpha-connection). One workgroup per pair;
// all arithmetic fp32. The states are read once, advanced by a.T tokens in registers and written once, so the state
// traffic of a call does not grow with the number of tokens. The same kernel is gka_forward's recurrent path (any
// number of tokens, separate initial and final states, ||H_t||_F and the solve's result as optional outputs), the
// only one for the head dimension 256 and for float32 tensors at 16 and 32.
//
// The d x d states are distributed as float4 pieces in flat row-major order, piece (it*NTHR + t) on thread
// t, so that state reads and writes are fully coalesced: thread t holds, for each of its ITS pieces, row
// i = it*RPI + t / C4 and columns 4*(t % C4) .. +3 (C4 = d/4 pieces per row, RPI = NTHR/C4 rows per sweep).
// H is symmetric, so H x is evaluated column-wise, (H x)_j = sum_i H[i][j] x_i: every thread accumulates
// its rows into its four columns, and the NTHR/C4 partial sums per column are combined through LDS.
// NTHR = 256 threads (d = 16 has a kernel of its own below); 1024 for d = 256, where a thread holds 16 pieces of H and U does
// not fit beside them: U is then streamed, each piece read, advanced, used for the readout and written back
// once per token (STREAM_U).
#include "gka_device.hpp"
#include "gka_kernels.hpp"

namespace gka {

template <int D>
struct DecodeShape {
    static constexpr int NTHR = D == 256 ? 1024 : 256;
    static constexpr int C4 = D / 4, RPI = NTHR / C4, ITS = D / RPI, NW = NTHR / 64;
    static constexpr bool STREAM_U = D == 256;
    static_assert(ITS * NTHR * 4 == D * D && ITS >= 1 && RPI * C4 == NTHR, "every thread holds ITS pieces of a state");
};

// MULTI = false: the single-step kernel, a.T == 1 known at compile time.
// LOWER: of H_in / H_state only the 32 x 32 blocks on and below the block diagonal are read and written; the blocks
// above are rebuilt in registers from their mirror images (through LDS, once per call), so the arithmetic is the same.
// STREAM: U is streamed (as always at d = 256) although it would fit: the single-token kernel at d = 128, which
// then has room for a fourth workgroup per CU.
template <class IO, int D, bool MULTI, bool LOWER, bool STREAM = false>
__global__ __launch_bounds__(DecodeShape<D>::NTHR) void decode_step_kernel(DecodeArgs a)
{
    typedef DecodeShape<D> SH;
    const int T = MULTI ? a.T : 1;
    constexpr int NTHR = SH::NTHR, C4 = SH::C4, RPI = SH::RPI, ITS = SH::ITS, NW = SH::NW;
    constexpr bool STREAM_U = SH::STREAM_U || STREAM;
    static_assert(!STREAM || !MULTI, "U is streamed once per token: at d < 256 only where a call is one token");
    const int t = threadIdx.x;
    const int pair = blockIdx.x;
    const int col4 = t % C4, rgrp = t / C4;

    __shared__ float s_q[D], s_k[D], s_v[D];
    __shared__ float s_x[D];                 // operand of the current product (delta_i or xhat)
    __shared__ float s_part[RPI][D];         // per row-group partial column sums
    __shared__ float s_red[NW];

    const int64_t state_off = (int64_t)pair * D * D;
    const float *Hin = a.H_in ? a.H_in + state_off : nullptr;      // nullptr: zero initial states
    const float *Uin = a.U_in ? a.U_in + state_off : nullptr;
    float *Hs = a.H_state ? a.H_state + state_off : nullptr;       // nullptr: the final states are not wanted
    float *Us = a.U_state ? a.U_state + state_off : nullptr;
    const int b = pair / a.H, h = pair - b * a.H;
    f32x4 hreg[ITS], ureg[STREAM_U ? 1 : ITS];
    // piece `it` of this thread lies in block row (it * RPI) / 32 (RPI divides 32) and block column bj
    const int bj = col4 / 8;
    auto held = [&](int it) { return !LOWER || bj <= (it * RPI) / 32; };
#pragma unroll
    for (int it = 0; it < ITS; ++it) {
        hreg[it] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
        if (Hin && held(it)) hreg[it] = __builtin_nontemporal_load((const f32x4 *)(Hin + (int64_t)(it * NTHR + t) * 4));
        if constexpr (!STREAM_U) {
            ureg[it] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
            if (Uin) ureg[it] = __builtin_nontemporal_load((const f32x4 *)(Uin + (int64_t)(it * NTHR + t) * 4));
        }
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
    // H is written in full where the caller of the forward pass wants the final state (valid under either layout)
    auto stored = [&](int it) { return held(it) || a.h_out_full; };
    for (int tok = 0; tok < T; ++tok) {
        const int64_t bth = ((int64_t)b * T + tok) * a.H + h;      // [B,T,H] index of this token
        // d = 256: addresses of the state pieces are recomputed per token (hoisted out of the loop they would take
        // registers that H needs)
        int tv = t;
        if constexpr (STREAM_U) asm volatile("" : "+v"(tv));
        const int64_t row0 = b * a.stride_b + tok * a.stride_t + h * a.stride_h;   // its row of q, k, v, o
        if (t < D) {
            s_q[t] = IO::load(a.q, row0 + t);
            s_k[t] = IO::load(a.k, row0 + t);
            s_v[t] = IO::load(a.v, row0 + t);
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
                // (the multiply-add written out: held or streamed, U gets the same bits)
                if constexpr (!STREAM_U) ureg[it][e] = __builtin_fmaf(gamma, ureg[it][e], vr * kc[e]);
                ss += hreg[it][e] * hreg[it][e];
            }
            if (tok == T - 1) {              // the stores drain while the last token is solved
                if (Hs && stored(it)) __builtin_nontemporal_store(hreg[it], (f32x4 *)(Hs + (int64_t)(it * NTHR + tv) * 4));
                if constexpr (!STREAM_U) {
                    if (Us) __builtin_nontemporal_store(ureg[it], (f32x4 *)(Us + (int64_t)(it * NTHR + t) * 4));
                }
            }
        }
        ss = wave_sum(ss);
        if ((t & 63) == 0) s_red[t >> 6] = ss;
        __syncthreads();
        float fro2 = 0.0f;
#pragma unroll
        for (int w = 0; w < NW; ++w) fro2 += s_red[w];
        const float fro = sqrtf(fro2);
        const float lam = a.lambda ? a.lambda[bth] : a.lambda_scale * fro;   // Section 4.1: lambda_t = a ||H_t||_F
        if (a.fro_out && t == 0) a.fro_out[bth] = fro;

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
        if (t < D) {
            s_x[t] = alpha * xi + (1.0f - alpha) * s_q[t];
            if (a.xhat_out) a.xhat_out[bth * D + t] = xi;
        }
        __syncthreads();
        float xc[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) xc[e] = s_x[4 * col4 + e];
        // (streamed U: four pieces in flight at d = 256, where all sixteen would not fit beside H; eight at d = 128)
        constexpr int kReadoutUnroll = SH::STREAM_U ? 4 : STREAM ? 8 : ITS;
#pragma unroll kReadoutUnroll
        for (int it = 0; it < ITS; ++it) {
            f32x4 u;
            if constexpr (STREAM_U) {
                // this thread's piece of U: from the caller's initial state at the first token, afterwards what this
                // same thread stored at the previous token
                const int64_t at = (int64_t)(it * NTHR + tv) * 4;
                u = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
                if constexpr (MULTI) {
                    if (tok > 0) u = *(const f32x4 *)(Us + at);
                    else if (Uin) u = *(const f32x4 *)(Uin + at);
                } else {
                    if (Uin) u = __builtin_nontemporal_load((const f32x4 *)(Uin + at));
                }
                const float vr = beta * s_v[it * RPI + rgrp];
#pragma unroll
                for (int e = 0; e < 4; ++e) u[e] = __builtin_fmaf(gamma, u[e], vr * kc[e]);
                if constexpr (MULTI) *(f32x4 *)(Us + at) = u;
                else __builtin_nontemporal_store(u, (f32x4 *)(Us + at));
            } else {
                u = ureg[it];
            }
            float y = u[0] * xc[0] + u[1] * xc[1] + u[2] * xc[2] + u[3] * xc[3];
#pragma unroll
            for (int off = C4 / 2; off > 0; off >>= 1) y += __shfl_xor(y, off, 64);
            if (col4 == 0) IO::store1(a.o, row0 + it * RPI + rgrp, y);
        }
        // the next token overwrites s_q, s_k, s_v and (two barriers later) s_x: every thread must be done with xc
        __syncthreads();
    }
}

// Head dimension 16 (the vision models of Appendix L: many pairs, short sequences): one wave per pair and no LDS. A
// state is 64 float4 pieces, lane l holds columns 4 (l % 4) .. + 3 of row l / 4 of H and of U; per-component
// quantities of the solve (xi, delta, residual) live in the four lanes of the component's row. A product H x is taken
// row-wise: the lane's four elements times the four components of x it needs (fetched from the lanes that hold them by
// lane shuffles), then a sum over the four lanes of the row. Four pairs share a workgroup only to fill it; the waves
// never synchronise. The arithmetic is that of decode_step_kernel in another order of summation.
template <class IO>
__global__ __launch_bounds__(256) void decode_step_kernel_d16(DecodeArgs a, int n_pairs)
{
    constexpr int D = 16;
    const int lane = threadIdx.x & 63;
    const int pair = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (pair >= n_pairs) return;                 // (wave-uniform)
    const int r = lane >> 2, c4 = lane & 3;
    const int T = a.T;
    const int64_t state_off = (int64_t)pair * D * D + lane * 4;
    const int b = pair / a.H, h = pair - b * a.H;
    f32x4 hreg = {0.0f, 0.0f, 0.0f, 0.0f}, ureg = {0.0f, 0.0f, 0.0f, 0.0f};
    if (a.H_in) hreg = *(const f32x4 *)(a.H_in + state_off);
    if (a.U_in) ureg = *(const f32x4 *)(a.U_in + state_off);
    // the components 4 c4 .. 4 c4 + 3 of a vector whose component i is held by the lanes of row i
    auto my_columns = [&](float x, float (&out)[4]) {
#pragma unroll
        for (int e = 0; e < 4; ++e) out[e] = __shfl(x, (4 * c4 + e) * 4, 64);
    };
    // sum over the four lanes of a row (a quad): two cross-lane moves within quads
    auto row_sum = [&](float x) {
        x += __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, x), 0xB1, 0xF, 0xF, true));   // quad_perm [1,0,3,2]
        x += __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, x), 0x4E, 0xF, 0xF, true));   // quad_perm [2,3,0,1]
        return x;
    };
    // inputs of a token are fetched while the token before it is solved
    struct TokenIn { float q, k, v, gamma, beta, alpha, lam; };
    auto fetch = [&](int tok) {
        const int64_t bth = ((int64_t)b * T + tok) * a.H + h;
        const int64_t row0 = b * a.stride_b + tok * a.stride_t + h * a.stride_h;
        TokenIn t;
        t.q = IO::load(a.q, row0 + r);
        t.k = IO::load(a.k, row0 + r);
        t.v = IO::load(a.v, row0 + r);
        t.gamma = a.gate[bth];
        t.beta = a.beta ? a.beta[bth] : 1.0f;
        t.alpha = a.alpha ? a.alpha[bth] : 1.0f;
        t.lam = a.lambda ? a.lambda[bth] : 0.0f;
        return t;
    };
    TokenIn next = fetch(0);
    for (int tok = 0; tok < T; ++tok) {
        const int64_t bth = ((int64_t)b * T + tok) * a.H + h;
        const int64_t row0 = b * a.stride_b + tok * a.stride_t + h * a.stride_h;
        const TokenIn in = next;
        next = fetch(min(tok + 1, T - 1));
        const float qr = in.q, kr = in.k, vr = in.v, gamma = in.gamma, beta = in.beta, alpha = in.alpha;
        float kc[4];
        my_columns(kr, kc);
        // ---- state update (Eq. (CH)) and ||H_t||_F
        float ss = 0.0f;
        const float bv = beta * vr;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            hreg[e] = gamma * hreg[e] + beta * (kr * kc[e]);
            ureg[e] = gamma * ureg[e] + bv * kc[e];
            ss += hreg[e] * hreg[e];
        }
        const float fro = sqrtf(wave_sum(ss));
        const float lam = a.lambda ? in.lam : a.lambda_scale * fro;          // Section 4.1: lambda_t = a ||H_t||_F
        if (a.fro_out && lane == 0) a.fro_out[bth] = fro;
        // ---- Algorithm 1 in residual form, component r in the four lanes of row r
        // (the kernel is bound by its instruction count: reciprocals by the hardware instruction, 1 ulp)
        const float L = fro + lam, mu = lam;
        const float rcp = __builtin_amdgcn_rcpf(L + mu);
        const float s0 = 2.0f * rcp;
        const float rho = (L - mu) * rcp;
        const float rho2 = rho * rho;
        float xi = s0 * qr, dl = xi, rs = qr, omega = 2.0f;
        for (int i = 0; i < a.n_iter; ++i) {
            float xc[4];
            my_columns(dl, xc);
            const float hx = row_sum(hreg[0] * xc[0] + hreg[1] * xc[1] + hreg[2] * xc[2] + hreg[3] * xc[3]);
            omega = 4.0f * __builtin_amdgcn_rcpf(4.0f - rho2 * omega);
            rs -= hx + lam * dl;
            dl = (omega - 1.0f) * dl + (omega * s0) * rs;
            xi += dl;
        }
        if (a.xhat_out && c4 == 0) a.xhat_out[bth * D + r] = xi;
        // ---- readout y = U (alpha xhat + (1 - alpha) q)
        float xc[4];
        my_columns(alpha * xi + (1.0f - alpha) * qr, xc);
        const float y = row_sum(ureg[0] * xc[0] + ureg[1] * xc[1] + ureg[2] * xc[2] + ureg[3] * xc[3]);
        if (c4 == 0) IO::store1(a.o, row0 + r, y);
    }
    if (a.H_state) *(f32x4 *)(a.H_state + state_off) = hreg;
    if (a.U_state) *(f32x4 *)(a.U_state + state_off) = ureg;
}

template <class IO, int D, bool MULTI, bool LOWER>
static void launch_one(const DecodeArgs &a, int n_pairs, hipStream_t stream)
{
    // One token at d = 128: U is streamed through the readout instead of being held beside H (102 registers instead
    // of 158: four workgroups per CU instead of three). Measured on two boxes of the pool, 8192 pairs: full layout
    // 0.380 / 0.389 ms against 0.423 / 0.386 ms, block-lower layout 0.310 / 0.313 ms against 0.368 / 0.330 ms.
    if constexpr (D == 128 && !MULTI) {
        if (a.U_state) {
            hipLaunchKernelGGL((decode_step_kernel<IO, D, MULTI, LOWER, true>), dim3((unsigned)n_pairs),
                               dim3(DecodeShape<D>::NTHR), 0, stream, a);
            return;
        }
    }
    hipLaunchKernelGGL((decode_step_kernel<IO, D, MULTI, LOWER>), dim3((unsigned)n_pairs), dim3(DecodeShape<D>::NTHR), 0,
                       stream, a);
}

template <class IO, bool MULTI>
static void launch_decode(const DecodeArgs &a, int n_pairs, int d, hipStream_t stream)
{
    // (up to d = 32 the state is a single 32 x 32 block: both layouts are the full one)
    if (a.h_lower_blocks && d >= 64) {
        if (d == 128) launch_one<IO, 128, MULTI, true>(a, n_pairs, stream);
        else launch_one<IO, 64, MULTI, true>(a, n_pairs, stream);
        return;
    }
    switch (d) {
    case 16:
        hipLaunchKernelGGL((decode_step_kernel_d16<IO>), dim3((unsigned)((n_pairs + 3) / 4)), dim3(256), 0, stream, a,
                           n_pairs);
        break;
    case 32: launch_one<IO, 32, MULTI, false>(a, n_pairs, stream); break;
    case 64: launch_one<IO, 64, MULTI, false>(a, n_pairs, stream); break;
    case 128: launch_one<IO, 128, MULTI, false>(a, n_pairs, stream); break;
    default: launch_one<IO, 256, MULTI, false>(a, n_pairs, stream); break;
    }
}

// d in {16, 32, 64, 128, 256}; the block-lower layout of H only up to d = 128; d = 256 needs U_state (checked by the
// callers).
hipError_t launch_decode_step(const DecodeArgs &a, int n_pairs, int d, bool io_bf16, hipStream_t stream)
{
    if (d != 16 && d != 32 && d != 64 && d != 128 && d != 256) return hipErrorInvalidValue;
    if ((a.h_lower_blocks && d == 256) || (d == 256 && !a.U_state)) return hipErrorInvalidValue;
    if (io_bf16) {
        if (a.T == 1) launch_decode<IOBF16, false>(a, n_pairs, d, stream);
        else launch_decode<IOBF16, true>(a, n_pairs, d, stream);
    } else {
        if (a.T == 1) launch_decode<IOF32, false>(a, n_pairs, d, stream);
        else launch_decode<IOF32, true>(a, n_pairs, d, stream);
    }
    return hipGetLastError();
}

}  // namespace gka
