// Elementwise and per-token kernels of the backward pass (Section 4.2.2 "Backward Pass", Appendix B.2). The heavy
// parts of the backward pass run on the forward kernels: two solves (the forward solve for xhat_t and the solve of the
// incoming gradient, dq_t = CH(H_t + lambda_t I, dxhat_t, r)) and six gated-linear-attention readouts, four of them
// on time-reversed sequences, which are the reverse recurrences of Section 4.2.2 (Eq. (Ai) and the like for U). What
// remains is here: mixing, conversions, the time reversal, the per-token combination of the pieces and the reverse
// cumulative sum that gives the gradient of the gates.
//
// All tensors are packed: [B,T,H,d] for vectors, [B,T,H] for scalars.
#include "gka_device.hpp"
#include "gka_kernels.hpp"

namespace gka {

// After the forward solve: x in the tensors' dtype, the readout operand xt = alpha x + (1 - alpha) q, and the
// per-token constants of the later passes.
template <class IO>
__global__ __launch_bounds__(256) void bwd_mix_kernel(BackwardGlueArgs a)
{
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= a.n_elems) return;
    const int64_t tok = i / a.d;
    const float al = a.alpha ? a.alpha[tok] : 1.0f;
    const float x = a.x_f32[i];
    IO::store1(a.x_io, i, x);
    IO::store1(a.xt_io, i, al * x + (1.0f - al) * IO::load(a.q, i));
    // once per token: the all-zero alpha of the plain readouts and the gates of the reverse recurrences,
    // gate'_tau = gate_{T - tau} for tau >= 1 (gate'_0 multiplies a zero state: 1)
    if (i - tok * a.d == 0) {
        const int64_t bt = tok / a.H, h = tok - bt * a.H;
        const int64_t b = bt / a.T, tau = bt - b * a.T;
        a.zeros[tok] = 0.0f;
        a.gate_rev[tok] = tau == 0 ? 1.0f : a.gate[(b * a.T + (a.T - tau)) * a.H + h];
    }
}

// Right-hand side of the backward solve: alpha_t dxt_t.
template <class IO>
__global__ __launch_bounds__(256) void bwd_rhs_kernel(BackwardGlueArgs a)
{
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= a.n_elems) return;
    const float al = a.alpha ? a.alpha[i / a.d] : 1.0f;
    IO::store1(a.rhs_io, i, al * IO::load(a.dxt_io, i));
}

// Time reversal tau = T - 1 - t of k, v, dy, x, p, xt (p converted from float32 on the way).
template <class IO>
__global__ __launch_bounds__(256) void bwd_reverse_kernel(BackwardGlueArgs a)
{
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= a.n_elems) return;
    const int64_t hd = (int64_t)a.H * a.d;
    const int64_t b = i / (hd * a.T), rem = i - b * hd * a.T;
    const int64_t tau = rem / hd, within = rem - tau * hd;
    const int64_t src = (b * a.T + (a.T - 1 - tau)) * hd + within;
    IO::store1(a.k_rev, i, IO::load(a.k, src));
    IO::store1(a.v_rev, i, IO::load(a.v, src));
    IO::store1(a.dy_rev, i, IO::load(a.dy, src));
    IO::store1(a.x_rev, i, IO::load(a.x_io, src));
    IO::store1(a.xt_rev, i, IO::load(a.xt_io, src));
    IO::store1(a.p_rev, i, a.p_f32[src]);
    if (a.rule_a > 0.0f) {
        const int64_t stok = src / a.d;
        IO::store1(a.vp_rev, i, (a.beta ? a.beta[stok] : 1.0f) * a.C[stok] * IO::load(a.k, src));
    }
}

// The rule lambda_t = a ||H_t||_F: c_t = a (x_t . p_t) / ||H_t||_F, one wave per token.
template <int D>
__global__ __launch_bounds__(256) void bwd_rule_scalar_kernel(BackwardGlueArgs a)
{
    constexpr int E = D / 64;
    const int lane = threadIdx.x & 63;
    const int64_t tok = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (tok >= a.n_tokens) return;
    float dot = 0.0f;
#pragma unroll
    for (int e = 0; e < E; ++e) dot += a.x_f32[tok * D + lane * E + e] * a.p_f32[tok * D + lane * E + e];
    dot = wave_sum(dot);
    if (lane == 0) a.c[tok] = a.rule_a * dot / a.fro[tok];
}

// C_t = c_t + gate_{t+1}^2 C_{t+1}: one wave per (batch, head) pair walks its sequence backwards 64 tokens at a time;
// inside a block the affine maps C -> c + w C are composed by a Hillis-Steele scan over the lanes (lane 0 the latest
// token).
__global__ __launch_bounds__(64) void bwd_rule_scan_kernel(BackwardGlueArgs a)
{
    const int lane = threadIdx.x;
    const int64_t b = blockIdx.x / a.H, h = blockIdx.x - b * a.H;
    float carry = 0.0f;
    for (int64_t t0 = a.T - 1; t0 >= 0; t0 -= 64) {
        const int64_t t = t0 - lane;
        const int64_t m = (b * a.T + (t >= 0 ? t : 0)) * a.H + h;
        float c = t >= 0 ? a.c[m] : 0.0f;
        const float gnext = (t >= 0 && t + 1 < a.T) ? a.gate[m + a.H] : 0.0f;
        float w = gnext * gnext;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const float cp = __shfl_up(c, off, 64), wp = __shfl_up(w, off, 64);
            if (lane >= off) { c = c + w * cp; w = w * wp; }
        }
        const float run = c + w * carry;
        if (t >= 0) a.C[m] = run;
        carry = lane_value(run, 63);
    }
}

// One wave per token: the pieces are combined into the gradients (Section 4.2.2, Appendix B.2):
//   dq = p + (1 - alpha) dxt,  dk = beta (-A k - A^T k + Ubar^T v),  dv = beta Ubar k,
//   dalpha = dxt . (x - q),  dlambda = -x . p,  dbeta = k^T Abar k + v . (Ubar k)  (Abar = -A without the rule),
//   s = -p . (H x) + dy . y - beta dbeta      (the gate gradient is the reverse cumulative sum of s over gamma)
// With the rule lambda_t = a ||H_t||_F the gradient at every H_t gets the term -c_t H_t (Appendix B.2,
// Eq. (dH_t-implicit)); summed over the later states it is C_t H_t for the keys up to t (C_t = sum_{s>=t} M[t,s]^2 c_s)
// plus a reverse recurrence over the later keys, both read from plain readouts.
// with A_t = sum_{s>=t} M[t,s] p_s x_s^T and Ubar_t = sum_{s>=t} M[t,s] dy_s xt_s^T read from the reversed passes.
template <class IO, int D>
__global__ __launch_bounds__(256) void bwd_combine_kernel(BackwardGlueArgs a)
{
    constexpr int E = D / 64;                    // elements per lane
    const int lane = threadIdx.x & 63;
    const int64_t tok = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);      // index into [B,T,H]
    if (tok >= a.n_tokens) return;
    const int64_t bt = tok / a.H, h = tok - bt * a.H;
    const int64_t b = bt / a.T, t = bt - b * a.T;
    const int64_t rtok = (b * a.T + (a.T - 1 - t)) * a.H + h;              // the same token in the reversed tensors
    const float al = a.alpha ? a.alpha[tok] : 1.0f;
    const float be = a.beta ? a.beta[tok] : 1.0f;
    float s_dalpha = 0.0f, s_dlam = 0.0f, s_ka1 = 0.0f, s_vd4 = 0.0f, s_phx = 0.0f, s_dyy = 0.0f;
    const bool rule = a.rule_a > 0.0f;
    const float Ct = rule ? a.C[tok] : 0.0f;
    float kk = 0.0f;                             // k_t . k_t (the rule's diagonal term)
    if (rule) {
#pragma unroll
        for (int e = 0; e < E; ++e) {
            const float kv = IO::load(a.k, tok * D + lane * E + e);
            kk += kv * kv;
        }
        kk = wave_sum(kk);
    }
#pragma unroll
    for (int e = 0; e < E; ++e) {
        const int64_t i = tok * D + lane * E + e, ri = rtok * D + lane * E + e;
        const float x = a.x_f32[i], p = a.p_f32[i];
        const float q = IO::load(a.q, i), k = IO::load(a.k, i), v = IO::load(a.v, i), dy = IO::load(a.dy, i);
        const float dxt = IO::load(a.dxt_io, i), y = IO::load(a.y_io, i), hx = IO::load(a.hx_io, i);
        const float a1 = IO::load(a.r1, ri), a2 = IO::load(a.r2, ri), u1 = IO::load(a.r3, ri), d4 = IO::load(a.r4, ri);
        // (Abar + Abar^T) k of the H state; with the rule, the -c_t H_t terms add -2 (C H k + sum_{j>t} ...)
        float dkh = -a1 - a2;
        if (rule) {
            const float hk = IO::load(a.hk_io, i), e2 = IO::load(a.r5, ri) - be * Ct * k * kk;
            dkh -= 2.0f * (Ct * hk + e2);
        }
        a.dq[i] = p + (1.0f - al) * dxt;
        a.dk[i] = be * (u1 + dkh);
        a.dv[i] = be * d4;
        s_dalpha += dxt * (x - q);
        s_dlam -= x * p;
        s_ka1 -= 0.5f * k * dkh;
        s_vd4 += v * d4;
        s_phx += p * hx;
        s_dyy += dy * y;
    }
    s_dalpha = wave_sum(s_dalpha); s_dlam = wave_sum(s_dlam); s_ka1 = wave_sum(s_ka1);
    s_vd4 = wave_sum(s_vd4); s_phx = wave_sum(s_phx); s_dyy = wave_sum(s_dyy);
    if (lane == 0) {
        const float dbeta = s_vd4 - s_ka1;       // s_ka1 = -k . (Abar + Abar^T) k / 2 = -k^T Abar k
        if (a.dalpha) a.dalpha[tok] = s_dalpha;
        if (a.dlambda && !rule) a.dlambda[tok] = s_dlam;
        if (a.dbeta) a.dbeta[tok] = dbeta;
        float D_t = s_dyy - s_phx;
        if (rule) D_t -= a.c[tok] * a.fro[tok] * a.fro[tok];
        a.s[tok] = D_t - be * dbeta;
    }
}

// One wave per (batch, head) pair: dgate_t = (sum_{s>=t} s_s) / gate_t, walking the sequence backwards 64 tokens at a
// time.
__global__ __launch_bounds__(64) void bwd_gate_scan_kernel(BackwardGlueArgs a)
{
    const int lane = threadIdx.x;
    const int64_t b = blockIdx.x / a.H, h = blockIdx.x - b * a.H;
    float carry = 0.0f;
    for (int64_t t0 = a.T - 1; t0 >= 0; t0 -= 64) {
        const int64_t t = t0 - lane;                       // lane 0 takes the latest token of the block
        const int64_t m = (b * a.T + (t >= 0 ? t : 0)) * a.H + h;
        const float sv = t >= 0 ? a.s[m] : 0.0f;
        const float run = wave_inclusive_scan(sv, lane) + carry;
        if (t >= 0) a.dgate[m] = run / a.gate[m];
        carry = lane_value(run, 63);
    }
}

template <class IO>
static void launch_glue_t(const BackwardGlueArgs &a, int which, hipStream_t stream)
{
    const unsigned blocks = (unsigned)((a.n_elems + 255) / 256);
    switch (which) {
    case 0: hipLaunchKernelGGL((bwd_mix_kernel<IO>), dim3(blocks), dim3(256), 0, stream, a); break;
    case 1: hipLaunchKernelGGL((bwd_rhs_kernel<IO>), dim3(blocks), dim3(256), 0, stream, a); break;
    case 2: hipLaunchKernelGGL((bwd_reverse_kernel<IO>), dim3(blocks), dim3(256), 0, stream, a); break;
    case 3: {
        const unsigned tb = (unsigned)((a.n_tokens + 3) / 4);
        if (a.d == 128) hipLaunchKernelGGL((bwd_combine_kernel<IO, 128>), dim3(tb), dim3(256), 0, stream, a);
        else hipLaunchKernelGGL((bwd_combine_kernel<IO, 64>), dim3(tb), dim3(256), 0, stream, a);
        break;
    }
    case 4:
        hipLaunchKernelGGL(bwd_gate_scan_kernel, dim3((unsigned)(a.n_tokens / a.T)), dim3(64), 0, stream, a);
        break;
    case 5: {
        const unsigned tb = (unsigned)((a.n_tokens + 3) / 4);
        if (a.d == 128) hipLaunchKernelGGL((bwd_rule_scalar_kernel<128>), dim3(tb), dim3(256), 0, stream, a);
        else hipLaunchKernelGGL((bwd_rule_scalar_kernel<64>), dim3(tb), dim3(256), 0, stream, a);
        break;
    }
    default:
        hipLaunchKernelGGL(bwd_rule_scan_kernel, dim3((unsigned)(a.n_tokens / a.T)), dim3(64), 0, stream, a);
    }
}

hipError_t launch_backward_glue(const BackwardGlueArgs &a, int which, bool io_bf16, hipStream_t stream)
{
    if (io_bf16) launch_glue_t<IOBF16>(a, which, stream);
    else launch_glue_t<IOF32>(a, which, stream);
    return hipGetLastError();
}

}  // namespace gka
