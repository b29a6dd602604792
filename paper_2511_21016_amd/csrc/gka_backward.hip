// Elementwise and per-token kernels of the backward pass (Section 4.2.2 "Backward Pass", Appendix B.2). The heavy
// parts of the backward pass run elsewhere: two solves on the forward kernels (the forward solve for xhat_t and the
// solve of the incoming gradient, dq_t = CH(H_t + lambda_t I, dxhat_t, r)) and the gated-linear-attention readouts,
// four of them walking the sequence backwards, which are the reverse recurrences of Section 4.2.2 (Eq. (Ai) and the
// like for U): one kernel with the state in registers for bf16 tensors, the forward kernels on time-reversed
// copies for float32 tensors. What remains is here: mixing, conversions, the time reversal (for the latter path),
// the per-token combination of the pieces and the reverse cumulative sum that gives the gradient of the gates.
//
// All tensors are packed: [B,T,H,d] for vectors, [B,T,H] for scalars.
#include "gka_device.hpp"
#include "gka_kernels.hpp"

namespace gka {

// The elementwise kernels take four consecutive features per thread (16-byte accesses to float32 tensors, 8-byte ones
// to bf16 tensors); d is a multiple of 4, so the four belong to one token.
__device__ __forceinline__ f32x4 load_f32x4(const float *p, int64_t i) { return *(const f32x4 *)(p + i); }

// After the forward solve: x in the tensors' dtype, the readout operand xt = alpha x + (1 - alpha) q, and the
// per-token constants of the later passes.
template <class IO>
__global__ __launch_bounds__(256) void bwd_mix_kernel(BackwardGlueArgs a)
{
    const int64_t i = ((int64_t)blockIdx.x * 256 + threadIdx.x) * 4;
    if (i >= a.n_elems) return;
    const int64_t tok = i / a.d;
    const float al = a.alpha ? a.alpha[tok] : 1.0f;
    const f32x4 x = load_f32x4(a.x_f32, i);
    const f32x4 q = IO::load4(a.q, i);
    const f32x4 xt = {al * x[0] + (1.0f - al) * q[0], al * x[1] + (1.0f - al) * q[1],
                      al * x[2] + (1.0f - al) * q[2], al * x[3] + (1.0f - al) * q[3]};
    IO::store4(a.x_io, i, x[0], x[1], x[2], x[3]);
    IO::store4(a.xt_io, i, xt[0], xt[1], xt[2], xt[3]);
    if (a.x_lo_io) {
        // bf16 tensors: the gradients at k and at the gates are small differences of sums over these operands, so
        // what their rounding leaves over goes along as a second operand
        const f32x4 xh = IO::load4(a.x_io, i), xth = IO::load4(a.xt_io, i);
        IO::store4(a.x_lo_io, i, x[0] - xh[0], x[1] - xh[1], x[2] - xh[2], x[3] - xh[3]);
        IO::store4(a.xt_lo_io, i, xt[0] - xth[0], xt[1] - xth[1], xt[2] - xth[2], xt[3] - xth[3]);
    }
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
    const int64_t i = ((int64_t)blockIdx.x * 256 + threadIdx.x) * 4;
    if (i >= a.n_elems) return;
    const float al = a.alpha ? a.alpha[i / a.d] : 1.0f;
    const f32x4 g = a.natural_order ? load_f32x4((const float *)a.dxt_io, i) : IO::load4(a.dxt_io, i);
    const f32x4 rhs = {al * g[0], al * g[1], al * g[2], al * g[3]};
    IO::store4(a.rhs_io, i, rhs[0], rhs[1], rhs[2], rhs[3]);
    if (a.rhs_lo_io) {
        // the solve amplifies a perturbation of its right-hand side: the rounding remainder goes along
        const f32x4 hi = IO::load4(a.rhs_io, i);
        IO::store4(a.rhs_lo_io, i, rhs[0] - hi[0], rhs[1] - hi[1], rhs[2] - hi[2], rhs[3] - hi[3]);
    }
}

// Time reversal tau = T - 1 - t of k, v, dy, x, p, xt (p converted from float32 on the way).
template <class IO>
__global__ __launch_bounds__(256) void bwd_reverse_kernel(BackwardGlueArgs a)
{
    const int64_t i = ((int64_t)blockIdx.x * 256 + threadIdx.x) * 4;
    if (i >= a.n_elems) return;
    if (a.natural_order) {                       // nothing to reverse: p in the tensors' dtype and beta C k
        const f32x4 pv = load_f32x4(a.p_f32, i);
        IO::store4(a.p_rev, i, pv[0], pv[1], pv[2], pv[3]);
        if (a.rule_a > 0.0f) {
            const int64_t tok = i / a.d;
            const float bc = (a.beta ? a.beta[tok] : 1.0f) * a.C[tok];
            const f32x4 kv = IO::load4(a.k, i);
            IO::store4(a.vp_rev, i, bc * kv[0], bc * kv[1], bc * kv[2], bc * kv[3]);
        }
        return;
    }
    const int64_t hd = (int64_t)a.H * a.d;
    const int64_t b = i / (hd * a.T), rem = i - b * hd * a.T;
    const int64_t tau = rem / hd, within = rem - tau * hd;
    const int64_t src = (b * a.T + (a.T - 1 - tau)) * hd + within;
    auto copy4 = [&](void *dst, const void *from) {
        const f32x4 v = IO::load4(from, src);
        IO::store4(dst, i, v[0], v[1], v[2], v[3]);
    };
    const f32x4 kv = IO::load4(a.k, src);
    IO::store4(a.k_rev, i, kv[0], kv[1], kv[2], kv[3]);
    copy4(a.v_rev, a.v);
    copy4(a.dy_rev, a.dy);
    copy4(a.x_rev, a.x_io);
    copy4(a.xt_rev, a.xt_io);
    const f32x4 pv = load_f32x4(a.p_f32, src);
    IO::store4(a.p_rev, i, pv[0], pv[1], pv[2], pv[3]);
    if (a.rule_a > 0.0f) {
        const int64_t stok = src / a.d;
        const float bc = (a.beta ? a.beta[stok] : 1.0f) * a.C[stok];
        IO::store4(a.vp_rev, i, bc * kv[0], bc * kv[1], bc * kv[2], bc * kv[3]);
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
    auto index = [&](int64_t t) { return (b * a.T + (t >= 0 ? t : 0)) * a.H + h; };
    auto next_gate = [&](int64_t t) { return (t >= 0 && t + 1 < a.T) ? a.gate[index(t + 1)] : 0.0f; };
    float carry = 0.0f;
    float c_next = a.c[index(a.T - 1 - lane)], g_next = next_gate(a.T - 1 - lane);   // read one block ahead
    for (int64_t t0 = a.T - 1; t0 >= 0; t0 -= 64) {
        const int64_t t = t0 - lane;
        float c = t >= 0 ? c_next : 0.0f;
        float w = g_next * g_next;
        c_next = a.c[index(t - 64)];
        g_next = next_gate(t - 64);
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const float cp = __shfl_up(c, off, 64), wp = __shfl_up(w, off, 64);
            if (lane >= off) { c = c + w * cp; w = w * wp; }
        }
        const float run = c + w * carry;
        if (t >= 0) a.C[index(t)] = run;
        carry = lane_value(run, 63);
    }
}

// d / 4 lanes per token: the pieces are combined into the gradients (Section 4.2.2, Appendix B.2):
//   dq = p + (1 - alpha) dxt,  dk = beta (-A k - A^T k + Ubar^T v),  dv = beta Ubar k,
//   dalpha = dxt . (x - q),  dlambda = -x . p,  dbeta = k^T Abar k + v . (Ubar k)  (Abar = -A without the rule),
//   s = -p . (H x) + dy . y - beta dbeta      (the gate gradient is the reverse cumulative sum of s over gamma),
//   with y = U_t xt_t read out from the stored (rounded) xt where the tensors are bf16: the sum telescopes against
//   v . (Ubar k), which the reversed passes form from that same xt; with the forward pass's own y (formed from the
//   unrounded xhat) the mismatch accumulates along the sequence
// With the rule lambda_t = a ||H_t||_F the gradient at every H_t gets the term -c_t H_t (Appendix B.2,
// Eq. (dH_t-implicit)); summed over the later states it is C_t H_t for the keys up to t (C_t = sum_{s>=t} M[t,s]^2 c_s)
// plus a reverse recurrence over the later keys, both read from plain readouts.
// with A_t = sum_{s>=t} M[t,s] p_s x_s^T and Ubar_t = sum_{s>=t} M[t,s] dy_s xt_s^T read from the reversed passes.
template <class IO, int D>
__global__ __launch_bounds__(256) void bwd_combine_kernel(BackwardGlueArgs a)
{
    constexpr int LPT = D / 4;                   // lanes per token, four features each
    constexpr int TPW = 64 / LPT;                // tokens per wave
    const int lane = threadIdx.x & 63;
    const int sub = lane % LPT;
    const int64_t tok_raw = ((int64_t)blockIdx.x * 4 + (threadIdx.x >> 6)) * TPW + lane / LPT;   // index into [B,T,H]
    const bool live = tok_raw < a.n_tokens;      // a dead group computes on the last token and stores nothing
    const int64_t tok = live ? tok_raw : a.n_tokens - 1;
    const int64_t bt = tok / a.H, h = tok - bt * a.H;
    const int64_t b = bt / a.T, t = bt - b * a.T;
    // the same token in the results of the reversed passes
    const int64_t rtok = a.natural_order ? tok : (b * a.T + (a.T - 1 - t)) * a.H + h;
    const int64_t i = tok * D + sub * 4, ri = rtok * D + sub * 4;
    auto group_sum = [](float x) {
#pragma unroll
        for (int off = LPT / 2; off > 0; off >>= 1) x += __shfl_xor(x, off, 64);
        return x;
    };
    const float al = a.alpha ? a.alpha[tok] : 1.0f;
    const float be = a.beta ? a.beta[tok] : 1.0f;
    const bool rule = a.rule_a > 0.0f;
    const float Ct = rule ? a.C[tok] : 0.0f;
    const f32x4 x = load_f32x4(a.x_f32, i), p = load_f32x4(a.p_f32, i);
    f32x4 q = {0.0f, 0.0f, 0.0f, 0.0f};
    if (a.dalpha) q = IO::load4(a.q, i);         // q enters dalpha only
    const f32x4 k = IO::load4(a.k, i), v = IO::load4(a.v, i), dy = IO::load4(a.dy, i);
    // with the fused readouts (natural_order) the pieces of the gate gradient's sum arrive in float32
    auto piece = [&](const void *ptr, int64_t idx) {
        return a.natural_order ? load_f32x4((const float *)ptr, idx) : IO::load4(ptr, idx);
    };
    const f32x4 dxt = piece(a.dxt_io, i), y = piece(a.y_io, i), hx = piece(a.hx_io, i);
    const f32x4 a1 = piece(a.r1, ri), a2 = piece(a.r2, ri), u1 = piece(a.r3, ri), d4 = piece(a.r4, ri);
    f32x4 hk = {0.0f, 0.0f, 0.0f, 0.0f}, r5 = hk;
    float kk = 0.0f;                             // k_t . k_t (the rule's diagonal term)
    if (rule) {
        hk = IO::load4(a.hk_io, i);
        r5 = IO::load4(a.r5, ri);
        kk = group_sum(k[0] * k[0] + k[1] * k[1] + k[2] * k[2] + k[3] * k[3]);
    }
    float s_dalpha = 0.0f, s_dlam = 0.0f, s_ka1 = 0.0f, s_vd4 = 0.0f, s_phx = 0.0f, s_dyy = 0.0f;
    f32x4 o_dq, o_dk, o_dv;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        // (Abar + Abar^T) k of the H state; with the rule, the -c_t H_t terms add -2 (C H k + sum_{j>t} ...)
        float dkh = -a1[e] - a2[e];
        if (rule) dkh -= 2.0f * (Ct * hk[e] + (r5[e] - be * Ct * k[e] * kk));
        o_dq[e] = p[e] + (1.0f - al) * dxt[e];
        o_dk[e] = be * (u1[e] + dkh);
        o_dv[e] = be * d4[e];
        s_dalpha += dxt[e] * (x[e] - q[e]);
        s_dlam -= x[e] * p[e];
        s_ka1 -= 0.5f * k[e] * dkh;
        s_vd4 += v[e] * d4[e];
        s_phx += p[e] * hx[e];
        s_dyy += dy[e] * y[e];
    }
    if (live) {
        *(f32x4 *)(a.dq + i) = o_dq;
        *(f32x4 *)(a.dk + i) = o_dk;
        *(f32x4 *)(a.dv + i) = o_dv;
    }
    s_dalpha = group_sum(s_dalpha); s_dlam = group_sum(s_dlam); s_ka1 = group_sum(s_ka1);
    s_vd4 = group_sum(s_vd4); s_phx = group_sum(s_phx); s_dyy = group_sum(s_dyy);
    if (live && sub == 0) {
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
// time. A gate of 0 starts a new packed sequence (it wipes the state): everything after it sums to gamma dgamma = 0
// exactly, so the sum restarts there instead of carrying that zero as rounding noise, G_t = s_t + w_t G_{t+1} with
// w_t = 0 where gate_{t+1} = 0; the gradient at such a gate itself is reported as 0. Inside a block the affine maps
// are composed by a Hillis-Steele scan over the lanes (lane 0 the latest token).
__global__ __launch_bounds__(64) void bwd_gate_scan_kernel(BackwardGlueArgs a)
{
    const int lane = threadIdx.x;
    const int64_t b = blockIdx.x / a.H, h = blockIdx.x - b * a.H;
    auto index = [&](int64_t t) { return (b * a.T + (t >= 0 ? t : 0)) * a.H + h; };
    auto gate_at = [&](int64_t t) { return (t >= 0 && t < a.T) ? a.gate[index(t)] : 1.0f; };
    float carry = 0.0f;
    // the next block's values are read before this block's scan, so that the walk does not pay a memory round trip
    // per block
    float sv_next = a.s[index(a.T - 1 - lane)], g_next = gate_at(a.T - 1 - lane), gn_next = gate_at(a.T - lane);
    for (int64_t t0 = a.T - 1; t0 >= 0; t0 -= 64) {
        const int64_t t = t0 - lane;                       // lane 0 takes the latest token of the block
        float c = t >= 0 ? sv_next : 0.0f;
        const float gv = g_next;
        float w = (t >= 0 && gn_next > 0.0f) ? 1.0f : 0.0f; // does the sum of the later tokens reach this one?
        sv_next = a.s[index(t - 64)];
        g_next = gate_at(t - 64);
        gn_next = gate_at(t - 63);
        float run;
        if (__ballot(t >= 0 && w == 0.0f) == 0) {          // (wave-uniform) no restart in this block: a plain prefix sum
            run = wave_inclusive_scan(c, lane) + carry;
        } else {
#pragma unroll
            for (int off = 1; off < 64; off <<= 1) {
                const float cp = __shfl_up(c, off, 64), wp = __shfl_up(w, off, 64);
                if (lane >= off) { c = c + w * cp; w = w * wp; }
            }
            run = c + w * carry;
        }
        if (t >= 0) a.dgate[index(t)] = gv > 0.0f ? run / gv : 0.0f;
        carry = lane_value(run, 63);
    }
}

// Gradients at the initial states (Section 4.2.2: the accumulated gradients at H_0 and U_0, times the first gate):
//   dH_init = gamma_0 Abar_0,  Abar_0 = -sum_t M[0,t] p_t xhat_t^T  [- gamma_0 C_0 H_init - sum_j M[0,j] beta_j C_j k_j k_j^T
//   with the rule lambda_t = a ||H_t||_F],   dU_init = gamma_0 sum_t M[0,t] dy_t xt_t^T,
// from the states that the reverse readouts hold after their last token (token 0).
__global__ __launch_bounds__(256) void bwd_init_grads_kernel(BackwardGlueArgs a)
{
    const int64_t dd = (int64_t)a.d * a.d;
    const int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (e >= (int64_t)a.n_pairs * dd) return;
    const int64_t pair = e / dd, ij = e - pair * dd;
    const int i = (int)(ij / a.d), j = (int)(ij - (int64_t)i * a.d);
    const int64_t b = pair / a.H, h = pair - b * a.H;
    const int64_t tok0 = (b * a.T) * a.H + h;            // the pair's first token
    const float g0 = a.gate[tok0];
    if (a.dH_init) {
        float acc = -a.fin_px[e];
        if (a.rule_a > 0.0f) acc -= g0 * a.C[tok0] * (a.H_init ? a.H_init[e] : 0.0f) + a.fin_ck[e];
        a.dH_init[e] = g0 * acc;
    }
    if (a.dU_init) a.dU_init[e] = g0 * a.fin_xtdy[pair * dd + (int64_t)j * a.d + i];
}

template <class IO>
static void launch_glue_t(const BackwardGlueArgs &a, int which, hipStream_t stream)
{
    const unsigned blocks = (unsigned)((a.n_elems / 4 + 255) / 256);
    switch (which) {
    case 0: hipLaunchKernelGGL((bwd_mix_kernel<IO>), dim3(blocks), dim3(256), 0, stream, a); break;
    case 1: hipLaunchKernelGGL((bwd_rhs_kernel<IO>), dim3(blocks), dim3(256), 0, stream, a); break;
    case 2: hipLaunchKernelGGL((bwd_reverse_kernel<IO>), dim3(blocks), dim3(256), 0, stream, a); break;
    case 3: {
        const int64_t per_block = 4 * (256 / a.d);         // 4 waves of 64 / (d / 4) tokens
        const unsigned tb = (unsigned)((a.n_tokens + per_block - 1) / per_block);
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
    case 6:
        hipLaunchKernelGGL(bwd_rule_scan_kernel, dim3((unsigned)(a.n_tokens / a.T)), dim3(64), 0, stream, a);
        break;
    default: {
        const int64_t n = (int64_t)a.n_pairs * a.d * a.d;
        hipLaunchKernelGGL(bwd_init_grads_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream, a);
    }
    }
}

// Rows of a strided [B,T,H,d] tensor (head dimension contiguous, 16-byte aligned rows) to the packed layout, 16 bytes
// per thread.
__global__ __launch_bounds__(256) void pack_rows_kernel(const unsigned char *src, unsigned char *dst, int64_t n_pieces,
                                                        int pieces_per_row, int T, int H, int64_t stride_b_bytes,
                                                        int64_t stride_t_bytes, int64_t stride_h_bytes)
{
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    const int64_t piece = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (piece >= n_pieces) return;
    const int64_t row = piece / pieces_per_row;
    const int part = (int)(piece - row * pieces_per_row);
    const int h = (int)(row % H);
    const int64_t bt = row / H;
    const int t = (int)(bt % T);
    const int64_t b = bt / T;
    const unsigned char *from = src + b * stride_b_bytes + t * stride_t_bytes + h * stride_h_bytes + (int64_t)part * 16;
    *(u32x4 *)(dst + piece * 16) = *(const u32x4 *)from;
}

hipError_t launch_pack_rows(const void *src, void *dst, int B, int T, int H, int d, int elem_bytes, int64_t stride_b,
                            int64_t stride_t, int64_t stride_h, hipStream_t stream)
{
    const int pieces_per_row = d * elem_bytes / 16;
    const int64_t n_pieces = (int64_t)B * T * H * pieces_per_row;
    hipLaunchKernelGGL(pack_rows_kernel, dim3((unsigned)((n_pieces + 255) / 256)), dim3(256), 0, stream,
                       (const unsigned char *)src, (unsigned char *)dst, n_pieces, pieces_per_row, T, H,
                       stride_b * elem_bytes, stride_t * elem_bytes, stride_h * elem_bytes);
    return hipGetLastError();
}

hipError_t launch_backward_glue(const BackwardGlueArgs &a, int which, bool io_bf16, hipStream_t stream)
{
    if (io_bf16) launch_glue_t<IOBF16>(a, which, stream);
    else launch_glue_t<IOF32>(a, which, stream);
    return hipGetLastError();
}

}  // namespace gka
