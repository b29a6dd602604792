// Chunk-wise forward pass (Section 4.2.1) for head dimensions up to 32, bf16 tensors and operands, float32 accumulation:
//   * the layer itself at d = 16 (the vision models of Appendix L) and d = 32: Eq. (CH), its Frobenius norm, Algorithm 1
//     and the readout y_t = U_t xhat_t;
//   * the solve of latent sketching (appendix "Latent Sketching for Approximate Solutions") in d_s <= 32 sketched
//     dimensions, z_t = CH(S H_t S^T + lambda_t I, S q_t, r), on the sketched keys and queries (no values, no readout).
// At these sizes a state is a 32 x 32 matrix (zero beyond d): one pair of accumulator tiles of the 16x16x32 matrix
// instruction, and a contraction over the features is a single 32-deep step. Every operand of a pass of Algorithm 1
// then lives in registers: a pass touches no memory at all. Three launches:
//   1. small_chunk_delta_kernel: per chunk, Delta H = sum_j w_j k_j k_j^T and Delta U = sum_j w_j v_j k_j^T (w_j: decay
//      from token j to the chunk's end, times the write gate) and the chunk's log2 decay; one wave per chunk.
//   2. small_state_scan_kernel: per pair, the states before every chunk, S_[n+1] = zeta_n S_[n] + Delta_n (elementwise
//      in float32, one float4 per thread and state, sixteen chunks in flight), from the caller's initial states if
//      given; the states after the last chunk are the final states.
//   3. small_solve_kernel: per chunk one workgroup of four waves, wave w = the 16 tokens 16 w .. 16 w + 15 on the
//      output lanes of the products (per-token scalars are per-lane scalars, the iterate stays in registers):
//      chunk-wise Frobenius norm, all passes of Algorithm 1 in residual form, then the readout.
// The arithmetic of 3 is that of the 128-dimensional kernels: the token's system is taken divided by its zeta_c,
//   g / zeta_c = H_[n] xi + K^T ((M / zeta_c) o (K xi)) - q / zeta_c,
//   delta' = (omega - 1) delta - omega s0 (zeta_c (g / zeta_c) + lambda xi'),  xi' = xi + delta,
// with bf16 operands (H_[n], K, the update delta, the masked products) and float32 accumulation; in the readout
// U_[n] and xhat enter as bf16 value + remainder.
//
// Fragment conventions (v_mfma_f32_16x16x32_bf16, lane l = 16 kg + n): an accumulator tile holds rows 4 kg + r
// (r = 0..3) of column n; an operand fragment holds eight contraction values of row (A) or column (B) n. Two
// accumulator tiles of the same columns convert in place into one B fragment, slot s <-> index 16 (s / 4) + 4 kg + s % 4
// of the 32 the fragment covers ("slot order"); every A fragment enumerates its contraction index in that order.
#include "gka_device.hpp"
#include "gka_kernels.hpp"

namespace gka {

namespace {

constexpr int kDs = 32;                    // features a fragment covers (rows of 16 features: the upper half is zero)
constexpr int kRow = 40;                   // LDS row of a key in 2-byte elements: 64 B of features + 16 B of padding
constexpr float kMinZeta = 0x1p-60f;       // floor of zeta_c where the system is divided by it
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ f32x4 mma16(bf16x8 a, bf16x8 b, f32x4 c)
{
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
}
__device__ __forceinline__ f32x4 zero4() { return f32x4{0.0f, 0.0f, 0.0f, 0.0f}; }
__device__ __forceinline__ bf16x8 pack8(f32x4 lo, f32x4 hi)
{
    bf16x8 f;
#pragma unroll
    for (int p = 0; p < 4; ++p) {
        f[p] = (__bf16)lo[p];
        f[4 + p] = (__bf16)hi[p];
    }
    return f;
}
__device__ __forceinline__ void unpack8(bf16x8 f, f32x4 &lo, f32x4 &hi)
{
#pragma unroll
    for (int p = 0; p < 4; ++p) {
        lo[p] = (float)f[p];
        hi[p] = (float)f[4 + p];
    }
}
// rounded value and what the rounding left over, both as fragments
__device__ __forceinline__ void split8(f32x4 lo, f32x4 hi, bf16x8 &val, bf16x8 &rem)
{
    val = pack8(lo, hi);
    f32x4 bl, bh;
    unpack8(val, bl, bh);
    rem = pack8(lo - bl, hi - bh);
}
__device__ __forceinline__ float sum_over_kg(float x)
{
    x += __shfl_xor(x, 16, 64);
    x += __shfl_xor(x, 32, 64);
    return x;
}
// the 32 features of one row (of 2-byte elements) in slot order, for the lane's kg; of a row that holds only 16
// features the upper half reads as zero
__device__ __forceinline__ bf16x8 row_in_slot_order(const uint16_t *row, int kg, bool upper = true)
{
    const u16x4 lo = *(const u16x4 *)(row + 4 * kg);
    u16x4 hi = {0, 0, 0, 0};
    if (upper) hi = *(const u16x4 *)(row + 16 + 4 * kg);
    const u16x8 v = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
    return __builtin_bit_cast(bf16x8, v);
}
// feature `col` of the eight keys 32 ks + (slot order) of an LDS tile of rows
__device__ __forceinline__ bf16x8 keys_in_slot_order(const uint16_t *rows, int ks, int kg, int col)
{
    u16x8 v;
#pragma unroll
    for (int s = 0; s < 8; ++s) v[s] = rows[(32 * ks + 16 * (s >> 2) + 4 * kg + (s & 3)) * kRow + col];
    return __builtin_bit_cast(bf16x8, v);
}
__device__ __forceinline__ int64_t row_offset(const SmallArgs &a, int b, int h, int tok)
{
    return b * a.stride_b + (int64_t)min(tok, a.T - 1) * a.stride_t + h * a.stride_h;
}
// The chunk's 64 rows of x (first 32 features; zeros from feature a.d on) into an LDS tile: 256 pieces of 16 bytes,
// `n_threads` at work. Rows past the end of the sequence repeat the last one (finite values that only meet zero
// weights and masked products).
__device__ __forceinline__ void stage_rows(const SmallArgs &a, const void *x, uint16_t *rows, int b, int h, int tok0, int t,
                                           int n_threads)
{
    for (int piece = t; piece < 256; piece += n_threads) {
        const int row = piece >> 2, part = piece & 3;
        u32x4 v = {0u, 0u, 0u, 0u};
        if (8 * part < a.d) v = *(const u32x4 *)((const uint16_t *)x + row_offset(a, b, h, tok0 + row) + 8 * part);
        *(u32x4 *)(rows + row * kRow + 8 * part) = v;
    }
}

}  // namespace

// ---- 1. chunk deltas ---------------------------------------------------------------------------------------------
// One wave per chunk (four chunks of consecutive pairs per workgroup). Delta H tile (fi, fj) = sum over the chunk's keys
// of K^T[fi] (w o K)[fj]: A = features x keys, B = keys x features, both gathered column-wise from the LDS tile of key
// rows; stored transposed (Delta H is symmetric up to the rounding of w o K), so that a lane holds four consecutive
// elements of a row. Delta U^T tile (fi, fj) = K^T[fi] (w o V)[fj], stored transposed likewise: row-major Delta U.
template <bool WITH_U, int D>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 8))) void small_chunk_delta_kernel(SmallArgs a)
{
    constexpr int NF = D / 16;                 // feature tiles that exist; a state is stored as D x D

    __shared__ __attribute__((aligned(16))) uint16_t s_k[4][64 * kRow];
    __shared__ __attribute__((aligned(16))) uint16_t s_v[WITH_U ? 4 : 1][WITH_U ? 64 * kRow : 8];
    __shared__ __attribute__((aligned(16))) float s_w[4][64];
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int n = lane & 15, kg = lane >> 4;
    const int64_t unit_raw = (int64_t)blockIdx.x * 4 + w;
    const int64_t n_units = (int64_t)a.n_pairs * a.n_chunks;
    const bool live = unit_raw < n_units;
    const int64_t unit = live ? unit_raw : n_units - 1;     // a dead wave repeats the last chunk and stores nothing
    const int pair = (int)(unit % a.n_pairs), chunk = (int)(unit / a.n_pairs);
    const int b = pair / a.H, h = pair % a.H;
    const int tok0 = chunk * kChunk;
    stage_rows(a, a.k, s_k[w], b, h, tok0, lane, 64);
    if constexpr (WITH_U) stage_rows(a, a.v, s_v[w], b, h, tok0, lane, 64);
    const bool valid = tok0 + lane < a.T;
    const int64_t gi = (b * (int64_t)a.T + min(tok0 + lane, a.T - 1)) * a.H + h;
    const float G = wave_inclusive_scan(valid ? log2_gate(a.gate[gi]) : 0.0f, lane);
    const float Gt = lane_value(G, 63);
    const float beta = a.beta ? a.beta[gi] : 1.0f;
    s_w[w][lane] = valid ? exp2f(Gt - G) * beta : 0.0f;
    __syncthreads();
    f32x4 accH[2][2] = {{zero4(), zero4()}, {zero4(), zero4()}}, accU[2][2] = {{zero4(), zero4()}, {zero4(), zero4()}};
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) {
        const f32x4 w0 = *(const f32x4 *)&s_w[w][32 * ks + 4 * kg], w1 = *(const f32x4 *)&s_w[w][32 * ks + 16 + 4 * kg];
        bf16x8 kt[2], wk[2], wv[2];
#pragma unroll
        for (int f = 0; f < NF; ++f) {
            f32x4 lo, hi;
            kt[f] = keys_in_slot_order(s_k[w], ks, kg, 16 * f + n);
            unpack8(kt[f], lo, hi);
            wk[f] = pack8(lo * w0, hi * w1);
            if constexpr (WITH_U) {
                unpack8(keys_in_slot_order(s_v[w], ks, kg, 16 * f + n), lo, hi);
                wv[f] = pack8(lo * w0, hi * w1);
            }
        }
#pragma unroll
        for (int fi = 0; fi < NF; ++fi)
#pragma unroll
            for (int fj = 0; fj < NF; ++fj) {
                accH[fi][fj] = mma16(kt[fi], wk[fj], accH[fi][fj]);
                if constexpr (WITH_U) accU[fi][fj] = mma16(kt[fi], wv[fj], accU[fi][fj]);
            }
    }
    if (live) {
        const int64_t at = (pair * (int64_t)a.n_chunks + chunk) * (D * D);
#pragma unroll
        for (int fi = 0; fi < NF; ++fi)
#pragma unroll
            for (int fj = 0; fj < NF; ++fj) {
                *(f32x4 *)(a.dH + at + (16 * fj + n) * D + 16 * fi + 4 * kg) = accH[fi][fj];
                if constexpr (WITH_U) *(f32x4 *)(a.dU + at + (16 * fj + n) * D + 16 * fi + 4 * kg) = accU[fi][fj];
            }
        if (lane == 0) a.chunk_log2_decay[pair * (int64_t)a.n_chunks + chunk] = Gt;
    }
}

// ---- 2. states before every chunk --------------------------------------------------------------------------------
// One workgroup per pair, thread t: elements 4 t .. 4 t + 3 of the D x D states (row-major, as the caller's initial
// and final states).
template <bool WITH_U, int D>
__global__ __launch_bounds__(D * D / 4) void small_state_scan_kernel(SmallArgs a)
{
    constexpr int kAhead = WITH_U ? 8 : 16;
    constexpr int SS = D * D;
    const int pair = blockIdx.x, t = threadIdx.x;
    const int64_t base = pair * (int64_t)a.n_chunks * SS + 4 * t;
    const float *decay = a.chunk_log2_decay + pair * (int64_t)a.n_chunks;
    const int64_t ext = (int64_t)pair * SS + 4 * t;          // this piece in the caller's states
    f32x4 H = zero4(), U = zero4();
    if (a.H_init) H = *(const f32x4 *)(a.H_init + ext);
    if (WITH_U && a.U_init) U = *(const f32x4 *)(a.U_init + ext);
    for (int c0 = 0; c0 < a.n_chunks; c0 += kAhead) {
        f32x4 dh[kAhead], du[WITH_U ? kAhead : 1];
        float z[kAhead];
#pragma unroll
        for (int i = 0; i < kAhead; ++i) {
            const int c = min(c0 + i, a.n_chunks - 1);
            dh[i] = *(const f32x4 *)(a.dH + base + (int64_t)c * SS);
            if constexpr (WITH_U) du[i] = *(const f32x4 *)(a.dU + base + (int64_t)c * SS);
            z[i] = decay[c];
        }
#pragma unroll
        for (int i = 0; i < kAhead; ++i) {
            if (c0 + i < a.n_chunks) {
                const float zeta = exp2f(z[i]);
                *(f32x4 *)(a.sH + base + (int64_t)(c0 + i) * SS) = H;
                H = zeta * H + dh[i];
                if constexpr (WITH_U) {
                    *(f32x4 *)(a.sU + base + (int64_t)(c0 + i) * SS) = U;
                    U = zeta * U + du[i];
                }
            }
        }
    }
    if (a.H_final) *(f32x4 *)(a.H_final + ext) = H;
    if (WITH_U && a.U_final) *(f32x4 *)(a.U_final + ext) = U;
}

// ---- 3. solve and readout ----------------------------------------------------------------------------------------
namespace {

// What a wave fetches from global memory before the workgroup's first barrier (the rows are on their way then).
struct TileInputs {
    f32x4 h[2][2];             // the state before the chunk: rows 16 fo + n, columns 4 kg .. and 16 + 4 kg ..
    bf16x8 qB;                 // the query of this lane's token as a B fragment
    float lam;                 // lambda of this lane's token (if given)
    int64_t ti;                // index of the token into [B,T,H]
    int64_t row;               // offset of its row in q, k, v, o
    bool valid;
};
// rows 16 fo + n of a D x D float32 state as the two runs of four columns a lane holds of them (zero beyond D)
template <int D>
__device__ __forceinline__ void state_row_runs(const float *S, int fo, int n, int kg, f32x4 &lo, f32x4 &hi)
{
    const float *row = S + (16 * fo + n) * D;
    lo = *(const f32x4 *)(row + 4 * kg);
    hi = zero4();
    if constexpr (D > 16) hi = *(const f32x4 *)(row + 16 + 4 * kg);
}
template <int D>
__device__ __forceinline__ TileInputs fetch_tile_inputs(const SmallArgs &a, int pair, int chunk, int w, int lane)
{
    const int n = lane & 15, kg = lane >> 4;
    const int b = pair / a.H, h = pair % a.H;
    const int tok = chunk * kChunk + 16 * w + n;
    TileInputs in;
    in.valid = tok < a.T;
    in.ti = (b * (int64_t)a.T + min(tok, a.T - 1)) * a.H + h;
    in.row = row_offset(a, b, h, tok);
    const float *Hn = a.sH + (pair * (int64_t)a.n_chunks + chunk) * (D * D);
#pragma unroll
    for (int fo = 0; fo < D / 16; ++fo) state_row_runs<D>(Hn, fo, n, kg, in.h[fo][0], in.h[fo][1]);
    in.qB = row_in_slot_order((const uint16_t *)a.q + in.row, kg, D > 16);
    in.lam = a.lambda ? a.lambda[in.ti] : 0.0f;
    return in;
}

// The work of the wave that owns token tile TT of the chunk: key tiles 0 .. TT are visible to it.
template <int TT, bool WITH_U, int D>
__device__ __forceinline__ void small_solve_tile(const SmallArgs &a, const TileInputs &in, const uint16_t *rows,
                                                 const uint16_t *vrows, const float *Gtab, const float *Btab, float *Wtab,
                                                 int64_t unit, int lane)
{
    constexpr int NJ = TT + 1;                 // key tiles
    constexpr int NKS = (TT + 2) / 2;          // steps of 32 keys in the products over keys
    constexpr int NF = D / 16;                 // feature tiles that exist (the second half of a fragment is zero at 16)
    const int n = lane & 15, kg = lane >> 4;
    const int c_local = 16 * TT + n;
    const bool valid = in.valid;
    const int64_t ti = in.ti;

    // ---- operands
    // the state before the chunk, rows as A fragments, and its squared norm
    bf16x8 Hf[NF];
    float hn2 = 0.0f;
#pragma unroll
    for (int fo = 0; fo < NF; ++fo) {
#pragma unroll
        for (int e = 0; e < 4; ++e) hn2 += in.h[fo][0][e] * in.h[fo][0][e] + in.h[fo][1][e] * in.h[fo][1][e];
        Hf[fo] = pack8(in.h[fo][0], in.h[fo][1]);
    }
    hn2 = wave_sum(hn2);
    const bf16x8 qB = in.qB;
    // decay mask of Section 4.2.1 (log-space form of Appendix B.2, base 2) with the write gate folded in:
    // m[j,c] = 2^(G_c - G_j) beta_j for j <= c; lane element (js, r) <-> key j = 16 js + 4 kg + r
    const float Gc = Gtab[c_local];
    float zeta = exp2f(Gc);
    const float beta_c = Btab[c_local];
    f32x4 mreg[NJ];
#pragma unroll
    for (int js = 0; js < NJ; ++js) {
        const f32x4 Gj = *(const f32x4 *)(Gtab + 16 * js + 4 * kg), bj = *(const f32x4 *)(Btab + 16 * js + 4 * kg);
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int j = 16 * js + 4 * kg + r;
            // hardware exp2: decays under 2^-126 are flushed to zero
            mreg[js][r] = (j <= c_local) ? __builtin_amdgcn_exp2f(Gc - Gj[r]) * bj[r] : 0.0f;
        }
    }
    // keys: rows as A fragments (products K x), columns as A fragments (products K^T p), this lane's own key as B
    bf16x8 kA[NJ], kT[NF][NKS];
#pragma unroll
    for (int js = 0; js < NJ; ++js) kA[js] = row_in_slot_order(rows + (16 * js + n) * kRow, kg);
#pragma unroll
    for (int fo = 0; fo < NF; ++fo)
#pragma unroll
        for (int ks = 0; ks < NKS; ++ks) kT[fo][ks] = keys_in_slot_order(rows, ks, kg, 16 * fo + n);
    const bf16x8 kB = kA[TT];                  // (row 16 TT + n: the same fragment read as a column of the B operand)

    // ---- chunk-wise Frobenius norm (Section 4.2.1, the double sum folded by M[i,c] M[j,c] = M[j,c]^2 M[i,j]):
    //   ||H_c||^2 = zeta_c^2 ||H_[n]||^2 + sum_{j<=c} m[j,c]^2 w_j,
    //   w_j = 2 (zeta_j k_j^T H_[n] k_j + sum_{i<j} m[i,j] G_ij^2) / beta_j + G_jj^2   (G = K K^T; w_j = 0 for beta_j = 0)
    {
        f32x4 kc[2];
        unpack8(kB, kc[0], kc[1]);
        float a_part = 0.0f;
#pragma unroll
        for (int fo = 0; fo < NF; ++fo) {
            const f32x4 hk = mma16(Hf[fo], kB, zero4());
#pragma unroll
            for (int r = 0; r < 4; ++r) a_part += hk[r] * kc[fo][r];
        }
        float b_part = 0.0f, d_part = 0.0f;
#pragma unroll
        for (int js = 0; js < NJ; ++js) {
            const f32x4 G = mma16(kA[js], kB, zero4());
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                b_part += mreg[js][r] * (G[r] * G[r]);
                if (js == TT && 4 * kg + r == n) d_part = G[r] * G[r];
            }
        }
        a_part = sum_over_kg(a_part);
        b_part = sum_over_kg(b_part);
        d_part = sum_over_kg(d_part);
        b_part -= beta_c * d_part;             // the sum runs over i < c: the diagonal term (m[c,c] = beta_c) is taken out
        const float wc = beta_c > 0.0f ? 2.0f * (zeta * a_part + b_part) / beta_c + d_part : 0.0f;
        if (kg == 0) Wtab[c_local] = wc;
    }
    __syncthreads();                           // every wave of the workgroup comes through here, whatever its TT
    float fro;
    {
        float f = 0.0f;
#pragma unroll
        for (int js = 0; js < NJ; ++js) {
            const f32x4 wv = *(const f32x4 *)(Wtab + 16 * js + 4 * kg);
#pragma unroll
            for (int r = 0; r < 4; ++r) f += mreg[js][r] * mreg[js][r] * wv[r];
        }
        f = sum_over_kg(f);
        fro = sqrtf(fmaxf(zeta * zeta * hn2 + f, 0.0f));
    }
    if (a.fro_out && valid && kg == 0) a.fro_out[ti] = fro;
    float lam = a.lambda ? in.lam : a.lambda_scale * fro;                // Section 4.1: lambda_t = a ||H_t||_F
    if (!valid) lam = 1.0f;

    // ---- Algorithm 1 in residual form; Section 4.1: L = ||H_t||_F + lambda_t, mu = lambda_t
    const float L = fro + lam, mu = lam;
    const float rcp = __builtin_amdgcn_rcpf(L + mu);
    const float s0 = 2.0f * rcp;
    const float rho = (L - mu) * rcp, rho2 = rho * rho;
    zeta = fmaxf(zeta, kMinZeta);
    const float rz = 1.0f / zeta;
#pragma unroll
    for (int js = 0; js < NJ; ++js) mreg[js] *= rz;
    f32x4 xi[NF], dl[NF], gn[NF];
    {
        f32x4 qv[2];
        unpack8(qB, qv[0], qv[1]);
#pragma unroll
        for (int fo = 0; fo < NF; ++fo)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const float qe = valid ? qv[fo][r] : 0.0f;
                xi[fo][r] = 0.0f;
                dl[fo][r] = s0 * qe;
                gn[fo][r] = -qe * rz;
            }
    }
    float omega = 2.0f;
    for (int it = 0; it < a.n_iter; ++it) {
        omega = 4.0f * __builtin_amdgcn_rcpf(4.0f - rho2 * omega);      // weight schedule
        const float cm = omega - 1.0f, ncs = -omega * s0 * zeta, ncl = -omega * s0 * lam;
        const bf16x8 dB = pack8(dl[0], NF > 1 ? dl[NF - 1] : zero4());
        f32x4 P[2 * NKS];                      // masked key products; a key tile beyond the token tile counts as zero
#pragma unroll
        for (int js = NJ; js < 2 * NKS; ++js) P[js] = zero4();
#pragma unroll
        for (int js = 0; js < NJ; ++js) P[js] = mma16(kA[js], dB, zero4()) * mreg[js];
#pragma unroll
        for (int fo = 0; fo < NF; ++fo) {
            gn[fo] = mma16(Hf[fo], dB, gn[fo]);
#pragma unroll
            for (int ks = 0; ks < NKS; ++ks) gn[fo] = mma16(kT[fo][ks], pack8(P[2 * ks], P[2 * ks + 1]), gn[fo]);
        }
#pragma unroll
        for (int fo = 0; fo < NF; ++fo) {
            xi[fo] += dl[fo];
            dl[fo] = cm * dl[fo] + ncs * gn[fo] + ncl * xi[fo];
        }
    }
    f32x4 x[NF];
#pragma unroll
    for (int fo = 0; fo < NF; ++fo) x[fo] = xi[fo] + dl[fo];
    if (a.xhat_out && valid) {
        float *z = a.xhat_out + ti * a.xhat_row;
#pragma unroll
        for (int fo = 0; fo < NF; ++fo) {
            *(f32x4 *)(z + 16 * fo + 4 * kg) = x[fo];
            if (a.xhat_zero_upper) *(f32x4 *)(z + kDs + 16 * fo + 4 * kg) = zero4();   // (a reader of 64 stored features)
        }
    }
    if constexpr (WITH_U) {
        // ---- readout y_c = zeta_c U_[n] x_c + sum_{j<=c} m[j,c] v_j (k_j . x_c), x = alpha xhat + (1 - alpha) q
        // (Section 4.3), formed with the mask divided by zeta_c and multiplied by zeta_c at the end
        if (a.alpha) {
            const float al = valid ? a.alpha[ti] : 1.0f;
            f32x4 qv[2];
            unpack8(qB, qv[0], qv[1]);
#pragma unroll
            for (int fo = 0; fo < NF; ++fo)
#pragma unroll
                for (int r = 0; r < 4; ++r) x[fo][r] = al * x[fo][r] + (1.0f - al) * (valid ? qv[fo][r] : 0.0f);
        }
        bf16x8 xv, xr;
        split8(x[0], NF > 1 ? x[NF - 1] : zero4(), xv, xr);
        f32x4 P[2 * NKS];
#pragma unroll
        for (int js = NJ; js < 2 * NKS; ++js) P[js] = zero4();
#pragma unroll
        for (int js = 0; js < NJ; ++js) P[js] = mma16(kA[js], xr, mma16(kA[js], xv, zero4())) * mreg[js];
        const float *Un = a.sU + unit * (D * D);
        const int64_t orow = in.row;
#pragma unroll
        for (int fo = 0; fo < NF; ++fo) {
            f32x4 ulo, uhi;
            state_row_runs<D>(Un, fo, n, kg, ulo, uhi);
            bf16x8 Uv, Ur;
            split8(ulo, uhi, Uv, Ur);
            f32x4 y = mma16(Uv, xr, mma16(Ur, xv, mma16(Uv, xv, zero4())));
#pragma unroll
            for (int ks = 0; ks < NKS; ++ks)
                y = mma16(keys_in_slot_order(vrows, ks, kg, 16 * fo + n), pack8(P[2 * ks], P[2 * ks + 1]), y);
            y *= zeta;
            if (valid) IOBF16::store4(a.o, orow + 16 * fo + 4 * kg, y[0], y[1], y[2], y[3]);
        }
    }
}

}  // namespace

// (the occupancy bound keeps the register budget at 128, within which the matrix instructions write plain vector
// registers; with the default budget of 512 the compiler gives them the accumulation file and a third of the pass
// loop is moves between the two files)
template <bool WITH_U, int D>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(4, 4))) void small_solve_kernel(SmallArgs a)
{
    __shared__ __attribute__((aligned(16))) uint16_t s_rows[64 * kRow];
    __shared__ __attribute__((aligned(16))) uint16_t s_vrows[WITH_U ? 64 * kRow : 8];
    __shared__ __attribute__((aligned(16))) float s_G[64], s_B[64], s_W[64];
    const int lane = threadIdx.x & 63;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    // consecutive workgroups: the same chunk of consecutive pairs (adjacent memory in the [B,T,H,d] layout)
    const int pair = blockIdx.x % a.n_pairs, chunk = blockIdx.x / a.n_pairs;
    const int b = pair / a.H, h = pair % a.H;
    const int tok0 = chunk * kChunk;
    stage_rows(a, a.k, s_rows, b, h, tok0, threadIdx.x, 256);
    if constexpr (WITH_U) stage_rows(a, a.v, s_vrows, b, h, tok0, threadIdx.x, 256);
    const TileInputs in = fetch_tile_inputs<D>(a, pair, chunk, w, lane);
    if (w == 0) {
        const int64_t gi = (b * (int64_t)a.T + min(tok0 + lane, a.T - 1)) * a.H + h;
        s_G[lane] = wave_inclusive_scan(tok0 + lane < a.T ? log2_gate(a.gate[gi]) : 0.0f, lane);
        s_B[lane] = a.beta ? a.beta[gi] : 1.0f;
    }
    __syncthreads();
    if (tok0 + 16 * w >= a.T) {                // none of this wave's tokens exists (the sequence's last chunk):
        __syncthreads();                       // the barrier that the other waves pass inside their tile's work
        return;
    }
    const int64_t unit = pair * (int64_t)a.n_chunks + chunk;
    switch (w) {
    case 0: small_solve_tile<0, WITH_U, D>(a, in, s_rows, s_vrows, s_G, s_B, s_W, unit, lane); break;
    case 1: small_solve_tile<1, WITH_U, D>(a, in, s_rows, s_vrows, s_G, s_B, s_W, unit, lane); break;
    case 2: small_solve_tile<2, WITH_U, D>(a, in, s_rows, s_vrows, s_G, s_B, s_W, unit, lane); break;
    default: small_solve_tile<3, WITH_U, D>(a, in, s_rows, s_vrows, s_G, s_B, s_W, unit, lane); break;
    }
}

namespace {
size_t state_array_bytes(int n_pairs, int n_chunks, int d)
{
    return ((size_t)n_pairs * n_chunks * d * d * sizeof(float) + 255) & ~(size_t)255;
}
template <bool WITH_U, int D>
void launch_all(const SmallArgs &a, hipStream_t stream)
{
    const int64_t n_units = (int64_t)a.n_pairs * a.n_chunks;
    hipLaunchKernelGGL((small_chunk_delta_kernel<WITH_U, D>), dim3((unsigned)((n_units + 3) / 4)), dim3(256), 0, stream, a);
    hipLaunchKernelGGL((small_state_scan_kernel<WITH_U, D>), dim3((unsigned)a.n_pairs), dim3(D * D / 4), 0, stream, a);
    hipLaunchKernelGGL((small_solve_kernel<WITH_U, D>), dim3((unsigned)n_units), dim3(256), 0, stream, a);
}
}  // namespace

// d: 16 or 32, the head dimension (32 for the solve of latent sketching)
size_t small_dim_workspace_bytes(int n_pairs, int n_chunks, int d, bool with_readout)
{
    const size_t decays = ((size_t)n_pairs * n_chunks * sizeof(float) + 255) & ~(size_t)255;
    return (with_readout ? 4 : 2) * state_array_bytes(n_pairs, n_chunks, d) + decays;
}

// `workspace`: small_dim_workspace_bytes(n_pairs, n_chunks, a.d, a.v != nullptr) bytes, 256-byte aligned.
hipError_t launch_small_dim_forward(SmallArgs a, void *workspace, hipStream_t stream)
{
    if (a.n_pairs < 1 || a.n_chunks < 1 || a.T < 1 || (a.d != 16 && a.d != 32)) return hipErrorInvalidValue;
    if ((int64_t)a.n_pairs * a.n_chunks > 0x7fffffff / 4) return hipErrorInvalidValue;
    const bool with_u = a.v != nullptr;
    if (with_u != (a.o != nullptr)) return hipErrorInvalidValue;
    if (!with_u && (a.alpha || a.U_init || a.U_final || a.d != 32)) return hipErrorInvalidValue;
    const size_t per_array = state_array_bytes(a.n_pairs, a.n_chunks, a.d);
    unsigned char *ws = (unsigned char *)workspace;
    a.dH = (float *)ws;
    a.sH = (float *)(ws + per_array);
    a.dU = with_u ? (float *)(ws + 2 * per_array) : nullptr;
    a.sU = with_u ? (float *)(ws + 3 * per_array) : nullptr;
    a.chunk_log2_decay = (float *)(ws + (with_u ? 4 : 2) * per_array);
    if (!with_u) launch_all<false, 32>(a, stream);
    else if (a.d == 32) launch_all<true, 32>(a, stream);
    else launch_all<true, 16>(a, stream);
    return hipGetLastError();
}

}  // namespace gka
