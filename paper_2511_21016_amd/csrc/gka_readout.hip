// Gated-linear-attention readout y_t = U_t q_t, U_t = gamma_t U_{t-1} + beta_t v_t k_t^T, with the state kept in
// registers: the reverse recurrences of the backward pass (Section 4.2.2, Eq. (Ai) and its counterpart for U) and its
// plain forward readouts (U_t^T dy_t, H_t xhat_t, H_t k_t) are all of this form. Unlike the forward pass of the layer
// there is no solve between the state and its readout, so nothing forces the chunk states through memory: one
// workgroup walks a segment of a pair's chunks, as the state pass does, and produces the chunk's outputs on the way,
//   y_c = zeta_c U_[n] q_c + sum_{s<=c} M[s,c] beta_s v_s (k_s . q_c)          (chunk-wise form, Section 4.2.1),
// then advances the state. Segment start states come from a first launch of the same kernel that only accumulates
// (SUMMARY), exactly as in the state pass. bf16 tensors and operands, d = 128 or 64. QLO: q is given as a bf16 value
// and a bf16 remainder (q + q_lo), for a q that was computed in float32 (latent sketching's projected solution).
//
// Layout. Wave w owns the 32 v-features 32w .. 32w+31 of U for all k-features: accumulator tile jb holds
// U[32w + n][32jb + kidx(r, g)] on lane (n, g), register r. In that layout a tile converts in place into the A operand
// of (U q): no transposition, the contraction index is enumerated in kidx order on both operands. All products have
// tokens on the output lanes (the layer's token-per-lane layout), so a token's decay is a per-lane scalar.
// With `reverse` the kernel walks the sequence backwards: token tau of its walk is token T-1-tau of the tensors, and
// gamma'_tau = gamma_{T-tau} (gamma'_0 multiplies a zero state), which is the recurrence of Eq. (Ai).
#include "gka_device.hpp"
#include "gka_kernels.hpp"

namespace gka {

namespace {

typedef MmaBF16 MMA;
typedef MMA::frag frag;

// DK: features of q and k; DV: features of v and of the output (U is DV x DK). DK = DV for the recurrences of the
// backward pass; DK = 64, DV = 128 for the readout of latent sketching in the sketched space.
template <int DK, int DV>
struct ReadoutShape {
    static constexpr int NB = DV / 32;             // 32-blocks of the v-features = waves
    static constexpr int NBK = DK / 32;            // 32-blocks of the k-features = state tiles per wave
    static constexpr int NT = NB * 64;             // threads
    static constexpr int RSQ = DK + 8;             // q rows: read along the row, two 8-byte runs per lane
    static constexpr int RSK = DK + 16;            // k and v rows: transpose reads (rows 32 bytes apart modulo 256)
    static constexpr int RSV = DV + 16;
    static constexpr int PK = kChunk * DK / 8 / NT;   // 16-byte pieces of a chunk's k (or bf16 q) rows per thread
    static constexpr int PV = kChunk * DV / 8 / NT;   // ... of its v rows
    static constexpr int PQ32 = kChunk * DK / 4 / NT; // ... of float32 q rows
    static constexpr size_t q_elems = (size_t)kChunk * RSQ;
    static constexpr size_t k_elems = (size_t)kChunk * RSK;
    static constexpr size_t v_elems = (size_t)kChunk * RSV;
    // masked P: three causal 32x32 tiles, two MFMA steps each; square states (the backward pass's recurrences) keep
    // the rounding remainder of P as a second set of fragments
    static constexpr bool kPrecise = DK == DV;
    static constexpr size_t p_frags = 3 * 2 * 64 * (kPrecise ? 2 : 1);
    static constexpr size_t tab_bytes = 3 * kChunk * sizeof(float);   // per-token G, state weight, beta of the chunk
    static constexpr size_t lds_bytes = (q_elems + k_elems + v_elems) * 2 + p_frags * sizeof(frag) + tab_bytes;
    static constexpr size_t lds_bytes_qlo = lds_bytes + q_elems * 2;   // with the remainder of q as a second tile
    static constexpr size_t lds_bytes_kvlo = lds_bytes + k_elems * 2;  // ... of k or v (square states: same size)
};

typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));

// Operand fragment whose 8 elements are two runs of 4 consecutive features of one row (cols j0.., j0+8..).
__device__ __forceinline__ frag row_runs(const uint16_t *row, int j0)
{
    const u32x2_t a = *(const u32x2_t *)(row + j0), b = *(const u32x2_t *)(row + j0 + 8);
    const u32x4_t u = {a[0], a[1], b[0], b[1]};
    return __builtin_bit_cast(frag, u);
}

struct PaddedTile {
    int rs;
    __device__ __forceinline__ int operator()(int row, int col) const { return row * rs + col; }
};

template <int DK, int DV>
__device__ __forceinline__ float *summary_tile(const ReadoutArgs &a, int pair, int sg, int w, int jb)
{
    return a.seg_buf + (((int64_t)(pair * a.n_segs + sg) * (DV / 32) + w) * (DK / 32) + jb) * 1024;
}

}  // namespace

// Waves per SIMD a variant is compiled for: two (256 registers each), but one (512 registers, half of them
// accumulation registers that the compiler uses as a second file) for the d = 128 variants with a second operand
// tensor, whose prefetch registers do not fit beside the state otherwise (they spilled 20-37 registers to memory).
constexpr int readout_waves_per_simd(int dk, bool summary, int qmode, int kvlo)
{
    return (dk == 128 && !summary && (qmode == 1 || kvlo != 0)) ? 1 : 2;
}

// QMODE: 0 q in bf16; 1 q as bf16 value + bf16 remainder (q_lo); 2 q in float32, split into value + remainder here.
// KVLO: 0 k and v as they are; 1 k comes with a remainder tensor (k_lo); 2 v does (v_lo). Not combined with QMODE != 0.
template <int DK, int DV, bool GATED, bool SUMMARY, int QMODE, int KVLO = 0>
__global__ __launch_bounds__(DV * 2)
    __attribute__((amdgpu_waves_per_eu(readout_waves_per_simd(DK, SUMMARY, QMODE, KVLO), readout_waves_per_simd(DK, SUMMARY, QMODE, KVLO))))
    void gla_readout_kernel(ReadoutArgs a)
{
    typedef ReadoutShape<DK, DV> SH;
    constexpr bool QLO = QMODE != 0, QF32 = QMODE == 2;
    constexpr bool KLO = KVLO == 1, VLO = KVLO == 2;
    static_assert(KVLO == 0 || (QMODE == 0 && DK == DV), "remainders of k / v: square states, plain q");
    // PRECISE: P and the weighted v rows enter their products as value + remainder, so that the outputs carry the
    // rounding of the tensors they are given and nothing else of that size: the gate gradient of the backward pass is
    // a long cumulative sum of differences of such outputs, and only errors common to all of them cancel in it
    constexpr bool PRECISE = SH::kPrecise;
    constexpr int NB = SH::NB, NBK = SH::NBK, NT = SH::NT, RSQ = SH::RSQ, RSK = SH::RSK, RSV = SH::RSV;
    constexpr int PK = SH::PK, PV = SH::PV, PQ = QF32 ? SH::PQ32 : SH::PK;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    uint16_t *sQ = (uint16_t *)smem;
    uint16_t *sK = sQ + SH::q_elems;
    uint16_t *sV = sK + SH::k_elems;
    frag *sP = (frag *)(sV + SH::v_elems);
    float *sG = (float *)(sP + SH::p_frags), *sW = sG + kChunk, *sB = sW + kChunk;
    uint16_t *sQ2 = (uint16_t *)(sB + kChunk);        // (QLO only)
    uint16_t *sKV2 = sQ2;                             // (KVLO only: the remainder rows of k or v, laid out like them)

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int n = lane & 31, g = lane >> 5;
    const int pair = blockIdx.x % a.n_pairs;
    const int seg = blockIdx.x / a.n_pairs;
    const int b = pair / a.H, h = pair % a.H;
    const int64_t base_v = (int64_t)b * a.stride_b + (int64_t)h * a.stride_h;            // v and the output
    const int64_t base_qk = (int64_t)b * a.qk_stride_b + (int64_t)h * a.qk_stride_h;    // q and k
    const int64_t gate_base = (int64_t)b * a.T * a.H + h;
    const int n_chunks = (a.T + kChunk - 1) / kChunk;
    const int chunk_begin = seg * a.seg_len;
    const int chunk_end = min(chunk_begin + a.seg_len, n_chunks);
    if (chunk_begin >= chunk_end) return;          // (whole workgroup)

    // token tau of the walk -> token of the tensors
    auto tensor_token = [&](int tau) {
        const int t = min(tau, a.T - 1);
        return a.reverse ? a.T - 1 - t : t;
    };

    // ---- state: start of the segment
    f32x16 acc[NBK];
#pragma unroll
    for (int jb = 0; jb < NBK; ++jb) {
        acc[jb] = zero16();
        if (!SUMMARY) {
            if (a.init_state) {
                // the caller's state before the first token of the walk (its first gate multiplies it), advanced over
                // the earlier segments below like a zero state
                const float *S0 = a.init_state + (int64_t)pair * DV * DK;
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int row = 32 * w + n, col = 32 * jb + kidx(r, g);
                    acc[jb][r] = a.init_transposed ? S0[(int64_t)col * DV + row] : S0[(int64_t)row * DK + col];
                }
            }
            for (int sg = 0; sg < seg; ++sg) {
                const float decay = exp2f(a.seg_logdecay[pair * a.n_segs + sg]);
                if (DK == DV && a.seg_mode == 2) {
                    // summaries of the transposed recurrence (k and v exchanged), left by the readout before this one:
                    // U[32w + n][32jb + kidx(r, g)] is its element [32jb + kidx(r, g)][32w + n], i.e. tile (jb, w),
                    // lane (kidx(r, g), g'), register r' with kidx(r', g') = n
                    const float *t = summary_tile<DK, DV>(a, pair, sg, jb, w);
                    const int gp = (n >> 2) & 1, rp = 4 * (n >> 3) + (n & 3);
#pragma unroll
                    for (int r = 0; r < 16; ++r) acc[jb][r] = decay * acc[jb][r] + t[rp * 64 + 32 * gp + kidx(r, g)];
                } else {
                    const float *t = summary_tile<DK, DV>(a, pair, sg, w, jb);
#pragma unroll
                    for (int r = 0; r < 16; ++r) acc[jb][r] = decay * acc[jb][r] + t[r * 64 + lane];
                }
            }
        }
    }

    // ---- rows of a chunk: global -> registers (one chunk ahead) -> LDS
    struct Rows {
        u32x4_t q[PQ], k[PK], v[PV], q2[QMODE == 1 ? PK : 1], kv2[KVLO != 0 ? PK : 1];
        float gate, beta;
    };
    auto fetch = [&](Rows &f, int c) {
#pragma unroll
        for (int i = 0; i < PK; ++i) {
            const int piece = i * NT + tid;
            const int64_t off = base_qk + (int64_t)tensor_token(c * kChunk + piece / (DK / 8)) * a.qk_stride_t +
                                8 * (piece % (DK / 8));
            if (!SUMMARY && !QF32) f.q[i] = *(const u32x4_t *)((const uint16_t *)a.q + off);
            if (QMODE == 1) f.q2[i] = *(const u32x4_t *)((const uint16_t *)a.q_lo + off);
            f.k[i] = *(const u32x4_t *)((const uint16_t *)a.k + off);
            if (KLO) f.kv2[i] = *(const u32x4_t *)((const uint16_t *)a.k_lo + off);
        }
        if (QF32) {
#pragma unroll
            for (int i = 0; i < PQ; ++i) {
                const int piece = i * NT + tid;
                const int64_t off = base_qk + (int64_t)tensor_token(c * kChunk + piece / (DK / 4)) * a.qk_stride_t +
                                    4 * (piece % (DK / 4));
                f.q[i] = *(const u32x4_t *)((const float *)a.q + off);
            }
        }
#pragma unroll
        for (int i = 0; i < PV; ++i) {
            const int piece = i * NT + tid;
            const int64_t off = base_v + (int64_t)tensor_token(c * kChunk + piece / (DV / 8)) * a.stride_t +
                                8 * (piece % (DV / 8));
            f.v[i] = *(const u32x4_t *)((const uint16_t *)a.v + off);
            if (VLO) f.kv2[i] = *(const u32x4_t *)((const uint16_t *)a.v_lo + off);
        }
        const int tau = min(c * kChunk + lane, a.T - 1);
        if (a.reverse) f.gate = tau == 0 ? 1.0f : a.gate[gate_base + (int64_t)(a.T - tau) * a.H];
        else f.gate = a.gate[gate_base + (int64_t)tau * a.H];
        f.beta = 1.0f;
        if (GATED) f.beta = a.beta[gate_base + (int64_t)tensor_token(tau) * a.H];
    };
    auto stage = [&](const Rows &f) {
#pragma unroll
        for (int i = 0; i < PK; ++i) {
            const int piece = i * NT + tid;
            const int row = piece / (DK / 8), col = 8 * (piece % (DK / 8));
            if (!SUMMARY && !QF32) *(u32x4_t *)(sQ + row * RSQ + col) = f.q[i];
            if (QMODE == 1) *(u32x4_t *)(sQ2 + row * RSQ + col) = f.q2[i];
            *(u32x4_t *)(sK + row * RSK + col) = f.k[i];
            if (KLO) *(u32x4_t *)(sKV2 + row * RSK + col) = f.kv2[i];
        }
        if (QF32) {
#pragma unroll
            for (int i = 0; i < PQ; ++i) {
                const int piece = i * NT + tid;
                const int row = piece / (DK / 4), col = 4 * (piece % (DK / 4));
                const f32x4 x = __builtin_bit_cast(f32x4, f.q[i]);
                float lo[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) lo[e] = x[e] - bf16_bits_to_f32(f32_to_bf16_bits(x[e]));
                MMA::store4(sQ + row * RSQ + col, x);
                MMA::store4(sQ2 + row * RSQ + col, f32x4{lo[0], lo[1], lo[2], lo[3]});
            }
        }
#pragma unroll
        for (int i = 0; i < PV; ++i) {
            const int piece = i * NT + tid;
            const int row = piece / (DV / 8), col = 8 * (piece % (DV / 8));
            *(u32x4_t *)(sV + row * RSV + col) = f.v[i];
            if (VLO) *(u32x4_t *)(sKV2 + row * RSV + col) = f.kv2[i];
        }
    };

    const int sub16 = 16 * ((lane >> 4) & 1);      // this lane's half of a 32-block in transpose reads
    float Gseg = 0.0f;
    Rows rows;
    fetch(rows, chunk_begin);
    for (int c = chunk_begin; c < chunk_end; ++c) {
        // ---- decays of the chunk (every wave for itself): lane j holds token j
        const bool valid = c * kChunk + lane < a.T;
        const float lg = valid ? log2_gate(rows.gate) : 0.0f;
        const float G = wave_inclusive_scan(lg, lane);
        const float Gtot = lane_value(G, 63);
        Gseg += Gtot;
        const float bj = GATED ? rows.beta : 1.0f;
        const float wj = valid ? exp2f(Gtot - G) * bj : 0.0f;      // weight of token j in the state after the chunk
        const float zetaC = exp2f(Gtot);
        lds_barrier();                             // the previous chunk's tiles have been read
        stage(rows);
        if (w == 0) {                              // per-token scalars of the chunk, read back in fragment order
            sG[lane] = G;
            sW[lane] = wj;
            if (GATED) sB[lane] = bj;
        }
        if (c + 1 < chunk_end) fetch(rows, c + 1);
        lds_barrier();                             // (no wait for the rows in flight)

        // V^T fragments, tokens of step (sb, h2) in kidx order: runs at 32 sb + 16 h2 + 4 g and 8 further
        frag vt[2][2], vt2[2][2];                  // (vt2: the remainder rows, VLO only)
#pragma unroll
        for (int sb = 0; sb < 2; ++sb)
#pragma unroll
            for (int h2 = 0; h2 < 2; ++h2) {
                const int t0 = 32 * sb + 16 * h2 + 4 * g;
                vt[sb][h2] = gather_transposed_bf16(sV, PaddedTile{RSV}, 32 * w + sub16, lane, t0, t0 + 8);
                if (VLO) vt2[sb][h2] = gather_transposed_bf16(sKV2, PaddedTile{RSV}, 32 * w + sub16, lane, t0, t0 + 8);
            }

        if (!SUMMARY) {
            // ---- P = K Q^T on the causal tiles (key block sb, token block tb), one tile per wave, masked and rounded
#pragma unroll
            for (int tile = 0; tile < 3; ++tile) {
                if (tile % NB != w) continue;      // (wave-uniform)
                const int sb = tile == 2 ? 1 : 0, tb = tile == 0 ? 0 : 1;
                f32x16 pacc = zero16();
                const uint16_t *krow = sK + (32 * sb + n) * RSK, *qrow = sQ + (32 * tb + n) * RSQ;
#pragma unroll
                for (int st = 0; st < 2 * NBK; ++st) {
                    const frag kf = row_runs(krow, 16 * st + 4 * g);
                    pacc = MMA::mma(kf, row_runs(qrow, 16 * st + 4 * g), pacc);
                    if (KLO)
                        pacc = MMA::mma(row_runs(sKV2 + (32 * sb + n) * RSK, 16 * st + 4 * g),
                                        row_runs(qrow, 16 * st + 4 * g), pacc);
                    if (QLO) pacc = MMA::mma(kf, row_runs(sQ2 + (32 * tb + n) * RSQ, 16 * st + 4 * g), pacc);
                }
                // M[s,t] beta_s = exp2(G_t - G_s) beta_s for s <= t (Appendix B.2, base 2)
                const float Gt = __shfl(G, 32 * tb + n, 64);
                float pm[16];
#pragma unroll
                for (int q4 = 0; q4 < 4; ++q4) {
                    // registers 4 q4 .. 4 q4 + 3 hold keys 32 sb + 8 q4 + 4 g + (0..3)
                    const int s0 = 32 * sb + 8 * q4 + 4 * g;
                    const f32x4 Gs = *(const f32x4 *)(sG + s0);
                    f32x4 bs = {1.0f, 1.0f, 1.0f, 1.0f};
                    if (GATED) bs = *(const f32x4 *)(sB + s0);
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        // hardware exp2: decays under 2^-126 are flushed to zero
                        const float m = __builtin_amdgcn_exp2f(Gt - Gs[e]) * bs[e];
                        pm[4 * q4 + e] = (s0 + e <= 32 * tb + n) ? pacc[4 * q4 + e] * m : 0.0f;
                    }
                }
#pragma unroll
                for (int h2 = 0; h2 < 2; ++h2) {
                    const frag hi = MMA::pack(pm + 8 * h2);
                    sP[(tile * 2 + h2) * 64 + lane] = hi;
                    if (PRECISE) {
                        float back[8];
                        MMA::unpack(hi, back);
#pragma unroll
                        for (int e = 0; e < 8; ++e) back[e] = pm[8 * h2 + e] - back[e];
                        sP[(6 + tile * 2 + h2) * 64 + lane] = MMA::pack(back);
                    }
                }
            }

            // ---- zeta_t U_[n] q_t for both token blocks: the state's tiles are the A operand (value + remainder)
            f32x16 y[2] = {zero16(), zero16()};
#pragma unroll
            for (int jb = 0; jb < NBK; ++jb)
#pragma unroll
                for (int hh = 0; hh < 2; ++hh) {
                    float hi_f[8], lo_f[8];
#pragma unroll
                    for (int e = 0; e < 8; ++e) hi_f[e] = acc[jb][8 * hh + e];
                    const frag uhi = MMA::pack(hi_f);
                    MMA::unpack(uhi, lo_f);
#pragma unroll
                    for (int e = 0; e < 8; ++e) lo_f[e] = hi_f[e] - lo_f[e];
                    const frag ulo = MMA::pack(lo_f);
#pragma unroll
                    for (int tb = 0; tb < 2; ++tb) {
                        const frag qf = row_runs(sQ + (32 * tb + n) * RSQ, 32 * jb + 16 * hh + 4 * g);
                        y[tb] = MMA::mma(uhi, qf, y[tb]);
                        y[tb] = MMA::mma(ulo, qf, y[tb]);
                        if (QLO)
                            y[tb] = MMA::mma(uhi, row_runs(sQ2 + (32 * tb + n) * RSQ, 32 * jb + 16 * hh + 4 * g), y[tb]);
                    }
                }
#pragma unroll
            for (int tb = 0; tb < 2; ++tb) {
                const float zt = exp2f(__shfl(G, 32 * tb + n, 64));
#pragma unroll
                for (int r = 0; r < 16; ++r) y[tb][r] *= zt;
            }
            lds_barrier();                         // P is visible
            // ---- + sum_s V[s] P[s,t] over the causal tiles
#pragma unroll
            for (int tile = 0; tile < 3; ++tile) {
                const int sb = tile == 2 ? 1 : 0, tb = tile == 0 ? 0 : 1;
#pragma unroll
                for (int h2 = 0; h2 < 2; ++h2) {
                    y[tb] = MMA::mma(vt[sb][h2], sP[(tile * 2 + h2) * 64 + lane], y[tb]);
                    if (PRECISE) y[tb] = MMA::mma(vt[sb][h2], sP[(6 + tile * 2 + h2) * 64 + lane], y[tb]);
                    if (VLO) y[tb] = MMA::mma(vt2[sb][h2], sP[(tile * 2 + h2) * 64 + lane], y[tb]);
                }
            }
            // ---- store: lane (n, g) holds features 32 w + kidx(r, g) of token 32 tb + n
#pragma unroll
            for (int tb = 0; tb < 2; ++tb) {
                const int tau = c * kChunk + 32 * tb + n;
                if (tau < a.T) {
                    const int64_t off = base_v + (int64_t)tensor_token(tau) * a.stride_t + 32 * w + 4 * g;
#pragma unroll
                    for (int q4 = 0; q4 < 4; ++q4) {
                        if (a.o_f32)
                            *(f32x4 *)(a.o_f32 + off + 8 * q4) =
                                f32x4{y[tb][4 * q4], y[tb][4 * q4 + 1], y[tb][4 * q4 + 2], y[tb][4 * q4 + 3]};
                        else
                            IOBF16::store4(a.o, off + 8 * q4, y[tb][4 * q4], y[tb][4 * q4 + 1], y[tb][4 * q4 + 2],
                                           y[tb][4 * q4 + 3]);
                    }
                }
            }
        }

        // ---- U <- zeta_C U + sum_s w_s v_s k_s^T: tile jb gets K^T (block jb) times the weighted V^T fragments
        frag vw[2][2], vwlo[2][2];
#pragma unroll
        for (int sb = 0; sb < 2; ++sb)
#pragma unroll
            for (int h2 = 0; h2 < 2; ++h2) {
                float x[8];
                MMA::unpack(vt[sb][h2], x);
                if (VLO) {
                    float x2[8];
                    MMA::unpack(vt2[sb][h2], x2);
#pragma unroll
                    for (int e = 0; e < 8; ++e) x[e] += x2[e];
                }
                const int t0 = 32 * sb + 16 * h2 + 4 * g;
                const f32x4 w0 = *(const f32x4 *)(sW + t0), w1 = *(const f32x4 *)(sW + t0 + 8);
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    x[e] *= w0[e];
                    x[4 + e] *= w1[e];
                }
                vw[sb][h2] = MMA::pack(x);
                if (PRECISE) {
                    float back[8];
                    MMA::unpack(vw[sb][h2], back);
#pragma unroll
                    for (int e = 0; e < 8; ++e) back[e] = x[e] - back[e];
                    vwlo[sb][h2] = MMA::pack(back);
                }
            }
#pragma unroll
        for (int jb = 0; jb < NBK; ++jb) {
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[jb][r] *= zetaC;
#pragma unroll
            for (int sb = 0; sb < 2; ++sb)
#pragma unroll
                for (int h2 = 0; h2 < 2; ++h2) {
                    const int t0 = 32 * sb + 16 * h2 + 4 * g;
                    const frag kt = gather_transposed_bf16(sK, PaddedTile{RSK}, 32 * jb + sub16, lane, t0, t0 + 8);
                    acc[jb] = MMA::mma(kt, vw[sb][h2], acc[jb]);
                    if (PRECISE) acc[jb] = MMA::mma(kt, vwlo[sb][h2], acc[jb]);
                    if (KLO)
                        acc[jb] = MMA::mma(gather_transposed_bf16(sKV2, PaddedTile{RSK}, 32 * jb + sub16, lane, t0, t0 + 8),
                                           vw[sb][h2], acc[jb]);
                }
        }
    }

    if (!SUMMARY && a.final_state && seg == a.n_segs - 1) {
        // the state after the last token of the walk, row-major [DV][DK]
        float *S1 = a.final_state + (int64_t)pair * DV * DK;
#pragma unroll
        for (int jb = 0; jb < NBK; ++jb)
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4)
                *(f32x4 *)(S1 + (int64_t)(32 * w + n) * DK + 32 * jb + 8 * q4 + 4 * g) =
                    f32x4{acc[jb][4 * q4], acc[jb][4 * q4 + 1], acc[jb][4 * q4 + 2], acc[jb][4 * q4 + 3]};
    }
    if (SUMMARY) {
#pragma unroll
        for (int jb = 0; jb < NBK; ++jb) {
            float *t = summary_tile<DK, DV>(a, pair, seg, w, jb);
#pragma unroll
            for (int r = 0; r < 16; ++r) t[r * 64 + lane] = acc[jb][r];
        }
        if (tid == 0) a.seg_logdecay[pair * a.n_segs + seg] = Gseg;
    }
}

template <int DK, int DV, bool GATED, int QMODE, int KVLO = 0>
static hipError_t launch_readout_d(const ReadoutArgs &a0, hipStream_t stream)
{
    typedef ReadoutShape<DK, DV> SH;
    ReadoutArgs a = a0;
    constexpr size_t lds_sum = KVLO != 0 ? SH::lds_bytes_kvlo : SH::lds_bytes;
    constexpr size_t lds_main = QMODE != 0 ? SH::lds_bytes_qlo : lds_sum;
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void *)gla_readout_kernel<DK, DV, GATED, false, QMODE, KVLO>,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_main);
        if (e != hipSuccess) return e;
        e = hipFuncSetAttribute((const void *)gla_readout_kernel<DK, DV, GATED, true, 0, KVLO>,
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_sum);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    if (a.n_segs > 1 && a.seg_mode == 0) {
        // summaries of every segment but the last, each from a zero state
        hipLaunchKernelGGL((gla_readout_kernel<DK, DV, GATED, true, 0, KVLO>), dim3(a.n_pairs * (a.n_segs - 1)),
                           dim3(SH::NT), lds_sum, stream, a);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL((gla_readout_kernel<DK, DV, GATED, false, QMODE, KVLO>), dim3(a.n_pairs * a.n_segs), dim3(SH::NT),
                       lds_main, stream, a);
    return hipGetLastError();
}

template <int D>
static hipError_t launch_readout_square(const ReadoutArgs &a, hipStream_t stream)
{
    if (a.k_lo || a.v_lo) {
        // (the reverse recurrences of the backward pass: no write gate inside them)
        if (a.q_lo || a.beta || (a.k_lo && a.v_lo)) return hipErrorInvalidValue;
        return a.k_lo ? launch_readout_d<D, D, false, 0, 1>(a, stream) : launch_readout_d<D, D, false, 0, 2>(a, stream);
    }
    if (a.q_lo)
        return a.beta ? launch_readout_d<D, D, true, 1>(a, stream) : launch_readout_d<D, D, false, 1>(a, stream);
    return a.beta ? launch_readout_d<D, D, true, 0>(a, stream) : launch_readout_d<D, D, false, 0>(a, stream);
}

hipError_t launch_gla_readout(const ReadoutArgs &a, int dk, int dv, hipStream_t stream)
{
    if (a.q_is_f32) {                          // the sketched readout: float32 q, 64 or 32 sketched features, full v
        if ((dk != 64 && dk != 32) || dv != 128 || a.q_lo || a.k_lo || a.v_lo) return hipErrorInvalidValue;
        if (dk == 32)
            return a.beta ? launch_readout_d<32, 128, true, 2>(a, stream) : launch_readout_d<32, 128, false, 2>(a, stream);
        return a.beta ? launch_readout_d<64, 128, true, 2>(a, stream) : launch_readout_d<64, 128, false, 2>(a, stream);
    }
    if (dk != dv) return hipErrorInvalidValue;
    return dk == 128 ? launch_readout_square<128>(a, stream) : launch_readout_square<64>(a, stream);
}

size_t gla_readout_workspace_bytes(int n_pairs, int n_segs, int dk, int dv)
{
    return (size_t)n_pairs * n_segs * dk * dv * sizeof(float) + (size_t)n_pairs * n_segs * sizeof(float);
}

}  // namespace gka
