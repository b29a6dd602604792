// Whole forward pass of Eq. (CH) in one kernel for bf16 tensors and operands at d = 128: a workgroup walks a run
// of consecutive chunks of one (batch, head) pair with the states H and U in registers, so that no chunk state
// crosses HBM (Section 4.2.1 computes the initial state of every chunk first and then treats the chunks
// independently; here the state is advanced and used chunk by chunk instead).
//
// Tiles. Everything is built from the 16x16x32 bf16 MFMA. Lane l = 16 kg + n (n = 0..15, kg = 0..3) of a
// 16 x 16 accumulator tile holds rows 4 kg + r (r = 0..3) of column n. An operand fragment holds, per lane (n, kg),
// eight contraction values ("slots" p = 0..7) of row / column n. Two accumulator tiles (rows 16 a .., rows 16 b ..)
// of the same columns convert in place into one B fragment whose slot p stands for row 16 (p < 4 ? a : b) + 4 kg +
// p % 4; with a = 2 f, b = 2 f + 1 this is "fragment f" of a 128-vector: slot p <-> index 32 f + 16 (p / 4) + 4 kg +
// p % 4. Every A operand enumerates its contraction index in the same slot order, so vectors go from accumulators
// to operands without leaving their lanes.
//
// Roles. The workgroup has eight waves and handles two consecutive chunks (A, B) per iteration.
//   * State role (all waves): wave w owns columns 16 w .. 16 w + 15 of H (as H[16 jt + row][16 w + n], eight tiles)
//     and of U^T (U[16 w + n][16 jt + row]). It converts H to the bf16 A operand of the solve, advances H and U by a
//     chunk (S <- zeta_C S + sum_j w_j k_j a_j^T, the weights on its own B fragments), and reads out
//     zeta-free U_[n] xhat for all tokens of a chunk from its registers (rounded value + remainder of both operands).
//   * Solver role: four waves per chunk, each wave 16 tokens with all 128 features: chunk-wise Frobenius norm, all
//     passes of Algorithm 1 and the intra-chunk part of the readout run without any barrier, the iterate never
//     leaves the wave's registers.
//
// SPLIT variant (GKA_COMPUTE_BF16_SPLIT), for ill-conditioned systems: the two operands whose rounding the
// iteration amplifies, H_[n] and the update delta, enter their products as bf16 value + bf16 remainder
// (H delta ~ Hv dv + Hv dr + Hr dv, K delta = K dv + K dr), and so do the masked intra-chunk products P o M (with
// H_[n] = 0 and a handful of tokens they are all of H_c); everything else is as above. The remainder of H_[n] takes
// the place of the second chunk's H_[n] in LDS, so an iteration handles one chunk, solved by waves 0-3 (one per
// SIMD) while waves 4-7 only play their state role.
#include "gka_device.hpp"
#include "gka_kernels.hpp"

namespace gka {
namespace {

constexpr int kFusedThreads = 512;
constexpr int kD = 128;

// LDS map (bytes). Regions are reused along an iteration; see the phase list in fused_forward_kernel.
constexpr int kOffH = 0;            // [2 chunks] 32 KiB: H_[n] as A fragments [ft 8][fb 4][64 lanes]
                                    //   later: xhat as B fragments [ts 4][hi/lo 2][fb 4][64 lanes]
constexpr int kOffK = 65536;        // [2] 16 KiB: key rows as A fragments [js 4][fb 4][64]
                                    //   later (both halves): state part of the readout [ts 4][ft 8][64] float4
constexpr int kOffKT = 98304;       // [2] 16 KiB: keys transposed as A fragments [ft 8][jb 2][64]
constexpr int kOffR = 131072;       // [2] 16 KiB: row-major tile of k rows, later of v rows (64 x 256 B, swizzled)
constexpr int kLdsBytes = 163840;
// per-token scalars of the Frobenius phase and the partial norms of H_[n]: last KiB of the second row tile
constexpr int kOffTab = kOffR + 2 * 16384 - 1024;

typedef SwizzledRows<256, 2> Rows;

template <int I, int N, class F>
__device__ __forceinline__ void static_for(F &&f)
{
    if constexpr (I < N) {
        f(std::integral_constant<int, I>{});
        static_for<I + 1, N>(f);
    }
}

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
    float x[8];
    MmaBF16::unpack(f, x);
    lo = f32x4{x[0], x[1], x[2], x[3]};
    hi = f32x4{x[4], x[5], x[6], x[7]};
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

// U is needed only for the state part of the readout and its own update, once per iteration; in between it is
// parked in a scratch block of this workgroup in global memory (1 KiB per wave and tile, written and read by the same
// lanes), so that the passes have its registers.
constexpr int kParkStores = 8;           // vector-memory instructions of park_store (one 16-byte store per tile)
__device__ __forceinline__ void park_store(f32x4 *slot, const f32x4 (&acc)[kParkStores])
{
#pragma unroll
    for (int jt = 0; jt < kParkStores; ++jt) slot[jt * 64] = acc[jt];
}
__device__ __forceinline__ void park_load(const f32x4 *slot, f32x4 (&acc)[8])
{
#pragma unroll
    for (int jt = 0; jt < 8; ++jt) acc[jt] = slot[jt * 64];
}

struct Ctx {
    const FusedArgs &a;
    unsigned char *smem;
    int tid, lane, w, n, kg;
    int64_t base_bh, gate_base;
    int T_eff;                       // tokens at or beyond this index do not exist for this workgroup
    f32x4 *park;                     // this lane's place in the workgroup's scratch block
};

// Lane-derived fields from a copy of the lane index that the compiler cannot trace back: addresses formed from it
// are formed anew instead of being kept in registers (or spilled) across the code in between.
__device__ __forceinline__ void refresh_lane(Ctx &c)
{
    int lane_now = threadIdx.x & 63;
    asm volatile("" : "+v"(lane_now));
    c.lane = lane_now;
    c.tid = c.w * 64 + lane_now;
    c.n = lane_now & 15;
    c.kg = lane_now >> 4;
    c.park = (f32x4 *)c.a.park + ((int64_t)blockIdx.x * 8 + c.w) * (8 * 64) + lane_now;
}

__device__ __forceinline__ bf16x8 *lds_frags(const Ctx &c, int off) { return (bf16x8 *)(c.smem + off); }
__device__ __forceinline__ uint16_t *lds_rows(const Ctx &c, int g) { return (uint16_t *)(c.smem + kOffR + g * 16384); }

// Per-token scalars of a chunk travel from "lane j holds the value of token j" to fragment order through a small
// table in LDS that every wave keeps for itself (written and read back by the same wave: no barrier; as lane
// broadcasts the same reads cost an LDS round trip each, 8 per fragment). Slots of 64 floats.
__device__ __forceinline__ float *wave_table(const Ctx &c, int byte_off, int slot)
{
    return (float *)(c.smem + byte_off) + (c.w * 4 + slot) * 64;
}

// ---- state role ------------------------------------------------------------------------------------------------
// (Loops that run once per chunk are kept rolled where that costs little: the loop body of the kernel is executed
// once per iteration, straight through, so its size is paid in instruction fetches.)

// This wave's B fragments of a chunk update: rows of the tile (k or v) transposed, columns 16 w .., each token
// scaled by its weight (wtab: the weights of the chunk's 64 tokens, a slot of this wave's table).
template <class Layout = Rows>
__device__ __forceinline__ void own_weighted_frags(const Ctx &c, const uint16_t *rows, const float *wtab,
                                                   bf16x8 (&out)[2], Layout at = Layout())
{
#pragma unroll
    for (int st = 0; st < 2; ++st) {
        const int t0 = 32 * st + 4 * c.kg;
        const bf16x8 raw = gather_transposed_bf16(rows, at, 16 * c.w, c.lane, t0, t0 + 16);
        const f32x4 w0 = *(const f32x4 *)(wtab + t0), w1 = *(const f32x4 *)(wtab + t0 + 16);
        f32x4 lo, hi;
        unpack8(raw, lo, hi);
        out[st] = pack8(lo * w0, hi * w1);
    }
}

// S <- zeta_C S + sum_j w_j k_j a_j^T for this wave's eight tiles (A: transposed keys of chunk g from LDS)
__device__ __forceinline__ void advance_state(const Ctx &c, f32x4 (&acc)[8], int g, float zetaC, const bf16x8 (&wB)[2])
{
    const bf16x8 *sKT = lds_frags(c, kOffKT + g * 16384) + c.lane;
#pragma unroll
    for (int half = 0; half < 2; ++half) {
        bf16x8 a[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) a[i] = sKT[(half * 8 + i) * 64];
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const int jt = 4 * half + t;
            acc[jt] *= zetaC;
            acc[jt] = mma16(a[2 * t], wB[0], acc[jt]);
            acc[jt] = mma16(a[2 * t + 1], wB[1], acc[jt]);
        }
    }
}

// H_[n] as the A operand of the solve (by symmetry the accumulators are rows 16 w .. of H in slot order) and this
// wave's share of ||H_[n]||_F^2.
// SPLIT: the rounding remainder goes to the second chunk's place (32 KiB further).
template <bool SPLIT>
__device__ __forceinline__ float publish_H(const Ctx &c, const f32x4 (&accH)[8], int g)
{
    bf16x8 *sH = lds_frags(c, kOffH + g * 32768) + (c.w * 4) * 64 + c.lane;
    float ss = 0.0f;
#pragma unroll
    for (int fb = 0; fb < 4; ++fb) {
        if constexpr (SPLIT) {
            bf16x8 val, rem;
            split8(accH[2 * fb], accH[2 * fb + 1], val, rem);
            sH[fb * 64] = val;
            sH[2048 + fb * 64] = rem;
        } else {
            sH[fb * 64] = pack8(accH[2 * fb], accH[2 * fb + 1]);
        }
#pragma unroll
        for (int r = 0; r < 4; ++r) ss += accH[2 * fb][r] * accH[2 * fb][r] + accH[2 * fb + 1][r] * accH[2 * fb + 1][r];
    }
    return lane_value(wave_inclusive_scan(ss, c.lane), 63);      // (DPP moves: no LDS round trips)
}

// State part of the readout for all 64 tokens of chunk g: rows 16 w .. of U_[n] xhat, with U and xhat as rounded
// value + remainder (three products), to the exchange region at byte offset y_off as [ts][w][lane] float4. The
// fragments of the next token block are requested before the products of the current one.
__device__ __forceinline__ void readout_state(const Ctx &c, const f32x4 (&accU)[8], int g, int y_off)
{
    bf16x8 Uv[4], Ur[4];
#pragma unroll
    for (int fb = 0; fb < 4; ++fb) split8(accU[2 * fb], accU[2 * fb + 1], Uv[fb], Ur[fb]);
    const bf16x8 *sX = lds_frags(c, kOffH + g * 32768) + c.lane;
    f32x4 *sY = (f32x4 *)(c.smem + y_off) + c.w * 64 + c.lane;
    bf16x8 x[2][8];
#pragma unroll
    for (int i = 0; i < 8; ++i) x[0][i] = sX[i * 64];
#pragma unroll
    for (int ts = 0; ts < 4; ++ts) {
        const int cur = ts & 1;
        if (ts + 1 < 4) {
#pragma unroll
            for (int i = 0; i < 8; ++i) x[cur ^ 1][i] = sX[((ts + 1) * 8 + i) * 64];
        }
        f32x4 y0 = zero4(), y1 = zero4(), y2 = zero4();
#pragma unroll
        for (int fb = 0; fb < 4; ++fb) {
            y0 = mma16(Uv[fb], x[cur][fb], y0);
            y1 = mma16(Ur[fb], x[cur][fb], y1);
            y2 = mma16(Uv[fb], x[cur][4 + fb], y2);
        }
        sY[ts * 8 * 64] = y0 + (y1 + y2);
    }
}

// ---- solver role -----------------------------------------------------------------------------------------------
// A wave's tokens see the key blocks js <= ts of their chunk (16 keys each). Two instantiations cover the four token
// blocks: NJ = 2 key blocks for ts = 0, 1 and NJ = 4 for ts = 2, 3; a block beyond ts is all future keys, its mask is
// zero and it costs a few products (four instantiations would cost more in instruction fetches than they save).

// Smallest zeta_c by which a token's system is divided (see solve_tokens).
constexpr float kMinSolveZeta = 0x1p-60f;

struct Solver {
    f32x4 mreg[4];                   // decay mask M[j][c], key block js: rows j = 16 js + 4 kg + r (from the passes on: / zeta)
    f32x4 yi[8];                     // intra-chunk part of the readout (/ zeta)
    float zeta, fro;
    float beta;                      // write gate of this lane's token (1 without the variant)
    int tok;                         // this lane's token (global index)
    bool valid;
};

// LDS reads of the pass loop are assembly statements with their own counted waits: the compiler would order every
// LDS read it knows of behind the copies of the v rows into LDS that are in flight during the passes (a full wait for
// them), whichever part of LDS they fill. A register loaded this way must be awaited before it is used or reused.
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
template <int BYTE_OFFSET>
__device__ __forceinline__ void lds_read16_untracked(u32x4 &dst, uint32_t addr)
{
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(dst) : "v"(addr), "n"(BYTE_OFFSET) : "memory");
}
// at most N LDS operations issued after the read into x are still outstanding: x has landed
template <int N>
__device__ __forceinline__ void lds_await(u32x4 &x)
{
    asm volatile("s_waitcnt lgkmcnt(%1)" : "+v"(x) : "n"(N) : "memory");
}
__device__ __forceinline__ uint32_t lds_address(const void *p)
{
    return (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const void *)p;
}

template <int NJ, bool SPLIT>
struct PassPlan {
    // steps of the loop body, one A fragment each: the tile phase (8 tiles x (HP state + NJB intra fragments)), then
    // the key fragments of the next pass. SPLIT: the state fragments of a tile are the four of the value (each
    // multiplied with the value and with the remainder of delta) and the four of the remainder of H_[n]; a key fragment
    // is multiplied with both parts of delta.
    static constexpr int NJB = NJ / 2, NP = 4 * NJ, HP = SPLIT ? 8 : 4, PER_TILE = HP + NJB, NT = 8 * PER_TILE,
                         NS = NT + NP;
    static constexpr int base(int i) { return i >= NT ? 1 : (i % PER_TILE < HP ? 0 : 2); }
    static constexpr int off(int i)
    {
        if (i >= NT) return (((i - NT) % NJ) * 4 + (i - NT) / NJ) * 64;       // keys [js][fb], fb-major order
        const int t = i / PER_TILE, u = i % PER_TILE;
        if (u < 4) return (t * 4 + u) * 64;
        if (u < HP) return 2048 + (t * 4 + (u - 4)) * 64;                     // remainder of H_[n]: 32 KiB further
        return (t * 2 + (u - HP)) * 64;
    }
};

// (P o M) of key blocks 2 jb, 2 jb + 1 as a B fragment
__device__ __forceinline__ bf16x8 masked_frag(const f32x4 &P0, const f32x4 &P1, const f32x4 (&mreg)[4], int jb)
{
    return pack8(P0 * mreg[2 * jb], P1 * mreg[2 * jb + 1]);
}
// the same as rounded value + remainder
__device__ __forceinline__ void masked_frag_split(const f32x4 &P0, const f32x4 &P1, const f32x4 (&mreg)[4], int jb,
                                                  bf16x8 &val, bf16x8 &rem)
{
    split8(P0 * mreg[2 * jb], P1 * mreg[2 * jb + 1], val, rem);
}

// P[js] = K[js] x for the key blocks js < NJ, x given as B fragments
template <int NJ, int NX>
__device__ __forceinline__ void key_products(const bf16x8 *sK, const bf16x8 (&x)[NX][4], f32x4 (&P)[NJ], int lane)
{
#pragma unroll
    for (int js = 0; js < NJ; ++js) P[js] = zero4();
#pragma unroll
    for (int fb = 0; fb < 4; ++fb) {
        bf16x8 a[NJ];
#pragma unroll
        for (int js = 0; js < NJ; ++js) a[js] = sK[(js * 4 + fb) * 64 + lane];
        bf16x8 b[NX];
#pragma unroll
        for (int v = 0; v < NX; ++v) b[v] = x[v][fb];
#pragma unroll
        for (int js = 0; js < NJ; ++js)
#pragma unroll
            for (int v = 0; v < NX; ++v) P[js] = mma16(a[js], b[v], P[js]);
    }
}

// Algorithm 1 in residual form for the 16 tokens of this wave:
//   delta_i = (omega_i - 1) delta_{i-1} - (2 omega_i / (L + mu)) (g_{i-1} + lambda xi_{i-1}),  xi_i = xi_{i-1} + delta_i,
// with g_i = H_c xi_i - q accumulated over the passes (H_c delta = zeta_c H_[n] delta + K^T (M o (K delta)), Section
// 4.2.1), so that the rounded operand of every product is the shrinking update, not the iterate.
// The system of a token is taken divided by its zeta_c: g / zeta_c = H_[n] xi + K^T ((M / zeta_c) o (K xi)) - q / zeta_c
// is one chain of matrix products per feature tile, with no vector instruction between the state part and the
// intra-chunk part (the caller passes the mask divided by zeta_c; the iterate itself is not scaled).
// On entry: xi = xi_{-1} = 0, dl = delta_0 = xi_0, gn = -q / zeta_c; s0z = 2 zeta_c / (L + mu), s0lam = 2 lambda /
// (L + mu). On exit xi + dl is the result.
// The loop body is one straight line of MFMA steps, each with its A fragment requested kDepth steps ahead and a slice
// of the vector work behind it.
// `start_copies` is called once, after the last LDS read that the compiler knows of: it issues the copies into LDS
// that overlap the passes.
template <int NJ, bool SPLIT, class StartCopies>
__device__ __forceinline__ void cheb_passes(const bf16x8 *sH, const bf16x8 *sK, const bf16x8 *sKT, f32x4 (&xi)[8],
                                            f32x4 (&dl)[8], f32x4 (&gn)[8], const f32x4 (&mreg)[4], float s0z,
                                            float s0lam, float rho2, int n_iter, int lane,
                                            StartCopies start_copies)
{
    typedef PassPlan<NJ, SPLIT> PL;
    constexpr int NJB = PL::NJB, PER_TILE = PL::PER_TILE, NT = PL::NT, NS = PL::NS, HP = PL::HP;
    static_assert((2048 + 31 * 64 + 63) * 16 < 65536, "the offset field of an LDS read holds 16 bits");
    // A fragments in flight. The request of step i + kDepth goes into the register that step i has just freed, also
    // across the end of the loop body, so the depth divides the number of steps (48, 64).
    constexpr int kDepth = 4;
    static_assert(NS % kDepth == 0 && kDepth <= 15, "queue registers rotate with the loop; the LDS counter holds 15 operations");
    if (n_iter <= 0) {
        start_copies();
        return;
    }
    const uint32_t bases[3] = {lds_address(sH + lane), lds_address(sK + lane), lds_address(sKT + lane)};
    u32x4 q[kDepth];
    bf16x8 dB[4], dR[SPLIT ? 4 : 1];         // delta as B fragments: rounded value and (SPLIT) remainder
    f32x4 P[NJ];
    auto pack_delta = [&](auto fbc) {
        constexpr int fb = decltype(fbc)::value;
        if constexpr (SPLIT) split8(dl[2 * fb], dl[2 * fb + 1], dB[fb], dR[fb]);
        else dB[fb] = pack8(dl[2 * fb], dl[2 * fb + 1]);
    };
    static_for<0, 4>(pack_delta);
    if constexpr (SPLIT) {
        // key products of the first pass
        bf16x8 x[2][4] = {{dB[0], dB[1], dB[2], dB[3]}, {dR[0], dR[1], dR[2], dR[3]}};
        key_products<NJ, 2>(sK, x, P, lane);
    } else {
        bf16x8 x[1][4] = {{dB[0], dB[1], dB[2], dB[3]}};
        key_products<NJ, 1>(sK, x, P, lane);
    }
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    start_copies();
    static_for<0, kDepth>([&](auto step) {
        constexpr int i = decltype(step)::value;
        lds_read16_untracked<PL::off(i) * 16>(q[i], bases[PL::base(i)]);
    });
    float omega = 2.0f;
    // A SIMD runs one wave of each instantiation. The one with more products per pass gets the higher priority for
    // the first seven tenths of the passes, so that the two finish together (measured: with equal priorities the
    // lighter wave finishes a third earlier, with the priority held throughout it finishes a fifth later; alone on
    // its SIMD a wave runs at half the rate of the two together).
    constexpr bool kBoost = NJ == 2 && !SPLIT;           // (SPLIT: one solver wave per SIMD)
    if (kBoost) __builtin_amdgcn_s_setprio(1);
    const int prio_passes = n_iter / 2;
#pragma unroll 1
    for (int it = 0; it < n_iter; ++it) {
        asm volatile("" ::: "memory");
        if (kBoost && it == prio_passes) __builtin_amdgcn_s_setprio(0);
        omega = 4.0f * __builtin_amdgcn_rcpf(4.0f - rho2 * omega);           // weight schedule
        const float cm = omega - 1.0f, ncs = -omega * s0z, ncl = -omega * s0lam;
        bf16x8 pm[NJB], pmR[SPLIT ? NJB : 1];
        f32x4 tcm;
        auto mask_products = [&](auto jbc) {
            constexpr int jb = decltype(jbc)::value;
            if constexpr (SPLIT) masked_frag_split(P[2 * jb], P[2 * jb + 1], mreg, jb, pm[jb], pmR[jb]);
            else pm[jb] = masked_frag(P[2 * jb], P[2 * jb + 1], mreg, jb);
        };
        // Update of a tile's four elements as sixteen single instructions, op = 2 r + {0, 1}: xi += delta and
        // (omega - 1) delta, which need no product of this pass; then op = 8 + 2 r + {0, 1}: the two multiply-adds
        // of the new delta. They are dealt out evenly over the steps of the next tile.
        auto upd_op = [&](auto ftc, auto opc) {
            constexpr int ft = decltype(ftc)::value, op = decltype(opc)::value, r = (op & 7) >> 1;
            if constexpr (op < 8 && (op & 1) == 0) xi[ft][r] += dl[ft][r];
            if constexpr (op < 8 && (op & 1) == 1) tcm[r] = cm * dl[ft][r];
            if constexpr (op >= 8 && (op & 1) == 0) tcm[r] = __builtin_fmaf(ncs, gn[ft][r], tcm[r]);
            if constexpr (op >= 8 && (op & 1) == 1) dl[ft][r] = __builtin_fmaf(ncl, xi[ft][r], tcm[r]);
        };
        auto upd_ops = [&](auto ftc, auto fromc, auto toc) {
            static_for<decltype(fromc)::value, decltype(toc)::value>([&](auto opc) { upd_op(ftc, opc); });
        };
        __builtin_amdgcn_sched_barrier(0);
        static_for<0, NS>([&](auto step) {
            constexpr int i = decltype(step)::value;
            lds_await<kDepth - 1>(q[i % kDepth]);
            const bf16x8 a = __builtin_bit_cast(bf16x8, q[i % kDepth]);
            if constexpr (i < NT) {
                constexpr int t = i / PER_TILE, u = i % PER_TILE;
                if constexpr (u < 4) {
                    gn[t] = mma16(a, dB[u], gn[t]);
                    if constexpr (SPLIT) gn[t] = mma16(a, dR[u], gn[t]);
                } else if constexpr (u < HP) {
                    gn[t] = mma16(a, dB[u - 4], gn[t]);
                } else {
                    gn[t] = mma16(a, pm[u - HP], gn[t]);
                    if constexpr (SPLIT) gn[t] = mma16(a, pmR[u - HP], gn[t]);
                }
            } else {
                constexpr int fb = (i - NT) / NJ, js = (i - NT) % NJ;
                P[js] = mma16(a, dB[fb], fb == 0 ? zero4() : P[js]);
                if constexpr (SPLIT) P[js] = mma16(a, dR[fb], P[js]);
            }
            {
                constexpr int nx = (i + kDepth) % NS;
                lds_read16_untracked<PL::off(nx) * 16>(q[i % kDepth], bases[PL::base(nx)]);
            }
            if constexpr (i < NT) {
                constexpr int t = i / PER_TILE, u = i % PER_TILE;
                if constexpr (t == 0 && u == 2) mask_products(std::integral_constant<int, 0>{});
                if constexpr (t == 0 && u == 3 && NJB == 2) mask_products(std::integral_constant<int, NJB - 1>{});
                if constexpr (t >= 1) {
                    // step u of the tile takes the operations [16 u / PER_TILE, 16 (u + 1) / PER_TILE)
                    upd_ops(std::integral_constant<int, t - 1>{}, std::integral_constant<int, 16 * u / PER_TILE>{},
                            std::integral_constant<int, 16 * (u + 1) / PER_TILE>{});
                }
            } else {
                // key products of the next pass: the last tile's update and the new operands meanwhile
                constexpr int k = i - NT;
                typedef std::integral_constant<int, 7> FT;
                if constexpr (k == 0) {
                    upd_ops(FT{}, std::integral_constant<int, 0>{}, std::integral_constant<int, 8>{});
                    pack_delta(std::integral_constant<int, 1>{});
                }
                if constexpr (k == NJ) {
                    upd_ops(FT{}, std::integral_constant<int, 8>{}, std::integral_constant<int, 16>{});
                    pack_delta(std::integral_constant<int, 2>{});
                }
                if constexpr (k == 2 * NJ) pack_delta(std::integral_constant<int, 3>{});
            }
            if constexpr (i == NT - 1) pack_delta(std::integral_constant<int, 0>{});
            __builtin_amdgcn_sched_barrier(0);
        });
    }
    if (kBoost) __builtin_amdgcn_s_setprio(0);
    // the reads issued for a pass that does not follow must have landed before their registers are used again
    static_for<0, kDepth>([&](auto step) { lds_await<0>(q[decltype(step)::value]); });
}

// Decay mask of Section 4.2.1 in the log-space form of Appendix B.2 (base 2): M[j][c] = 2^(G_c - G_j) for j <= c.
// (Gtab: G_j of the chunk's 64 tokens, a slot of this wave's table.) With the write gate of the Remark in Section 4.1,
// H_c = zeta_c H_[n] + sum_{j<=c} M[j,c] beta_j k_j k_j^T (the same for U): beta_j is folded into the mask,
// m[j,c] = M[j,c] beta_j, which every product uses (Btab: beta_j of the chunk's tokens).
template <bool GATED>
__device__ __forceinline__ void build_mask(const Ctx &c, Solver &s, const float *Gtab, const float *Btab, int ts)
{
    const int c_local = 16 * ts + c.n;
    const float Gc = Gtab[c_local];
    s.zeta = exp2f(Gc);
    s.beta = GATED ? Btab[c_local] : 1.0f;
#pragma unroll
    for (int js = 0; js < 4; ++js) {
        const f32x4 Gj = *(const f32x4 *)(Gtab + 16 * js + 4 * c.kg);
        f32x4 bj = {1.0f, 1.0f, 1.0f, 1.0f};
        if constexpr (GATED) bj = *(const f32x4 *)(Btab + 16 * js + 4 * c.kg);
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int j = 16 * js + 4 * c.kg + r;
            // hardware exp2: results below the normal range (decays under 2^-126) are flushed to zero
            s.mreg[js][r] = (j <= c_local) ? __builtin_amdgcn_exp2f(Gc - Gj[r]) * bj[r] : 0.0f;
        }
    }
}

// Chunk-wise Frobenius norm, first half: w_j of this wave's tokens to the table.
//   ||H_c||^2 = zeta_c^2 ||H_[n]||^2 + sum_{j<=c} M[j,c]^2 w_j,  w_j = 2 (zeta_j k_j^T H_[n] k_j + sum_{i<j} M[i,j] G_ij^2) + G_jj^2
// (G = K K^T): the three-term expansion of Section 4.2.1 with its double sum folded by M[i,c] M[j,c] = M[j,c]^2 M[i,j].
// With the write gate (mask m = M beta): w_j = 2 (zeta_j k_j^T H_[n] k_j + sum_{i<j} m[i,j] G_ij^2) / beta_j + G_jj^2,
// and w_j = 0 for beta_j = 0 (its column of m vanishes).
template <int NJ, bool GATED>
__device__ __forceinline__ void frobenius_terms(const Ctx &c, const Solver &s, int g, int ts)
{
    const bf16x8 *sH = lds_frags(c, kOffH + g * 32768) + c.lane;
    const bf16x8 *sK = lds_frags(c, kOffK + g * 16384);
    bf16x8 kB[1][4];
#pragma unroll
    for (int fb = 0; fb < 4; ++fb) kB[0][fb] = sK[(ts * 4 + fb) * 64 + c.lane];
    // this lane's elements of k_c as floats: tile ft, row r <-> slot 4 (ft & 1) + r of fragment ft / 2
    f32x4 kc[8];
#pragma unroll
    for (int fb = 0; fb < 4; ++fb) unpack8(kB[0][fb], kc[2 * fb], kc[2 * fb + 1]);
    // k_c^T H_[n] k_c (the fragments of the next tile are requested before the products of this one: the scheduler
    // would otherwise sink the reads to their uses, one LDS round trip per tile)
    f32x4 dot = zero4();
    bf16x8 a[2][4];
#pragma unroll
    for (int fb = 0; fb < 4; ++fb) a[0][fb] = sH[fb * 64];
#pragma unroll
    for (int ft = 0; ft < 8; ++ft) {
        if (ft + 1 < 8) {
#pragma unroll
            for (int fb = 0; fb < 4; ++fb) a[(ft + 1) & 1][fb] = sH[((ft + 1) * 4 + fb) * 64];
        }
        __builtin_amdgcn_sched_barrier(0);
        f32x4 acc = zero4();
#pragma unroll
        for (int fb = 0; fb < 4; ++fb) acc = mma16(a[ft & 1][fb], kB[0][fb], acc);
        dot += acc * kc[ft];
    }
    float a_part = dot[0] + dot[1] + dot[2] + dot[3];
    // Gram columns of this wave's tokens against the key blocks js <= ts
    f32x4 G[NJ];
    key_products<NJ, 1>(sK, kB, G, c.lane);
    float b_part = 0.0f, d_part = 0.0f;
#pragma unroll
    for (int js = 0; js < NJ; ++js)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            b_part += s.mreg[js][r] * (G[js][r] * G[js][r]);
            if (js == ts && 4 * c.kg + r == c.n) d_part = G[js][r] * G[js][r];
        }
    a_part = sum_over_kg(a_part);
    b_part = sum_over_kg(b_part);
    d_part = sum_over_kg(d_part);
    // the sum runs over i < c: the diagonal term (m[c][c] = beta_c) is taken out again
    float w;
    if constexpr (GATED) {
        b_part -= s.beta * d_part;
        w = s.beta > 0.0f ? 2.0f * (s.zeta * a_part + b_part) / s.beta + d_part : 0.0f;
    } else {
        b_part -= d_part;
        w = 2.0f * (s.zeta * a_part + b_part) + d_part;
    }
    float *sW = (float *)(c.smem + kOffTab) + g * 64;
    if (c.kg == 0) sW[16 * ts + c.n] = w;
}

// second half: ||H_c||_F of this lane's token
template <int NJ>
__device__ __forceinline__ float frobenius_norm(const Ctx &c, const Solver &s, int g)
{
    const float *sW = (const float *)(c.smem + kOffTab) + g * 64;
    const float *sN = (const float *)(c.smem + kOffTab) + 128 + g * 8;
    float hn2 = 0.0f;
#pragma unroll
    for (int i = 0; i < 8; ++i) hn2 += sN[i];
    float f = 0.0f;
#pragma unroll
    for (int js = 0; js < NJ; ++js) {
        const f32x4 wv = *(const f32x4 *)(sW + 16 * js + 4 * c.kg);
#pragma unroll
        for (int r = 0; r < 4; ++r) f += s.mreg[js][r] * s.mreg[js][r] * wv[r];
    }
    f = sum_over_kg(f);
    return sqrtf(fmaxf(s.zeta * s.zeta * hn2 + f, 0.0f));
}

__device__ __forceinline__ void copy_rows(const Ctx &c, const void *x, int g, int chunk);

// Everything between the Frobenius table and the published result: the passes, then (after the workgroup has
// passed the barrier inside) xhat to LDS and the intra-chunk part of the readout.
template <int NJ, bool SPLIT, bool GATED>
__device__ __forceinline__ void solve_tokens(Ctx &c, Solver &s, int g, int ts, const typename IOBF16::raw4 (&qraw)[8],
                                             float lam, f32x4 (&accU)[8], int c0)
{
    const bf16x8 *sH = lds_frags(c, kOffH + g * 32768);
    const bf16x8 *sK = lds_frags(c, kOffK + g * 16384);
    const bf16x8 *sKT = lds_frags(c, kOffKT + g * 16384);
    // Section 4.1: L = ||H_t||_F + lambda_t, mu = lambda_t
    const float L = s.fro + lam, mu = lam;
    const float rcp = __builtin_amdgcn_rcpf(L + mu);
    const float s0 = 2.0f * rcp;
    const float rho = (L - mu) * rcp;
    // From here on the token's system and its readout are taken divided by zeta_c (see cheb_passes): the mask
    // becomes m[j,c] / zeta_c and the results are multiplied by zeta_c at the end. zeta_c is floored for this purpose:
    // behind a gate that wipes the state inside the chunk, what was before it keeps a weight of 2^-60 relative to
    // the newest key (instead of less), far below the rounding of everything else, and 1 / zeta_c stays finite.
    s.zeta = fmaxf(s.zeta, kMinSolveZeta);
    const float rz = 1.0f / s.zeta;
#pragma unroll
    for (int js = 0; js < 4; ++js) s.mreg[js] *= rz;
    f32x4 xi[8], dl[8], gn[8];
#pragma unroll
    for (int ft = 0; ft < 8; ++ft) {
        const f32x4 qv = IOBF16::cvt4(qraw[ft]);
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const float qe = s.valid ? qv[r] : 0.0f;
            xi[ft][r] = 0.0f;
            dl[ft][r] = s0 * qe;
            gn[ft][r] = -qe * rz;
        }
    }
    cheb_passes<NJ, SPLIT>(sH, sK, sKT, xi, dl, gn, s.mreg, s0 * s.zeta, s0 * lam, rho * rho, c.a.n_iter, c.lane, [&]() {
        // v rows of the iteration's chunks replace the k rows; they land during the passes
        copy_rows(c, c.a.v, 0, c0);
        if constexpr (!SPLIT) copy_rows(c, c.a.v, 1, c0 + 1);
    });
    refresh_lane(c);
#pragma unroll
    for (int ft = 0; ft < 8; ++ft) xi[ft] += dl[ft];
    if constexpr (GATED) {
        // alpha-connection (Section 4.3): the readout is applied to alpha xhat + (1 - alpha) q; q is read again (it
        // was not kept through the passes)
        if (c.a.alpha) {
            const int tokc = min(s.tok, c.a.T - 1);
            const float al = s.valid ? c.a.alpha[c.gate_base + (int64_t)tokc * c.a.H] : 1.0f;
            const int64_t tok_off = c.base_bh + (int64_t)tokc * c.a.stride_t;
#pragma unroll
            for (int ft = 0; ft < 8; ++ft) {
                const f32x4 qv = IOBF16::load4(c.a.q, tok_off + 16 * ft + 4 * c.kg);
#pragma unroll
                for (int r = 0; r < 4; ++r) xi[ft][r] = al * xi[ft][r] + (1.0f - al) * (s.valid ? qv[r] : 0.0f);
            }
        }
    }

    // ---- readout, intra-chunk part: sum_{j<=c} M[j,c] v_j (k_j . xhat_c), xhat as value + remainder
    bf16x8 x[2][4];
#pragma unroll
    for (int fb = 0; fb < 4; ++fb) split8(xi[2 * fb], xi[2 * fb + 1], x[0][fb], x[1][fb]);
    f32x4 P[NJ];
    key_products<NJ, 2>(sK, x, P, c.lane);
    constexpr int NJB = NJ / 2;
    bf16x8 pm[NJB];
#pragma unroll
    for (int jb = 0; jb < NJB; ++jb) pm[jb] = masked_frag(P[2 * jb], P[2 * jb + 1], s.mreg, jb);
    wait_all_memory();               // this wave's copies of v rows have landed
    lds_barrier();                   // all of them have; every wave is through its passes: H_[n] is dead
    bf16x8 *sX = lds_frags(c, kOffH + g * 32768) + c.lane;
#pragma unroll
    for (int fb = 0; fb < 4; ++fb) {
        sX[((ts * 2 + 0) * 4 + fb) * 64] = x[0][fb];
        sX[((ts * 2 + 1) * 4 + fb) * 64] = x[1][fb];
    }
    park_load(c.park, accU);         // U comes back while the last products of this phase run
    const uint16_t *rowsV = lds_rows(c, g);
#pragma unroll
    for (int ft = 0; ft < 8; ++ft) {
        s.yi[ft] = zero4();
#pragma unroll
        for (int jb = 0; jb < NJB; ++jb) {
            const int t0 = 32 * jb + 4 * c.kg;
            const bf16x8 vt = gather_transposed_bf16(rowsV, Rows(), 16 * ft, c.lane, t0, t0 + 16);
            s.yi[ft] = mma16(vt, pm[jb], s.yi[ft]);
        }
    }
}

// y_c = zeta_c U_[n] xhat_c + intra part, stored
__device__ __forceinline__ void store_output(const Ctx &c, const Solver &s, int ts, int y_off)
{
    const f32x4 *sY = (const f32x4 *)(c.smem + y_off);
    if (!s.valid) return;
    const int64_t off = c.base_bh + (int64_t)s.tok * c.a.stride_t;
#pragma unroll
    for (int ft = 0; ft < 8; ++ft) {
        const f32x4 ys = sY[(ts * 8 + ft) * 64 + c.lane];
        const f32x4 y = s.zeta * (ys + s.yi[ft]);          // (yi was formed with the mask divided by zeta)
        IOBF16::store4(c.a.o, off + 16 * ft + 4 * c.kg, y[0], y[1], y[2], y[3]);
    }
}

// ---- data movement ---------------------------------------------------------------------------------------------

// Rows of chunk `chunk` of x (k or v) into row tile g: direct copies global -> LDS without staging registers, 1 KiB
// (four rows) per wave instruction; the lane picks the 16 source bytes that belong at its place of the swizzled row.
// Rows past the end of the sequence repeat the last row (finite values that only ever meet zero weights or masked
// products). The copies complete in the background; the compiler waits for them before the next LDS read it knows of.
template <bool UNTRACKED = false>
__device__ __forceinline__ void copy_rows_impl(const Ctx &c, const void *x, int g, int chunk)
{
    const int tok_base = min(chunk * kChunk, c.a.T - 1);
    const uint16_t *base = (const uint16_t *)x + c.base_bh + (int64_t)tok_base * c.a.stride_t;
    const int last_row = c.a.T - 1 - tok_base;
    const int row_bytes = (int)c.a.stride_t * 2;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const int i = c.w + 8 * h;
        const int row = 4 * i + (c.lane >> 4);
        const int sbyte = ((c.lane & 15) * 16) ^ ((row & 7) << 5);
        const int off = min(row, last_row) * row_bytes + sbyte;
        if constexpr (UNTRACKED) {
            async_copy16_to_lds_untracked(lds_address((char *)lds_rows(c, g) + i * 1024), raw_buffer_words(base), off);
        } else {
            async_copy16_to_lds((char *)lds_rows(c, g) + i * 1024, make_raw_buffer(base), off, 0);
        }
    }
}
__device__ __forceinline__ void copy_rows(const Ctx &c, const void *x, int g, int chunk)
{
    copy_rows_impl<false>(c, x, g, chunk);
}
// The same as copies that the compiler does not track (see async_copy16_to_lds_untracked): for the k rows of the
// next iteration, which are issued in the middle of an iteration and awaited at the top of the next.
__device__ __forceinline__ void copy_rows_untracked(const Ctx &c, const void *x, int g, int chunk)
{
    copy_rows_impl<true>(c, x, g, chunk);
}

// A fragments of the keys of both chunks from their row tiles: rows (K[js][fb]) and transposed (KT[ft][jb]); each
// wave builds four of the 32 fragments of either kind.
// (SPLIT: one chunk, two of its 16 fragments of either kind per wave.)
template <bool SPLIT>
__device__ __forceinline__ void build_key_frags(const Ctx &c)
{
    constexpr int PER_WAVE = SPLIT ? 2 : 4;
    // all reads first, then all writes: read-then-write per fragment would be one LDS round trip after the other
    bf16x8 rowf[PER_WAVE], trf[PER_WAVE];
#pragma unroll
    for (int q = 0; q < PER_WAVE; ++q) {
        const int idx = c.w * PER_WAVE + q;
        const int g = idx >> 4, f = idx & 15;
        const uint16_t *rows = lds_rows(c, g);
        {
            const int js = f >> 2, fb = f & 3;
            const u16x4 lo = *(const u16x4 *)(rows + Rows()(16 * js + c.n, 32 * fb + 4 * c.kg));
            const u16x4 hi = *(const u16x4 *)(rows + Rows()(16 * js + c.n, 32 * fb + 16 + 4 * c.kg));
            const u16x8 u = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
            rowf[q] = __builtin_bit_cast(bf16x8, u);
        }
        {
            const int ft = f >> 1, jb = f & 1;
            const int t0 = 32 * jb + 4 * c.kg;
            trf[q] = gather_transposed_bf16(rows, Rows(), 16 * ft, c.lane, t0, t0 + 16);
        }
    }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int q = 0; q < PER_WAVE; ++q) {
        const int idx = c.w * PER_WAVE + q;
        const int g = idx >> 4, f = idx & 15;
        lds_frags(c, kOffK + g * 16384)[f * 64 + c.lane] = rowf[q];
        lds_frags(c, kOffKT + g * 16384)[f * 64 + c.lane] = trf[q];
    }
}

// Start state of this wave's tiles: the caller's initial state advanced over the segments before this one.
__device__ __forceinline__ void load_start_state(const Ctx &c, f32x4 (&accH)[8], f32x4 (&accU)[8], int pair, int seg)
{
    const FusedArgs &a = c.a;
#pragma unroll
    for (int jt = 0; jt < 8; ++jt) {
        accH[jt] = zero4();
        accU[jt] = zero4();
    }
    if (a.H_init) {
        const float *Hi = a.H_init + (int64_t)pair * kD * kD;
        const float *Ui = a.U_init + (int64_t)pair * kD * kD;
#pragma unroll
        for (int jt = 0; jt < 8; ++jt) {
            // tile element (row 4 kg + r, column n) = H[16 jt + 4 kg + r][16 w + n] = H[16 w + n][16 jt + 4 kg + r]
            if (a.h_init_lower_blocks && (jt >> 1) > (c.w >> 1)) {
                // the 32 x 32 block above the block diagonal is not stored: take the mirror image
#pragma unroll
                for (int r = 0; r < 4; ++r) accH[jt][r] = Hi[(int64_t)(16 * jt + 4 * c.kg + r) * kD + 16 * c.w + c.n];
            } else {
                accH[jt] = *(const f32x4 *)(Hi + (int64_t)(16 * c.w + c.n) * kD + 16 * jt + 4 * c.kg);
            }
            accU[jt] = *(const f32x4 *)(Ui + (int64_t)(16 * c.w + c.n) * kD + 16 * jt + 4 * c.kg);
        }
    }
    for (int sg = 0; sg < seg; ++sg) {
        const f32x4 *t = (const f32x4 *)a.seg_buf + ((int64_t)(pair * a.n_segs + sg) * 2) * 4096 + (c.w * 8) * 64 + c.lane;
        const float decay = exp2f(a.seg_logdecay[pair * a.n_segs + sg]);
#pragma unroll
        for (int jt = 0; jt < 8; ++jt) {
            accH[jt] = decay * accH[jt] + t[jt * 64];
            accU[jt] = decay * accU[jt] + t[4096 + jt * 64];
        }
    }
}

}  // namespace

// One workgroup per (pair, segment of chunks). Per iteration (chunks A = c0, B = c0 + 1), with the barriers between
// the phases:
//   1. gate scans (the k rows, copied global -> LDS since the end of the previous iteration, land; solver B of the
//      previous iteration may still be storing)
//   2. H_[n] of A -> LDS; key fragments of both chunks; this wave's weighted k fragments
//   3. H advanced over A; H_[n] of B -> LDS; H advanced over B; partial norms -> table (in the dead k row tile)
//   4. solver: Frobenius terms -> table
//   5. solver: norms; copies of the v rows into the row tiles start; passes, intra-chunk readout products;
//      xhat -> LDS (over H_[n])
//   6. state part of the readout for A (over the key-row fragments), U advanced over A
//   7. solver A stores; state part of the readout for B (over A's xhat), U advanced over B and parked
//   8. solver B stores; copies of the next k rows into the row tiles start
// SPLIT: the same with chunk A alone (everything that concerns B drops out, phase 8 joins phase 7).
// GATED: the layer's variants (write gate beta, alpha-connection, the rule lambda_t = a ||H_t||_F), a compile-time
// flag so that the plain kernel carries none of their loads, registers or branches.
template <bool SPLIT, bool GATED>
__global__ __launch_bounds__(kFusedThreads) __attribute__((amdgpu_waves_per_eu(2, 2))) void fused_forward_kernel(FusedArgs a)
{
    extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
    Ctx c{a, smem};
    c.tid = threadIdx.x;
    c.lane = c.tid & 63;
    c.w = __builtin_amdgcn_readfirstlane(c.tid >> 6);
    c.n = c.lane & 15;
    c.kg = c.lane >> 4;
    const int pair = blockIdx.x % a.n_pairs, seg = blockIdx.x / a.n_pairs;
    const int b = pair / a.H, h = pair % a.H;
    c.base_bh = (int64_t)b * a.stride_b + (int64_t)h * a.stride_h;
    c.gate_base = (int64_t)b * a.T * a.H + h;
    const int chunk_begin = seg * a.seg_len;
    const int chunk_end = min(chunk_begin + a.seg_len, a.n_chunks);
    if (chunk_begin >= chunk_end) return;
    c.T_eff = min(a.T, chunk_end * kChunk);
    constexpr int kChunksPerIter = SPLIT ? 1 : 2;
    // Solver role: chunk of the pair and token block. Waves w and w + 4 share a SIMD, whose arbiter prefers the older
    // one: waves 0-3 take the token blocks with more key blocks (ts = 2, 3), waves 4-7 the others. SPLIT: waves 0-3
    // take the four token blocks of the one chunk, waves 4-7 none.
    const int grp = SPLIT ? 0 : (c.w >> 1) & 1;
    const int ts = SPLIT ? (c.w & 3) : (c.w < 4 ? 2 : 0) + (c.w & 1);
    const bool solver = !SPLIT || c.w < 4;

    c.park = (f32x4 *)a.park + ((int64_t)blockIdx.x * 8 + c.w) * (8 * 64) + c.lane;
    f32x4 accH[8];
    {
        f32x4 accU[8];
        load_start_state(c, accH, accU, pair, seg);
        park_store(c.park, accU);
    }
    copy_rows(c, a.k, 0, chunk_begin);
    if constexpr (!SPLIT) copy_rows(c, a.k, 1, chunk_begin + 1);
    float *sTab = (float *)(smem + kOffTab);

    const bool wide = ts >= 2;                              // which instantiation of the solver code this wave runs
    float gmA = a.gate[c.gate_base + (int64_t)min(chunk_begin * kChunk + c.lane, a.T - 1) * a.H];
    float gmB = 1.0f;
    if constexpr (!SPLIT) gmB = a.gate[c.gate_base + (int64_t)min((chunk_begin + 1) * kChunk + c.lane, a.T - 1) * a.H];
    // write gates of the chunks' tokens (lane j: token j), fetched with the gates
    float bmA = 1.0f, bmB = 1.0f;
    auto fetch_beta = [&](int chunk0) {
        if constexpr (GATED) {
            if (a.beta) {
                bmA = a.beta[c.gate_base + (int64_t)min(chunk0 * kChunk + c.lane, a.T - 1) * a.H];
                if constexpr (!SPLIT) bmB = a.beta[c.gate_base + (int64_t)min((chunk0 + 1) * kChunk + c.lane, a.T - 1) * a.H];
            }
        }
    };
    fetch_beta(chunk_begin);
    wait_all_memory();                   // the first k rows (the loop's own wait counts on a whole iteration before it)
#pragma unroll 1
    for (int c0 = chunk_begin; c0 < chunk_end; c0 += kChunksPerIter) {
        // Addresses are formed anew in every iteration from a copy of the lane index that the compiler cannot trace
        // back: hoisted out of the loop they would occupy registers across the passes (or be spilled and reloaded).
        refresh_lane(c);
        // ---- 1
        // Gates of the chunks (fetched during the previous iteration): G_j, the weight of token j in the chunk's
        // update 2^(G_C - G_j) (times its write gate), and the chunk's decay 2^(G_C). Before the passes one wave per
        // chunk scans (waves 0 and 1: among the first to arrive here, while others still store their tokens) and
        // leaves the per-token scalars in a table that all waves read after the barrier; slots of 64 floats: weights
        // of A, of B, G of A, of B, write gates of A, of B. The table lies in a part of LDS that is free from the last
        // barrier of the previous iteration to the second of this one (the second chunk's H_[n]; SPLIT: the second
        // chunk's key fragments, which do not exist).
        constexpr int kTabBefore = SPLIT ? kOffK + 16384 : kOffH + 32768;
        constexpr int kTabAfter = kOffK + 16384;             // after the passes: the key-row fragments are dead
        float *gtab = (float *)(smem + kTabBefore);
        auto scan_chunk = [&](float gm, float bm, int chunk, float &wj, float &zeta) {
            const bool valid = chunk * kChunk + c.lane < c.T_eff;
            const float G = wave_inclusive_scan(valid ? log2_gate(gm) : 0.0f, c.lane);
            const float Gt = lane_value(G, 63);
            wj = valid ? exp2f(Gt - G) * bm : 0.0f;
            zeta = exp2f(Gt);
            return G;
        };
        float wjA, wjB = 0.0f, zetaA, zetaB = 1.0f;
        if (c.w == 0) {
            const float GA = scan_chunk(gmA, bmA, c0, wjA, zetaA);
            gtab[0 * 64 + c.lane] = wjA;
            gtab[2 * 64 + c.lane] = GA;
            if constexpr (GATED) gtab[4 * 64 + c.lane] = bmA;
        }
        if constexpr (!SPLIT) {
            if (c.w == 1) {
                const float GB = scan_chunk(gmB, bmB, c0 + 1, wjB, zetaB);
                gtab[1 * 64 + c.lane] = wjB;
                gtab[3 * 64 + c.lane] = GB;
                if constexpr (GATED) gtab[5 * 64 + c.lane] = bmB;
            }
        }
        // This wave's copies of the k rows have landed: they were issued before the kParkStores stores of U that
        // every wave issues in every iteration, so once no more than that many vector-memory instructions are
        // outstanding the copies are complete. (The stores of the last tokens, which follow, need not be: waiting
        // for them cost 3 % of the step.)
        wait_vector_memory_but<kParkStores>();
        lds_barrier();                   // ... and everybody else's; the table is complete
        // ---- 2
        zetaA = exp2f(gtab[2 * 64 + 63]);
        if constexpr (!SPLIT) zetaB = exp2f(gtab[3 * 64 + 63]);
        const float hnA = publish_H<SPLIT>(c, accH, 0);
        build_key_frags<SPLIT>(c);
        bf16x8 wBA[2], wBB[2];
        own_weighted_frags(c, lds_rows(c, 0), gtab, wBA);
        if constexpr (!SPLIT) own_weighted_frags(c, lds_rows(c, 1), gtab + 64, wBB);
        // solver inputs of this lane's token
        f32x4 accU[8];
        Solver s;
        s.tok = (c0 + grp) * kChunk + 16 * ts + c.n;
        s.valid = solver && s.tok < c.T_eff;
        const int64_t tok_off = c.base_bh + (int64_t)min(s.tok, a.T - 1) * a.stride_t;
        IOBF16::raw4 qraw[8];
        float lam = 1.0f;
        if (solver) {                    // (wave-uniform)
#pragma unroll
            for (int ft = 0; ft < 8; ++ft) qraw[ft] = IOBF16::load_raw4(a.q, tok_off + 16 * ft + 4 * c.kg);
            if (!GATED || a.lambda) lam = a.lambda[c.gate_base + (int64_t)min(s.tok, a.T - 1) * a.H];
            build_mask<GATED>(c, s, gtab + (2 + grp) * 64, gtab + (4 + grp) * 64, ts);
        }
        lds_barrier();
        // ---- 3
        advance_state(c, accH, 0, zetaA, wBA);
        float hnB = 0.0f;
        if constexpr (!SPLIT) {
            hnB = publish_H<false>(c, accH, 1);
            advance_state(c, accH, 1, zetaB, wBB);
        }
        if (c.lane == 0) {
            sTab[128 + c.w] = hnA;
            if constexpr (!SPLIT) sTab[128 + 8 + c.w] = hnB;
        }
        lds_barrier();
        // ---- 4
        if (solver) {
            if (wide) frobenius_terms<4, GATED>(c, s, grp, ts);
            else frobenius_terms<2, GATED>(c, s, grp, ts);
        }
        lds_barrier();
        // ---- 5
        if (solver) {
            s.fro = wide ? frobenius_norm<4>(c, s, grp) : frobenius_norm<2>(c, s, grp);
            if (a.fro_out && s.valid && c.kg == 0) a.fro_out[c.gate_base + (int64_t)s.tok * a.H] = s.fro;
            if constexpr (GATED) {
                if (!a.lambda) lam = a.lambda_scale * s.fro;       // the rule of Section 4.1
            }
            if (!s.valid) lam = 1.0f;
        }
        lds_barrier();                   // the table is dead: the row tiles may be overwritten
        if (solver) {
            if (wide) solve_tokens<4, SPLIT, GATED>(c, s, grp, ts, qraw, lam, accU, c0);
            else solve_tokens<2, SPLIT, GATED>(c, s, grp, ts, qraw, lam, accU, c0);
        } else {
            // (SPLIT, waves 4-7) this wave's share of the copies of the v rows, the barrier that the solver waves pass
            // after their passes, and U back from its parking place
            copy_rows(c, a.v, 0, c0);
            wait_all_memory();
            lds_barrier();
            park_load(c.park, accU);
        }
        // (after the passes every wave scans the gates for itself: no barrier separates this from the use of the
        // results, and the raw gates cost two registers across the passes; the opaque copy keeps the compiler from
        // merging these scans with those of waves 0 and 1 above)
        asm volatile("" : "+v"(gmA), "+v"(gmB));
        scan_chunk(gmA, bmA, c0, wjA, zetaA);
        if constexpr (!SPLIT) scan_chunk(gmB, bmB, c0 + 1, wjB, zetaB);
        // this wave's weighted v fragments of the chunks
        bf16x8 wVA[2], wVB[2];
        wave_table(c, kTabAfter, 0)[c.lane] = wjA;
        if constexpr (!SPLIT) wave_table(c, kTabAfter, 1)[c.lane] = wjB;
        own_weighted_frags(c, lds_rows(c, 0), wave_table(c, kTabAfter, 0), wVA);
        if constexpr (!SPLIT) own_weighted_frags(c, lds_rows(c, 1), wave_table(c, kTabAfter, 1), wVB);
        lds_barrier();                   // xhat of the chunks is visible; the key-row fragments are dead
        // ---- 6
        // k rows of the next chunks: the row tiles are free from here on (every wave has formed its v fragments); the
        // copies land during the readout.
        // U, on its way back from its parking place since before the last barrier but one, is awaited first: the
        // compiler does not count the copies, so the wait it would otherwise place before the first use of U (for all
        // but the loads it knows to be younger) would also wait for copies to land (1 % of the kernel).
        wait_all_memory();
        copy_rows_untracked(c, a.k, 0, c0 + kChunksPerIter);
        if constexpr (!SPLIT) copy_rows_untracked(c, a.k, 1, c0 + 3);
        // gates of the next chunks
        gmA = a.gate[c.gate_base + (int64_t)min((c0 + kChunksPerIter) * kChunk + c.lane, a.T - 1) * a.H];
        if constexpr (!SPLIT) gmB = a.gate[c.gate_base + (int64_t)min((c0 + 3) * kChunk + c.lane, a.T - 1) * a.H];
        fetch_beta(c0 + kChunksPerIter);
        readout_state(c, accU, 0, kOffK);
        advance_state(c, accU, 0, zetaA, wVA);
        lds_barrier();
        // ---- 7: solver A stores while the state part of B is read out into the place of A's xhat
        if (solver && grp == 0) store_output(c, s, ts, kOffK);
        if constexpr (!SPLIT) {
            readout_state(c, accU, 1, kOffH);
            advance_state(c, accU, 1, zetaB, wVB);
        }
        park_store(c.park, accU);
        if constexpr (!SPLIT) {
            lds_barrier();
            // ---- 8
            if (grp == 1) store_output(c, s, ts, kOffH);
        }
    }
    wait_all_memory();               // no copy into this workgroup's LDS may be in flight when it ends

    if (a.H_final && seg == a.n_segs - 1) {
        float *Hf = a.H_final + (int64_t)pair * kD * kD;
        float *Uf = a.U_final + (int64_t)pair * kD * kD;
        f32x4 accU[8];
        park_load(c.park, accU);
#pragma unroll
        for (int jt = 0; jt < 8; ++jt) {
            *(f32x4 *)(Hf + (int64_t)(16 * c.w + c.n) * kD + 16 * jt + 4 * c.kg) = accH[jt];
            *(f32x4 *)(Uf + (int64_t)(16 * c.w + c.n) * kD + 16 * jt + 4 * c.kg) = accU[jt];
        }
    }
}

// Summary (prod gamma, Delta H, Delta U from a zero state) of every segment but the last: the start states of the
// fused kernel's workgroups follow from these by a short scan. One chunk per iteration; its k and v rows were fetched
// kSummaryAhead iterations earlier into registers and are stored into the other half of a double buffer, so an
// iteration is one barrier followed by wave-local work: every wave reads the transposed operands of its tiles
// straight from the row tiles. (The kernel is bound by the latency of its loads: what counts is the bytes in flight.)
// The tiles are padded, not swizzled: the reads of a wave's eight tiles then differ by constant offsets.
constexpr int kSummaryRowElems = kD + MmaBF16::kRowPad;    // rows 32 bytes apart modulo 256
constexpr int kSummaryTile = kChunk * kSummaryRowElems * 2; // bytes
constexpr int kSummaryAhead = 2;                           // chunks whose rows are in flight
constexpr int kSummaryTables = 2 * 2 * kSummaryTile;       // offset of the waves' tables of per-token weights
constexpr int kSummaryLds = kSummaryTables + 8 * 4 * 64 * 4;   // [buffer][k, v] row tiles + tables
__global__ __launch_bounds__(kFusedThreads) __attribute__((amdgpu_waves_per_eu(2, 2))) void fused_summary_kernel(FusedArgs a)
{
    extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
    Ctx c{a, smem};
    c.w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    refresh_lane(c);
    const int pair = blockIdx.x % a.n_pairs, seg = blockIdx.x / a.n_pairs;
    const int b = pair / a.H, h = pair % a.H;
    c.base_bh = (int64_t)b * a.stride_b + (int64_t)h * a.stride_h;
    c.gate_base = (int64_t)b * a.T * a.H + h;
    const int chunk_begin = seg * a.seg_len;
    const int chunk_end = min(chunk_begin + a.seg_len, a.n_chunks);
    c.T_eff = min(a.T, chunk_end * kChunk);

    f32x4 accH[8], accU[8];
#pragma unroll
    for (int jt = 0; jt < 8; ++jt) {
        accH[jt] = zero4();
        accU[jt] = zero4();
    }
    // Rows of k and v travel global memory -> registers -> padded LDS tiles, kSummaryAhead chunks ahead of their use
    // (one stage of registers per chunk in flight). Piece i of a thread: tile (i / 2: k, v), 16 bytes of row
    // (i % 2) * 32 + tid / 16.
    u32x4 regs[kSummaryAhead][4];        // (a native vector type: arrays of HIP's uint4 struct stay in memory)
    float gm[kSummaryAhead], bm[kSummaryAhead];  // gates and write gates (1 if none) of the chunks, lane j: token j
    auto fetch = [&](auto stagec, int chunk) {
        constexpr int st = decltype(stagec)::value;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int row = (i & 1) * 32 + (c.tid >> 4), piece = c.tid & 15;
            const int tok = min(chunk * kChunk + row, a.T - 1);
            const uint16_t *x = (const uint16_t *)((i >> 1) ? a.v : a.k);
            regs[st][i] = *(const u32x4 *)(x + c.base_bh + (int64_t)tok * a.stride_t + 8 * piece);
        }
        const int64_t at = c.gate_base + (int64_t)min(chunk * kChunk + c.lane, a.T - 1) * a.H;
        gm[st] = a.gate[at];
        bm[st] = a.beta ? a.beta[at] : 1.0f;         // (uniform branch)
    };
    float Gseg = 0.0f;
    static_for<0, kSummaryAhead>([&](auto stagec) { fetch(stagec, chunk_begin + decltype(stagec)::value); });
    int buf = 0;
#pragma unroll 1
    for (int c0 = chunk_begin; c0 < chunk_end; c0 += kSummaryAhead) {
        static_for<0, kSummaryAhead>([&](auto stagec) {
            constexpr int st = decltype(stagec)::value;
            const int chunk = c0 + st;
            if (chunk >= chunk_end) return;          // (uniform)
            refresh_lane(c);
            unsigned char *tiles = smem + buf * (2 * kSummaryTile);
            buf ^= 1;
            const PaddedRows at{kSummaryRowElems};
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int row = (i & 1) * 32 + (c.tid >> 4), piece = c.tid & 15;
                *(u32x4 *)((uint16_t *)(tiles + (i >> 1) * kSummaryTile) + at(row, 8 * piece)) = regs[st][i];
            }
            const float gmc = gm[st], bmc = bm[st];
            lds_barrier();               // the tiles are complete; the other buffer's readers are done
            fetch(stagec, chunk + kSummaryAhead);    // (past the end of the segment: harmless reads of rows that exist)
            // (the scheduler must not sink these loads to where their data is stored, kSummaryAhead chunks later)
            __builtin_amdgcn_sched_barrier(0);
            const bool valid = chunk * kChunk + c.lane < c.T_eff;
            const float G = wave_inclusive_scan(valid ? log2_gate(gmc) : 0.0f, c.lane);
            const float Gtot = lane_value(G, 63);
            Gseg += Gtot;
            const float wj = valid ? exp2f(Gtot - G) * bmc : 0.0f;
            const float zetaC = exp2f(Gtot);
            const uint16_t *rowsK = (const uint16_t *)tiles;
            const uint16_t *rowsV = (const uint16_t *)(tiles + kSummaryTile);
            bf16x8 wK[2], wV[2];
            float *wtab = wave_table(c, kSummaryTables, buf);
            wtab[c.lane] = wj;
            own_weighted_frags(c, rowsK, wtab, wK, at);
            own_weighted_frags(c, rowsV, wtab, wV, at);
#pragma unroll
            for (int jt = 0; jt < 8; ++jt) {
                // (operand reads of four tiles at a time in flight: more would take the registers of the prefetch)
                if (jt == 4) __builtin_amdgcn_sched_barrier(0);
                accH[jt] *= zetaC;
                accU[jt] *= zetaC;
#pragma unroll
                for (int ks = 0; ks < 2; ++ks) {
                    const int t0 = 32 * ks + 4 * c.kg;
                    const bf16x8 kt = gather_transposed_bf16(rowsK, at, 16 * jt, c.lane, t0, t0 + 16);
                    accH[jt] = mma16(kt, wK[ks], accH[jt]);
                    accU[jt] = mma16(kt, wV[ks], accU[jt]);
                }
            }
            __builtin_amdgcn_sched_barrier(0);
        });
    }
    f32x4 *t = (f32x4 *)a.seg_buf + ((int64_t)(pair * a.n_segs + seg) * 2) * 4096 + (c.w * 8) * 64 + c.lane;
#pragma unroll
    for (int jt = 0; jt < 8; ++jt) {
        t[jt * 64] = accH[jt];
        t[4096 + jt * 64] = accU[jt];
    }
    if (c.tid == 0) a.seg_logdecay[pair * a.n_segs + seg] = Gseg;
}

size_t fused_workspace_bytes(int n_pairs, int n_segs)
{
    // per (pair, segment): Delta H, Delta U in the kernels' tile order, the segment's log2 decay, and the scratch
    // block that holds U between its uses
    const size_t n = (size_t)n_pairs * n_segs;
    return n * (2 * kD * kD * sizeof(float)) + ((n * sizeof(float) + 255) / 256) * 256 + n * (kD * kD * sizeof(float));
}

hipError_t launch_fused_forward(const FusedArgs &a0, void *workspace, hipStream_t stream, int which, bool split)
{
    FusedArgs a = a0;
    a.seg_buf = (float *)workspace;
    const size_t n = (size_t)a.n_pairs * a.n_segs;
    a.seg_logdecay = (float *)((char *)workspace + n * (2 * kD * kD * sizeof(float)));
    a.park = (float *)((char *)a.seg_logdecay + ((n * sizeof(float) + 255) / 256) * 256);
    // (the attribute is kept per device)
    static bool attr_set_on[64] = {};
    int dev = 0;
    hipError_t ed = hipGetDevice(&dev);
    if (ed != hipSuccess) return ed;
    bool unused = false;
    bool &attr_set = (dev >= 0 && dev < 64) ? attr_set_on[dev] : unused;
    if (!attr_set) {
        const void *walks[4] = {(const void *)fused_forward_kernel<false, false>,
                                (const void *)fused_forward_kernel<false, true>,
                                (const void *)fused_forward_kernel<true, false>,
                                (const void *)fused_forward_kernel<true, true>};
        hipError_t e = hipSuccess;
        for (const void *f : walks) {
            e = hipFuncSetAttribute(f, hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes);
            if (e != hipSuccess) return e;
        }
        e = hipFuncSetAttribute((const void *)fused_summary_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, kSummaryLds);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    if (a.n_segs > 1 && (which & 1)) {
        hipLaunchKernelGGL(fused_summary_kernel, dim3((unsigned)(a.n_pairs * (a.n_segs - 1))), dim3(kFusedThreads),
                           kSummaryLds, stream, a);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    if (which & 2) {
        const dim3 grid((unsigned)(a.n_pairs * a.n_segs));
        const bool gated = a.beta || a.alpha || !a.lambda;
        const dim3 block(kFusedThreads);
        if (split && gated) hipLaunchKernelGGL((fused_forward_kernel<true, true>), grid, block, kLdsBytes, stream, a);
        else if (split) hipLaunchKernelGGL((fused_forward_kernel<true, false>), grid, block, kLdsBytes, stream, a);
        else if (gated) hipLaunchKernelGGL((fused_forward_kernel<false, true>), grid, block, kLdsBytes, stream, a);
        else hipLaunchKernelGGL((fused_forward_kernel<false, false>), grid, block, kLdsBytes, stream, a);
    }
    return hipGetLastError();
}

}  // namespace gka
