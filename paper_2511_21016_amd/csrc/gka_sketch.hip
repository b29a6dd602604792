// Latent sketching (appendix "Latent Sketching for Approximate Solutions"): the two projections around the solve.
//   down:  qs_t = S q_t, ks_t = S k_t     (d_s <= 64 sketched features, written as 64 with zeros above d_s)
//   up:    xhat_t = S^T z_t               (z_t: the solve's result in the subspace, float32)
// Both are skinny matrix products over all tokens, written for the matrix cores with tokens on the output lanes:
// a wave takes 32 consecutive tokens of one head. The sketch S is float32 and is used as value + remainder (two bf16
// operands), so the products carry no rounding of S; q and k are bf16 already; z is split the same way. Packed
// [B,T,H,d] tensors.
#include "gka_device.hpp"
#include "gka_kernels.hpp"

namespace gka {

namespace {

typedef MmaBF16 MMA;
typedef MMA::frag frag;
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
constexpr int kSketchPad = 64;                     // sketched features as stored (zeros above d_s)
constexpr int kSketchReps = 1;                     // groups of 128 tokens per workgroup of the up-projection
constexpr int kDownGroups = 4;                     // groups of 64 tokens per workgroup of the down-projection

__device__ __forceinline__ void split_bf16(float x, uint16_t &hi, uint16_t &lo)
{
    hi = f32_to_bf16_bits(x);
    lo = f32_to_bf16_bits(x - bf16_bits_to_f32(hi));
}

}  // namespace

// One workgroup: 64 tokens of one (batch, head) pair; wave w takes token block w & 1 and the 32 sketched features
// w >> 1. LDS: S as bf16 value and remainder, row-major [64][D + 8], and a staging tile [64][D + 8] through which the
// rows of q, then of k, pass: they are read from memory as whole rows (16 lanes x 16 bytes) and taken from the tile one
// token per lane, as the B operand wants them.
template <int D>
__global__ __launch_bounds__(256) void sketch_down_kernel(SketchArgs a)
{
    constexpr int RS = D + 8;
    constexpr int PPR = D / 8;                     // 16-byte pieces per row
    constexpr int TOK = 64;                        // tokens per workgroup
    constexpr int PIECES = TOK * PPR / 256;        // per thread and tensor
    __shared__ __attribute__((aligned(16))) uint16_t s_hi[kSketchPad * RS];
    __shared__ __attribute__((aligned(16))) uint16_t s_lo[kSketchPad * RS];
    __shared__ __attribute__((aligned(16))) uint16_t s_x[TOK * RS];
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int n = lane & 31, g = lane >> 5;
    const int pair = blockIdx.x, b = pair / a.H, h = pair % a.H;
    int t0 = 0;
    const int tb = w & 1, mt = w >> 1;
    auto fetch = [&](const void *x, u32x4_t (&r)[PIECES]) {
#pragma unroll
        for (int i = 0; i < PIECES; ++i) {
            const int piece = i * 256 + tid;
            const int tc = min(t0 + piece / PPR, a.T - 1);
            r[i] = *(const u32x4_t *)((const uint16_t *)x + (((int64_t)b * a.T + tc) * a.H + h) * D + 8 * (piece % PPR));
        }
    };
    auto stage = [&](const u32x4_t (&r)[PIECES]) {
#pragma unroll
        for (int i = 0; i < PIECES; ++i) {
            const int piece = i * 256 + tid;
            *(u32x4_t *)(s_x + (piece / PPR) * RS + 8 * (piece % PPR)) = r[i];
        }
    };
    auto project = [&](f32x16 &acc) {
        acc = zero16();
#pragma unroll
        for (int st = 0; st < D / 16; ++st) {
            const frag x = *(const frag *)(s_x + (32 * tb + n) * RS + 16 * st + 8 * g);
            acc = MMA::mma(*(const frag *)(s_hi + (32 * mt + n) * RS + 16 * st + 8 * g), x, acc);
            acc = MMA::mma(*(const frag *)(s_lo + (32 * mt + n) * RS + 16 * st + 8 * g), x, acc);
        }
    };
    auto store = [&](void *out, const f32x16 &acc) {
        const int t = t0 + 32 * tb + n;
        if (t >= a.T) return;
        const int64_t orow = (((int64_t)b * a.T + t) * a.H + h) * a.out_width;
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4)
            IOBF16::store4(out, orow + 32 * mt + 8 * q4 + 4 * g, acc[4 * q4], acc[4 * q4 + 1], acc[4 * q4 + 2],
                           acc[4 * q4 + 3]);
    };

    const float *S = a.S + (a.per_head ? (int64_t)h * a.d_s * D : 0);
    for (int e = tid * 4; e < kSketchPad * D; e += 256 * 4) {
        const int i = e / D, j = e % D;
        f32x4 sv = {0.0f, 0.0f, 0.0f, 0.0f};
        if (i < a.d_s) sv = *(const f32x4 *)(S + (int64_t)i * D + j);
        float lo[4];
#pragma unroll
        for (int c = 0; c < 4; ++c) lo[c] = sv[c] - bf16_bits_to_f32(f32_to_bf16_bits(sv[c]));
        MMA::store4(s_hi + i * RS + j, sv);
        MMA::store4(s_lo + i * RS + j, f32x4{lo[0], lo[1], lo[2], lo[3]});
    }
    // kDownGroups groups of 64 tokens per workgroup: S is staged once for them
    for (int rep = 0; rep < kDownGroups; ++rep) {
        t0 = (blockIdx.y * kDownGroups + rep) * TOK;
        if (t0 >= a.T) break;                      // (whole workgroup)
        u32x4_t rq[PIECES], rk[PIECES];
        fetch(a.q, rq);
        fetch(a.k, rk);
        __syncthreads();                           // S is staged; the previous group's k rows have been read
        stage(rq);
        __syncthreads();
        // (32 stored features: the waves of the upper 32 have nothing to compute or store)
        const bool mine = 32 * mt < a.out_width;   // (wave-uniform)
        f32x16 acc;
        if (mine) project(acc);
        __syncthreads();                           // every wave has read its q rows
        stage(rk);
        if (mine) store(a.qs, acc);
        __syncthreads();
        if (mine) project(acc);
        if (mine) store(a.ks, acc);
    }
}

// xhat_t = S^T z_t as bf16 value (xhat_hi) and remainder (xhat_lo, optional). LDS: S^T as bf16 value and remainder,
// row-major [D][64 + 8].
template <int D>
__global__ __launch_bounds__(256) void sketch_up_kernel(SketchArgs a)
{
    constexpr int RS = kSketchPad + 8;
    constexpr int NB = D / 32;
    __shared__ __attribute__((aligned(16))) uint16_t s_hi[D * RS];
    __shared__ __attribute__((aligned(16))) uint16_t s_lo[D * RS];
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int n = lane & 31, g = lane >> 5;
    const int pair = blockIdx.x, b = pair / a.H, h = pair % a.H;
    const float *S = a.S + (a.per_head ? (int64_t)h * a.d_s * D : 0);
    for (int e = tid; e < kSketchPad * D; e += 256) {
        const int i = e / D, j = e % D;
        uint16_t hi, lo;
        split_bf16(i < a.d_s ? S[(int64_t)i * D + j] : 0.0f, hi, lo);
        s_hi[j * RS + i] = hi;
        s_lo[j * RS + i] = lo;
    }
    __syncthreads();
    for (int rep = 0; rep < kSketchReps; ++rep) {
    const int t = (blockIdx.y * kSketchReps + rep) * 128 + w * 32 + n;
    if (t - n >= a.T) break;                       // (wave-uniform)
    const int tc = min(t, a.T - 1);
    const float *zrow = a.z + (((int64_t)b * a.T + tc) * a.H + h) * kSketchPad;
    f32x16 acc[NB];
#pragma unroll
    for (int mt = 0; mt < NB; ++mt) acc[mt] = zero16();
#pragma unroll
    for (int st = 0; st < kSketchPad / 16; ++st) {
        float zf[8], back[8];
        const f32x4 z0 = *(const f32x4 *)(zrow + 16 * st + 8 * g), z1 = *(const f32x4 *)(zrow + 16 * st + 8 * g + 4);
#pragma unroll
        for (int e = 0; e < 4; ++e) { zf[e] = z0[e]; zf[4 + e] = z1[e]; }
        const frag zhi = MMA::pack(zf);
        MMA::unpack(zhi, back);
#pragma unroll
        for (int e = 0; e < 8; ++e) back[e] = zf[e] - back[e];
        const frag zlo = MMA::pack(back);
#pragma unroll
        for (int mt = 0; mt < NB; ++mt) {
            const frag shi = *(const frag *)(s_hi + (32 * mt + n) * RS + 16 * st + 8 * g);
            const frag slo = *(const frag *)(s_lo + (32 * mt + n) * RS + 16 * st + 8 * g);
            acc[mt] = MMA::mma(shi, zhi, acc[mt]);
            acc[mt] = MMA::mma(slo, zhi, acc[mt]);
            acc[mt] = MMA::mma(shi, zlo, acc[mt]);
        }
    }
    if (t < a.T) {
        const int64_t orow = (((int64_t)b * a.T + t) * a.H + h) * D;
#pragma unroll
        for (int mt = 0; mt < NB; ++mt)
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
                const int64_t o = orow + 32 * mt + 8 * q4 + 4 * g;
                float x[4], lo[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    x[e] = acc[mt][4 * q4 + e];
                    lo[e] = x[e] - bf16_bits_to_f32(f32_to_bf16_bits(x[e]));
                }
                IOBF16::store4(a.xhat_hi, o, x[0], x[1], x[2], x[3]);
                if (a.xhat_lo) IOBF16::store4(a.xhat_lo, o, lo[0], lo[1], lo[2], lo[3]);
            }
    }
    }
}

hipError_t launch_sketch(const SketchArgs &a, int n_pairs, int d, bool up, hipStream_t stream)
{
    if (!up && a.out_width != kSketchPad && !(a.out_width == 32 && a.d_s <= 32)) return hipErrorInvalidValue;
    const dim3 grid(n_pairs, (a.T + 127) / 128), grid_down(n_pairs, (a.T + 64 * kDownGroups - 1) / (64 * kDownGroups)), block(256);
    if (up) {
        if (d == 128) hipLaunchKernelGGL(sketch_up_kernel<128>, grid, block, 0, stream, a);
        else hipLaunchKernelGGL(sketch_up_kernel<64>, grid, block, 0, stream, a);
    } else {
        if (d == 128) hipLaunchKernelGGL(sketch_down_kernel<128>, grid_down, block, 0, stream, a);
        else hipLaunchKernelGGL(sketch_down_kernel<64>, grid_down, block, 0, stream, a);
    }
    return hipGetLastError();
}

}  // namespace gka
