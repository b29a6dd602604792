// Chunk initial states of Section 4.2.1: H_[n], U_[n] for every chunk of every (batch, head) pair.
//
// One workgroup owns a 32-wide slab of both states of one pair: H0[32*rb .. +32][:] and
// U0[32*rb .. +32][:], held as fp32 MFMA accumulators (wave w owns columns 32*w .. +32 of the slab),
// and walks a contiguous run of the pair's chunks in order. Per chunk it
//   1. (if asked) writes the slab, as it stands before the chunk, to the workspace in the fragment order
//      the solve kernel consumes, plus the slab's contribution to ||H_[n]||_F^2,
//   2. applies the chunk: S <- zeta_C S + sum_j (zeta_C / zeta_j) a_j k_j^T  (a = k for H, a = v for U),
//      the decay weights built in log space (Appendix B.2), as one MFMA contraction over the
//      chunk's tokens. The chunk's k rows and the slab's v columns are staged row-major in LDS and read
//      back transposed as MFMA operands; the next chunk's rows are fetched while the current one is used.
//
// The recurrence over chunks is an affine scan, S_[n+1] = zeta^(n) S_[n] + Delta_n. Long sequences are cut
// into segments: a first launch reduces every segment to (prod zeta, Delta) from a zero state; a second launch
// walks every segment again, from its true start state (a short scan over the summaries of the segments before
// it), and writes the chunk states.
#include "gka_device.hpp"
#include "gka_kernels.hpp"

namespace gka {

#ifdef GKA_DEBUG_TIMERS
__device__ unsigned long long g_dbg_state_timers[64 * 16];
#define GKA_STSTAMP(i)                                                                          \
    do {                                                                                        \
        if (threadIdx.x == 0 && blockIdx.x >= 1024 && blockIdx.x < 1088)                         \
            g_dbg_state_timers[(blockIdx.x - 1024) * 16 + (i)] = __builtin_amdgcn_s_memtime();  \
    } while (0)
extern "C" int gka_debug_read_state_timers(unsigned long long *host)
{
    return (int)hipMemcpyFromSymbol(host, HIP_SYMBOL(g_dbg_state_timers), sizeof(g_dbg_state_timers));
}
#else
#define GKA_STSTAMP(i) do {} while (0)
#endif

#ifndef GKA_STATE_WAVES
#define GKA_STATE_WAVES 2          // waves per SIMD the state-pass kernel is compiled for (register cap)
#endif

template <class MMA, class IO, int D>
__global__ __launch_bounds__(D * 2) __attribute__((amdgpu_waves_per_eu(GKA_STATE_WAVES))) void state_pass_kernel(StatePassArgs a)
{
    constexpr int NB = D / 32;
    constexpr int VEC = MMA::VEC;
    constexpr int HS = MMA::HS;
    constexpr int STEPS = kChunk / (2 * VEC);     // MFMA steps over the chunk's tokens
    constexpr int NT = D * 2;                     // threads
    constexpr int RS = D + MMA::kRowPad;
    constexpr int RSV = 32 + MMA::kRowPad;
    constexpr int KP = kChunk * (D / 4) / NT;     // 4-element pieces of k per thread (= 8)
    constexpr int VP = kChunk * 8 / NT;           // 4-element pieces of the v slab per thread
    typedef typename MMA::frag frag;
    typedef typename MMA::elem_t elem_t;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int w = tid >> 6;                       // column block of the slab owned by this wave
    const int n = lane & 31, g = lane >> 5;
    // Workgroups are dealt round-robin to the 8 XCDs, each with its own L2. The NB slabs of one (pair, segment)
    // read the same k rows, so they are given block indices that are equal modulo 8.
    int rb, group;
    {
        const int id = blockIdx.x;
        const int full = (gridDim.x / (8 * NB)) * (8 * NB);
        if (id < full) {
            const int within = id % (8 * NB);
            rb = within / 8;                       // slab index (row block of H0 / U0)
            group = (id / (8 * NB)) * 8 + within % 8;
        } else {
            rb = (id - full) % NB;
            group = full / NB + (id - full) / NB;
        }
    }
    // pairs vary fastest: workgroups that run together then read adjacent memory ([B,T,H,d]: heads are adjacent)
    const int pair = group % a.n_pairs;           // within this launch; indexes the workspace
    const int seg = group / a.n_pairs;
    const int b = (a.pair0 + pair) / a.H, h = (a.pair0 + pair) % a.H;

    // Both operands of S += sum_j w_j a_j k_j^T carry sqrt(w_j): (sqrt(w_j) a_j)(sqrt(w_j) k_j)^T.
    __shared__ __attribute__((aligned(16))) elem_t s_k[kChunk * RS];    // k rows of the chunk, scaled
    __shared__ __attribute__((aligned(16))) elem_t s_v[kChunk * RSV];   // the slab's 32 columns of the v rows, scaled

    const int64_t base_bh = (int64_t)b * a.stride_b + (int64_t)h * a.stride_h;
    const int64_t gate_base = (int64_t)b * a.T * a.H + h;
    const int chunk_begin = seg * a.seg_len;
    const int chunk_end = min(chunk_begin + a.seg_len, a.n_chunks_total);
    // per (pair, segment, slab, wave): two 16x64 float tiles in accumulator order
    auto seg_tile = [&](int sg) {
        return a.seg_buf + ((((int64_t)(pair * a.n_segs + sg) * NB + rb) * NB + w) * 2) * 1024;
    };

    // accumulators: element (row = 32*w + kidx(r,g), col n) = S0[32*rb + n][32*w + kidx(r,g)]
    f32x16 accH = zero16(), accU = zero16();
    if (a.init_mode != 0) {
        if (a.H_init) {
            const float *Hi = a.H_init + (int64_t)(a.pair0 + pair) * D * D;
            const float *Ui = a.U_init + (int64_t)(a.pair0 + pair) * D * D;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                int col = 32 * w + kidx(r, g);
                accH[r] = Hi[(int64_t)(32 * rb + n) * D + col];
                accU[r] = Ui[(int64_t)(32 * rb + n) * D + col];
            }
        }
        // start state of this segment: scan of the summaries (decay, Delta) of the segments before it
        for (int sg = 0; sg < seg; ++sg) {
            const float *t = seg_tile(sg);
            const float decay = exp2f(a.seg_logdecay[pair * a.n_segs + sg]);
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                accH[r] = decay * accH[r] + t[r * 64 + lane];
                accU[r] = decay * accU[r] + t[1024 + r * 64 + lane];
            }
        }
    }

    // Register prefetch, two chunks deep. Rows past the end of the sequence are read from the last valid row (a
    // divergent branch around a load would force a wait on it) and zeroed when they are stored to LDS.
    struct Fetch {
        typename IO::raw4 k[KP], v[VP];
        float gate;
    };
    auto fetch = [&](Fetch &f, int c) {
#pragma unroll
        for (int i = 0; i < KP; ++i) {
            const int piece = i * NT + tid;
            const int row = piece / (D / 4), c4 = piece % (D / 4);
            const int t = min(c * kChunk + row, a.T - 1);
            f.k[i] = IO::load_raw4(a.k, base_bh + (int64_t)t * a.stride_t + 4 * c4);
        }
#pragma unroll
        for (int i = 0; i < VP; ++i) {
            const int piece = i * NT + tid;
            const int row = piece / 8, c4 = piece % 8;
            const int t = min(c * kChunk + row, a.T - 1);
            f.v[i] = IO::load_raw4(a.v, base_bh + (int64_t)t * a.stride_t + 32 * rb + 4 * c4);
        }
        const int t = min(c * kChunk + lane, a.T - 1);
        f.gate = a.gate[gate_base + (int64_t)t * a.H];
    };
    float Gseg = 0.0f;

    auto process = [&](const Fetch &f, int c) {
        const bool stamp = (c == chunk_begin + 2);
        if (stamp) GKA_STSTAMP(1);
        // ---- gates of the chunk: G_j = sum_{i<=j} log2 gamma_i, weights 2^(G_C - G_j)
        const float lg = (c * kChunk + lane < a.T) ? log2_gate(f.gate) : 0.0f;
        const float G = wave_inclusive_scan(lg, lane);
        const float Gtot = __shfl(G, 63, 64);
        Gseg += Gtot;
        const float swd = exp2f(0.5f * (Gtot - G));   // lane j: sqrt(zeta_C / zeta_j)
        if (stamp) GKA_STSTAMP(2);
        __syncthreads();                          // previous chunk's LDS readers are done
        if (stamp) GKA_STSTAMP(3);
#pragma unroll
        for (int i = 0; i < KP; ++i) {
            const int piece = i * NT + tid;
            const int row = piece / (D / 4);
            f32x4 kv = IO::cvt4(f.k[i]);
            if (c * kChunk + row >= a.T) kv = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
            MMA::store4(s_k + row * RS + 4 * (piece % (D / 4)), kv * __shfl(swd, row, 64));
        }
#pragma unroll
        for (int i = 0; i < VP; ++i) {
            const int piece = i * NT + tid;
            const int row = piece / 8;
            f32x4 vv = IO::cvt4(f.v[i]);
            if (c * kChunk + row >= a.T) vv = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
            MMA::store4(s_v + row * RSV + 4 * (piece % 8), vv * __shfl(swd, row, 64));
        }
        const float zetaC = exp2f(Gtot);
        if (stamp) GKA_STSTAMP(4);

        // ---- write the state before the chunk, fragment order
        if (a.write_frags) {
            const int64_t chunk_id = (int64_t)pair * a.n_chunks_total + c;
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
                frag fr = MMA::pack(vals + hh * VEC);
                Uw[((rb * NB + w) * HS + hh) * 64 + lane] = fr;
                if (NSPL == 2) {
#pragma unroll
                    for (int p = 0; p < VEC; ++p) lo[hh * VEC + p] = vals[hh * VEC + p] - MMA::elem(fr, p);
                }
            }
            if (NSPL == 2) {
#pragma unroll
                for (int hh = 0; hh < HS; ++hh)
                    Uw[(NB * NB * HS + (rb * NB + w) * HS + hh) * 64 + lane] = MMA::pack(lo + hh * VEC);
            }
        }
        if (stamp) GKA_STSTAMP(5);
        __syncthreads();                          // s_k, s_v visible
        if (stamp) GKA_STSTAMP(6);

        // ---- S <- zeta_C S + sum_j w_j a_j k_j^T
#pragma unroll
        for (int r = 0; r < 16; ++r) { accH[r] *= zetaC; accU[r] *= zetaC; }
#pragma unroll
        for (int s = 0; s < STEPS; ++s) {
            // lane (n, g): tokens j = s*2*VEC + g*VEC + p of the chunk
            const int j0 = s * 2 * VEC + g * VEC;
            frag fa, fk, fv;
            if constexpr (MMA::VEC == 8) {
                const int sub = 16 * ((lane >> 4) & 1);      // this 16-lane block's columns within the 32
                fa = gather_transposed_bf16(s_k, PaddedRows{RS}, 32 * w + sub, lane, j0, j0 + 4);
                fk = gather_transposed_bf16(s_k, PaddedRows{RS}, 32 * rb + sub, lane, j0, j0 + 4);
                fv = gather_transposed_bf16(s_v, PaddedRows{RSV}, sub, lane, j0, j0 + 4);
            } else {
                auto tok_of = [&](int p) { return j0 + p; };
                fa = gather_transposed<MMA>(s_k, PaddedRows{RS}, 32 * w + n, tok_of);
                fk = gather_transposed<MMA>(s_k, PaddedRows{RS}, 32 * rb + n, tok_of);
                fv = gather_transposed<MMA>(s_v, PaddedRows{RSV}, n, tok_of);
            }
            accH = MMA::mma(fa, fk, accH);
            accU = MMA::mma(fa, fv, accU);
        }
        if (stamp) GKA_STSTAMP(7);
    };

    // two fetch buffers in flight: while chunk c is processed, chunks c + 1 and c + 2 are on their way
    Fetch f0, f1;
    GKA_STSTAMP(0);
    if (chunk_begin < chunk_end) fetch(f0, chunk_begin);
    if (chunk_begin + 1 < chunk_end) fetch(f1, chunk_begin + 1);
    for (int c = chunk_begin; c < chunk_end; c += 2) {
        process(f0, c);
        if (c + 2 < chunk_end) fetch(f0, c + 2);
        if (c + 1 < chunk_end) {
            process(f1, c + 1);
            if (c + 3 < chunk_end) fetch(f1, c + 3);
        }
    }

    GKA_STSTAMP(8);
    if (a.final_mode == 1) {
        if (a.H_final && seg == a.n_segs - 1) {
            float *Hf = a.H_final + (int64_t)(a.pair0 + pair) * D * D;
            float *Uf = a.U_final + (int64_t)(a.pair0 + pair) * D * D;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                int col = 32 * w + kidx(r, g);
                Hf[(int64_t)(32 * rb + n) * D + col] = accH[r];
                Uf[(int64_t)(32 * rb + n) * D + col] = accU[r];
            }
        }
    } else if (a.final_mode == 2) {
        float *t = seg_tile(seg);
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            t[r * 64 + lane] = accH[r];
            t[1024 + r * 64 + lane] = accU[r];
        }
        if (rb == 0 && tid == 0) a.seg_logdecay[pair * a.n_segs + seg] = Gseg;
    }
}

template <class MMA, class IO, int D>
static hipError_t launch_state_pass_t(const StatePassArgs &a0, int n_pairs, hipStream_t stream)
{
    constexpr int NB = D / 32;
    dim3 block(D * 2);
    StatePassArgs a = a0;
    a.n_pairs = n_pairs;
    if (a.n_segs <= 1) {
        a.n_segs = 1;
        a.seg_len = a.n_chunks_total;
    } else {
        // summaries (decay, Delta from a zero state) of every segment but the last
        a.init_mode = 0;
        a.final_mode = 2;
        a.write_frags = 0;
        hipLaunchKernelGGL((state_pass_kernel<MMA, IO, D>), dim3(n_pairs * NB * (a.n_segs - 1)), block, 0, stream, a);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    // every segment from its true start state (H_init / U_init scanned with the summaries before it)
    a.init_mode = 1;
    a.final_mode = 1;
    a.write_frags = 1;
    hipLaunchKernelGGL((state_pass_kernel<MMA, IO, D>), dim3(n_pairs * NB * a.n_segs), block, 0, stream, a);
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
