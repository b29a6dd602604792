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
// into segments: a first launch reduces every segment to (prod zeta, Delta) from a zero state, a small
// combine kernel scans the segment summaries into segment start states, and a second launch walks every
// segment from its true start state and writes the chunk states.
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

    __shared__ __attribute__((aligned(16))) elem_t s_k[kChunk * RS];    // k rows of the chunk
    __shared__ __attribute__((aligned(16))) elem_t s_ks[kChunk * RS];   // k rows scaled by zeta_C / zeta_j
    __shared__ __attribute__((aligned(16))) elem_t s_v[kChunk * RSV];   // the slab's 32 columns of the v rows

    const int64_t base_bh = (int64_t)b * a.stride_b + (int64_t)h * a.stride_h;
    const int64_t gate_base = (int64_t)b * a.T * a.H + h;
    const int chunk_begin = seg * a.seg_len;
    const int chunk_end = min(chunk_begin + a.seg_len, a.n_chunks_total);
    float *segH = a.seg_buf + ((((int64_t)(pair * a.n_segs + seg) * NB + rb) * NB + w) * 2 + 0) * 1024;
    float *segU = segH + 1024;

    // accumulators: element (row = 32*w + kidx(r,g), col n) = S0[32*rb + n][32*w + kidx(r,g)]
    f32x16 accH = zero16(), accU = zero16();
    if (a.init_mode == 1) {
        const float *Hi = a.H_init + (int64_t)(a.pair0 + pair) * D * D;
        const float *Ui = a.U_init + (int64_t)(a.pair0 + pair) * D * D;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            int col = 32 * w + kidx(r, g);
            accH[r] = Hi[(int64_t)(32 * rb + n) * D + col];
            accU[r] = Ui[(int64_t)(32 * rb + n) * D + col];
        }
    } else if (a.init_mode == 2) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            accH[r] = segH[r * 64 + lane];
            accU[r] = segU[r * 64 + lane];
        }
    }

    // prefetch registers for the next chunk's rows
    // Rows past the end of the sequence are read from the last valid row (a divergent branch around a load
    // would force a wait on it) and zeroed when they are stored to LDS.
    typename IO::raw4 kreg[KP], vreg[VP];
    float gate_next = 1.0f;
    auto fetch = [&](int c) {
#pragma unroll
        for (int i = 0; i < KP; ++i) {
            const int piece = i * NT + tid;
            const int row = piece / (D / 4), c4 = piece % (D / 4);
            const int t = min(c * kChunk + row, a.T - 1);
            kreg[i] = IO::load_raw4(a.k, base_bh + (int64_t)t * a.stride_t + 4 * c4);
        }
#pragma unroll
        for (int i = 0; i < VP; ++i) {
            const int piece = i * NT + tid;
            const int row = piece / 8, c4 = piece % 8;
            const int t = min(c * kChunk + row, a.T - 1);
            vreg[i] = IO::load_raw4(a.v, base_bh + (int64_t)t * a.stride_t + 32 * rb + 4 * c4);
        }
        const int t = min(c * kChunk + lane, a.T - 1);
        gate_next = a.gate[gate_base + (int64_t)t * a.H];
    };
    if (chunk_begin < chunk_end) fetch(chunk_begin);
    float Gseg = 0.0f;

    for (int c = chunk_begin; c < chunk_end; ++c) {
        // ---- gates of the chunk: G_j = sum_{i<=j} log gamma_i, weights exp(G_C - G_j)
        const float lg = (c * kChunk + lane < a.T) ? log2_gate(gate_next) : 0.0f;
        const float G = wave_inclusive_scan(lg, lane);
        const float Gtot = __shfl(G, 63, 64);
        Gseg += Gtot;
        const float wd = exp2f(Gtot - G);          // lane j: zeta_C / zeta_j
        __syncthreads();                          // previous chunk's LDS readers are done
#pragma unroll
        for (int i = 0; i < KP; ++i) {
            const int piece = i * NT + tid;
            const int row = piece / (D / 4);
            f32x4 kv = IO::cvt4(kreg[i]);
            if (c * kChunk + row >= a.T) kv = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
            MMA::store4(s_k + row * RS + 4 * (piece % (D / 4)), kv);
            const float wrow = __shfl(wd, row, 64);
            MMA::store4(s_ks + row * RS + 4 * (piece % (D / 4)), kv * wrow);
        }
#pragma unroll
        for (int i = 0; i < VP; ++i) {
            const int piece = i * NT + tid;
            f32x4 vv = IO::cvt4(vreg[i]);
            if (c * kChunk + piece / 8 >= a.T) vv = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
            MMA::store4(s_v + (piece / 8) * RSV + 4 * (piece % 8), vv);
        }
        if (c + 1 < chunk_end) fetch(c + 1);      // in flight while this chunk is processed
        const float zetaC = exp2f(Gtot);

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
        __syncthreads();                          // s_k, s_ks, s_v visible

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
                fa = gather_transposed_bf16(s_ks, RS, 32 * w + sub, lane, j0, j0 + 4);
                fk = gather_transposed_bf16(s_k, RS, 32 * rb + sub, lane, j0, j0 + 4);
                fv = gather_transposed_bf16(s_v, RSV, sub, lane, j0, j0 + 4);
            } else {
                auto tok_of = [&](int p) { return j0 + p; };
                fa = gather_transposed<MMA>(s_ks, RS, 32 * w + n, tok_of);
                fk = gather_transposed<MMA>(s_k, RS, 32 * rb + n, tok_of);
                fv = gather_transposed<MMA>(s_v, RSV, n, tok_of);
            }
            accH = MMA::mma(fa, fk, accH);
            accU = MMA::mma(fa, fv, accU);
        }
    }

    if (a.final_mode == 1) {
        float *Hf = a.H_final + (int64_t)(a.pair0 + pair) * D * D;
        float *Uf = a.U_final + (int64_t)(a.pair0 + pair) * D * D;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            int col = 32 * w + kidx(r, g);
            Hf[(int64_t)(32 * rb + n) * D + col] = accH[r];
            Uf[(int64_t)(32 * rb + n) * D + col] = accU[r];
        }
    } else if (a.final_mode == 2) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            segH[r * 64 + lane] = accH[r];
            segU[r * 64 + lane] = accU[r];
        }
        if (rb == 0 && tid == 0) a.seg_logdecay[pair * a.n_segs + seg] = Gseg;
    }
}

// Scan of the segment summaries: seg_buf[s] holds Delta_s on entry and the start state of segment s on
// exit; the state after the last segment goes to H_final / U_final when requested.
template <int D>
__global__ __launch_bounds__(D * 2) void segment_combine_kernel(StatePassArgs a)
{
    constexpr int NB = D / 32;
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int n = lane & 31, g = lane >> 5;
    const int rb = blockIdx.x % NB;
    const int pair = blockIdx.x / NB;
    float sH[16], sU[16];
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        sH[r] = 0.0f;
        sU[r] = 0.0f;
        if (a.H_init) {
            int col = 32 * w + kidx(r, g);
            sH[r] = a.H_init[(int64_t)(a.pair0 + pair) * D * D + (int64_t)(32 * rb + n) * D + col];
            sU[r] = a.U_init[(int64_t)(a.pair0 + pair) * D * D + (int64_t)(32 * rb + n) * D + col];
        }
    }
    for (int seg = 0; seg < a.n_segs; ++seg) {
        float *segH = a.seg_buf + ((((int64_t)(pair * a.n_segs + seg) * NB + rb) * NB + w) * 2 + 0) * 1024;
        float *segU = segH + 1024;
        const float decay = exp2f(a.seg_logdecay[pair * a.n_segs + seg]);
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const float dH = segH[r * 64 + lane], dU = segU[r * 64 + lane];
            segH[r * 64 + lane] = sH[r];
            segU[r * 64 + lane] = sU[r];
            sH[r] = decay * sH[r] + dH;
            sU[r] = decay * sU[r] + dU;
        }
    }
    if (a.H_final) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            int col = 32 * w + kidx(r, g);
            a.H_final[(int64_t)(a.pair0 + pair) * D * D + (int64_t)(32 * rb + n) * D + col] = sH[r];
            a.U_final[(int64_t)(a.pair0 + pair) * D * D + (int64_t)(32 * rb + n) * D + col] = sU[r];
        }
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
        a.init_mode = a.H_init ? 1 : 0;
        a.final_mode = a.H_final ? 1 : 0;
        a.write_frags = 1;
        hipLaunchKernelGGL((state_pass_kernel<MMA, IO, D>), dim3(n_pairs * NB), block, 0, stream, a);
        return hipGetLastError();
    }
    dim3 grid(n_pairs * NB * a.n_segs);
    a.init_mode = 0;
    a.final_mode = 2;
    a.write_frags = 0;
    hipLaunchKernelGGL((state_pass_kernel<MMA, IO, D>), grid, block, 0, stream, a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL((segment_combine_kernel<D>), dim3(n_pairs * NB), block, 0, stream, a);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    a.init_mode = 2;
    a.final_mode = 0;
    a.write_frags = 1;
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
