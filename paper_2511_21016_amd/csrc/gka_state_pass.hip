// Chunk initial states of Section 4.2.1: H_[n], U_[n] for every chunk of every (batch, head) pair.
//
// One workgroup owns a 32-wide slab of ONE of the two states of one pair, H0[32*rb .. +32][:] or
// U0[32*rb .. +32][:], held as fp32 MFMA accumulators (wave w owns columns 32*w .. +32 of the slab),
// and walks a contiguous run of the pair's chunks in order. Per chunk it
//   1. (if asked) writes the slab, as it stands before the chunk, to the workspace in the fragment order
//      the solve kernel consumes (H: bf16 or fp32 operands plus the slab's share of ||H_[n]||_F^2; U: the operand
//      and, for bf16, what the rounding left over as a second operand),
//   2. applies the chunk: S <- zeta_C S + sum_j (zeta_C / zeta_j) a_j k_j^T  (a = k for H, a = v for U),
//      the decay weights built in log space (Appendix B.2), as one MFMA contraction over the chunk's tokens.
// Two bodies implement the walk. The generic one (fp32 operands, one workgroup per slab as above) stages the k rows
// and the slab's columns of a, each scaled by the square root of the weight, through registers into padded LDS tiles.
// The bf16 one owns all row blocks of a state in one workgroup, copies the k rows from global memory straight into
// LDS one chunk ahead and puts the whole weight on the a tile; see state_pass_body_bf16_tile.
//
// The recurrence over chunks is an affine scan, S_[n+1] = zeta^(n) S_[n] + Delta_n. Long sequences are cut
// into segments: a first launch reduces every segment to (prod zeta, Delta) from a zero state; a second launch
// walks every segment again, from its true start state (a short scan over the summaries of the segments before
// it), and writes the chunk states.
#include "gka_device.hpp"
#include "gka_kernels.hpp"

namespace gka {

// Chunk states are written once and read once, by another kernel, after hundreds of megabytes of other states:
// non-temporal stores (measured: the state phase of configuration 2 goes from 0.160 to 0.134 ms).
template <class T>
__device__ __forceinline__ void store_once(T *dst, T value) { __builtin_nontemporal_store(value, dst); }


constexpr int kStateWavesPerSimd = 2;      // waves per SIMD the state-pass kernels are compiled for (register cap)

// Start state of a workgroup's slab: the caller's initial state scanned with the summaries (decay, Delta) of the
// segments before this one. Accumulator element (r, lane (n, g)) = S0[32*rb + n][32*w + kidx(r, g)].
template <int D>
__device__ __forceinline__ float *segment_tile(const StatePassArgs &a, int pair, int sg, int rb, int w)
{
    constexpr int NB = D / 32;
    return a.seg_buf + ((((int64_t)(pair * a.n_segs + sg) * NB + rb) * NB + w) * 2) * 1024;
}
template <int D, bool DOH>
__device__ __forceinline__ void load_start_state(const StatePassArgs &a, f32x16 &acc, int pair, int seg, int rb, int w,
                                                 int lane)
{
    if (a.init_mode == 0) return;
    const int n = lane & 31, g = lane >> 5;
    if (a.H_init) {
        const float *Si = (DOH ? a.H_init : a.U_init) + (int64_t)(a.init_pair0 + pair) * D * D;
        if (DOH && a.h_init_lower_blocks && w > rb) {      // H is symmetric: block (rb, w) = block (w, rb) transposed
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[r] = Si[(int64_t)(32 * w + kidx(r, g)) * D + 32 * rb + n];
        } else {
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[r] = Si[(int64_t)(32 * rb + n) * D + 32 * w + kidx(r, g)];
        }
    }
    for (int sg = 0; sg < seg; ++sg) {
        const float *t = segment_tile<D>(a, pair, sg, rb, w) + (DOH ? 0 : 1024);
        const float decay = exp2f(a.seg_logdecay[pair * a.n_segs + sg]);
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[r] = decay * acc[r] + t[r * 64 + lane];
    }
}
// End of the walk: the final state (last segment of the full pass) or this segment's summary.
template <int D, bool DOH>
__device__ __forceinline__ void store_end_state(const StatePassArgs &a, const f32x16 &acc, float Gseg, int pair, int seg,
                                                int rb, int w, int lane)
{
    const int n = lane & 31, g = lane >> 5;
    if (a.final_mode == 1) {
        if (a.H_final && seg == a.n_segs - 1) {
            float *Sf = (DOH ? a.H_final : a.U_final) + (int64_t)(a.final_pair0 + pair) * D * D;
#pragma unroll
            for (int r = 0; r < 16; ++r) Sf[(int64_t)(32 * rb + n) * D + 32 * w + kidx(r, g)] = acc[r];
        }
    } else if (a.final_mode == 2) {
        float *t = segment_tile<D>(a, pair, seg, rb, w) + (DOH ? 0 : 1024);
#pragma unroll
        for (int r = 0; r < 16; ++r) t[r * 64 + lane] = acc[r];
        // (the H workgroup's job; in a launch without H workgroups the U workgroup's)
        if (rb == 0 && (DOH || a.only_u) && threadIdx.x == 0) a.seg_logdecay[pair * a.n_segs + seg] = Gseg;
    }
}

// DOH: this workgroup owns the H slab (else the U slab); WRITE: chunk states are written to the workspace. Both are
// compile-time so that the chunk loop is straight-line code and the in-flight prefetches are never drained by a
// conservative wait.
template <class MMA, class IO, int D, bool DOH, bool WRITE, bool GATED>
__device__ __forceinline__ void state_pass_body(const StatePassArgs &a, int rb, int group,
                                                typename MMA::elem_t *s_k, typename MMA::elem_t *s_v)
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
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);   // column block of the slab owned by this wave (uniform)
    const int n = lane & 31, g = lane >> 5;
    constexpr bool doH = DOH;
    // pairs vary fastest: workgroups that run together then read adjacent memory ([B,T,H,d]: heads are adjacent)
    const int pair = group % a.n_pairs;           // within this launch; indexes the workspace
    const int seg = group / a.n_pairs;
    const int b = (a.pair0 + pair) / a.H, h = (a.pair0 + pair) % a.H;

    // Both operands of S += sum_j w_j a_j k_j^T carry sqrt(w_j): (sqrt(w_j) a_j)(sqrt(w_j) k_j)^T.
    // s_k: k rows of the chunk, scaled; s_v: the slab's 32 columns of the v rows, scaled.

    const int64_t base_bh = (int64_t)b * a.stride_b + (int64_t)h * a.stride_h;
    const int64_t gate_base = (int64_t)b * a.T * a.H + h;
    const int chunk_begin = a.chunk0 + seg * a.seg_len;
    const int chunk_end = min(chunk_begin + a.seg_len, a.chunk0 + a.n_chunks);
    // per (pair, segment, slab, wave): two 16x64 float tiles in accumulator order
    auto seg_tile = [&](int sg) {
        return a.seg_buf + ((((int64_t)(pair * a.n_segs + sg) * NB + rb) * NB + w) * 2) * 1024;
    };

    // accumulators: element (row = 32*w + kidx(r,g), col n) = S0[32*rb + n][32*w + kidx(r,g)]
    f32x16 acc = zero16();                        // this workgroup's state: H (doH) or U
    const int tile_off = doH ? 0 : 1024;
    load_start_state<D, DOH>(a, acc, pair, seg, rb, w, lane);

    // Register prefetch, two chunks deep. Rows past the end of the sequence are read from the last valid row (a
    // divergent branch around a load would force a wait on it) and zeroed when they are stored to LDS.
    struct Fetch {
        typename IO::raw4 k[KP], v[VP];
        float gate, beta;
    };
    // without a write gate the gates are read a second time and the value is replaced by 1: no branch around a load
    const float *beta_src = a.beta ? a.beta : a.gate;
    auto fetch = [&](Fetch &f, int c) {
#pragma unroll
        for (int i = 0; i < KP; ++i) {
            const int piece = i * NT + tid;
            const int row = piece / (D / 4), c4 = piece % (D / 4);
            const int t = min(c * kChunk + row, a.T - 1);
            f.k[i] = IO::load_raw4(a.k, base_bh + (int64_t)t * a.stride_t + 4 * c4);
        }
        if (!doH) {
#pragma unroll
            for (int i = 0; i < VP; ++i) {
                const int piece = i * NT + tid;
                const int row = piece / 8, c4 = piece % 8;
                const int t = min(c * kChunk + row, a.T - 1);
                f.v[i] = IO::load_raw4(a.v, base_bh + (int64_t)t * a.stride_t + 32 * rb + 4 * c4);
            }
        }
        const int t = min(c * kChunk + lane, a.T - 1);
        f.gate = a.gate[gate_base + (int64_t)t * a.H];
        if constexpr (GATED) f.beta = beta_src[gate_base + (int64_t)t * a.H];
    };
    float Gseg = 0.0f;

    auto process = [&](const Fetch &f, int c) {
        // ---- gates of the chunk: G_j = sum_{i<=j} log2 gamma_i, weights beta_j 2^(G_C - G_j)
        const float lg = (c * kChunk + lane < a.T) ? log2_gate(f.gate) : 0.0f;
        const float G = wave_inclusive_scan(lg, lane);
        const float Gtot = lane_value(G, 63);
        Gseg += Gtot;
        float swd = exp2f(0.5f * (Gtot - G));          // lane j: sqrt(beta_j zeta_C / zeta_j)
        if constexpr (GATED) swd *= sqrtf(a.beta ? f.beta : 1.0f);
        lds_barrier();                          // previous chunk's LDS readers are done
#pragma unroll
        for (int i = 0; i < KP; ++i) {
            const int piece = i * NT + tid;
            const int row = piece / (D / 4);
            f32x4 kv = IO::cvt4(f.k[i]);
            if (c * kChunk + row >= a.T) kv = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
            // the wave's 64 pieces of this sweep lie in two consecutive rows
            const int row0 = (i * NT + 64 * w) / (D / 4);
            const float sw = (D / 4 == 32) ? ((lane < 32) ? lane_value(swd, row0) : lane_value(swd, row0 + 1))
                                           : __shfl(swd, row, 64);
            MMA::store4(s_k + row * RS + 4 * (piece % (D / 4)), kv * sw);
        }
        if (!doH) {
#pragma unroll
            for (int i = 0; i < VP; ++i) {
                const int piece = i * NT + tid;
                const int row = piece / 8;
                f32x4 vv = IO::cvt4(f.v[i]);
                if (c * kChunk + row >= a.T) vv = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
                MMA::store4(s_v + row * RSV + 4 * (piece % 8), vv * __shfl(swd, row, 64));
            }
        }
        const float zetaC = exp2f(Gtot);

        // ---- write the state before the chunk, fragment order
        if (WRITE) {
            const int64_t chunk_id = (int64_t)(c - a.chunk0) * a.n_pairs + pair;   // chunk-major: pairs adjacent
            float vals[16];
#pragma unroll
            for (int r = 0; r < 16; ++r) vals[r] = acc[r];
            if (doH) {
                frag *Hw = (frag *)a.ws_H + chunk_id * (NB * NB * HS * 64);
                float ss = 0.0f;
#pragma unroll
                for (int r = 0; r < 16; ++r) ss += acc[r] * acc[r];
#pragma unroll
                for (int hh = 0; hh < HS; ++hh)
                    store_once(&Hw[((rb * NB + w) * HS + hh) * 64 + lane], MMA::pack(vals + hh * VEC));
                ss = wave_sum(ss);
                if (lane == 0) a.ws_hn[chunk_id * (NB * NB) + rb * NB + w] = ss;
            } else {
                constexpr int NSPL = MMA::kSplitReadout ? 2 : 1;
                frag *Uw = (frag *)a.ws_U + chunk_id * (NSPL * NB * NB * HS * 64);
                float lo[16];
#pragma unroll
                for (int hh = 0; hh < HS; ++hh) {
                    frag fr = MMA::pack(vals + hh * VEC);
                    store_once(&Uw[((rb * NB + w) * HS + hh) * 64 + lane], fr);
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
        }
        lds_barrier();                          // s_k, s_v visible

        // ---- S <- zeta_C S + sum_j w_j a_j k_j^T
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[r] *= zetaC;
#pragma unroll
        for (int s = 0; s < STEPS; ++s) {
            // lane (n, g): tokens j = s*2*VEC + g*VEC + p of the chunk
            const int j0 = s * 2 * VEC + g * VEC;
            // B operand: the slab's columns of the scaled k rows (H) or of the scaled v rows (U)
            const elem_t *bt = doH ? s_k : s_v;
            const PaddedRows bl{doH ? RS : RSV};
            const int bcol = doH ? 32 * rb : 0;
            frag fa, fb;
            if constexpr (MMA::VEC == 8) {
                const int sub = 16 * ((lane >> 4) & 1);      // this 16-lane block's columns within the 32
                fa = gather_transposed_bf16(s_k, PaddedRows{RS}, 32 * w + sub, lane, j0, j0 + 4);
                fb = gather_transposed_bf16(bt, bl, bcol + sub, lane, j0, j0 + 4);
            } else {
                auto tok_of = [&](int p) { return j0 + p; };
                fa = gather_transposed<MMA>(s_k, PaddedRows{RS}, 32 * w + n, tok_of);
                fb = gather_transposed<MMA>(bt, bl, bcol + n, tok_of);
            }
            acc = MMA::mma(fa, fb, acc);
        }
    };

    // two fetch buffers in flight: while chunk c is processed, chunks c + 1 and c + 2 are on their way
    // (fetches past the end of the run re-read its last chunk: harmless, and it keeps the loop free of branches
    // around memory operations)
    // An odd chunk count is evened out in front of the loop, with a fetch of its own, so that the loop body is the
    // only user of the two prefetch buffers.
    const int c_last = max(chunk_end - 1, chunk_begin);
    int c = chunk_begin;
    if ((chunk_end - chunk_begin) & 1) {
        Fetch fp;
        fetch(fp, c);
        process(fp, c);
        ++c;
    }
    if (c < chunk_end) {
        Fetch f0, f1;
        fetch(f0, c);
        fetch(f1, c + 1);
        for (; c < chunk_end; c += 2) {
            process(f0, c);
            fetch(f0, min(c + 2, c_last));
            process(f1, c + 1);
            fetch(f1, min(c + 3, c_last));
        }
    }

    if (a.final_mode == 1) {
        if (a.H_final && seg == a.n_segs - 1) {
            float *Sf = (doH ? a.H_final : a.U_final) + (int64_t)(a.final_pair0 + pair) * D * D;
#pragma unroll
            for (int r = 0; r < 16; ++r) Sf[(int64_t)(32 * rb + n) * D + 32 * w + kidx(r, g)] = acc[r];
        }
    } else if (a.final_mode == 2) {
        float *t = seg_tile(seg);
#pragma unroll
        for (int r = 0; r < 16; ++r) t[tile_off + r * 64 + lane] = acc[r];
        if (rb == 0 && (doH || a.only_u) && tid == 0) a.seg_logdecay[pair * a.n_segs + seg] = Gseg;
    }
}

// vmcnt(n) wait with the other counters left alone (gfx9 encoding: vmcnt in bits 3:0 and 15:14, expcnt 6:4,
// lgkmcnt 11:8). The compiler moves no memory operation across it.
template <int N>
__device__ __forceinline__ void wait_vector_memory_upto()
{
    static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
    asm volatile("s_waitcnt %0" ::"n"((N & 15) | ((N >> 4) << 14) | (7 << 4) | (15 << 8)) : "memory");
}
// Everything this wave has issued to vector memory has completed. The intrinsic tells the compiler's own wait
// bookkeeping so (it does not look inside assembly statements); the assembly statement keeps memory operations
// from moving across.
__device__ __forceinline__ void drain_vector_memory()
{
    __builtin_amdgcn_s_waitcnt(0 | (7 << 4) | (15 << 8));
    asm volatile("" ::: "memory");
}

__device__ __forceinline__ uint32_t lds_address(const void *p)
{
    return (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const void *)p;
}

// ---------------------------------------------------------------------------------------------------------------
// Whole-tile variant of the bf16 body: one workgroup owns all row blocks of one state (H or U) of a pair and walks
// a segment of its chunks. Wave w keeps column block w of every row block (NB accumulators), so its A fragments (the
// chunk's unscaled k columns of block w) are read once and used NB times, and the latency of a chunk step (barriers,
// LDS round trips, the wait for the copies) is paid once for NB times the work of a slab step. The B tile holds all
// D columns of the scaled k (H) or v (U) rows. Two k buffers (copy one chunk ahead).
typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));

// Four transpose reads (one per MFMA step, STEP bytes apart) from one lane address; not waited for here.
template <int STEP>
__device__ __forceinline__ void issue_tr4(uint32_t addr, u32x2_t (&r)[4])
{
    asm volatile("ds_read_b64_tr_b16 %0, %4\n\t"
                 "ds_read_b64_tr_b16 %1, %4 offset:%5\n\t"
                 "ds_read_b64_tr_b16 %2, %4 offset:%6\n\t"
                 "ds_read_b64_tr_b16 %3, %4 offset:%7"
                 : "=&v"(r[0]), "=&v"(r[1]), "=&v"(r[2]), "=&v"(r[3])
                 : "v"(addr), "n"(STEP), "n"(2 * STEP), "n"(3 * STEP)
                 : "memory");
}
// At most N LDS operations issued after the reads into lo / hi are still outstanding: those reads have landed. The
// registers pass through the statement so that their uses stay behind it.
template <int N>
__device__ __forceinline__ void await_tr8(u32x2_t (&lo)[4], u32x2_t (&hi)[4])
{
    asm volatile("s_waitcnt lgkmcnt(%8)"
                 : "+v"(lo[0]), "+v"(lo[1]), "+v"(lo[2]), "+v"(lo[3]), "+v"(hi[0]), "+v"(hi[1]), "+v"(hi[2]), "+v"(hi[3])
                 : "n"(N)
                 : "memory");
}
__device__ __forceinline__ bf16x8 join_runs(const u32x2_t &lo, const u32x2_t &hi)
{
    const u32x4_t u = {lo[0], lo[1], hi[0], hi[1]};
    return __builtin_bit_cast(bf16x8, u);
}

template <class IO, int D, bool DOH, bool WRITE, bool GATED>
__device__ __forceinline__ void state_pass_body_bf16_tile(const StatePassArgs &a, int group, uint16_t *s_k, uint16_t *s_b)
{
    typedef MmaBF16 MMA;
    typedef typename MMA::frag frag;
    constexpr int NB = D / 32;
    constexpr int HS = MMA::HS;
    constexpr int STEPS = kChunk / 16;            // MFMA steps over the chunk's tokens
    constexpr int NT = D * 2;                     // threads
    constexpr int NW = NT / 64;                   // waves = column blocks
    constexpr int RSB = D + MMA::kRowPad;         // row stride of the B tile (elements)
    constexpr int ROWB = D * 2;                   // bytes per k row
    constexpr int KBUF = kChunk * D;              // elements per k buffer
    constexpr int NA = kChunk * ROWB / (NT * 16); // 16-byte copies per thread per chunk
    constexpr int LPR = ROWB / 16;                // lanes (16-byte pieces) per row
    constexpr int RPI = 64 / LPR;                 // rows per wave-wide copy instruction
    constexpr int PPR = D / 4;                    // 4-element pieces per row of the B tile
    constexpr int VP = kChunk * PPR / NT;         // pieces of the B tile per thread
    constexpr int NSPL = MMA::kSplitReadout ? 2 : 1;
    constexpr int NS = WRITE ? NB * (DOH ? HS + 1 : HS * NSPL) : 0;   // state stores per chunk
    static_assert(NW == NB && STEPS == 4, "one wave per column block, four MFMA steps per chunk");
    static_assert(NA + NS < 64, "the counted wait below fits the counter");
    typedef SwizzledRows<ROWB, 2> KRows;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);   // column block owned by this wave (uniform)
    const int g = lane >> 5;
    const int pair = group % a.n_pairs;
    const int seg = group / a.n_pairs;
    const int b = (a.pair0 + pair) / a.H, h = (a.pair0 + pair) % a.H;
    const int64_t base_bh = (int64_t)b * a.stride_b + (int64_t)h * a.stride_h;
    const int64_t gate_base = (int64_t)b * a.T * a.H + h;
    const int chunk_begin = a.chunk0 + seg * a.seg_len;
    const int chunk_end = min(chunk_begin + a.seg_len, a.chunk0 + a.n_chunks);
    const int c_last = max(chunk_end - 1, chunk_begin);
    const void *bsrc = DOH ? a.k : a.v;

    f32x16 acc[NB];
#pragma unroll
    for (int rb = 0; rb < NB; ++rb) {
        acc[rb] = zero16();
        load_start_state<D, DOH>(a, acc[rb], pair, seg, rb, w, lane);
    }

    const int lrow = lane / LPR, lbyte = (lane % LPR) * 16;
    const int row_bytes = (int)a.stride_t * 2;
    auto issue_k = [&](int c, int buf) {
        const uint16_t *base = (const uint16_t *)a.k + base_bh + (int64_t)c * kChunk * a.stride_t;
        const buffer_rsrc rsrc = make_raw_buffer(base);
        const int last_row = a.T - 1 - c * kChunk;
#pragma unroll
        for (int q = 0; q < NA; ++q) {
            const int row = (q * NW + w) * RPI + lrow;
            const int sbyte = lbyte ^ ((row & KRows::kMask) << 5);
            async_copy16_to_lds(s_k + buf * KBUF + (q * NW + w) * 512, rsrc, min(row, last_row) * row_bytes + sbyte, 0);
        }
    };
    struct Fetch {
        typename IO::raw4 b[VP];
        float gate, beta;
    };
    const float *beta_src = a.beta ? a.beta : a.gate;
    auto fetch = [&](Fetch &f, int c) {
#pragma unroll
        for (int i = 0; i < VP; ++i) {
            const int piece = i * NT + tid;
            const int t = min(c * kChunk + piece / PPR, a.T - 1);
            f.b[i] = IO::load_raw4(bsrc, base_bh + (int64_t)t * a.stride_t + 4 * (piece % PPR));
        }
        const int t = min(c * kChunk + lane, a.T - 1);
        f.gate = a.gate[gate_base + (int64_t)t * a.H];
        if constexpr (GATED) f.beta = beta_src[gate_base + (int64_t)t * a.H];
    };
    float Gseg = 0.0f;
    int kb = 0;                                   // buffer that holds the chunk being processed
    // transpose-read addresses of this lane, as in the slab body; the B tile's row blocks are 64 bytes apart
    const int sub = 16 * ((lane >> 4) & 1);
    const int li = lane & 15;
    const uint32_t ka0 = lds_address(s_k + KRows{}(8 * g + (li >> 2), 32 * w + sub + 4 * (li & 3)));
    const uint32_t ka1 = lds_address(s_k + KRows{}(8 * g + 4 + (li >> 2), 32 * w + sub + 4 * (li & 3)));
    const uint32_t kb0 = lds_address(s_b + (8 * g + (li >> 2)) * RSB + sub + 4 * (li & 3));

    auto process = [&](const Fetch &f, int c) {
        __builtin_amdgcn_sched_barrier(0);
        const bool valid = c * kChunk + lane < a.T;
        const float lg = valid ? log2_gate(f.gate) : 0.0f;
        const float G = wave_inclusive_scan(lg, lane);
        const float Gtot = lane_value(G, 63);
        Gseg += Gtot;
        float wj = valid ? exp2f(Gtot - G) : 0.0f;     // lane j: weight of token j
        if constexpr (GATED) wj *= a.beta ? f.beta : 1.0f;
        const float zetaC = exp2f(Gtot);
        lds_barrier();                          // the previous chunk's operand reads are done
        issue_k(min(c + 1, c_last), kb ^ 1);
#pragma unroll
        for (int i = 0; i < VP; ++i) {
            const int piece = i * NT + tid;
            const int row = piece / PPR;
            MMA::store4(s_b + row * RSB + 4 * (piece % PPR), IO::cvt4(f.b[i]) * __shfl(wj, row, 64));
        }
        // ---- write the state before the chunk, fragment order
        if (WRITE) {
            const int64_t chunk_id = (int64_t)(c - a.chunk0) * a.n_pairs + pair;   // chunk-major: pairs adjacent
#pragma unroll
            for (int rb = 0; rb < NB; ++rb) {
                float vals[16];
#pragma unroll
                for (int r = 0; r < 16; ++r) vals[r] = acc[rb][r];
                if (DOH) {
                    frag *Hw = (frag *)a.ws_H + chunk_id * (NB * NB * HS * 64);
                    float ss = 0.0f;
#pragma unroll
                    for (int r = 0; r < 16; ++r) ss += vals[r] * vals[r];
#pragma unroll
                    for (int hh = 0; hh < HS; ++hh)
                        store_once(&Hw[((rb * NB + w) * HS + hh) * 64 + lane], MMA::pack(vals + hh * MMA::VEC));
                    ss = wave_inclusive_scan(ss, lane);           // lane 63: the wave's total
                    if (lane == 63) a.ws_hn[chunk_id * (NB * NB) + rb * NB + w] = ss;
                } else {
                    frag *Uw = (frag *)a.ws_U + chunk_id * (NSPL * NB * NB * HS * 64);
                    float lo[16];
#pragma unroll
                    for (int hh = 0; hh < HS; ++hh) {
                        frag fr = MMA::pack(vals + hh * MMA::VEC);
                        store_once(&Uw[((rb * NB + w) * HS + hh) * 64 + lane], fr);
                        float back[MMA::VEC];
                        MMA::unpack(fr, back);
#pragma unroll
                        for (int p = 0; p < MMA::VEC; ++p) lo[hh * MMA::VEC + p] = vals[hh * MMA::VEC + p] - back[p];
                    }
                    if (NSPL == 2) {
#pragma unroll
                        for (int hh = 0; hh < HS; ++hh)
                            store_once(&Uw[(NB * NB * HS + (rb * NB + w) * HS + hh) * 64 + lane],
                                       MMA::pack(lo + hh * MMA::VEC));
                    }
                }
            }
        }
        // This chunk's copy was issued one iteration ago, right after a barrier, followed by that iteration's stores
        // and prefetch loads; this iteration has added its copies and stores. (Letting the older stores stay in
        // flight as well, by issuing the prefetch loads ahead of the stores, was measured and is slower.)
        wait_vector_memory_upto<NA + NS>();
        lds_barrier();                          // k rows (all waves' copies) and the B tile are visible

        // ---- S <- zeta_C S + sum_j w_j a_j k_j^T. The LDS counter holds 15 operations, so the operand reads go in
        // groups: A and the first row block's B, then each further row block's B while the products of the block
        // before it run.
        u32x2_t fa0[4], fa1[4], fb0[NB][4], fb1[NB][4];
        issue_tr4<16 * ROWB>(ka0 + kb * (KBUF * 2), fa0);
        issue_tr4<16 * ROWB>(ka1 + kb * (KBUF * 2), fa1);
        issue_tr4<16 * RSB * 2>(kb0, fb0[0]);
        issue_tr4<16 * RSB * 2>(kb0 + 4 * RSB * 2, fb1[0]);
#pragma unroll
        for (int rb = 0; rb < NB; ++rb)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[rb][r] *= zetaC;
        await_tr8<0>(fa0, fa1);
#pragma unroll
        for (int rb = 0; rb < NB; ++rb) {
            await_tr8<0>(fb0[rb], fb1[rb]);
            if (rb + 1 < NB) {
                issue_tr4<16 * RSB * 2>(kb0 + 64 * (rb + 1), fb0[rb + 1]);
                issue_tr4<16 * RSB * 2>(kb0 + 64 * (rb + 1) + 4 * RSB * 2, fb1[rb + 1]);
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int s = 0; s < STEPS; ++s)
                acc[rb] = MMA::mma(join_runs(fa0[s], fa1[s]), join_runs(fb0[rb][s], fb1[rb][s]), acc[rb]);
            __builtin_amdgcn_sched_barrier(0);
        }
        kb ^= 1;
    };

    int c = chunk_begin;
    issue_k(c, 0);
    if ((chunk_end - chunk_begin) & 1) {
        Fetch fp;
        fetch(fp, c);
        drain_vector_memory();
        process(fp, c);
        ++c;
    }
    if (c < chunk_end) {
        Fetch f0, f1;
        fetch(f0, c);
        fetch(f1, c + 1);
        drain_vector_memory();
        for (; c < chunk_end; c += 2) {
            process(f0, c);
            fetch(f0, min(c + 2, c_last));
            process(f1, c + 1);
            fetch(f1, min(c + 3, c_last));
        }
    }
    // no copy into this workgroup's LDS may still be in flight when it ends
    drain_vector_memory();
#pragma unroll
    for (int rb = 0; rb < NB; ++rb) store_end_state<D, DOH>(a, acc[rb], Gseg, pair, seg, rb, w, lane);
}

// One workgroup per (pair, segment, H or U). The two workgroups of a (pair, segment) read the same k rows: they get
// block indices that are equal modulo 8, i.e. the same XCD and L2.
template <class IO, int D, bool GATED>
__global__ __launch_bounds__(D * 2) __attribute__((amdgpu_waves_per_eu(kStateWavesPerSimd))) void state_pass_tile_kernel(StatePassArgs a)
{
    constexpr int PER = 2;
    const int id = blockIdx.x;
    const int full = (gridDim.x / (8 * PER)) * (8 * PER);
    int sub, group;
    if (id < full) {
        const int within = id % (8 * PER);
        sub = within / 8;
        group = (id / (8 * PER)) * 8 + within % 8;
    } else {
        sub = (id - full) % PER;
        group = full / PER + (id - full) / PER;
    }
    if (a.only_u && !(sub & 1)) return;            // nobody reads the H states of this launch
    if (a.only_h && (sub & 1)) return;             // ... or its U states
    __shared__ __attribute__((aligned(1024))) uint16_t s_k[2 * kChunk * D];
    __shared__ __attribute__((aligned(16))) uint16_t s_b[kChunk * (D + MmaBF16::kRowPad)];
    if (a.write_frags) {
        if (sub & 1) state_pass_body_bf16_tile<IO, D, false, true, GATED>(a, group, s_k, s_b);
        else state_pass_body_bf16_tile<IO, D, true, true, GATED>(a, group, s_k, s_b);
    } else {
        if (sub & 1) state_pass_body_bf16_tile<IO, D, false, false, GATED>(a, group, s_k, s_b);
        else state_pass_body_bf16_tile<IO, D, true, false, GATED>(a, group, s_k, s_b);
    }
}

template <class MMA, class IO, int D, bool GATED>
__global__ __launch_bounds__(D * 2) __attribute__((amdgpu_waves_per_eu(kStateWavesPerSimd))) void state_pass_kernel(StatePassArgs a)
{
    constexpr int NB = D / 32;
    // Workgroups are dealt round-robin to the 8 XCDs, each with its own L2. The 2 NB workgroups of one
    // (pair, segment) read the same k rows, so they are given block indices that are equal modulo 8.
    // Each workgroup owns one of the two states of its slab (H or U): twice the workgroups, each with half the
    // accumulators and half the state writes per chunk.
    constexpr int PER = 2 * NB;                    // workgroups per (pair, segment)
    const int id = blockIdx.x;
    const int full = (gridDim.x / (8 * PER)) * (8 * PER);
    int sub, group;
    if (id < full) {
        const int within = id % (8 * PER);
        sub = within / 8;
        group = (id / (8 * PER)) * 8 + within % 8;
    } else {
        sub = (id - full) % PER;
        group = full / PER + (id - full) / PER;
    }
    if (a.only_u && !(sub & 1)) return;            // nobody reads the H states of this launch
    if (a.only_h && (sub & 1)) return;             // ... or its U states
    const int rb = sub >> 1;                       // slab index (row block of H0 / U0)
    typedef typename MMA::elem_t elem_t;
    __shared__ __attribute__((aligned(1024))) elem_t s_k[kChunk * (D + MMA::kRowPad)];
    __shared__ __attribute__((aligned(16))) elem_t s_v[kChunk * (32 + MMA::kRowPad)];
    if (a.write_frags) {
        if (sub & 1) state_pass_body<MMA, IO, D, false, true, GATED>(a, rb, group, s_k, s_v);
        else state_pass_body<MMA, IO, D, true, true, GATED>(a, rb, group, s_k, s_v);
    } else {
        if (sub & 1) state_pass_body<MMA, IO, D, false, false, GATED>(a, rb, group, s_k, s_v);
        else state_pass_body<MMA, IO, D, true, false, GATED>(a, rb, group, s_k, s_v);
    }
}

// Workgroups per (pair, segment): bf16 operands use the whole-tile kernel (one workgroup for H, one for U), fp32
// operands the slab kernel (one per 32-row slab and state).
template <class MMA, int D>
constexpr bool uses_tile_kernel() { return std::is_same<MMA, MmaBF16>::value; }

template <class MMA, class IO, int D, bool GATED>
static void launch_state_kernel(const StatePassArgs &a, int n_groups, hipStream_t stream)
{
    constexpr int NB = D / 32;
    dim3 block(D * 2);
    if constexpr (uses_tile_kernel<MMA, D>())
        hipLaunchKernelGGL((state_pass_tile_kernel<IO, D, GATED>), dim3(n_groups * 2), block, 0, stream, a);
    else
        hipLaunchKernelGGL((state_pass_kernel<MMA, IO, D, GATED>), dim3(n_groups * 2 * NB), block, 0, stream, a);
}

template <class MMA, class IO, int D, bool GATED>
static hipError_t launch_state_pass_g(const StatePassArgs &a0, int n_pairs, hipStream_t stream)
{
    StatePassArgs a = a0;
    a.n_pairs = n_pairs;
    if (a.n_segs <= 1) {
        a.n_segs = 1;
        a.seg_len = a.n_chunks;
    } else {
        // summaries (decay, Delta from a zero state) of every segment but the last
        a.init_mode = 0;
        a.final_mode = 2;
        a.write_frags = 0;
        launch_state_kernel<MMA, IO, D, GATED>(a, n_pairs * (a.n_segs - 1), stream);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    // every segment from its true start state (H_init / U_init scanned with the summaries before it)
    a.init_mode = 1;
    a.final_mode = 1;
    a.write_frags = 1;
    launch_state_kernel<MMA, IO, D, GATED>(a, n_pairs * a.n_segs, stream);
    return hipGetLastError();
}

template <class MMA, class IO, int D>
static hipError_t launch_state_pass_t(const StatePassArgs &a, int n_pairs, hipStream_t stream)
{
    // the write gate is the only variant of the layer that reaches this kernel
    if (a.beta) return launch_state_pass_g<MMA, IO, D, true>(a, n_pairs, stream);
    return launch_state_pass_g<MMA, IO, D, false>(a, n_pairs, stream);
}

int state_pass_workgroups_per_segment(int n_pairs, int d, bool compute_bf16)
{
    const bool tile = compute_bf16;
    return n_pairs * 2 * (tile ? 1 : d / 32);
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
