// Host-visible argument blocks and launchers of the libgka kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace gka {

constexpr int kChunk = 64;   // chunk size C of Section 4.2.1

struct StatePassArgs {
    const void *k, *v;            // [B,T,H,d] tensors (element strides below)
    const float *gate;            // [B,T,H]
    const float *beta;            // [B,T,H] write gate or nullptr (= 1)
    const float *H_init, *U_init; // [pairs,d,d] or nullptr
    float *H_final, *U_final;     // [pairs,d,d] or nullptr
    void *ws_H, *ws_U;            // chunk initial states, fragment order
    float *ws_hn;                 // partial sums of ||H_[n]||_F^2
    int64_t stride_b, stride_t, stride_h;
    int H, T;
    int pair0;                    // first (batch, head) pair of this launch; workspace is indexed from 0
    int chunk0, n_chunks;         // this launch covers chunks chunk0 .. chunk0 + n_chunks - 1 of every pair;
                                  // the workspace is indexed from 0 in both pairs and chunks
    int init_pair0, final_pair0;  // pair index of element 0 of H_init/U_init and of H_final/U_final
    bool h_init_lower_blocks;     // H_init: blocks above the block diagonal are taken from their mirror images
    int n_segs, seg_len;          // segments per pair and chunks per segment (n_segs <= 1: one pass)
    int n_pairs;                  // pairs of this launch (set by the launcher)
    float *seg_buf;               // [pairs, n_segs, 2, d*d] segment summaries / start states
    float *seg_logdecay;          // [pairs, n_segs] sum of log2 gates over each segment
    // set by the launcher:
    int init_mode;                // 0 zero state, 1 H_init/U_init (or zero) advanced over the earlier segments
    int final_mode;               // 1 last segment writes H_final/U_final, 2 segment summary to seg_buf
    int write_frags;              // store chunk states to ws_H / ws_U / ws_hn
    bool only_u;                  // the H states are not needed (plain readout y_t = U_t q_t): their workgroups exit
    bool only_h;                  // the U states are not needed (solve without readout): their workgroups exit
};

struct SolveArgs {
    const void *q, *k, *v;
    const void *q_lo;             // variants' kernel: optional remainder of q in the tensors' dtype (the right-hand side
                                  // of the solve is q + q_lo), or nullptr
    const float *gate, *lambda;   // lambda nullptr: lambda_t = lambda_scale ||H_t||_F
    const float *beta, *alpha;    // [B,T,H] write gate / alpha-connection, each nullptr (= 1)
    float lambda_scale;
    void *o;
    float *fro_out;               // [B,T,H] or nullptr
    float *xhat_out;              // [B,T,H,d] packed float32 or nullptr: the solve's result
    const void *ws_H, *ws_U;
    const float *ws_hn;
    int64_t stride_b, stride_t, stride_h;
    int H, T, n_iter;
    int chunk0, n_chunks;         // chunks of every pair covered by this launch (workspace indexed from 0)
    int n_pairs;                  // pairs of this launch (set by the launcher)
    int pair0;                    // first (batch, head) pair of this launch; workspace is indexed from 0
    bool readout_only;            // variants' kernel: no solve (its result is discarded by alpha = 0): H_[n] is not read
    bool solve_only;              // variants' kernel: xhat_out is all the caller wants: U_[n] is not read, o not written
};

struct DecodeArgs {
    const float *H_in, *U_in;     // [B,H,d,d] states before the first token (decode: the same buffers as H_state,
                                  //   U_state); nullptr: zero
    float *H_state, *U_state;     // [B,H,d,d] states after the last token; nullptr: not written (d = 256 needs U_state)
    bool h_out_full;              // H_state is written in full whatever h_lower_blocks says
    const void *q, *k, *v;        // [B,T,H,d] with the element strides below
    int64_t stride_b, stride_t, stride_h;
    float *fro_out, *xhat_out;    // ||H_t||_F [B,T,H] and the solve's result [B,T,H,d], each nullptr or written
    const float *gate, *lambda;   // [B,T,H]; lambda nullptr: lambda = lambda_scale ||H||_F
    const float *beta, *alpha;    // [B,T,H] or nullptr (= 1)
    float lambda_scale;
    void *o;                      // [B,T,H,d]
    int n_iter;
    int T, H;                     // tokens per call (1 for a single step), heads
    bool h_lower_blocks;          // H_state: only the 32 x 32 blocks on and below the block diagonal are read / written
};

// Elementwise / per-token kernels of the backward pass. Packed tensors: vectors [B,T,H,d] in the tensors' dtype unless
// named _f32, scalars [B,T,H] float32.
struct BackwardGlueArgs {
    int64_t n_elems, n_tokens;    // B*T*H*d, B*T*H
    int T, H, d;
    const void *q, *k, *v, *dy;   // inputs
    const float *gate, *alpha, *beta;                      // alpha, beta may be nullptr (= 1)
    const float *x_f32, *p_f32;   // results of the two solves
    void *x_io, *xt_io, *rhs_io;  // x, alpha x + (1 - alpha) q, alpha dxt
    void *rhs_lo_io;              // bf16 tensors: what rounding alpha dxt to rhs_io left over (nullptr: not kept)
    void *x_lo_io, *xt_lo_io;     // likewise for x_io and xt_io
    const void *dxt_io, *y_io, *hx_io;                     // U_t^T dy_t, forward output, H_t x_t
    void *k_rev, *v_rev, *dy_rev, *x_rev, *p_rev, *xt_rev; // time-reversed copies
    float *gate_rev, *zeros;      // gates of the reverse recurrences; an all-zero alpha
    const void *r1, *r2, *r3, *r4;                         // reversed passes: A k, A^T k, Ubar^T v, Ubar k
    float *dq, *dk, *dv, *dgate, *dlambda, *dbeta, *dalpha, *s;
    // the rule lambda_t = a ||H_t||_F (rule_a > 0): its extra gradient -c_t H_t at every state, c_t = a x_t.p_t / ||H_t||_F
    float rule_a;
    const float *fro;             // ||H_t||_F of the forward pass
    float *c, *C;                 // c_t and C_t = sum_{s>=t} M[t,s]^2 c_s
    void *vp_rev;                 // time-reversed beta_t C_t k_t
    bool natural_order;           // the reversed passes read and write the tensors in place (gla_readout `reverse`):
                                  // nothing is reversed here, p_rev and vp_rev are plain conversions, and dxt_io, y_io,
                                  // hx_io, r1, r2, r3, r4 are float32
    const void *hk_io, *r5;       // H_t k_t; reversed pass sum_{j>=t} M[t,j] beta_j C_j k_j (k_j . k_t)
    // gradients at the initial states (which = 7): the final states of three reverse readouts, each [pairs, d, d]
    const float *H_init;          // the caller's initial H (the rule's term needs it)
    const float *fin_px, *fin_xtdy, *fin_ck;   // sum p xhat^T, sum xt dy^T, sum (beta C k) k^T at token 0
    float *dH_init, *dU_init;     // [pairs, d, d], each written if not nullptr
    int n_pairs;
};
// which: 0 mix, 1 right-hand side, 2 reverse, 3 combine, 4 gate scan, 5 rule scalars (c_t), 6 rule scan (C_t),
// 7 gradients at the initial states
hipError_t launch_backward_glue(const BackwardGlueArgs &a, int which, bool io_bf16, hipStream_t stream);
// Copy of a strided [B,T,H,d] tensor (element strides; rows 16-byte aligned) into the packed layout.
hipError_t launch_pack_rows(const void *src, void *dst, int B, int T, int H, int d, int elem_bytes, int64_t stride_b,
                            int64_t stride_t, int64_t stride_h, hipStream_t stream);

// Gated-linear-attention readout y_t = U_t q_t, U_t = gate_t U_{t-1} + beta_t v_t k_t^T with the state in registers
// (bf16 tensors, packed or strided like the forward pass's; U is dv x dk). reverse: the recurrence runs from the last token to
// the first with gate'_tau = gate_{T-tau}; tensors are read and written at their own positions.
struct ReadoutArgs {
    const void *q, *k, *v;        // q, k: [B,T,H,dk]; v: [B,T,H,dv]
    const void *q_lo;             // optional bf16 remainder of q (y_t = U_t (q_t + q_lo_t)), or nullptr
    const void *k_lo, *v_lo;      // optional bf16 remainder of k or of v (at most one of the two; dk = dv only), laid out
                                  // like k / v: the recurrence is that of k + k_lo (v + v_lo). For operands that were
                                  // computed in float32 (the solves' results in the backward pass)
    bool q_is_f32;                // q is float32 (split into value + remainder inside); dk = 64, dv = 128 only
    void *o;                      // [B,T,H,dv]
    float *o_f32;                 // if not nullptr the output goes here in float32 instead (same strides)
    const float *gate, *beta;     // [B,T,H]; beta nullptr (= 1)
    int64_t stride_b, stride_t, stride_h;            // element strides of v and o
    int64_t qk_stride_b, qk_stride_t, qk_stride_h;   // ... of q (q_lo) and k
    int H, T;
    int n_pairs;                  // B * H
    int n_segs, seg_len;          // segments of the chunk scan per pair, chunks per segment
    float *seg_buf;               // [pairs, n_segs, dv*dk] segment summaries
    float *seg_logdecay;          // [pairs, n_segs]
    int seg_mode;                 // 0: the summaries are computed by this call; 1: they are in seg_buf already (the call
                                  // before had the same k, v, gate, beta, direction); 2: likewise, with k and v exchanged
                                  // (the transposed state; dk = dv only)
    bool reverse;
    const float *init_state;      // [pairs, dv, dk] float32 or nullptr (zero): the state before the first token of the walk
    bool init_transposed;         // init_state holds the transposed state, [pairs, dk, dv] (dk = dv only)
    float *final_state;           // [pairs, dv, dk] float32 or nullptr: the state after the last token of the walk
};
hipError_t launch_gla_readout(const ReadoutArgs &a, int dk, int dv, hipStream_t stream);
size_t gla_readout_workspace_bytes(int n_pairs, int n_segs, int dk, int dv);

// Projections of latent sketching: down (qs = S q, ks = S k, 64 sketched features stored, zeros above d_s) and up
// (xhat = S^T z as bf16 value and optional remainder). Packed bf16 tensors [B,T,H,d]; z float32 [B,T,H,64].
struct SketchArgs {
    const void *q, *k;
    const float *S;               // [d_s, d] float32, or [H, d_s, d] with per_head
    int d_s;
    bool per_head;
    void *qs, *ks;                // [B,T,H,out_width] bf16
    int out_width;                // stored sketched features per token: 64, or 32 (down-projection with d_s <= 32 only)
    const float *z;               // [B,T,H,64]
    void *xhat_hi, *xhat_lo;      // [B,T,H,d] bf16; xhat_lo may be nullptr
    int T, H;
};
hipError_t launch_sketch(const SketchArgs &a, int n_pairs, int d, bool up, hipStream_t stream);

// Chunk-wise forward pass for head dimensions up to 32 (gka_small_dim.hip): the layer at d = 16 and 32, and, without
// values and output, the solve of latent sketching in at most 32 sketched dimensions. bf16 tensors.
struct SmallArgs {
    const void *q, *k;            // rows of d features
    const void *v;                // rows of d features, or nullptr: no readout (then o is nullptr too)
    void *o;
    int64_t stride_b, stride_t, stride_h;   // of q, k, v, o, in elements (multiples of 8)
    int d;                        // 16 or 32 features per row exist; the kernels work in 32
    const float *gate;            // [B,T,H]
    const float *lambda;          // [B,T,H], or nullptr: lambda_t = lambda_scale ||H_t||_F
    const float *beta, *alpha;    // [B,T,H] write gate / alpha-connection, or nullptr
    float lambda_scale;
    float *xhat_out;              // optional float32 out, xhat_row elements per token, features 0 .. d - 1 written
    int64_t xhat_row;
    bool xhat_zero_upper;         // also write zeros to features 32..63 of a row (for a reader of 64 stored features)
    float *fro_out;               // optional [B,T,H]
    const float *H_init, *U_init; // optional [pairs, d, d] float32
    float *H_final, *U_final;     // optional
    int T, H, n_pairs, n_chunks, n_iter;
    float *dH, *sH, *dU, *sU, *chunk_log2_decay;   // carved from the workspace by the launcher
};
size_t small_dim_workspace_bytes(int n_pairs, int n_chunks, int d, bool with_readout);
hipError_t launch_small_dim_forward(SmallArgs a, void *workspace, hipStream_t stream);

hipError_t launch_state_pass(const StatePassArgs &a, int n_pairs, int d, bool io_bf16, bool compute_bf16,
                             hipStream_t stream);
// Workgroups the state pass launches per segment of the chunk scan (the plan sizes the segments with it).
int state_pass_workgroups_per_segment(int n_pairs, int d, bool compute_bf16);
hipError_t launch_chunk_solve(const SolveArgs &a, int n_pairs, int d, bool io_bf16, bool compute_bf16,
                              hipStream_t stream);
hipError_t launch_decode_step(const DecodeArgs &a, int n_pairs, int d, bool io_bf16, hipStream_t stream);

// Forward pass in one kernel with the states in registers (bf16 tensors and operands, d = 128, Eq. (CH) as printed).
struct FusedArgs {
    const void *q, *k, *v;
    const float *gate, *lambda;   // [B,T,H]; lambda nullptr: lambda_t = lambda_scale ||H_t||_F
    const float *beta, *alpha;    // [B,T,H] write gate / alpha-connection, each nullptr (= 1)
    float lambda_scale;
    void *o;
    float *fro_out;               // [B,T,H] or nullptr
    const float *H_init, *U_init; // [pairs,d,d] or nullptr
    float *H_final, *U_final;     // [pairs,d,d] or nullptr
    bool h_init_lower_blocks;
    int64_t stride_b, stride_t, stride_h;
    int H, T, n_iter;
    int n_pairs, n_chunks;
    int n_segs, seg_len;          // segments of the chunk walk per pair (one workgroup each), chunks per segment
    float *seg_buf, *seg_logdecay, *park; // set by the launcher (carved from the workspace)
};
size_t fused_workspace_bytes(int n_pairs, int n_segs);
// which: bit 0 the summary launch (segment summaries for the start states), bit 1 the chunk walk; split: H_[n], delta
// and the masked products as bf16 value + remainder. (beta, alpha or a missing lambda select the kernels' variant with
// the write gate, the alpha-connection and the rule for lambda.)
hipError_t launch_fused_forward(const FusedArgs &a, void *workspace, hipStream_t stream, int which, bool split);

// Workspace sizes in bytes per (pair, chunk).
size_t ws_H_bytes_per_chunk(int d, bool compute_bf16);
size_t ws_U_bytes_per_chunk(int d, bool compute_bf16);
size_t ws_hn_bytes_per_chunk(int d);

}  // namespace gka
