// Host side of the C ABI declared in include/gka.h: argument validation, workspace carving and kernel
// launches on the caller's stream. No device allocation and no synchronisation (gka_forward_profile aside); the only
// state kept between calls is the address of gka_forward_static's scratch array on each device.
#include "../../include/gka.h"
#include "gka_kernels.hpp"

#include <mutex>
#include <vector>

namespace {

struct Plan {
    int n_pairs, n_chunks, d;
    bool io_bf16, compute_bf16;
    int64_t stride_b, stride_t, stride_h;
    size_t off_H, off_U, off_hn, off_seg, off_segdecay, off_carry, total;
    int n_segs, seg_len;
    int pairs_per_batch;          // (batch, head) pairs per launch
    int slab_chunks;              // chunks of every pair per launch
    bool recurrent;               // token-by-token kernel: no chunks, no launch plan
    bool small;                   // chunk-wise kernels of the head dimensions 16 and 32 (bf16 tensors and operands)
    bool split;                   // GKA_COMPUTE_BF16_SPLIT (fused kernel only)
    bool fused_shape;             // dtype, operands and head dimension of the fused kernel
    int fused_n_segs, fused_seg_len;
    size_t fused_bytes;           // workspace of the fused kernels alone
};

size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

constexpr int kStateMinWorkgroups = 512;   // two state-pass workgroups per CU
constexpr int kStateMaxWalk = 64;          // chunks a state-pass workgroup walks before segments are added
// Chunk states one launch pair keeps in the workspace unless gka_params::slab_state_bytes says otherwise (tests use
// that to force several slabs on small problems).
constexpr size_t kDefaultSlabStateBytes = (size_t)1 << 30;
// Workgroups the fused kernel should at least have: one per compute unit.
constexpr int kFusedMinWorkgroups = 256;
constexpr size_t kMaxPairsPerBatch = 1024;
constexpr size_t kMinSlabChunks = 4;

gka_status check_common(const gka_params *p, bool decode)
{
    if (!p) return GKA_ERR_NULL;
    if (p->B <= 0 || p->H <= 0 || p->n_iter < 0) return GKA_ERR_SHAPE;
    if (!decode && p->T <= 0) return GKA_ERR_SHAPE;
    if (p->d_k <= 0 || p->d_v <= 0) return GKA_ERR_SHAPE;
    if (p->phase < GKA_PHASE_ALL || p->phase > GKA_PHASE_SOLVE) return GKA_ERR_UNSUPPORTED;
    if (p->d_k != p->d_v) return GKA_ERR_UNSUPPORTED;
    if (p->d_k != 16 && p->d_k != 32 && p->d_k != 64 && p->d_k != 128 && p->d_k != 256) return GKA_ERR_UNSUPPORTED;
    if (p->io_dtype != GKA_F32 && p->io_dtype != GKA_BF16) return GKA_ERR_UNSUPPORTED;
    if (p->compute < GKA_COMPUTE_F32 || p->compute > GKA_COMPUTE_BF16_SPLIT) return GKA_ERR_UNSUPPORTED;
    if (p->io_dtype == GKA_F32 && p->compute != GKA_COMPUTE_F32) return GKA_ERR_UNSUPPORTED;
    if (!decode && p->chunk != gka::kChunk) return GKA_ERR_UNSUPPORTED;
    if ((int64_t)p->B * p->H > (int64_t)1 << 24) return GKA_ERR_SHAPE;
    if (!(p->lambda_scale >= 0.0f)) return GKA_ERR_SHAPE;
    if (p->state_layout != GKA_STATE_FULL && p->state_layout != GKA_STATE_H_LOWER_BLOCKS) return GKA_ERR_UNSUPPORTED;
    if (p->slab_state_bytes < 0 || p->walk_chunks < 0) return GKA_ERR_SHAPE;
    if (p->state_layout == GKA_STATE_H_LOWER_BLOCKS && p->d_k == 256) return GKA_ERR_UNSUPPORTED;
    if (p->path < GKA_PATH_AUTO || p->path > GKA_PATH_RECURRENT) return GKA_ERR_UNSUPPORTED;
    return GKA_OK;
}

// head dimensions of the chunk-wise kernels (the others run token by token)
bool chunked_dim(int d) { return d == 64 || d == 128; }

gka_status make_plan(const gka_params *p, Plan *pl, bool readout_only = false)
{
    gka_status s = check_common(p, false);
    if (s != GKA_OK) return s;
    pl->d = p->d_k;
    pl->n_pairs = p->B * p->H;
    pl->n_chunks = (p->T + gka::kChunk - 1) / gka::kChunk;
    pl->io_bf16 = p->io_dtype == GKA_BF16;
    pl->compute_bf16 = p->compute != GKA_COMPUTE_F32;
    pl->split = p->compute == GKA_COMPUTE_BF16_SPLIT;
    // d = 16, 32: chunk-wise kernels of their own for bf16 tensors with bf16 operands (what GKA_PATH_AUTO and
    // GKA_PATH_TWO_PHASE select there), else token by token
    pl->small = pl->d <= 32 && pl->io_bf16 && p->compute == GKA_COMPUTE_BF16 && !readout_only &&
                (p->path == GKA_PATH_AUTO || p->path == GKA_PATH_TWO_PHASE);
    pl->recurrent = !pl->small && (p->path == GKA_PATH_RECURRENT || !chunked_dim(pl->d));
    if (pl->recurrent && (p->path == GKA_PATH_TWO_PHASE || p->path == GKA_PATH_FUSED || readout_only))
        return GKA_ERR_UNSUPPORTED;
    if ((int64_t)pl->n_pairs * pl->n_chunks > (int64_t)0x7fffffff) return GKA_ERR_SHAPE;
    if (p->stride_b == 0 && p->stride_t == 0 && p->stride_h == 0) {
        pl->stride_h = p->d_k;
        pl->stride_t = (int64_t)p->H * p->d_k;
        pl->stride_b = (int64_t)p->T * p->H * p->d_k;
    } else {
        if (p->stride_b <= 0 || p->stride_t <= 0 || p->stride_h <= 0) return GKA_ERR_SHAPE;
        if (p->stride_h < p->d_k && p->H > 1) return GKA_ERR_SHAPE;
        if (p->stride_t % 4 || p->stride_h % 4 || p->stride_b % 4) return GKA_ERR_SHAPE;  // vector stores
        // bf16 operands: k rows are copied 16 bytes at a time, addressed with 32-bit byte offsets within a chunk
        if (pl->compute_bf16 && (p->stride_t % 8 || p->stride_h % 8 || p->stride_b % 8)) return GKA_ERR_SHAPE;
        if (pl->compute_bf16 && p->stride_t >= (1 << 23)) return GKA_ERR_UNSUPPORTED;
        pl->stride_b = p->stride_b;
        pl->stride_t = p->stride_t;
        pl->stride_h = p->stride_h;
    }
    if (pl->small) {
        if ((int64_t)pl->n_pairs * pl->n_chunks > (int64_t)0x7fffffff / 4) return GKA_ERR_SHAPE;
        pl->fused_shape = false;
        pl->fused_bytes = 0;
        pl->total = align_up(gka::small_dim_workspace_bytes(pl->n_pairs, pl->n_chunks, pl->d, true), 256);
        return GKA_OK;
    }
    if (pl->recurrent) {
        // states stay in registers; only d = 256 streams U through memory and needs room for it when the caller does
        // not ask for U_final
        pl->fused_shape = false;
        pl->fused_bytes = 0;
        pl->total = 256 + (pl->d == 256 ? align_up((size_t)pl->n_pairs * pl->d * pl->d * sizeof(float), 256) : 0);
        return GKA_OK;
    }
    // The work is cut into launches of (a batch of pairs) x (a slab of consecutive chunks), slabs in sequence order,
    // so that the chunk states one launch pair writes and reads (state pass, then solve) fit a bounded workspace,
    // which every launch pair reuses; the running states are carried between slabs in fp32. (Slabs small enough to
    // stay in the last-level cache were measured slower than one launch pair: more launches, shorter walks.)
    const size_t per_chunk = gka::ws_H_bytes_per_chunk(pl->d, pl->compute_bf16) +
                             gka::ws_U_bytes_per_chunk(pl->d, pl->compute_bf16);
    size_t ppb = pl->n_pairs < kMaxPairsPerBatch ? pl->n_pairs : kMaxPairsPerBatch;
    const size_t budget = p->slab_state_bytes > 0 ? (size_t)p->slab_state_bytes : kDefaultSlabStateBytes;
    size_t slab = budget / (ppb * per_chunk);
    if (slab < kMinSlabChunks) slab = kMinSlabChunks;
    if (slab > (size_t)pl->n_chunks) slab = pl->n_chunks;
    pl->pairs_per_batch = (int)ppb;
    pl->slab_chunks = (int)slab;
    const size_t nc = ppb * slab;
    pl->off_H = 0;
    pl->off_U = align_up(pl->off_H + nc * gka::ws_H_bytes_per_chunk(pl->d, pl->compute_bf16), 256);
    pl->off_hn = align_up(pl->off_U + nc * gka::ws_U_bytes_per_chunk(pl->d, pl->compute_bf16), 256);
    pl->off_seg = align_up(pl->off_hn + nc * gka::ws_hn_bytes_per_chunk(pl->d), 256);
    // Segments of the chunk scan. A workgroup walks its chunks one after the other (a few microseconds each), and a
    // segmented pass reads k and v twice, so: one segment unless that leaves CUs idle or makes the walk longer than
    // about 64 chunks; never fewer than two chunks per segment.
    // (a plain readout walks U only: half the workgroups of a segment have nothing to do)
    int wg_per_seg = gka::state_pass_workgroups_per_segment(pl->pairs_per_batch, pl->d, pl->compute_bf16);
    if (readout_only && wg_per_seg > 1) wg_per_seg /= 2;
    int n_segs = (kStateMinWorkgroups + wg_per_seg - 1) / wg_per_seg;
    if (n_segs < pl->slab_chunks / kStateMaxWalk) n_segs = pl->slab_chunks / kStateMaxWalk;
    if (n_segs > pl->slab_chunks / 2) n_segs = pl->slab_chunks / 2;
    if (n_segs < 1) n_segs = 1;
    pl->seg_len = (pl->slab_chunks + n_segs - 1) / n_segs;
    pl->n_segs = (pl->slab_chunks + pl->seg_len - 1) / pl->seg_len;
    pl->off_segdecay = align_up(pl->off_seg + (size_t)pl->pairs_per_batch * pl->n_segs * 2 * pl->d * pl->d * sizeof(float), 256);
    pl->off_carry = align_up(pl->off_segdecay + (size_t)pl->pairs_per_batch * pl->n_segs * sizeof(float), 256);
    // two ping-pong pairs of fp32 (H, U) carried from slab to slab
    pl->total = align_up(pl->off_carry + (size_t)4 * pl->pairs_per_batch * pl->d * pl->d * sizeof(float), 256);
    // Fused kernel: one workgroup per (pair, segment of the chunk walk). As few segments as give every compute unit a
    // workgroup (every segment but the last costs a second read of its k and v rows for the summary launch); an even
    // number of chunks per segment, because a workgroup takes its chunks two at a time.
    pl->fused_shape = pl->io_bf16 && pl->compute_bf16 && pl->d == 128 && !readout_only;
    pl->fused_bytes = 0;
    if (pl->fused_shape) {
        int seg_len;
        if (p->walk_chunks > 0) {
            seg_len = p->walk_chunks;
        } else {
            int n_segs = (kFusedMinWorkgroups + pl->n_pairs - 1) / pl->n_pairs;
            const int min_walk = pl->split ? 1 : 2;
            if (n_segs > pl->n_chunks / min_walk) n_segs = pl->n_chunks / min_walk;
            if (n_segs < 1) n_segs = 1;
            seg_len = (pl->n_chunks + n_segs - 1) / n_segs;
        }
        if (!pl->split) seg_len += seg_len & 1;
        pl->fused_seg_len = seg_len;
        pl->fused_n_segs = (pl->n_chunks + seg_len - 1) / seg_len;
        if ((int64_t)pl->n_pairs * pl->fused_n_segs > (int64_t)0x7fffffff) return GKA_ERR_SHAPE;
        pl->fused_bytes = align_up(gka::fused_workspace_bytes(pl->n_pairs, pl->fused_n_segs), 256);
        // (a caller that insists on the fused kernels needs no room for the two-phase kernels' chunk states)
        if (p->path == GKA_PATH_FUSED || pl->split || pl->fused_bytes > pl->total) pl->total = pl->fused_bytes;
    }
    return GKA_OK;
}

}  // namespace

extern "C" {

size_t gka_forward_workspace_bytes(const gka_params *p)
{
    Plan pl;
    if (make_plan(p, &pl) != GKA_OK) return 0;
    return pl.total;
}

}  // extern "C"

namespace {

// Events around the two phases of every batch (profiling entry point only).
struct PhaseEvents {
    std::vector<hipEvent_t> ev;
    bool ok = true;
    void mark(hipStream_t stream)
    {
        hipEvent_t e;
        if (hipEventCreate(&e) != hipSuccess) { ok = false; return; }
        if (hipEventRecord(e, stream) != hipSuccess) ok = false;
        ev.push_back(e);
    }
    ~PhaseEvents()
    {
        for (hipEvent_t e : ev) (void)hipEventDestroy(e);
    }
};

gka_status forward_impl(const gka_params *p, const void *q, const void *k, const void *v, const float *gate,
                        const float *lambda, void *o, const float *H_init, const float *U_init, float *H_final,
                        float *U_final, float *fro_out, void *workspace, size_t workspace_bytes,
                        void *hip_stream, PhaseEvents *prof, bool readout_only = false, bool solve_only = false,
                        const void *q_lo = nullptr)
{
    Plan pl;
    gka_status s = make_plan(p, &pl, readout_only);
    if (s != GKA_OK) return s;
    if (!q || !k || !v || !gate || !o) return GKA_ERR_NULL;
    if (!lambda && !(p->lambda_scale > 0.0f)) return GKA_ERR_NULL;      // neither lambda_t nor the rule for it
    if ((H_init == nullptr) != (U_init == nullptr)) return GKA_ERR_NULL;
    if ((H_final == nullptr) != (U_final == nullptr)) return GKA_ERR_NULL;
    if (!workspace || workspace_bytes < pl.total || ((uintptr_t)workspace & 255)) return GKA_ERR_WORKSPACE;
    hipStream_t stream = (hipStream_t)hip_stream;
    char *ws = (char *)workspace;

    if (pl.small) {
        if (p->phase != GKA_PHASE_ALL || solve_only || q_lo) return GKA_ERR_UNSUPPORTED;
        gka::SmallArgs sm = {};
        sm.q = q; sm.k = k; sm.v = v; sm.o = o;
        sm.stride_b = pl.stride_b; sm.stride_t = pl.stride_t; sm.stride_h = pl.stride_h;
        sm.d = pl.d;
        sm.gate = gate; sm.lambda = lambda; sm.beta = p->beta; sm.alpha = p->alpha; sm.lambda_scale = p->lambda_scale;
        sm.xhat_out = p->xhat_out; sm.xhat_row = pl.d; sm.xhat_zero_upper = false;
        sm.fro_out = fro_out;
        sm.H_init = H_init; sm.U_init = U_init; sm.H_final = H_final; sm.U_final = U_final;
        sm.T = p->T; sm.H = p->H; sm.n_pairs = pl.n_pairs; sm.n_chunks = pl.n_chunks; sm.n_iter = p->n_iter;
        // (profiling: all of it is reported as the solve phase)
        if (prof) { prof->mark(stream); prof->mark(stream); }
        if (gka::launch_small_dim_forward(sm, ws, stream) != hipSuccess) return GKA_ERR_LAUNCH;
        if (prof) prof->mark(stream);
        return GKA_OK;
    }
    if (pl.recurrent) {
        if (p->phase != GKA_PHASE_ALL || pl.split || solve_only || q_lo) return GKA_ERR_UNSUPPORTED;
        gka::DecodeArgs da = {};
        da.H_in = H_init; da.U_in = U_init;
        da.H_state = H_final;
        da.U_state = U_final ? U_final : (pl.d == 256 ? (float *)(ws + 256) : nullptr);
        da.h_out_full = true;
        da.h_lower_blocks = p->state_layout == GKA_STATE_H_LOWER_BLOCKS && chunked_dim(pl.d);
        da.q = q; da.k = k; da.v = v; da.gate = gate; da.lambda = lambda; da.o = o;
        da.stride_b = pl.stride_b; da.stride_t = pl.stride_t; da.stride_h = pl.stride_h;
        da.beta = p->beta; da.alpha = p->alpha; da.lambda_scale = p->lambda_scale;
        da.fro_out = fro_out; da.xhat_out = p->xhat_out;
        da.n_iter = p->n_iter; da.T = p->T; da.H = p->H;
        // (profiling: all of it is reported as the solve phase)
        if (prof) { prof->mark(stream); prof->mark(stream); }
        if (gka::launch_decode_step(da, pl.n_pairs, pl.d, pl.io_bf16, stream) != hipSuccess) return GKA_ERR_LAUNCH;
        if (prof) prof->mark(stream);
        return GKA_OK;
    }
    const bool fused_ok = pl.fused_shape && !p->xhat_out && !solve_only && !q_lo && p->phase == GKA_PHASE_ALL;
    if ((p->path == GKA_PATH_FUSED || pl.split) && !fused_ok) return GKA_ERR_UNSUPPORTED;
    if (pl.split && p->path == GKA_PATH_TWO_PHASE) return GKA_ERR_UNSUPPORTED;     // only the fused kernel splits
    if (fused_ok && p->path != GKA_PATH_TWO_PHASE) {
        gka::FusedArgs fa = {};
        fa.q = q; fa.k = k; fa.v = v; fa.gate = gate; fa.lambda = lambda; fa.o = o; fa.fro_out = fro_out;
        fa.beta = p->beta; fa.alpha = p->alpha; fa.lambda_scale = p->lambda_scale;
        fa.H_init = H_init; fa.U_init = U_init; fa.H_final = H_final; fa.U_final = U_final;
        fa.h_init_lower_blocks = p->state_layout == GKA_STATE_H_LOWER_BLOCKS;
        fa.stride_b = pl.stride_b; fa.stride_t = pl.stride_t; fa.stride_h = pl.stride_h;
        fa.H = p->H; fa.T = p->T; fa.n_iter = p->n_iter;
        fa.n_pairs = pl.n_pairs; fa.n_chunks = pl.n_chunks;
        fa.n_segs = pl.fused_n_segs; fa.seg_len = pl.fused_seg_len;
        fa.seg_buf = nullptr; fa.seg_logdecay = nullptr;
        // (profiling: the summary launch is reported as the state phase, the chunk walk as the solve phase)
        if (prof) prof->mark(stream);
        if (gka::launch_fused_forward(fa, ws, stream, 1, pl.split) != hipSuccess) return GKA_ERR_LAUNCH;
        if (prof) prof->mark(stream);
        if (gka::launch_fused_forward(fa, ws, stream, 2, pl.split) != hipSuccess) return GKA_ERR_LAUNCH;
        if (prof) prof->mark(stream);
        return GKA_OK;
    }

    gka::StatePassArgs sa = {};
    sa.k = k; sa.v = v; sa.gate = gate; sa.beta = p->beta;
    sa.H_init = H_init; sa.U_init = U_init;
    sa.H_final = H_final; sa.U_final = U_final;
    sa.ws_H = ws + pl.off_H; sa.ws_U = ws + pl.off_U; sa.ws_hn = (float *)(ws + pl.off_hn);
    sa.stride_b = pl.stride_b; sa.stride_t = pl.stride_t; sa.stride_h = pl.stride_h;
    sa.H = p->H; sa.T = p->T;
    sa.n_segs = pl.n_segs; sa.seg_len = pl.seg_len;
    sa.seg_buf = (float *)(ws + pl.off_seg); sa.seg_logdecay = (float *)(ws + pl.off_segdecay);
    sa.init_mode = 0; sa.final_mode = 0; sa.write_frags = 1;
    gka::SolveArgs so = {};
    so.q = q; so.q_lo = q_lo; so.k = k; so.v = v; so.gate = gate; so.lambda = lambda; so.o = o; so.fro_out = fro_out;
    so.beta = p->beta; so.alpha = p->alpha; so.lambda_scale = p->lambda_scale;
    so.xhat_out = p->xhat_out;
    // plain readout y_t = U_t q_t (used by the backward pass): needs alpha = 0 from the caller; no H states, no solve
    sa.only_u = readout_only; so.readout_only = readout_only;
    // the solve alone (latent sketching): needs xhat_out; no U states, no readout, o is left untouched
    sa.only_h = solve_only; so.solve_only = solve_only;
    so.ws_H = sa.ws_H; so.ws_U = sa.ws_U; so.ws_hn = sa.ws_hn;
    so.stride_b = pl.stride_b; so.stride_t = pl.stride_t; so.stride_h = pl.stride_h;
    so.H = p->H; so.T = p->T; so.n_iter = p->n_iter;
    const bool one_launch = pl.pairs_per_batch >= pl.n_pairs && pl.slab_chunks >= pl.n_chunks;
    // With a single phase requested the workspace must cover the whole problem.
    if (p->phase != GKA_PHASE_ALL && !one_launch) return GKA_ERR_UNSUPPORTED;
    const size_t state_elems = (size_t)pl.pairs_per_batch * pl.d * pl.d;
    float *carry = (float *)(ws + pl.off_carry);               // [2][2][pairs_per_batch, d, d]
    for (int pair0 = 0; pair0 < pl.n_pairs; pair0 += pl.pairs_per_batch) {
        const int np = pl.n_pairs - pair0 < pl.pairs_per_batch ? pl.n_pairs - pair0 : pl.pairs_per_batch;
        int slab_index = 0;
        for (int chunk0 = 0; chunk0 < pl.n_chunks; chunk0 += pl.slab_chunks, ++slab_index) {
            const int nch = pl.n_chunks - chunk0 < pl.slab_chunks ? pl.n_chunks - chunk0 : pl.slab_chunks;
            const bool first = chunk0 == 0, last = chunk0 + nch >= pl.n_chunks;
            sa.pair0 = so.pair0 = pair0;
            sa.chunk0 = so.chunk0 = chunk0;
            sa.n_chunks = so.n_chunks = nch;
            // states enter from the caller (first slab) or from the previous slab, and leave to the next slab or to
            // the caller (last slab)
            float *in = carry + (size_t)((slab_index + 1) & 1) * 2 * state_elems;
            float *out = carry + (size_t)(slab_index & 1) * 2 * state_elems;
            sa.H_init = first ? H_init : in;
            sa.U_init = first ? U_init : in + state_elems;
            sa.init_pair0 = first ? pair0 : 0;
            // states carried between slabs are always complete
            sa.h_init_lower_blocks = first && p->state_layout == GKA_STATE_H_LOWER_BLOCKS;
            sa.H_final = last ? H_final : out;
            sa.U_final = last ? U_final : out + state_elems;
            sa.final_pair0 = last ? pair0 : 0;
            if (prof) prof->mark(stream);
            if (p->phase != GKA_PHASE_SOLVE &&
                gka::launch_state_pass(sa, np, pl.d, pl.io_bf16, pl.compute_bf16, stream) != hipSuccess)
                return GKA_ERR_LAUNCH;
            if (prof) prof->mark(stream);
            if (p->phase != GKA_PHASE_STATES &&
                gka::launch_chunk_solve(so, np, pl.d, pl.io_bf16, pl.compute_bf16, stream) != hipSuccess)
                return GKA_ERR_LAUNCH;
            if (prof) prof->mark(stream);
        }
    }
    return GKA_OK;
}

}  // namespace

extern "C" {

gka_status gka_forward(const gka_params *p, const void *q, const void *k, const void *v, const float *gate,
                       const float *lambda, void *o, const float *H_init, const float *U_init, float *H_final,
                       float *U_final, float *fro_out, void *workspace, size_t workspace_bytes,
                       void *hip_stream)
{
    return forward_impl(p, q, k, v, gate, lambda, o, H_init, U_init, H_final, U_final, fro_out, workspace,
                        workspace_bytes, hip_stream, nullptr);
}

gka_status gka_forward_profile(const gka_params *p, const void *q, const void *k, const void *v, const float *gate,
                               const float *lambda, void *o, const float *H_init, const float *U_init,
                               float *H_final, float *U_final, float *fro_out, void *workspace,
                               size_t workspace_bytes, void *hip_stream, float *ms_states, float *ms_solve,
                               int32_t *n_solve_launches)
{
    if (!ms_states || !ms_solve || !n_solve_launches) return GKA_ERR_NULL;
    PhaseEvents prof;
    gka_status s = forward_impl(p, q, k, v, gate, lambda, o, H_init, U_init, H_final, U_final, fro_out, workspace,
                                workspace_bytes, hip_stream, &prof);
    if (s != GKA_OK) return s;
    if (!prof.ok || prof.ev.empty() || hipEventSynchronize(prof.ev.back()) != hipSuccess) return GKA_ERR_LAUNCH;
    float t_states = 0.0f, t_solve = 0.0f;
    for (size_t i = 0; i + 2 < prof.ev.size(); i += 3) {
        float a = 0.0f, b = 0.0f;
        if (hipEventElapsedTime(&a, prof.ev[i], prof.ev[i + 1]) != hipSuccess) return GKA_ERR_LAUNCH;
        if (hipEventElapsedTime(&b, prof.ev[i + 1], prof.ev[i + 2]) != hipSuccess) return GKA_ERR_LAUNCH;
        t_states += a;
        t_solve += b;
    }
    *ms_states = t_states;
    *ms_solve = t_solve;
    *n_solve_launches = (int32_t)(prof.ev.size() / 3);
    return GKA_OK;
}

// ---- gka_forward_static: the fused kernels with their scratch in a fixed device array --------------------------
namespace {
// Segment summaries and parked states of the fused kernels. Every GPU the library runs on holds its own copy until
// the process ends. In host code the array's name is only a handle: its device address comes from
// hipGetSymbolAddress, once per device, and is what kernels and copies are given.
static __device__ __align__(256) unsigned char scratch[GKA_STATIC_SCRATCH_BYTES];
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void *g_scratch_ptr[kMaxDevices] = {};

gka_status static_scratch(void **ptr)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return GKA_ERR_LAUNCH;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return GKA_ERR_LAUNCH;
        g_scratch_ptr[dev] = p;
    }
    *ptr = g_scratch_ptr[dev];
    return GKA_OK;
}
}  // namespace

gka_status gka_forward_static(const gka_params *p, const void *q, const void *k, const void *v, const float *gate,
                              const float *lambda, void *o, const float *H_init, const float *U_init, float *H_final,
                              float *U_final, float *fro_out, void *hip_stream)
{
    Plan pl;
    gka_status s = make_plan(p, &pl);
    if (s != GKA_OK) return s;
    if (!pl.fused_shape || p->path == GKA_PATH_TWO_PHASE) return GKA_ERR_UNSUPPORTED;
    if (pl.fused_bytes > (size_t)GKA_STATIC_SCRATCH_BYTES) return GKA_ERR_STATIC_SCRATCH;
    void *ws = nullptr;
    s = static_scratch(&ws);
    if (s != GKA_OK) return s;
    gka_params pf = *p;
    pf.path = GKA_PATH_FUSED;            // (anything the fused kernels do not cover: GKA_ERR_UNSUPPORTED)
    return forward_impl(&pf, q, k, v, gate, lambda, o, H_init, U_init, H_final, U_final, fro_out, ws,
                        GKA_STATIC_SCRATCH_BYTES, hip_stream, nullptr);
}

namespace {
gka_status decode_impl(const gka_params *p, int n_tokens, float *H_state, float *U_state, const void *q, const void *k,
                       const void *v, const float *gate, const float *lambda, void *o, void *hip_stream)
{
    gka_status s = check_common(p, true);
    if (s != GKA_OK) return s;
    if (n_tokens <= 0) return GKA_ERR_SHAPE;
    if (!H_state || !U_state || !q || !k || !v || !gate || !o) return GKA_ERR_NULL;
    if (!lambda && !(p->lambda_scale > 0.0f)) return GKA_ERR_NULL;
    gka::DecodeArgs da = {};
    da.H_in = H_state; da.U_in = U_state;
    da.H_state = H_state; da.U_state = U_state;
    da.q = q; da.k = k; da.v = v; da.gate = gate; da.lambda = lambda; da.o = o;
    da.stride_h = p->d_k; da.stride_t = (int64_t)p->H * p->d_k; da.stride_b = (int64_t)n_tokens * p->H * p->d_k;
    da.beta = p->beta; da.alpha = p->alpha; da.lambda_scale = p->lambda_scale;
    da.n_iter = p->n_iter;
    da.T = n_tokens; da.H = p->H;
    da.h_lower_blocks = p->state_layout == GKA_STATE_H_LOWER_BLOCKS && chunked_dim(p->d_k);
    if (gka::launch_decode_step(da, p->B * p->H, p->d_k, p->io_dtype == GKA_BF16, (hipStream_t)hip_stream) !=
        hipSuccess)
        return GKA_ERR_LAUNCH;
    return GKA_OK;
}
}  // namespace

gka_status gka_decode_step(const gka_params *p, float *H_state, float *U_state, const void *q, const void *k,
                           const void *v, const float *gate, const float *lambda, void *o, void *hip_stream)
{
    return decode_impl(p, 1, H_state, U_state, q, k, v, gate, lambda, o, hip_stream);
}

gka_status gka_decode_tokens(const gka_params *p, float *H_state, float *U_state, const void *q, const void *k,
                             const void *v, const float *gate, const float *lambda, void *o, void *hip_stream)
{
    if (!p) return GKA_ERR_NULL;
    if (p->stride_b != 0 || p->stride_t != 0 || p->stride_h != 0) return GKA_ERR_UNSUPPORTED;
    return decode_impl(p, p->T, H_state, U_state, q, k, v, gate, lambda, o, hip_stream);
}

namespace {
// Segments of the fused readout's chunk scan: two workgroups per CU when the pairs alone do not give that many,
// never fewer than two chunks per segment.
constexpr int kReadoutMinWorkgroups = 512;
void plan_readout_segments(int n_pairs, int n_chunks, int *n_segs, int *seg_len)
{
    int ns = (kReadoutMinWorkgroups + n_pairs - 1) / n_pairs;
    if (ns > n_chunks / 2) ns = n_chunks / 2;
    if (ns < 1) ns = 1;
    *seg_len = (n_chunks + ns - 1) / ns;
    *n_segs = (n_chunks + *seg_len - 1) / *seg_len;
}

struct BackwardPlan {
    size_t n_elems, n_tokens, esz;
    size_t off_f32[9];        // xhat, p; with the fused readouts also y, H x, A k, A^T k, Ubar k, U^T dy, Ubar^T v
    size_t off_io[23];
    size_t off_m[6];          // gate_rev, zeros, s, fro, c, C
    size_t off_fin[3];        // final states of three reverse readouts (gradients at the initial states)
    size_t off_fwd, fwd_bytes, total;
    bool reuse_states;        // the second solve runs on the chunk states of the first
    size_t off_rws;           // scratch of the readouts (the forward workspace itself unless reuse_states)
    bool strided;             // q, k, v, dy come with explicit strides
    size_t off_pack[4];       // their packed copies
};
enum { IO_Y, IO_DXT, IO_RHS, IO_HX, IO_X, IO_XT, IO_KR, IO_VR, IO_DYR, IO_XR, IO_PR, IO_XTR, IO_R1, IO_R2, IO_R3, IO_R4,
       IO_SCRATCH, IO_HK, IO_VPR, IO_R5, IO_RHS_LO, IO_X_LO, IO_XT_LO };

gka_status make_backward_plan(const gka_params *p, BackwardPlan *bp)
{
    gka_status s = check_common(p, false);
    if (s != GKA_OK) return s;
    if (!chunked_dim(p->d_k) || p->path == GKA_PATH_RECURRENT) return GKA_ERR_UNSUPPORTED;
    if (p->phase != GKA_PHASE_ALL || p->compute == GKA_COMPUTE_BF16_SPLIT) return GKA_ERR_UNSUPPORTED;
    bp->n_tokens = (size_t)p->B * p->T * p->H;
    bp->n_elems = bp->n_tokens * p->d_k;
    bp->esz = p->io_dtype == GKA_BF16 ? 2 : 4;
    // Strided q, k, v, dy are copied into the packed layout first (four tensors at the head of the workspace): every
    // kernel of the pass works on packed tensors.
    bp->strided = p->stride_b != 0 || p->stride_t != 0 || p->stride_h != 0;
    size_t off = 0;
    if (bp->strided) {
        const int64_t align = 16 / (int64_t)bp->esz;         // rows are copied 16 bytes at a time
        if (p->stride_b <= 0 || p->stride_t <= 0 || p->stride_h <= 0) return GKA_ERR_SHAPE;
        if (p->stride_h < p->d_k && p->H > 1) return GKA_ERR_SHAPE;
        if (p->stride_b % align || p->stride_t % align || p->stride_h % align) return GKA_ERR_SHAPE;
        for (int i = 0; i < 4; ++i) { bp->off_pack[i] = off; off = align_up(off + bp->n_elems * bp->esz, 256); }
    }
    for (int i = 0; i < 9; ++i) { bp->off_f32[i] = off; off = align_up(off + bp->n_elems * 4, 256); }
    for (int i = 0; i < 23; ++i) { bp->off_io[i] = off; off = align_up(off + bp->n_elems * bp->esz, 256); }
    for (int i = 0; i < 6; ++i) { bp->off_m[i] = off; off = align_up(off + bp->n_tokens * 4, 256); }
    for (int i = 0; i < 3; ++i) {
        bp->off_fin[i] = off;
        off = align_up(off + (size_t)p->B * p->H * p->d_k * p->d_k * 4, 256);
    }
    bp->off_fwd = off;
    gka_params pf = *p;
    pf.xhat_out = nullptr;
    pf.stride_b = pf.stride_t = pf.stride_h = 0;
    Plan full, plain;                              // the plain readouts cut the scan into more segments
    if (make_plan(&pf, &full) != GKA_OK || make_plan(&pf, &plain, true) != GKA_OK) return GKA_ERR_SHAPE;
    bp->fwd_bytes = full.total > plain.total ? full.total : plain.total;
    int rs_n, rs_len;
    plan_readout_segments(p->B * p->H, (p->T + gka::kChunk - 1) / gka::kChunk, &rs_n, &rs_len);
    const size_t rbytes = align_up(gka::gla_readout_workspace_bytes(p->B * p->H, rs_n, p->d_k, p->d_v), 256);
    // bf16 tensors, one launch per phase: the second solve reuses the chunk states H_[n] that the first one left in the
    // forward workspace (the same H_t), so the readouts in between get a scratch region of their own
    bp->reuse_states = p->io_dtype == GKA_BF16 && full.pairs_per_batch >= full.n_pairs && full.slab_chunks >= full.n_chunks;
    if (bp->reuse_states) {
        bp->off_rws = off + bp->fwd_bytes;
        bp->total = bp->off_rws + rbytes;
    } else {
        if (rbytes > bp->fwd_bytes) bp->fwd_bytes = rbytes;
        bp->off_rws = bp->off_fwd;
        bp->total = off + bp->fwd_bytes;
    }
    return GKA_OK;
}
}  // namespace

size_t gka_backward_workspace_bytes(const gka_params *p)
{
    BackwardPlan bp;
    if (make_backward_plan(p, &bp) != GKA_OK) return 0;
    return bp.total;
}

gka_status gka_backward(const gka_params *p, const void *q, const void *k, const void *v, const float *gate,
                        const float *lambda, const void *dy, float *dq, float *dk, float *dv, float *dgate,
                        float *dlambda, float *dbeta, float *dalpha, void *workspace, size_t workspace_bytes,
                        void *hip_stream)
{
    return gka_backward_from_state(p, q, k, v, gate, lambda, dy, nullptr, nullptr, dq, dk, dv, dgate, dlambda, dbeta,
                                   dalpha, nullptr, nullptr, workspace, workspace_bytes, hip_stream);
}

gka_status gka_backward_from_state(const gka_params *p, const void *q, const void *k, const void *v,
                                   const float *gate, const float *lambda, const void *dy, const float *H_init,
                                   const float *U_init, float *dq, float *dk, float *dv, float *dgate,
                                   float *dlambda, float *dbeta, float *dalpha, float *dH_init, float *dU_init,
                                   void *workspace, size_t workspace_bytes, void *hip_stream)
{
    BackwardPlan bp;
    gka_status st = make_backward_plan(p, &bp);
    if (st != GKA_OK) return st;
    if (!q || !k || !v || !gate || !dy || !dq || !dk || !dv || !dgate) return GKA_ERR_NULL;
    if ((H_init == nullptr) != (U_init == nullptr)) return GKA_ERR_NULL;
    const bool with_state = H_init != nullptr || dH_init != nullptr || dU_init != nullptr;
    // initial states: bf16 tensors (the readouts that keep their state in registers), complete H_init
    if (with_state && (p->io_dtype != GKA_BF16 || p->state_layout != GKA_STATE_FULL)) return GKA_ERR_UNSUPPORTED;
    const bool rule = lambda == nullptr;          // lambda_t = lambda_scale ||H_t||_F
    if (rule && !(p->lambda_scale > 0.0f)) return GKA_ERR_NULL;
    if (!workspace || ((uintptr_t)workspace & 255) || workspace_bytes < bp.total) return GKA_ERR_WORKSPACE;
    hipStream_t stream = (hipStream_t)hip_stream;
    unsigned char *ws = (unsigned char *)workspace;
    gka_params packed_params;
    if (bp.strided) {
        const void *src[4] = {q, k, v, dy};
        for (int i = 0; i < 4; ++i) {
            if (gka::launch_pack_rows(src[i], ws + bp.off_pack[i], p->B, p->T, p->H, p->d_k, (int)bp.esz, p->stride_b,
                                      p->stride_t, p->stride_h, stream) != hipSuccess)
                return GKA_ERR_LAUNCH;
        }
        q = ws + bp.off_pack[0]; k = ws + bp.off_pack[1]; v = ws + bp.off_pack[2]; dy = ws + bp.off_pack[3];
        packed_params = *p;
        packed_params.stride_b = packed_params.stride_t = packed_params.stride_h = 0;
        p = &packed_params;
    }
    auto io = [&](int i) { return (void *)(ws + bp.off_io[i]); };
    float *xf = (float *)(ws + bp.off_f32[0]), *pf32 = (float *)(ws + bp.off_f32[1]);
    auto f32buf = [&](int i) { return (float *)(ws + bp.off_f32[i]); };
    float *gate_rev = (float *)(ws + bp.off_m[0]), *zeros = (float *)(ws + bp.off_m[1]), *sbuf = (float *)(ws + bp.off_m[2]);
    float *fro = (float *)(ws + bp.off_m[3]), *cbuf = (float *)(ws + bp.off_m[4]), *Cbuf = (float *)(ws + bp.off_m[5]);
    void *fws = ws + bp.off_fwd;
    const bool io_bf16 = p->io_dtype == GKA_BF16;

    gka::BackwardGlueArgs g = {};
    g.n_elems = (int64_t)bp.n_elems; g.n_tokens = (int64_t)bp.n_tokens;
    g.T = p->T; g.H = p->H; g.d = p->d_k;
    g.q = q; g.k = k; g.v = v; g.dy = dy; g.gate = gate; g.alpha = p->alpha; g.beta = p->beta;
    g.x_f32 = xf; g.p_f32 = pf32;
    g.x_io = io(IO_X); g.xt_io = io(IO_XT); g.rhs_io = io(IO_RHS);
    g.dxt_io = io(IO_DXT); g.y_io = io(IO_Y); g.hx_io = io(IO_HX);
    g.k_rev = io(IO_KR); g.v_rev = io(IO_VR); g.dy_rev = io(IO_DYR); g.x_rev = io(IO_XR); g.p_rev = io(IO_PR);
    g.xt_rev = io(IO_XTR);
    g.gate_rev = gate_rev; g.zeros = zeros;
    g.r1 = io(IO_R1); g.r2 = io(IO_R2); g.r3 = io(IO_R3); g.r4 = io(IO_R4);
    g.dq = dq; g.dk = dk; g.dv = dv; g.dgate = dgate; g.dlambda = dlambda; g.dbeta = dbeta; g.dalpha = dalpha; g.s = sbuf;
    g.rule_a = rule ? p->lambda_scale : 0.0f; g.fro = fro; g.c = cbuf; g.C = Cbuf;
    g.vp_rev = io(IO_VPR); g.hk_io = io(IO_HK); g.r5 = io(IO_R5);

    // a forward pass with the roles given; alpha = zeros makes it the plain readout y_t = U_t q_t of the gated
    // recurrence U_t = gate_t U_{t-1} + beta_t v_t k_t^T (the solve is reduced to its starting point and discarded)
    auto fwd = [&](const void *qq, const void *kk, const void *vv, const float *gg, const float *beta,
                   const float *alpha, int n_iter, void *out, float *xhat, float *fro_out = nullptr,
                   bool solve_only = false, const void *q_lo = nullptr, int phase = GKA_PHASE_ALL) {
        gka_params pp = *p;                      // lambda (or its rule) as given: only the two solves use it
        pp.beta = beta; pp.alpha = alpha; pp.n_iter = n_iter; pp.xhat_out = xhat; pp.phase = phase;
        pp.state_layout = GKA_STATE_FULL;
        const bool plain_readout = alpha == zeros;
        // (initial states reach the two solves; the composition of plain readouts for float32 tensors has none)
        const bool is_solve = xhat != nullptr;
        return forward_impl(&pp, qq, kk, vv, gg, lambda, out, is_solve ? H_init : nullptr, is_solve ? U_init : nullptr,
                            nullptr, nullptr, fro_out, fws, bp.fwd_bytes, hip_stream, nullptr, plain_readout, solve_only,
                            q_lo);
    };
    auto glue = [&](int which) {
        return gka::launch_backward_glue(g, which, io_bf16, stream) == hipSuccess ? GKA_OK : GKA_ERR_LAUNCH;
    };
    // the plain readout y_t = U_t qq_t, U_t = gate_t U_{t-1} + beta_t vv_t kk_t^T, in one kernel with the state in
    // registers (bf16 tensors); `reverse`: the recurrence runs from the last token to the first
    // (bf16 tensors: whatever operands the two solves use, the readouts take the stored bf16 tensors as they are)
    const bool fused = io_bf16;
    // out_f32: the output in float32 (the pieces of the gate gradient's sum), else in the tensors' dtype
    // q_lo, k_lo, v_lo: the bf16 remainder of an operand that was computed in float32 (x, xt), or nullptr
    // init / init_transposed: the state before the first token (forward readouts); fin: where the state after the last
    // token of the walk goes (reverse readouts: the accumulated gradient at the initial state)
    auto readout = [&](const void *qq, const void *kk, const void *vv, const float *beta, bool reverse, void *out,
                       int seg_mode = 0, float *out_f32 = nullptr, const void *q_lo = nullptr,
                       const void *k_lo = nullptr, const void *v_lo = nullptr, const float *init = nullptr,
                       bool init_transposed = false, float *fin = nullptr) {
        gka::ReadoutArgs r = {};                     // (optional pointers default to nullptr)
        r.init_state = init; r.init_transposed = init_transposed; r.final_state = fin;
        r.q = qq; r.q_lo = q_lo; r.k_lo = k_lo; r.v_lo = v_lo; r.q_is_f32 = false; r.k = kk; r.v = vv; r.o = out;
        r.o_f32 = out_f32;
        r.gate = gate; r.beta = beta;
        r.stride_h = p->d_k; r.stride_t = (int64_t)p->H * p->d_k; r.stride_b = (int64_t)p->T * p->H * p->d_k;
        r.qk_stride_h = r.stride_h; r.qk_stride_t = r.stride_t; r.qk_stride_b = r.stride_b;
        r.H = p->H; r.T = p->T; r.n_pairs = p->B * p->H;
        plan_readout_segments(r.n_pairs, (p->T + gka::kChunk - 1) / gka::kChunk, &r.n_segs, &r.seg_len);
        r.seg_buf = (float *)(ws + bp.off_rws);
        r.seg_logdecay = r.seg_buf + (size_t)r.n_pairs * r.n_segs * p->d_k * p->d_v;
        r.reverse = reverse; r.seg_mode = seg_mode;
        return gka::launch_gla_readout(r, p->d_k, p->d_v, stream) == hipSuccess ? GKA_OK : GKA_ERR_LAUNCH;
    };
    g.natural_order = fused;
    if (fused) {                                  // these seven arrive in float32 (see the combine kernel)
        g.y_io = f32buf(2); g.hx_io = f32buf(3); g.r1 = f32buf(4); g.r2 = f32buf(5); g.r4 = f32buf(6);
        g.dxt_io = f32buf(7); g.r3 = f32buf(8);
        // bf16 tensors: the second solve takes alpha dxt, and the readouts take x and xt, as value + remainder
        g.rhs_lo_io = io(IO_RHS_LO); g.x_lo_io = io(IO_X_LO); g.xt_lo_io = io(IO_XT_LO);
    }
#define GKA_TRY(expr) do { gka_status e_ = (expr); if (e_ != GKA_OK) return e_; } while (0)
    // the forward solve and output; then x, xt in the tensors' dtype, the all-zero alpha and the reversed gates
    // (with the fused readouts y is read out again below, and the solves run without U states and readout)
    GKA_TRY(fwd(q, k, v, gate, p->beta, p->alpha, p->n_iter, io(IO_Y), xf, rule ? fro : nullptr, fused));
    GKA_TRY(glue(0));
    // y_t again, from the stored xt (see the combine kernel)
    if (fused) GKA_TRY(readout(io(IO_XT), k, v, p->beta, false, nullptr, 0, f32buf(2), io(IO_XT_LO), nullptr, nullptr,
                               U_init));
    // dxt_t = U_t^T dy_t: the recurrence with the roles of k and v exchanged, read out with dy
    // (its state is the transpose of the one just read out: the segment summaries are reused)
    if (fused) GKA_TRY(readout(dy, v, k, p->beta, false, nullptr, 2, f32buf(7), nullptr, nullptr, nullptr, U_init, true));
    else GKA_TRY(fwd(dy, v, k, gate, p->beta, zeros, 0, io(IO_DXT), nullptr));
    GKA_TRY(glue(1));
    // p_t = CH(H_t + lambda_t I, alpha_t dxt_t, r)
    // (the chunk states H_[n] of the first solve are still in the forward workspace where the plan says so)
    GKA_TRY(fwd(io(IO_RHS), k, v, gate, p->beta, nullptr, p->n_iter, io(IO_SCRATCH), pf32, nullptr, fused,
                fused ? io(IO_RHS_LO) : nullptr, fused && bp.reuse_states ? GKA_PHASE_SOLVE : GKA_PHASE_ALL));
    // H_t x_t
    if (fused) GKA_TRY(readout(io(IO_X), k, k, p->beta, false, nullptr, 0, f32buf(3), io(IO_X_LO), nullptr, nullptr,
                               H_init));
    else GKA_TRY(fwd(io(IO_X), k, k, gate, p->beta, zeros, 0, io(IO_HX), nullptr));
    // the rule's extra gradient -c_t H_t at every state: c_t, C_t = sum_{s>=t} M[t,s]^2 c_s, and H_t k_t
    if (rule) {
        GKA_TRY(glue(5));
        GKA_TRY(glue(6));
        if (fused) GKA_TRY(readout(k, k, k, p->beta, false, io(IO_HK), 1, nullptr, nullptr, nullptr, nullptr, H_init));
        else GKA_TRY(fwd(k, k, k, gate, p->beta, zeros, 0, io(IO_HK), nullptr));
    }
    // reverse recurrences: A_t k_t, A_t^T k_t, Ubar_t^T v_t, Ubar_t k_t (no write gate inside them)
    GKA_TRY(glue(2));
    if (fused) {
        float *fin_px = with_state ? (float *)(ws + bp.off_fin[0]) : nullptr;
        float *fin_xtdy = with_state ? (float *)(ws + bp.off_fin[1]) : nullptr;
        float *fin_ck = with_state && rule ? (float *)(ws + bp.off_fin[2]) : nullptr;
        if (rule) GKA_TRY(readout(k, k, io(IO_VPR), nullptr, true, io(IO_R5), 0, nullptr, nullptr, nullptr, nullptr,
                                  nullptr, false, fin_ck));
        GKA_TRY(readout(k, io(IO_X), io(IO_PR), nullptr, true, nullptr, 0, f32buf(4), nullptr, io(IO_X_LO), nullptr,
                        nullptr, false, fin_px));
        GKA_TRY(readout(k, io(IO_PR), io(IO_X), nullptr, true, nullptr, 2, f32buf(5), nullptr, nullptr, io(IO_X_LO)));
        GKA_TRY(readout(v, dy, io(IO_XT), nullptr, true, nullptr, 0, f32buf(8), nullptr, nullptr, io(IO_XT_LO),
                        nullptr, false, fin_xtdy));
        g.fin_px = fin_px; g.fin_xtdy = fin_xtdy; g.fin_ck = fin_ck;
        GKA_TRY(readout(k, io(IO_XT), dy, nullptr, true, nullptr, 2, f32buf(6), nullptr, io(IO_XT_LO), nullptr));
    } else {
        if (rule) GKA_TRY(fwd(io(IO_KR), io(IO_KR), io(IO_VPR), gate_rev, nullptr, zeros, 0, io(IO_R5), nullptr));
        GKA_TRY(fwd(io(IO_KR), io(IO_XR), io(IO_PR), gate_rev, nullptr, zeros, 0, io(IO_R1), nullptr));
        GKA_TRY(fwd(io(IO_KR), io(IO_PR), io(IO_XR), gate_rev, nullptr, zeros, 0, io(IO_R2), nullptr));
        GKA_TRY(fwd(io(IO_VR), io(IO_DYR), io(IO_XTR), gate_rev, nullptr, zeros, 0, io(IO_R3), nullptr));
        GKA_TRY(fwd(io(IO_KR), io(IO_XTR), io(IO_DYR), gate_rev, nullptr, zeros, 0, io(IO_R4), nullptr));
    }
    GKA_TRY(glue(3));
    GKA_TRY(glue(4));
    if (dH_init || dU_init) {
        g.H_init = H_init; g.dH_init = dH_init; g.dU_init = dU_init; g.n_pairs = p->B * p->H;
        GKA_TRY(glue(7));
    }
#undef GKA_TRY
    return GKA_OK;
}

// ---- latent sketching: down-projection, the solve in the sketched space (up to 32 dimensions on the kernels of
// gka_small_dim.hip, else in 64 zero-padded dimensions on the forward kernels), readout in the sketched space (d = 128)
// or up-projection and plain readout with the full U_t (d = 64)
namespace {
struct SketchPlan {
    size_t n_tokens;
    size_t off_qs, off_ks, off_scratch, off_z, off_xhat, off_xhat_lo, off_fwd, fwd_bytes, total;
    gka_params inner;             // the solve's problem: d = 64, packed
    int rs_n, rs_len;
    bool small;                   // d_s <= 32: the solve runs on the kernels of gka_small_dim.hip
};
constexpr int kSketchDim = 64;
constexpr int kSketchSmall = 32;
gka_status make_sketch_plan(const gka_params *p, int d_s, SketchPlan *sp)
{
    gka_status s = check_common(p, false);
    if (s != GKA_OK) return s;
    if (p->io_dtype != GKA_BF16 || p->compute != GKA_COMPUTE_BF16) return GKA_ERR_UNSUPPORTED;
    if (!chunked_dim(p->d_k) || p->path == GKA_PATH_RECURRENT) return GKA_ERR_UNSUPPORTED;
    if (p->stride_b != 0 || p->stride_t != 0 || p->stride_h != 0) return GKA_ERR_UNSUPPORTED;
    if (p->phase != GKA_PHASE_ALL || p->alpha) return GKA_ERR_UNSUPPORTED;
    if (d_s < 1 || d_s > kSketchDim) return GKA_ERR_SHAPE;
    sp->n_tokens = (size_t)p->B * p->T * p->H;
    sp->inner = *p;
    sp->inner.d_k = sp->inner.d_v = kSketchDim;
    sp->inner.xhat_out = nullptr;
    sp->inner.state_layout = GKA_STATE_FULL;
    size_t off = 0;
    sp->off_qs = off; off = align_up(off + sp->n_tokens * kSketchDim * 2, 256);
    sp->off_ks = off; off = align_up(off + sp->n_tokens * kSketchDim * 2, 256);
    sp->off_scratch = off; off = align_up(off + sp->n_tokens * kSketchDim * 2, 256);
    sp->off_z = off; off = align_up(off + sp->n_tokens * kSketchDim * 4, 256);
    sp->off_xhat = off; off = align_up(off + sp->n_tokens * p->d_k * 2, 256);
    sp->off_xhat_lo = off; off = align_up(off + sp->n_tokens * p->d_k * 2, 256);
    sp->off_fwd = off;
    Plan pl;
    if (make_plan(&sp->inner, &pl) != GKA_OK) return GKA_ERR_SHAPE;
    sp->fwd_bytes = pl.total;
    plan_readout_segments(p->B * p->H, (p->T + gka::kChunk - 1) / gka::kChunk, &sp->rs_n, &sp->rs_len);
    const size_t rbytes = align_up(gka::gla_readout_workspace_bytes(p->B * p->H, sp->rs_n, p->d_k, p->d_v), 256);
    if (rbytes > sp->fwd_bytes) sp->fwd_bytes = rbytes;
    // up to 32 sketched dimensions the solve has kernels of its own (their chunk states: 2 x 4 KiB per chunk)
    sp->small = d_s <= kSketchSmall;
    if (sp->small) {
        const size_t sbytes = gka::small_dim_workspace_bytes(p->B * p->H, (p->T + gka::kChunk - 1) / gka::kChunk, kSketchSmall, false);
        if (sbytes > sp->fwd_bytes) sp->fwd_bytes = sbytes;
    }
    sp->total = off + sp->fwd_bytes;
    return GKA_OK;
}
}  // namespace

size_t gka_forward_sketched_workspace_bytes(const gka_params *p, int d_s)
{
    SketchPlan sp;
    if (make_sketch_plan(p, d_s, &sp) != GKA_OK) return 0;
    return sp.total;
}

gka_status gka_forward_sketched(const gka_params *p, const void *q, const void *k, const void *v, const float *gate,
                                const float *lambda, const float *S, int d_s, int sketch_per_head, void *o,
                                void *workspace, size_t workspace_bytes, void *hip_stream)
{
    SketchPlan sp;
    gka_status st = make_sketch_plan(p, d_s, &sp);
    if (st != GKA_OK) return st;
    if (!q || !k || !v || !gate || !S || !o) return GKA_ERR_NULL;
    if (!lambda && !(p->lambda_scale > 0.0f)) return GKA_ERR_NULL;
    if (!workspace || ((uintptr_t)workspace & 255) || workspace_bytes < sp.total) return GKA_ERR_WORKSPACE;
    hipStream_t stream = (hipStream_t)hip_stream;
    unsigned char *ws = (unsigned char *)workspace;
    gka::SketchArgs sa = {};
    // stored width of the sketched tensors: 32 where everything downstream works in 32 dimensions
    const int sw = sp.small && p->d_v == 128 ? kSketchSmall : kSketchDim;
    sa.q = q; sa.k = k; sa.S = S; sa.d_s = d_s; sa.per_head = sketch_per_head != 0; sa.out_width = sw;
    sa.qs = ws + sp.off_qs; sa.ks = ws + sp.off_ks; sa.z = (const float *)(ws + sp.off_z);
    sa.xhat_hi = ws + sp.off_xhat; sa.xhat_lo = ws + sp.off_xhat_lo;
    sa.T = p->T; sa.H = p->H;
    const int n_pairs = p->B * p->H;
    if (gka::launch_sketch(sa, n_pairs, p->d_k, false, stream) != hipSuccess) return GKA_ERR_LAUNCH;
    // z_t = CH(S H_t S^T + lambda_t I, S q_t, r): the forward pass on the sketched keys and queries, its own readout
    // discarded (the sketched keys stand in for its values)
    if (sp.small) {
        gka::SmallArgs ss = {};                  // (no values, no output: the solve alone)
        ss.q = sa.qs; ss.k = sa.ks;
        ss.stride_h = sw; ss.stride_t = (int64_t)p->H * sw; ss.stride_b = (int64_t)p->T * p->H * sw;
        ss.d = kSketchSmall;
        ss.gate = gate; ss.lambda = lambda; ss.beta = p->beta; ss.lambda_scale = p->lambda_scale;
        ss.xhat_out = (float *)(ws + sp.off_z); ss.xhat_row = sw;
        ss.xhat_zero_upper = sw == kSketchDim;   // (the up-projection of the d = 64 path reads all 64 stored features)
        ss.T = p->T; ss.H = p->H; ss.n_pairs = n_pairs; ss.n_chunks = (p->T + gka::kChunk - 1) / gka::kChunk;
        ss.n_iter = p->n_iter;
        if (gka::launch_small_dim_forward(ss, ws + sp.off_fwd, stream) != hipSuccess) return GKA_ERR_LAUNCH;
    } else {
        gka_params inner = sp.inner;
        inner.xhat_out = (float *)(ws + sp.off_z);
        st = forward_impl(&inner, sa.qs, sa.ks, sa.ks, gate, lambda, ws + sp.off_scratch, nullptr, nullptr, nullptr,
                          nullptr, nullptr, ws + sp.off_fwd, sp.fwd_bytes, hip_stream, nullptr, false, true);
        if (st != GKA_OK) return st;
    }
    gka::ReadoutArgs r = {};                     // (optional pointers default to nullptr)
    r.k_lo = nullptr; r.v_lo = nullptr;
    r.v = v; r.o = o; r.o_f32 = nullptr; r.gate = gate; r.beta = p->beta;
    r.stride_h = p->d_v; r.stride_t = (int64_t)p->H * p->d_v; r.stride_b = (int64_t)p->T * p->H * p->d_v;
    r.H = p->H; r.T = p->T; r.n_pairs = n_pairs;
    r.n_segs = sp.rs_n; r.seg_len = sp.rs_len;
    r.seg_buf = (float *)(ws + sp.off_fwd);
    r.reverse = false; r.seg_mode = 0;
    if (p->d_v == 128) {
        // y_t = U_t S^T z_t = (sum_i eta_{t,i} beta_i v_i (S k_i)^T) z_t: the readout runs in the sketched space, on the
        // stored sketched keys and the float32 z_t (split into value + remainder inside the kernel), with a d_v x 64
        // state; the projected solution xhat_t is never formed
        r.q = sa.z; r.q_lo = nullptr; r.q_is_f32 = true; r.k = sa.ks;
        r.qk_stride_h = sw; r.qk_stride_t = (int64_t)p->H * sw;
        r.qk_stride_b = (int64_t)p->T * p->H * sw;
        r.seg_logdecay = r.seg_buf + (size_t)n_pairs * r.n_segs * kSketchDim * p->d_v;
        // (up to 32 sketched dimensions: a d_v x 32 state on the first 32 stored features)
        return gka::launch_gla_readout(r, sp.small ? kSketchSmall : kSketchDim, p->d_v, stream) == hipSuccess
                   ? GKA_OK : GKA_ERR_LAUNCH;
    }
    // d = 64: xhat_t = S^T z_t as value + remainder, then y_t = U_t xhat_t with the state of Eq. (CH)
    if (gka::launch_sketch(sa, n_pairs, p->d_k, true, stream) != hipSuccess) return GKA_ERR_LAUNCH;
    r.q = sa.xhat_hi; r.q_lo = sa.xhat_lo; r.q_is_f32 = false; r.k = k;
    r.qk_stride_h = r.stride_h; r.qk_stride_t = r.stride_t; r.qk_stride_b = r.stride_b;
    r.seg_logdecay = r.seg_buf + (size_t)n_pairs * r.n_segs * p->d_k * p->d_v;
    return gka::launch_gla_readout(r, p->d_k, p->d_v, stream) == hipSuccess ? GKA_OK : GKA_ERR_LAUNCH;
}

const char *gka_status_string(gka_status s)
{
    switch (s) {
    case GKA_OK: return "ok";
    case GKA_ERR_NULL: return "required pointer is NULL";
    case GKA_ERR_SHAPE: return "invalid size or stride";
    case GKA_ERR_UNSUPPORTED: return "unsupported head dimension, chunk, dtype or compute mode";
    case GKA_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case GKA_ERR_LAUNCH: return "HIP launch failed";
    case GKA_ERR_STATIC_SCRATCH: return "problem needs more scratch than gka_forward_static's fixed array holds";
    }
    return "unknown status";
}

int gka_version(void) { return 810; }

}  // extern "C"
