// Whole decode step of one token row as ONE kernel: every workgroup walks the
// same list of phases (row table + embedding, then per layer QKV / attention /
// O-proj / gate-up / down, then LM head and router merge) and the phases are
// separated by a grid-wide barrier; on top of it, Algorithm 1's whole loop as one
// kernel (k_stitch_loop).  On MI355X a software barrier across the eight XCDs
// (agent-scope release + acquire per workgroup, several dependent round trips to
// memory-side atomics) costs 12-16 us against the ~2 us of a kernel boundary, so
// both are slower than one kernel per phase; they exist for callers that cannot
// put the host between invocations, and as a measured answer to that question.
//
// The kernels are launched cooperatively (all workgroups co-resident), and every
// wait in them is bounded: a workgroup that polls longer than `spin_limit` times
// raises a sticky abort word; every other workgroup leaves at its next poll, the
// record is flagged RS_FLAG_ABORTED (the loop: status RS_STITCH_ABORTED) and, for
// the single step, later launches return at once.
#pragma once

#include "model_kernels.h"

namespace rs {

struct LayerPtrs { const uint16_t *attn_norm, *w_qkv, *w_o, *mlp_norm, *w_gate_up, *w_down; };

// Words of the grid-wide barrier, each on a cache line of its own: arrivals are counted per group of
// workgroups and the last of a group reports to the root, so that no counter sees more than
// SYNC_GROUPS (or a group's size) back-to-back atomics; waiting workgroups poll their group's `release`
// word, which the arrivals do not touch and at most a group's workgroups read.  All counters only grow:
// after barrier number b the root holds b * groups.
constexpr int SYNC_GROUPS = 16;
struct alignas(128) SyncLine { unsigned long long v; unsigned long long pad[15]; };
struct SyncState {
    SyncLine root;               // groups that have arrived, over all barriers so far
    SyncLine release[SYNC_GROUPS];   // per group: number of the last completed barrier
    SyncLine abort;              // sticky (low word): a bounded wait ran out
    SyncLine grp[SYNC_GROUPS];   // workgroups of the group that have arrived, over all barriers so far
};

struct PersistArgs {
    PrepArgs prep;
    GemvArgs gemv;               // shape fields and per-call pointers; per-phase fields are set in the kernel
    AttnArgs attn;
    const LayerPtrs *layers; int n_layers;
    int qkv_rows, qdim;
    const uint16_t *lm_head, *final_norm;
    int qkv_rt, o_rt, down_rt;   // rows per wave tile chosen on the host for this shape
    int n_splits;
    int vocab; float tau; int active;
    int *seq_bad; rs_route_out *out;
    SyncState *sync; unsigned long long bar_base; unsigned int spin_limit;   // bar_base: barriers completed before this launch
};

__device__ __forceinline__ unsigned long long sync_load(const unsigned long long *p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Barrier number `gen` (1, 2, ... since the words were cleared) of a grid of nwg co-resident workgroups.
// Returns false if the wait was abandoned.
__device__ __forceinline__ bool grid_barrier(SyncState *s, unsigned long long gen, int wg, int nwg, unsigned int spin_limit) {
    __shared__ int ok_sh;
    __syncthreads();
    if (threadIdx.x == 0) {
        const int ng = nwg < SYNC_GROUPS ? nwg : SYNC_GROUPS;
        const int g = wg % ng;
        const unsigned long long gs = (unsigned long long)(nwg / ng + (g < nwg % ng ? 1 : 0));
        __threadfence();                                      // this workgroup's writes are out before it counts as arrived
        if (atomicAdd(&s->grp[g].v, 1ULL) + 1ULL == gen * gs)
            if (atomicAdd(&s->root.v, 1ULL) + 1ULL == gen * (unsigned long long)ng)
                for (int i = 0; i < ng; ++i)
                    __hip_atomic_store(&s->release[i].v, gen, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        unsigned int spins = 0;
        int ok = 1;
        while (sync_load(&s->release[g].v) < gen) {
            __builtin_amdgcn_s_sleep(1);
            ++spins;
            if (spins >= spin_limit || ((spins & 63u) == 0u && sync_load(&s->abort.v) != 0ULL)) {
                ok = 0;
                break;
            }
        }
        if (!ok) __hip_atomic_store(&s->abort.v, 1ULL, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __threadfence();
        ok_sh = ok;
    }
    __syncthreads();
    return ok_sh != 0;
}

__device__ __forceinline__ void write_aborted(rs_route_out *out, int active) {
    if (threadIdx.x == 0) {
        const float qnan = __uint_as_float(0x7fc00000u);
        rs_route_out r;
        r.token = -1; r.h_nats = qnan; r.h_norm = qnan; r.max_logit = qnan; r.log_z = qnan;
        r.flags = RS_FLAG_ABORTED | RS_FLAG_HI | RS_FLAG_NEXT_LLM | (active == RS_LLM ? RS_FLAG_ACCEPT : 0u);
        out[0] = r;
    }
}

// The decoder layers and, if asked for, the LM head with its router record for the token row that
// `prepare_row` / `loop_prepare_row` has just set up (a barrier included).  `gen` is the number of the last barrier
// the grid has passed.  Returns false when a wait was abandoned.
template <int HD>
__device__ __forceinline__ bool persistent_row(const PersistArgs &p, unsigned char *smem, int wg, int nwg,
                                               unsigned long long &gen, bool lm_head, float tau, int active,
                                               rs_route_out *out) {
#define RS_BARRIER()                                                          \
    do {                                                                      \
        ++gen;                                                                \
        if (!grid_barrier(p.sync, gen, wg, nwg, p.spin_limit)) return false;  \
    } while (0)
    RS_BARRIER();                                             // row table and embedding are in place
    GemvArgs g = p.gemv;
    AttnArgs at = p.attn;
    float *h = p.prep.h;
    const int d = p.prep.d_model;
    for (int l = 0; l < p.n_layers; ++l) {
        const LayerPtrs lp = p.layers[l];
        g.layer = l; at.layer = l;
        // QKV (+ RMSNorm, RoPE, KV write)
        g.W = lp.w_qkv; g.N = p.qkv_rows; g.K = d; g.h_in = h; g.gain = lp.attn_norm; g.x_in = nullptr;
        gemv_phase<G_QKV, 2, 1, 2, 1>(g, smem, wg, nwg);
        RS_BARRIER();
        // attention: (slice, kv head) units, then one merge unit per query head
        for (int u = wg; u < p.n_splits * at.n_kv; u += nwg) {
            attn_partial_unit<HD>(at, smem, u % p.n_splits, p.n_splits, u / p.n_splits, 0);
            __syncthreads();
        }
        RS_BARRIER();
        for (int u = wg; u < at.n_q; u += nwg) {
            attn_combine_unit<HD>(at, smem, u, 0);
            __syncthreads();
        }
        RS_BARRIER();
        // O projection + residual
        g.W = lp.w_o; g.N = d; g.K = p.qdim; g.h_in = nullptr; g.gain = nullptr; g.x_in = at.out;
        gemv_phase<G_OPROJ, 2, 1, 2, 1>(g, smem, wg, nwg);
        RS_BARRIER();
        // gate/up (+ RMSNorm, SwiGLU)
        g.W = lp.w_gate_up; g.N = 2 * g.d_ffn; g.K = d; g.h_in = h; g.gain = lp.mlp_norm; g.x_in = nullptr;
        gemv_phase<G_GATEUP, 4, 1, 4, 1>(g, smem, wg, nwg);
        RS_BARRIER();
        // down + residual
        g.W = lp.w_down; g.N = d; g.K = g.d_ffn; g.h_in = nullptr; g.gain = nullptr; g.x_in = g.act;
        if (p.down_rt == 2) gemv_phase<G_DOWN, 2, 4, 2, 1>(g, smem, wg, nwg);
        else if (p.down_rt == 4) gemv_phase<G_DOWN, 4, 4, 2, 1>(g, smem, wg, nwg);
        else gemv_phase<G_DOWN, 8, 4, 1, 1>(g, smem, wg, nwg);
        RS_BARRIER();
    }
    if (!lm_head) return true;
    // LM head + single-pass softmax statistics, one partial per workgroup
    g.W = p.lm_head; g.N = p.vocab; g.K = d; g.h_in = h; g.gain = p.final_norm; g.x_in = nullptr;
    g.n_parts = nwg;
    gemv_phase<G_LMHEAD, 8, 1, 2, 1>(g, smem, wg, nwg);
    RS_BARRIER();
    if (wg == 0) route_merge_row(g.parts, nwg, p.vocab, tau, active, p.seq_bad, out, 0, reinterpret_cast<SoftPartial *>(smem));
#undef RS_BARRIER
    return true;
}

template <int HD>
__global__ void __launch_bounds__(256) k_decode_persistent(PersistArgs p) {
    extern __shared__ __align__(16) unsigned char smem[];
    const int wg = blockIdx.x, nwg = gridDim.x;
    if (sync_load(&p.sync->abort.v) != 0ULL) {
        if (wg == 0) write_aborted(p.out, p.active);
        return;
    }
    unsigned long long gen = p.bar_base;
    if (wg == 0) prepare_row(p.prep, 0, reinterpret_cast<int *>(smem));
    if (!persistent_row<HD>(p, smem, wg, nwg, gen, true, p.tau, p.active, p.out)) write_aborted(p.out, p.active);
}

// ------------------------------------------------------------------------------------------------
// Algorithm 1 ("Inference procedure") as ONE kernel: the loop state (sequence length, how many rows
// each model has cached, which model runs next) lives in device memory, workgroup 0 applies the
// routing flags of every invocation to it, and the host reads nothing until the run is over.  The
// active model's unseen suffix is fed one token row at a time through `persistent_row`; only its
// last row runs the LM head and the router.  Every wait is bounded as in the single-step kernel, the
// number of invocations is bounded by the trace capacity, and every workgroup takes the same exits.
// ------------------------------------------------------------------------------------------------
struct LoopArgs {
    PersistArgs m[2];            // RS_SLM, RS_LLM (prep.tokens / pos0 / scale are not used)
    int *seq;                    // prompt followed by the accepted tokens
    const float *scale;          // entry p scales the logits that predict position p, or null (1.0)
    float tau; int eos; int slot;
    rs_stitch_record *trace; int max_records;
    rs_stitch_result *state;     // live loop state and, at the end, the result
    SyncState *sync; unsigned int spin_limit;
};

// Row table of a one-row call and the embedding row, by one workgroup.
__device__ __forceinline__ void loop_prepare_row(const PrepArgs &a, int token, int pos, int slot, float scale) {
    const int tid = threadIdx.x;
    const int bad = (token < 0 || token >= a.vocab || pos < 0 || pos >= a.max_ctx || slot < 0 || slot >= a.max_seqs) ? 1 : 0;
    if (tid == 0) {
        a.row_bad[0] = bad; a.row_slot[0] = bad ? 0 : slot; a.row_pos[0] = bad ? 0 : pos;
        a.out_row[0] = 0; a.seq_bad[0] = bad; a.seq_scale[0] = scale;
        a.seq_info[0] = bad ? make_int4(-1, 0, 0, 0) : make_int4(0, 1, slot, pos);
    }
    if (bad) { for (int i = tid; i < a.d_model; i += 256) a.h[i] = 0.f; return; }
    const uint16_t *e = a.embed + (size_t)token * a.d_model;
    for (int i = tid; i < a.d_model; i += 256) a.h[i] = bf16_to_f32(e[i]);
}

__device__ __forceinline__ int loop_load(const int32_t *p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// one thread: the state a run starts from, and the barrier words cleared
__global__ void k_stitch_init(rs_stitch_result *st, SyncState *sync, int n_prompt, int n_target, int seen_slm, int seen_llm) {
    if (blockIdx.x != 0 || threadIdx.x != 0) return;
    st->status = RS_STITCH_RUNNING; st->n_tokens = n_prompt; st->n_records = 0;
    st->seen_slm = seen_slm; st->seen_llm = seen_llm; st->active = RS_SLM; st->n_target = n_target; st->reserved = 0;
    sync->root.v = 0ULL; sync->abort.v = 0ULL;
    for (int g = 0; g < SYNC_GROUPS; ++g) { sync->grp[g].v = 0ULL; sync->release[g].v = 0ULL; }
}

template <int HD>
__global__ void __launch_bounds__(256) k_stitch_loop(LoopArgs a) {
    extern __shared__ __align__(16) unsigned char smem[];
    const int wg = blockIdx.x, nwg = gridDim.x;
    rs_stitch_result *st = a.state;
    unsigned long long gen = 0;                               // the barrier words are cleared before every launch
    for (int it = 0; it < a.max_records; ++it) {
        // the state is stable here: its last writer passed a barrier after writing it
        if (loop_load(&st->status) != RS_STITCH_RUNNING) return;
        const int active = loop_load(&st->active) != 0 ? RS_LLM : RS_SLM;
        const int n_tok = loop_load(&st->n_tokens), n_rec = loop_load(&st->n_records);
        const int pos0 = active == RS_LLM ? loop_load(&st->seen_llm) : loop_load(&st->seen_slm);
        const PersistArgs &p = a.m[active];
        rs_stitch_record *rec = a.trace + n_rec;
        // Algorithm 1 keeps at least one unseen token in front of the model it activates; a state that
        // says otherwise (or lies outside the buffers) ends the run
        const bool sane = pos0 >= 0 && pos0 < n_tok && n_tok < loop_load(&st->n_target) && n_rec >= 0 && n_rec < a.max_records;
        if (!sane) {
            if (wg == 0 && threadIdx.x == 0) __hip_atomic_store(&st->status, RS_STITCH_FLAGGED, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            return;
        }
        for (int pos = pos0; pos < n_tok; ++pos) {
            const bool last = pos == n_tok - 1;
            if (wg == 0) loop_prepare_row(p.prep, a.seq[pos], pos, a.slot, last && a.scale ? a.scale[n_tok] : 1.f);
            if (!persistent_row<HD>(p, smem, wg, nwg, gen, last, a.tau, active, &rec->out)) {
                if (threadIdx.x == 0) __hip_atomic_store(&st->status, RS_STITCH_ABORTED, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                return;
            }
        }
        if (wg == 0 && threadIdx.x == 0) {
            // Algorithm 1's bookkeeping from the flag bits of the record this thread has just written
            const unsigned int flags = rec->out.flags;
            const int token = rec->out.token;
            rec->model = active; rec->pos0 = pos0; rec->n_rows = n_tok - pos0; rec->reserved = 0;
            if (active == RS_LLM) st->seen_llm = n_tok; else st->seen_slm = n_tok;
            int status = RS_STITCH_RUNNING, n_new_tok = n_tok;
            if (flags & (RS_FLAG_BADARG | RS_FLAG_NONFINITE | RS_FLAG_ABORTED)) status = RS_STITCH_FLAGGED;
            else if (flags & RS_FLAG_ACCEPT) {
                a.seq[n_tok] = token;
                n_new_tok = n_tok + 1;
                if (n_new_tok >= st->n_target || token == a.eos) status = RS_STITCH_DONE;
            }
            if (status == RS_STITCH_RUNNING && n_rec + 1 >= a.max_records) status = RS_STITCH_TRACE_FULL;
            st->n_tokens = n_new_tok;
            st->n_records = n_rec + 1;
            st->active = (flags & RS_FLAG_NEXT_LLM) ? RS_LLM : RS_SLM;
            st->status = status;
        }
        ++gen;
        if (!grid_barrier(a.sync, gen, wg, nwg, a.spin_limit)) {
            if (threadIdx.x == 0) __hip_atomic_store(&st->status, RS_STITCH_ABORTED, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            return;
        }
    }
}

}  // namespace rs
