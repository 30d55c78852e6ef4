// Whole decode step of one token row as ONE kernel: every workgroup walks the
// same list of phases (row table + embedding, then per layer QKV / attention /
// O-proj / gate-up / down, then LM head and router merge) and the phases are
// separated by a grid-wide barrier.  This removes ~140 kernel launches per
// step, each of which costs several microseconds of launch and ramp-up latency
// that a 0.4 ms step cannot afford.
//
// The kernel is launched cooperatively (all workgroups co-resident), and every
// wait in it is bounded: a workgroup that polls longer than `spin_limit` times
// raises a sticky abort word; every other workgroup leaves at its next poll, the
// record is flagged RS_FLAG_ABORTED and later launches return at once.
#pragma once

#include "model_kernels.h"

namespace rs {

struct LayerPtrs { const uint16_t *attn_norm, *w_qkv, *w_o, *mlp_norm, *w_gate_up, *w_down; };

struct SyncState {
    unsigned long long arrive;   // arrivals at all barriers since the model was created
    unsigned int abort;          // sticky: a bounded wait ran out
    unsigned int pad;
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
    SyncState *sync; unsigned long long bar_base; unsigned int spin_limit;
};

// returns false if the wait was abandoned
__device__ __forceinline__ bool grid_barrier(SyncState *s, unsigned long long target, unsigned int spin_limit) {
    __shared__ int ok_sh;
    __syncthreads();
    if (threadIdx.x == 0) {
        __threadfence();
        atomicAdd(&s->arrive, 1ULL);
        unsigned int spins = 0;
        int ok = 1;
        while (__hip_atomic_load(&s->arrive, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < target) {
            __builtin_amdgcn_s_sleep(1);
            ++spins;
            if (spins >= spin_limit ||
                ((spins & 63u) == 0u && __hip_atomic_load(&s->abort, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0u)) {
                ok = 0;
                break;
            }
        }
        if (!ok) __hip_atomic_store(&s->abort, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
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

template <int HD>
__global__ void __launch_bounds__(256) k_decode_persistent(PersistArgs p) {
    extern __shared__ __align__(16) unsigned char smem[];
    const int wg = blockIdx.x, nwg = gridDim.x;
    if (__hip_atomic_load(&p.sync->abort, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0u) {
        if (wg == 0) write_aborted(p.out, p.active);
        return;
    }
    unsigned long long target = p.bar_base;
#define RS_BARRIER()                                                          \
    do {                                                                      \
        target += (unsigned long long)nwg;                                    \
        if (!grid_barrier(p.sync, target, p.spin_limit)) { write_aborted(p.out, p.active); return; } \
    } while (0)

    // ---- row table and embedding
    if (wg == 0) prepare_row(p.prep, 0, reinterpret_cast<int *>(smem));
    RS_BARRIER();

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
    // LM head + single-pass softmax statistics, one partial per workgroup
    g.W = p.lm_head; g.N = p.vocab; g.K = d; g.h_in = h; g.gain = p.final_norm; g.x_in = nullptr;
    g.n_parts = nwg;
    gemv_phase<G_LMHEAD, 8, 1, 2, 1>(g, smem, wg, nwg);
    RS_BARRIER();
    if (wg == 0) route_merge_row(g.parts, nwg, p.vocab, p.tau, p.active, p.seq_bad, p.out, 0, reinterpret_cast<SoftPartial *>(smem));
#undef RS_BARRIER
}

}  // namespace rs
