// C ABI of the stitched-decoding hot path (see include/rstitch.h): argument
// checks, workspace layout, launch sequencing.  All arithmetic of the path runs
// in the kernels included below; the only host arithmetic is the rotary
// cos/sin table, which is input-independent and built once per model.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <new>
#include <vector>

#include "../../include/rstitch.h"
#include "device_utils.h"
#include "router.h"
#include "model_kernels.h"
#include "mrow_kernels.h"

namespace {

thread_local char g_err[512] = "";

rs_status fail(rs_status code, const char *fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}

#define RS_HIP(expr)                                                                         \
    do {                                                                                     \
        hipError_t e_ = (expr);                                                              \
        if (e_ != hipSuccess) return fail(RS_EHIP, "%s: %s", #expr, hipGetErrorString(e_));  \
    } while (0)

#define RS_LAUNCHED(name)                                                                    \
    do {                                                                                     \
        hipError_t e_ = hipGetLastError();                                                   \
        if (e_ != hipSuccess) return fail(RS_EHIP, "launch %s: %s", name, hipGetErrorString(e_)); \
    } while (0)

constexpr size_t ALIGN = 256;
size_t align_up(size_t v) { return (v + ALIGN - 1) / ALIGN * ALIGN; }

const char *check_config(const rs_config *c) {
    if (!c) return "null config";
    if (c->n_layers < 1 || c->d_model < 1 || c->n_q_heads < 1 || c->n_kv_heads < 1) return "non-positive shape";
    if (c->head_dim != 32 && c->head_dim != 64 && c->head_dim != 128) return "head_dim must be 32, 64 or 128";
    if (c->n_q_heads % c->n_kv_heads) return "n_kv_heads must divide n_q_heads";
    if (c->n_q_heads / c->n_kv_heads > rs::ATT_GMAX) return "more than 8 query heads per kv head";
    if (c->d_model % 128 || c->d_ffn % 128 || (c->n_q_heads * c->head_dim) % 128)
        return "d_model, d_ffn and n_q_heads*head_dim must be multiples of 128";
    if (c->d_ffn < 128) return "d_ffn too small";
    if (c->vocab < 2) return "vocab must be at least 2";
    if (c->max_ctx < 1) return "max_ctx must be positive";
    if (c->max_seqs < 1 || c->max_seqs > 8) return "max_seqs must be in 1..8";
    if (c->max_rows < 1 || c->max_rows > 64) return "max_rows must be in 1..64";
    if (!(c->rms_eps > 0.f) || !(c->rope_theta > 1.f)) return "rms_eps must be > 0 and rope_theta > 1";
    if (c->d_model > rs::GEMV_KSEG || c->n_q_heads * c->head_dim > rs::GEMV_KSEG)
        return "d_model and n_q_heads*head_dim must not exceed 12288";
    return nullptr;
}

struct Layout {
    size_t rope_cos, rope_sin, row_slot, row_pos, row_bad, out_row, seq_bad, seq_scale, h, xn, qkv_raw, qbuf,
        attn_out, attn_pl, act, act_pl, attn_part, attn_cnt, lm_pl, lm_parts, total;
    int attn_rows_x_splits;   // capacity of attn_part in (row, split) pairs
    int lm_parts_cap;         // partial states per sequence
};

int attn_pairs_cap(const rs_config &c) { return c.max_rows > 256 ? c.max_rows : 256; }

constexpr int LM_PARTS_CAP = 4096;

Layout make_layout(const rs_config &c) {
    Layout L{};
    size_t o = 0;
    auto take = [&](size_t bytes) { size_t at = o; o = align_up(o + bytes); return at; };
    const size_t half = c.head_dim / 2, qdim = (size_t)c.n_q_heads * c.head_dim;
    const size_t qkv = (size_t)(c.n_q_heads + 2 * c.n_kv_heads) * c.head_dim;
    L.rope_cos = take((size_t)c.max_ctx * half * 4);
    L.rope_sin = take((size_t)c.max_ctx * half * 4);
    L.row_slot = take(c.max_rows * 4);
    L.row_pos = take(c.max_rows * 4);
    L.row_bad = take(c.max_rows * 4);
    L.out_row = take(c.max_seqs * 4);
    L.seq_bad = take(c.max_seqs * 4);
    L.seq_scale = take(c.max_seqs * 4);
    L.h = take((size_t)c.max_rows * c.d_model * 4);
    L.xn = take((size_t)3 * c.max_rows * c.d_model * 2);
    L.qkv_raw = take((size_t)c.max_rows * qkv * 4);
    L.qbuf = take((size_t)c.max_rows * qdim * 4);
    L.attn_out = take((size_t)c.max_rows * qdim * 4);
    L.attn_pl = take((size_t)3 * c.max_rows * qdim * 2);
    L.act = take((size_t)c.d_ffn * 4);
    L.act_pl = take((size_t)3 * c.max_rows * c.d_ffn * 2);
    L.attn_rows_x_splits = attn_pairs_cap(c);
    L.attn_part = take((size_t)L.attn_rows_x_splits * c.n_q_heads * (c.head_dim + 4) * 4);
    L.attn_cnt = take((size_t)c.max_rows * c.n_kv_heads * 4);
    L.lm_pl = take((size_t)3 * c.max_seqs * c.d_model * 2);
    L.lm_parts_cap = LM_PARTS_CAP;
    L.lm_parts = take((size_t)c.max_seqs * L.lm_parts_cap * sizeof(rs::SoftPartial));
    L.total = o;
    return L;
}

}  // namespace

struct rs_model {
    rs_config cfg;
    Layout lay;
    int n_cu;
    const uint16_t *embed, *lm_head, *final_norm;
    std::vector<const uint16_t *> attn_norm, w_qkv, w_o, mlp_norm, w_gate_up, w_down;
    uint16_t *kv_k, *kv_v;
    unsigned char *ws;
    int timer_phase = -1, timer_layer = 0;
    hipEvent_t timer_start = nullptr, timer_stop = nullptr;

    template <typename T> T *at(size_t off) const { return reinterpret_cast<T *>(ws + off); }
};

namespace {

using namespace rs;

int gemv_blocks(int n_units_per_wg_granularity, int n_cu, int per_cu) {
    int cap = n_cu * per_cu;
    return n_units_per_wg_granularity < cap ? (n_units_per_wg_granularity < 1 ? 1 : n_units_per_wg_granularity) : cap;
}

template <int MODE, int RT, int KS>
rs_status launch_gemv(const rs_model *m, GemvArgs &a, int n_tiles, hipStream_t st, const char *name,
                      int *blocks_out = nullptr) {
    const int units = (KS == 1) ? (n_tiles + 3) / 4 : n_tiles;
    const size_t lds = (size_t)(a.K < GEMV_KSEG ? a.K : GEMV_KSEG) * 4;
    const int per_cu = lds > 40 * 1024 ? 2 : 4;
    int blocks = gemv_blocks(units, m->n_cu, per_cu);
    if (a.K > GEMV_KSEG) {                 // x is restaged per tile: one tile per workgroup
        if (KS != 4) return fail(RS_EINVAL, "internal: segmented K needs the split-K launch");
        blocks = units;
    }
    if (MODE == G_LMHEAD && blocks * 4 > LM_PARTS_CAP) blocks = LM_PARTS_CAP / 4;   // one partial per wave
    if (blocks_out) *blocks_out = blocks;
    hipLaunchKernelGGL((k_gemv<MODE, RT, KS>), dim3(blocks), dim3(256), lds, st, a);
    RS_LAUNCHED(name);
    return RS_OK;
}

template <int HD>
rs_status launch_attn(AttnArgs &a, int n_splits, int n_kv, int n_rows, hipStream_t st) {
    hipLaunchKernelGGL((k_attn_decode<HD>), dim3(n_splits, n_kv, n_rows), dim3(256), 0, st, a);
    RS_LAUNCHED("attn_decode");
    return RS_OK;
}

template <int MODE, int NB>
rs_status launch_gemm_nb(GemmArgs &a, int blocks, int nw, hipStream_t st, const char *name) {
    switch (nw) {
        case 1: hipLaunchKernelGGL((k_gemm_rows<MODE, NB, 1>), dim3(blocks), dim3(64), 0, st, a); break;
        case 4: hipLaunchKernelGGL((k_gemm_rows<MODE, NB, 4>), dim3(blocks), dim3(256), 0, st, a); break;
        case 8: hipLaunchKernelGGL((k_gemm_rows<MODE, NB, 8>), dim3(blocks), dim3(512), 0, st, a); break;
        default: hipLaunchKernelGGL((k_gemm_rows<MODE, NB, 16>), dim3(blocks), dim3(1024), 0, st, a); break;
    }
    RS_LAUNCHED(name);
    return RS_OK;
}

// n_tiles = number of 16-column output tiles
template <int MODE>
rs_status launch_gemm(const rs_model *m, GemmArgs &a, int n_tiles, hipStream_t st, const char *name) {
    const int nb = (a.M + 15) / 16;
    const int nt = (MODE == G_GATEUP) ? 2 : 1;
    const int kblocks = a.K / 128;
    // waves per workgroup: enough to put ~2000 waves on the chip, bounded by K and by the LDS
    // used for the cross-wave sum (1 KB per wave, tile and token block)
    int nw = n_tiles >= 512 ? 4 : (n_tiles >= 256 ? 8 : 16);
    while (nw > 1 && (nw > kblocks || nw * nt * nb > 32)) nw >>= 1;
    if (nw == 2) nw = 1;
    int blocks = n_tiles < 2048 ? n_tiles : 2048;
    if (MODE == G_LMHEAD) {
        if (blocks > LM_PARTS_CAP) blocks = LM_PARTS_CAP;                 // one partial per workgroup
        a.n_parts = blocks;
    }
    (void)m;
    if (MODE == G_LMHEAD) return launch_gemm_nb<MODE, 1>(a, blocks, nw, st, name);
    switch (nb) {
        case 1: return launch_gemm_nb<MODE, 1>(a, blocks, nw, st, name);
        case 2: return launch_gemm_nb<MODE, 2>(a, blocks, nw, st, name);
        case 3: return launch_gemm_nb<MODE, 3>(a, blocks, nw, st, name);
        default: return launch_gemm_nb<MODE, 4>(a, blocks, nw, st, name);
    }
}

// One forward invocation over n_rows token rows of n_seqs sequences.
rs_status forward(rs_model *m, int n_seqs, int n_rows, const int *d_seq_slot, const int *d_tokens,
                  const int *d_span_off, const int *d_pos0, const float *d_scale, float tau, int active,
                  rs_route_out *d_out, float *d_logits, hipStream_t st) {
    const rs_config &c = m->cfg;
    const Layout &L = m->lay;
    const int hd = c.head_dim, qdim = c.n_q_heads * hd, qkv_rows = (c.n_q_heads + 2 * c.n_kv_heads) * hd;
    int *row_slot = m->at<int>(L.row_slot), *row_pos = m->at<int>(L.row_pos), *row_bad = m->at<int>(L.row_bad);
    float *h = m->at<float>(L.h);

    PrepArgs pa{};
    pa.n_seqs = n_seqs; pa.n_rows = n_rows; pa.d_model = c.d_model; pa.vocab = c.vocab;
    pa.max_ctx = c.max_ctx; pa.max_seqs = c.max_seqs;
    pa.seq_slot = d_seq_slot; pa.tokens = d_tokens; pa.span_off = d_span_off; pa.pos0 = d_pos0; pa.scale = d_scale;
    pa.embed = m->embed;
    pa.row_slot = row_slot; pa.row_pos = row_pos; pa.row_bad = row_bad;
    pa.out_row = m->at<int>(L.out_row); pa.seq_bad = m->at<int>(L.seq_bad); pa.seq_scale = m->at<float>(L.seq_scale);
    pa.h = h;
    hipLaunchKernelGGL(k_prepare, dim3(n_rows), dim3(256), 0, st, pa);
    RS_LAUNCHED("prepare");

    // attention launch shape
    const int att_ts = 16384 / c.head_dim;                 // tokens one attention workgroup takes per round trip
    int n_splits = (c.max_ctx + att_ts - 1) / att_ts;
    if (n_splits > ATT_SMAX) n_splits = ATT_SMAX;
    if (n_splits * n_rows > L.attn_rows_x_splits) n_splits = L.attn_rows_x_splits / n_rows;
    if (n_splits < 1) n_splits = 1;

    const bool single = (n_rows == 1);
    rs_status rc;
    // optional event pair around one chosen kernel (rs_set_phase_timer)
    auto tic = [&](int phase, int layer) {
        if (m->timer_phase == phase && (phase == RS_PHASE_LMHEAD || m->timer_layer == layer)) (void)hipEventRecord(m->timer_start, st);
    };
    auto toc = [&](int phase, int layer) {
        if (m->timer_phase == phase && (phase == RS_PHASE_LMHEAD || m->timer_layer == layer)) (void)hipEventRecord(m->timer_stop, st);
    };
    for (int l = 0; l < c.n_layers; ++l) {
        AttnArgs aa{};
        aa.qbuf = m->at<float>(L.qbuf); aa.kcache = m->kv_k; aa.vcache = m->kv_v;
        aa.partials = m->at<float>(L.attn_part); aa.counters = m->at<int>(L.attn_cnt);
        aa.out = m->at<float>(L.attn_out);
        aa.out_planes = single ? nullptr : m->at<uint16_t>(L.attn_pl);
        aa.out_plane = (size_t)c.max_rows * qdim;
        aa.row_pos = row_pos; aa.row_slot = row_slot; aa.row_bad = row_bad;
        aa.n_q = c.n_q_heads; aa.n_kv = c.n_kv_heads; aa.max_ctx = c.max_ctx; aa.max_seqs = c.max_seqs; aa.layer = l;

        if (single) {
            GemvArgs g{};
            g.eps = c.rms_eps; g.n_q = c.n_q_heads; g.n_kv = c.n_kv_heads; g.head_dim = hd; g.max_ctx = c.max_ctx;
            g.max_seqs = c.max_seqs; g.layer = l; g.d_ffn = c.d_ffn;
            g.row_pos = row_pos; g.row_slot = row_slot; g.row_bad = row_bad;
            g.rope_cos = m->at<float>(L.rope_cos); g.rope_sin = m->at<float>(L.rope_sin);
            g.qbuf = m->at<float>(L.qbuf); g.kcache = m->kv_k; g.vcache = m->kv_v;
            g.act = m->at<float>(L.act); g.h_out = h;

            // QKV (+ RMSNorm, RoPE, KV write)
            g.W = m->w_qkv[l]; g.N = qkv_rows; g.K = c.d_model; g.h_in = h; g.gain = m->attn_norm[l]; g.x_in = nullptr;
            tic(RS_PHASE_QKV, l);
            if (qkv_rows <= 4096) {
                const int tiles = (c.n_q_heads + c.n_kv_heads) * (hd / 2) + (c.n_kv_heads * hd) / 2;
                rc = launch_gemv<G_QKV, 2, 1>(m, g, tiles, st, "gemv_qkv");
            } else {
                const int tiles = (c.n_q_heads + c.n_kv_heads) * (hd / 4) + (c.n_kv_heads * hd) / 4;
                rc = launch_gemv<G_QKV, 4, 1>(m, g, tiles, st, "gemv_qkv");
            }
            toc(RS_PHASE_QKV, l);
            if (rc) return rc;
            // attention
            tic(RS_PHASE_ATTN, l);
            switch (hd) {
                case 32: rc = launch_attn<32>(aa, n_splits, c.n_kv_heads, 1, st); break;
                case 64: rc = launch_attn<64>(aa, n_splits, c.n_kv_heads, 1, st); break;
                default: rc = launch_attn<128>(aa, n_splits, c.n_kv_heads, 1, st); break;
            }
            toc(RS_PHASE_ATTN, l);
            if (rc) return rc;
            // O projection + residual
            g.W = m->w_o[l]; g.N = c.d_model; g.K = qdim; g.h_in = nullptr; g.gain = nullptr;
            g.x_in = m->at<float>(L.attn_out);
            tic(RS_PHASE_OPROJ, l);
            if (c.d_model <= 2048) rc = launch_gemv<G_OPROJ, 2, 1>(m, g, (c.d_model + 1) / 2, st, "gemv_oproj");
            else rc = launch_gemv<G_OPROJ, 4, 1>(m, g, (c.d_model + 3) / 4, st, "gemv_oproj");
            toc(RS_PHASE_OPROJ, l);
            if (rc) return rc;
            // gate/up (+ RMSNorm, SwiGLU)
            g.W = m->w_gate_up[l]; g.N = 2 * c.d_ffn; g.K = c.d_model; g.h_in = h; g.gain = m->mlp_norm[l]; g.x_in = nullptr;
            tic(RS_PHASE_GATEUP, l);
            rc = launch_gemv<G_GATEUP, 4, 1>(m, g, c.d_ffn / 2, st, "gemv_gateup");
            toc(RS_PHASE_GATEUP, l);
            if (rc) return rc;
            // down + residual
            g.W = m->w_down[l]; g.N = c.d_model; g.K = c.d_ffn; g.h_in = nullptr; g.gain = nullptr;
            g.x_in = m->at<float>(L.act);
            tic(RS_PHASE_DOWN, l);
            if (c.d_ffn > GEMV_KSEG) rc = launch_gemv<G_DOWN, 8, 4>(m, g, (c.d_model + 7) / 8, st, "gemv_down");
            else if (c.d_model <= 2048) rc = launch_gemv<G_DOWN, 2, 4>(m, g, (c.d_model + 1) / 2, st, "gemv_down");
            else rc = launch_gemv<G_DOWN, 4, 4>(m, g, (c.d_model + 3) / 4, st, "gemv_down");
            toc(RS_PHASE_DOWN, l);
            if (rc) return rc;
        } else {
            uint16_t *xn = m->at<uint16_t>(L.xn);
            const size_t xn_plane = (size_t)c.max_rows * c.d_model;
            GemmArgs g{};
            g.M = n_rows; g.d_ffn = c.d_ffn;
            hipLaunchKernelGGL(k_rmsnorm_rows, dim3(n_rows), dim3(256), 0, st, (const float *)h, m->attn_norm[l], c.rms_eps,
                               c.d_model, (const int *)nullptr, xn, xn_plane);
            RS_LAUNCHED("rmsnorm_rows");
            g.W = m->w_qkv[l]; g.N = qkv_rows; g.K = c.d_model; g.X = xn; g.x_plane = xn_plane;
            g.out_f32 = m->at<float>(L.qkv_raw); g.ld_out = qkv_rows;
            tic(RS_PHASE_QKV, l);
            if ((rc = launch_gemm<G_QKV>(m, g, (qkv_rows + 15) / 16, st, "gemm_qkv"))) return rc;
            toc(RS_PHASE_QKV, l);
            RopeArgs ra{};
            ra.qkv = m->at<float>(L.qkv_raw); ra.qbuf = m->at<float>(L.qbuf); ra.kcache = m->kv_k; ra.vcache = m->kv_v;
            ra.rope_cos = m->at<float>(L.rope_cos); ra.rope_sin = m->at<float>(L.rope_sin);
            ra.row_pos = row_pos; ra.row_slot = row_slot; ra.row_bad = row_bad;
            ra.n_q = c.n_q_heads; ra.n_kv = c.n_kv_heads; ra.head_dim = hd; ra.max_ctx = c.max_ctx;
            ra.max_seqs = c.max_seqs; ra.layer = l;
            hipLaunchKernelGGL(k_rope_kv_rows, dim3(n_rows), dim3(256), 0, st, ra);
            RS_LAUNCHED("rope_kv_rows");
            tic(RS_PHASE_ATTN, l);
            switch (hd) {
                case 32: rc = launch_attn<32>(aa, n_splits, c.n_kv_heads, n_rows, st); break;
                case 64: rc = launch_attn<64>(aa, n_splits, c.n_kv_heads, n_rows, st); break;
                default: rc = launch_attn<128>(aa, n_splits, c.n_kv_heads, n_rows, st); break;
            }
            toc(RS_PHASE_ATTN, l);
            if (rc) return rc;
            g.W = m->w_o[l]; g.N = c.d_model; g.K = qdim;
            g.X = m->at<uint16_t>(L.attn_pl); g.x_plane = (size_t)c.max_rows * qdim;
            g.h_out = h; g.ld_h = c.d_model;
            tic(RS_PHASE_OPROJ, l);
            if ((rc = launch_gemm<G_OPROJ>(m, g, (c.d_model + 15) / 16, st, "gemm_oproj"))) return rc;
            toc(RS_PHASE_OPROJ, l);
            hipLaunchKernelGGL(k_rmsnorm_rows, dim3(n_rows), dim3(256), 0, st, (const float *)h, m->mlp_norm[l], c.rms_eps,
                               c.d_model, (const int *)nullptr, xn, xn_plane);
            RS_LAUNCHED("rmsnorm_rows");
            g.W = m->w_gate_up[l]; g.N = 2 * c.d_ffn; g.K = c.d_model; g.X = xn; g.x_plane = xn_plane;
            g.act = m->at<uint16_t>(L.act_pl); g.act_plane = (size_t)c.max_rows * c.d_ffn;
            tic(RS_PHASE_GATEUP, l);
            if ((rc = launch_gemm<G_GATEUP>(m, g, (c.d_ffn + 15) / 16, st, "gemm_gateup"))) return rc;
            toc(RS_PHASE_GATEUP, l);
            g.W = m->w_down[l]; g.N = c.d_model; g.K = c.d_ffn;
            g.X = m->at<uint16_t>(L.act_pl); g.x_plane = (size_t)c.max_rows * c.d_ffn;
            tic(RS_PHASE_DOWN, l);
            if ((rc = launch_gemm<G_DOWN>(m, g, (c.d_model + 15) / 16, st, "gemm_down"))) return rc;
            toc(RS_PHASE_DOWN, l);
        }
    }

    // LM head + single-pass softmax statistics
    SoftPartial *parts = m->at<SoftPartial>(L.lm_parts);
    int n_parts;
    if (single) {
        GemvArgs g{};
        g.eps = c.rms_eps; g.W = m->lm_head; g.N = c.vocab; g.K = c.d_model; g.h_in = h; g.gain = m->final_norm;
        g.seq_scale = m->at<float>(L.seq_scale); g.parts = parts; g.logits = d_logits;
        int blocks = 0;
        tic(RS_PHASE_LMHEAD, 0);
        if ((rc = launch_gemv<G_LMHEAD, 8, 1>(m, g, (c.vocab + 7) / 8, st, "gemv_lmhead", &blocks))) return rc;
        toc(RS_PHASE_LMHEAD, 0);
        n_parts = blocks * 4;
    } else {
        uint16_t *lm_pl = m->at<uint16_t>(L.lm_pl);
        const size_t lm_plane = (size_t)c.max_seqs * c.d_model;
        hipLaunchKernelGGL(k_rmsnorm_rows, dim3(n_seqs), dim3(256), 0, st, (const float *)h, m->final_norm, c.rms_eps,
                           c.d_model, (const int *)m->at<int>(L.out_row), lm_pl, lm_plane);
        RS_LAUNCHED("rmsnorm_rows");
        GemmArgs g{};
        g.M = n_seqs; g.W = m->lm_head; g.N = c.vocab; g.K = c.d_model; g.X = lm_pl; g.x_plane = lm_plane;
        g.seq_scale = m->at<float>(L.seq_scale); g.parts = parts; g.logits = d_logits;
        tic(RS_PHASE_LMHEAD, 0);
        if ((rc = launch_gemm<G_LMHEAD>(m, g, (c.vocab + 15) / 16, st, "gemm_lmhead"))) return rc;
        toc(RS_PHASE_LMHEAD, 0);
        n_parts = g.n_parts;
    }
    if (n_parts > L.lm_parts_cap) return fail(RS_EINVAL, "internal: %d router partials exceed capacity", n_parts);
    hipLaunchKernelGGL(k_route_merge, dim3(n_seqs), dim3(256), 0, st, (const SoftPartial *)parts, n_parts, c.vocab, tau,
                       active, (const int *)m->at<int>(L.seq_bad), d_out);
    RS_LAUNCHED("route_merge");
    return RS_OK;
}

}  // namespace

// ================================================================================================
extern "C" {

const char *rs_last_error(void) { return g_err; }

int32_t rs_abi_version(void) { return 1; }

size_t rs_workspace_bytes(const rs_config *cfg) {
    if (const char *why = check_config(cfg)) { fail(RS_EINVAL, "%s", why); return 0; }
    return make_layout(*cfg).total;
}

size_t rs_kv_bytes(const rs_config *cfg) {
    if (const char *why = check_config(cfg)) { fail(RS_EINVAL, "%s", why); return 0; }
    return (size_t)cfg->n_layers * cfg->max_seqs * cfg->n_kv_heads * cfg->max_ctx * cfg->head_dim * 2;
}

rs_status rs_create_model(const rs_config *cfg, const rs_weights *w, void *kv_k, void *kv_v, void *workspace,
                          size_t workspace_bytes, rs_model **out) {
    if (!out) return fail(RS_EINVAL, "null output handle");
    *out = nullptr;
    if (const char *why = check_config(cfg)) return fail(RS_EINVAL, "%s", why);
    if (!w || !w->embed || !w->lm_head || !w->final_norm || !w->attn_norm || !w->w_qkv || !w->w_o || !w->mlp_norm ||
        !w->w_gate_up || !w->w_down)
        return fail(RS_EINVAL, "null weight pointer");
    if (!kv_k || !kv_v || !workspace) return fail(RS_EINVAL, "null KV or workspace pointer");
    if (((uintptr_t)kv_k | (uintptr_t)kv_v | (uintptr_t)workspace) % ALIGN) return fail(RS_EINVAL, "KV/workspace must be 256-byte aligned");
    const Layout L = make_layout(*cfg);
    if (workspace_bytes < L.total) return fail(RS_EINVAL, "workspace of %zu bytes is smaller than the %zu needed", workspace_bytes, L.total);
    for (int l = 0; l < cfg->n_layers; ++l)
        if (!w->attn_norm[l] || !w->w_qkv[l] || !w->w_o[l] || !w->mlp_norm[l] || !w->w_gate_up[l] || !w->w_down[l])
            return fail(RS_EINVAL, "null weight pointer in layer %d", l);
    const void *ptrs[] = {w->embed, w->lm_head, w->final_norm};
    for (const void *p : ptrs)
        if ((uintptr_t)p % 16) return fail(RS_EINVAL, "weight tensors must be 16-byte aligned");
    for (int l = 0; l < cfg->n_layers; ++l) {
        const void *lp[] = {w->attn_norm[l], w->w_qkv[l], w->w_o[l], w->mlp_norm[l], w->w_gate_up[l], w->w_down[l]};
        for (const void *p : lp)
            if ((uintptr_t)p % 16) return fail(RS_EINVAL, "weight tensors must be 16-byte aligned (layer %d)", l);
    }

    rs_model *m = new (std::nothrow) rs_model();
    if (!m) return fail(RS_EINVAL, "out of host memory");
    m->cfg = *cfg; m->lay = L;
    m->embed = (const uint16_t *)w->embed; m->lm_head = (const uint16_t *)w->lm_head; m->final_norm = (const uint16_t *)w->final_norm;
    for (int l = 0; l < cfg->n_layers; ++l) {
        m->attn_norm.push_back((const uint16_t *)w->attn_norm[l]); m->w_qkv.push_back((const uint16_t *)w->w_qkv[l]);
        m->w_o.push_back((const uint16_t *)w->w_o[l]); m->mlp_norm.push_back((const uint16_t *)w->mlp_norm[l]);
        m->w_gate_up.push_back((const uint16_t *)w->w_gate_up[l]); m->w_down.push_back((const uint16_t *)w->w_down[l]);
    }
    m->kv_k = (uint16_t *)kv_k; m->kv_v = (uint16_t *)kv_v; m->ws = (unsigned char *)workspace;

    int dev = 0;
    hipDeviceProp_t prop;
    hipError_t e = hipGetDevice(&dev);
    if (e == hipSuccess) e = hipGetDeviceProperties(&prop, dev);
    if (e != hipSuccess) { delete m; return fail(RS_EHIP, "device query: %s", hipGetErrorString(e)); }
    m->n_cu = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;

    // rotary table: angle(pos, i) = pos * theta^(-2 i / head_dim), evaluated in double
    const int half = cfg->head_dim / 2;
    std::vector<float> cs((size_t)cfg->max_ctx * half), sn((size_t)cfg->max_ctx * half);
    std::vector<double> inv_freq(half);
    for (int i = 0; i < half; ++i) inv_freq[i] = std::pow((double)cfg->rope_theta, -2.0 * i / cfg->head_dim);
    for (int p = 0; p < cfg->max_ctx; ++p)
        for (int i = 0; i < half; ++i) {
            const double ang = (double)p * inv_freq[i];
            cs[(size_t)p * half + i] = (float)std::cos(ang);
            sn[(size_t)p * half + i] = (float)std::sin(ang);
        }
    e = hipMemcpy(m->ws + L.rope_cos, cs.data(), cs.size() * 4, hipMemcpyHostToDevice);
    if (e == hipSuccess) e = hipMemcpy(m->ws + L.rope_sin, sn.data(), sn.size() * 4, hipMemcpyHostToDevice);
    if (e == hipSuccess) e = hipMemset(m->ws + L.attn_cnt, 0, (size_t)cfg->max_rows * cfg->n_kv_heads * 4);
    if (e == hipSuccess) e = hipDeviceSynchronize();
    if (e != hipSuccess) { delete m; return fail(RS_EHIP, "workspace initialisation: %s", hipGetErrorString(e)); }
    *out = m;
    return RS_OK;
}

rs_status rs_destroy_model(rs_model *model) {
    delete model;
    return RS_OK;
}

rs_status rs_decode_step(rs_model *m, int32_t n_seqs, const int32_t *d_seq_slot, const int32_t *d_token,
                         const int32_t *d_pos, const float *d_logit_scale, float tau, int32_t active,
                         rs_route_out *d_out, float *d_logits, void *stream) {
    if (!m) return fail(RS_EINVAL, "null model");
    if (!d_seq_slot || !d_token || !d_pos || !d_out) return fail(RS_EINVAL, "null argument");
    if (n_seqs < 1) return fail(RS_EINVAL, "n_seqs must be at least 1");
    if (n_seqs > m->cfg.max_seqs || n_seqs > m->cfg.max_rows)
        return fail(RS_ECAPACITY, "n_seqs %d exceeds max_seqs %d / max_rows %d", n_seqs, m->cfg.max_seqs, m->cfg.max_rows);
    if (active != RS_SLM && active != RS_LLM) return fail(RS_EINVAL, "active must be RS_SLM or RS_LLM");
    return forward(m, n_seqs, n_seqs, d_seq_slot, d_token, nullptr, d_pos, d_logit_scale, tau, active, d_out, d_logits,
                   (hipStream_t)stream);
}

rs_status rs_catchup_prefill(rs_model *m, int32_t n_seqs, int32_t n_rows, const int32_t *d_seq_slot,
                             const int32_t *d_tokens, const int32_t *d_span_offset, const int32_t *d_pos0,
                             const float *d_logit_scale, float tau, int32_t active, rs_route_out *d_out,
                             float *d_logits, void *stream) {
    if (!m) return fail(RS_EINVAL, "null model");
    if (!d_seq_slot || !d_tokens || !d_span_offset || !d_pos0 || !d_out) return fail(RS_EINVAL, "null argument");
    if (n_seqs < 1 || n_rows < n_seqs) return fail(RS_EINVAL, "need n_seqs >= 1 and at least one row per sequence");
    if (n_seqs > m->cfg.max_seqs) return fail(RS_ECAPACITY, "n_seqs %d exceeds max_seqs %d", n_seqs, m->cfg.max_seqs);
    if (n_rows > m->cfg.max_rows) return fail(RS_ECAPACITY, "n_rows %d exceeds max_rows %d", n_rows, m->cfg.max_rows);
    if (active != RS_SLM && active != RS_LLM) return fail(RS_EINVAL, "active must be RS_SLM or RS_LLM");
    return forward(m, n_seqs, n_rows, d_seq_slot, d_tokens, d_span_offset, d_pos0, d_logit_scale, tau, active, d_out,
                   d_logits, (hipStream_t)stream);
}

rs_status rs_set_phase_timer(rs_model *m, int32_t phase, int32_t layer, void *start_event, void *stop_event) {
    if (!m) return fail(RS_EINVAL, "null model");
    if (phase < 0) { m->timer_phase = -1; m->timer_start = m->timer_stop = nullptr; return RS_OK; }
    if (phase > RS_PHASE_ATTN) return fail(RS_EINVAL, "unknown phase %d", phase);
    if (!start_event || !stop_event) return fail(RS_EINVAL, "null event");
    if (phase != RS_PHASE_LMHEAD && (layer < 0 || layer >= m->cfg.n_layers)) return fail(RS_EINVAL, "layer %d out of range", layer);
    m->timer_phase = phase; m->timer_layer = layer;
    m->timer_start = (hipEvent_t)start_event; m->timer_stop = (hipEvent_t)stop_event;
    return RS_OK;
}

static int route_parts(int vocab) {
    int p = (vocab / 4 + 255) / 256;      // one float4 per thread and pass
    if (p < 1) p = 1;
    return p > 128 ? 128 : p;
}

size_t rs_route_scratch_bytes(int32_t n, int32_t vocab) {
    if (n < 1 || vocab < 2) { fail(RS_EINVAL, "need n >= 1 and vocab >= 2"); return 0; }
    return align_up((size_t)n * route_parts(vocab) * sizeof(rs::SoftPartial));
}

rs_status rs_route(const float *d_logits, int32_t n, int32_t vocab, const float *d_logit_scale, float tau,
                   int32_t active, rs_route_out *d_out, void *d_scratch, size_t scratch_bytes, void *stream) {
    if (n < 1 || n > 65535) return fail(RS_EINVAL, "n must be in 1..65535");
    if (vocab < 2) return fail(RS_EINVAL, "vocab must be at least 2");
    if (!d_logits || !d_out || !d_scratch) return fail(RS_EINVAL, "null argument");
    if (active != RS_SLM && active != RS_LLM) return fail(RS_EINVAL, "active must be RS_SLM or RS_LLM");
    if ((uintptr_t)d_scratch % 16 || (uintptr_t)d_logits % 16) return fail(RS_EINVAL, "logits and scratch must be 16-byte aligned");
    const size_t need = rs_route_scratch_bytes(n, vocab);
    if (scratch_bytes < need) return fail(RS_EINVAL, "scratch of %zu bytes is smaller than the %zu needed", scratch_bytes, need);
    const int parts = route_parts(vocab);
    hipStream_t st = (hipStream_t)stream;
    hipLaunchKernelGGL(rs::k_route_partials, dim3(parts, n), dim3(256), 0, st, d_logits, vocab, d_logit_scale,
                       (rs::SoftPartial *)d_scratch);
    RS_LAUNCHED("route_partials");
    hipLaunchKernelGGL(rs::k_route_merge, dim3(n), dim3(256), 0, st, (const rs::SoftPartial *)d_scratch, parts, vocab, tau,
                       active, (const int *)nullptr, d_out);
    RS_LAUNCHED("route_merge");
    return RS_OK;
}

}  // extern "C"
