// C ABI of the stitched-decoding hot path (see include/rstitch.h): argument
// checks, workspace layout, launch sequencing.  All arithmetic of the path runs
// in the kernels included below; the only host arithmetic is the rotary
// cos/sin table, which is input-independent and built once per model.
#include <hip/hip_runtime.h>

#include <atomic>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

#include "../../include/rstitch.h"
#include "../../include/rstitch_aids.h"
#include "device_utils.h"
#include "router.h"
#include "model_kernels.h"
#include "mrow_kernels.h"
#include "persistent.h"

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
    if (c->max_ctx < 8 || c->max_ctx % 8) return "max_ctx must be a positive multiple of 8";
    if (c->max_seqs < 1 || c->max_seqs > rs::MAX_SEQS) return "max_seqs must be in 1..128";
    if (c->max_rows < 1 || c->max_rows > rs::MAX_ROWS) return "max_rows must be in 1..128";
    if (!(c->rms_eps > 0.f) || !(c->rope_theta > 1.f)) return "rms_eps must be > 0 and rope_theta > 1";
    if (c->d_model > 12288 || c->n_q_heads * c->head_dim > 12288)
        return "d_model and n_q_heads*head_dim must not exceed 12288";
    return nullptr;
}

struct Layout {
    size_t rope_cos, rope_sin, row_slot, row_pos, row_bad, out_row, seq_bad, seq_scale, seq_info, h, qkv_raw, qbuf,
        attn_out, act, attn_part, attn_cnt, lm_parts, sync, layer_ptrs, gemm_part, xn32, lm32, total;
    int attn_rows_x_splits;   // capacity of attn_part in (row, split) pairs
    int lm_parts_cap;         // partial states per sequence
};

struct GemvPlan {
    int qkv_rt, qkv_blocks, o_rt, o_blocks, gu_blocks, down_rt, down_blocks, lm_blocks;
    bool o_all_early;     // O-proj of a mid-sized matrix: every chunk of a wave's first tile requested before the prologue
    bool gu_early;      // gate/up single-row kernel with the early weight request
};

// (row, context slice) pairs the attention partial buffer holds: every row of a full call may use
// slices of one 64-position pass, up to 72 of them (short dependent chains matter more than the
// buffer: 528 bytes per pair and query head)
int attn_pairs_cap(const rs_config &c) {
    int slices = (c.max_ctx + 63) / 64;
    if (slices > 72) slices = 72;
    const int want = c.max_rows * slices;
    return want > 512 ? want : 512;
}

constexpr int LM_PARTS_CAP = 4096;                  // multiple of 8
constexpr int FMA_MAX_ROWS = 4;                     // calls of up to this many token rows run on the FMA GEMV kernels
constexpr int GEMM_KSPLIT_MAX = rs::KSPLIT_MAX;     // workgroup-level K splits of the multi-row projections, at most

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
    L.seq_info = take((size_t)c.max_seqs * 16);
    L.h = take((size_t)c.max_rows * c.d_model * 4);
    L.qkv_raw = take((size_t)c.max_rows * qkv * 4);
    L.qbuf = take((size_t)c.max_rows * qdim * 4);
    L.attn_out = take((size_t)c.max_rows * qdim * 4);
    L.act = take((size_t)c.max_rows * c.d_ffn * 4);                               // fp32 SwiGLU rows
    L.attn_rows_x_splits = attn_pairs_cap(c);
    L.attn_part = take((size_t)L.attn_rows_x_splits * c.n_q_heads * (c.head_dim + 4) * 4);
    L.attn_cnt = take((size_t)c.max_rows * c.n_kv_heads * 4);
    L.lm_parts_cap = LM_PARTS_CAP;
    L.lm_parts = take((size_t)c.max_seqs * L.lm_parts_cap * sizeof(rs::SoftPartial));
    L.gemm_part = take((size_t)GEMM_KSPLIT_MAX * c.max_rows * (qkv > (size_t)c.d_model ? qkv : (size_t)c.d_model) * 4);
    L.xn32 = take((size_t)c.max_rows * c.d_model * 4);                            // normalised rows of a multi-row call (fp32)
    L.lm32 = take((size_t)c.max_seqs * c.d_model * 4);                            // normalised last rows for the LM head
    L.sync = take(2 * sizeof(rs::SyncState));          // [0] single-kernel step, [1] device-resident loop
    L.layer_ptrs = take((size_t)c.n_layers * sizeof(rs::LayerPtrs));
    L.total = o;
    return L;
}

}  // namespace

struct rs_model {
    rs_config cfg;
    Layout lay;
    int n_cu;
    int device = 0;                               // ordinal the model was created on
    const uint16_t *embed, *lm_head, *final_norm;
    std::vector<const uint16_t *> attn_norm, w_qkv, w_o, mlp_norm, w_gate_up, w_down;
    uint16_t *kv_k, *kv_v;
    unsigned char *ws;
    int timer_phase = -1, timer_layer = 0;
    hipEvent_t timer_start = nullptr, timer_stop = nullptr;
    GemvPlan plan{};
    // replayable launch sequences, one per distinct call signature (see forward())
    struct GraphEntry {
        int n_seqs, n_rows, active; float tau;
        const void *slot, *tok, *off, *pos, *scale, *out, *logits; hipStream_t st;
        hipGraph_t graph; hipGraphExec_t exec;
        unsigned long long last_used;
    };
    unsigned long long graph_clock = 0;
    std::vector<GraphEntry> graphs;
    std::vector<size_t> seen_once;                 // signatures launched eagerly once (ring buffer)
    size_t seen_next = 0;
    bool use_graphs = true;
    int sample_on = 0;                             // rs_set_sampling
    unsigned long long sample_key = 0;
    // single-kernel decode step (experimental: slower than one kernel per phase on MI355X, where a
    // grid-wide software barrier costs more than a kernel boundary)
    bool use_persistent = false;
    int persist_blocks = 0;
    size_t persist_lds = 0;
    unsigned long long barriers_done = 0;         // grid barriers of all single-kernel steps so far
    unsigned int spin_limit = 1u << 22;

    template <typename T> T *at(size_t off) const { return reinterpret_cast<T *>(ws + off); }
};

namespace {

using namespace rs;

int clamp_blocks(int want, int n_tiles_per_wg_unit) {
    if (want > n_tiles_per_wg_unit) want = n_tiles_per_wg_unit;
    return want < 1 ? 1 : want;
}

// `blocks` workgroups share the phase; every workgroup takes a contiguous range of tiles
template <int MODE, int RT, int KS, int UNR, int MP, int PRE = 0>
rs_status launch_gemv_mp(GemvArgs &a, int blocks, hipStream_t st, const char *name) {
    const size_t lds = gemv_lds_bytes<MP>(a.K);
    if (lds > 64 * 1024) {
        static std::atomic<bool> raised{false};           // per instantiation; setting the attribute twice is harmless
        if (!raised) {
            hipError_t e = hipFuncSetAttribute((const void *)k_gemv<MODE, RT, KS, UNR, MP, PRE>,
                                               hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024 - 4096);
            if (e != hipSuccess) return fail(RS_EHIP, "raising the LDS limit of %s: %s", name, hipGetErrorString(e));
            raised = true;
        }
    }
    if (gemv_seg<MP>(a.K) != a.K && KS != 4) return fail(RS_EINVAL, "internal: segmented K needs the split-K launch");
    hipLaunchKernelGGL((k_gemv<MODE, RT, KS, UNR, MP, PRE>), dim3(blocks), dim3(256), lds, st, a);
    RS_LAUNCHED(name);
    return RS_OK;
}


// register-resident x (k_gemv_reg): K must be 512 * NCH with NCH one of 3, 7, 10 (d_model 1536, 3584, 5120);
// MP token rows need MP * K / 64 registers per lane for x, so MP * NCH stays at or below 14
template <int MODE, int RT, int MP = 1>
rs_status launch_gemv_reg(GemvArgs &a, int blocks, hipStream_t st, const char *name) {
    if (a.K == 1536) hipLaunchKernelGGL((k_gemv_reg<MODE, RT, 3, 3, MP>), dim3(blocks), dim3(256), 0, st, a);
    else if (a.K == 3584 && MP <= 2) {
        if constexpr (MP <= 2) hipLaunchKernelGGL((k_gemv_reg<MODE, RT, 7, (RT >= 8 ? 2 : 4), MP>), dim3(blocks), dim3(256), 0, st, a);
    } else if (a.K == 5120 && MP == 1) {
        if constexpr (MP == 1) hipLaunchKernelGGL((k_gemv_reg<MODE, RT, 10, (RT >= 8 ? 2 : 5), MP>), dim3(blocks), dim3(256), 0, st, a);
    } else return fail(RS_EINVAL, "internal: %s with K = %d and %d rows", name, a.K, MP);
    RS_LAUNCHED(name);
    return RS_OK;
}
inline bool reg_fits(int K, int mp) { return (K == 1536 && mp <= 4) || (K == 3584 && mp <= 2) || (K == 5120 && mp == 1); }

// Launch shapes from sweeps on MI355X: about three workgroups per CU for matrices under ~128 MB,
// two above; the down projection gets one tile per workgroup.
GemvPlan make_plan(const rs_config &c, int n_cu) {
    GemvPlan p{};
    const int hd = c.head_dim, qkv_rows = (c.n_q_heads + 2 * c.n_kv_heads) * hd;
    auto pick = [&](size_t bytes) { return bytes >= ((size_t)128 << 20) ? 2 * n_cu : 3 * n_cu; };
    // QKV: two rows per wave tile; a large matrix (14B/32B shapes: 73 MB) takes four rows (two rotary pairs) with
    // three early weight chunks at two workgroups per CU.  A small matrix (1.5B shape: 6 MB) runs best with one
    // workgroup per CU (5.8 us against 6.4 us with three).
    const size_t qkv_bytes = (size_t)qkv_rows * c.d_model * 2;
    p.qkv_rt = qkv_bytes >= ((size_t)64 << 20) ? 4 : 2;
    const int qkv_tiles = (c.n_q_heads + c.n_kv_heads) * (hd / p.qkv_rt) + (c.n_kv_heads * hd) / p.qkv_rt;
    p.qkv_blocks = clamp_blocks(p.qkv_rt == 4 ? 2 * n_cu : qkv_bytes < ((size_t)16 << 20) ? n_cu : pick(qkv_bytes), (qkv_tiles + 3) / 4);
    p.o_rt = 2;
    p.o_blocks = clamp_blocks(pick((size_t)c.d_model * c.n_q_heads * hd * 2), ((c.d_model + 1) / 2 + 3) / 4);
    p.gu_early = (size_t)2 * c.d_ffn * c.d_model * 2 >= ((size_t)128 << 20);
    // gate/up: large matrices take two gate/up pairs per wave tile at two workgroups per CU; small ones one pair
    // per tile and two tiles per wave (1.5B shape: 1120 workgroups), 1.5B decode step -2.5 % against four-row
    // tiles at three workgroups per CU
    p.gu_blocks = p.gu_early ? clamp_blocks(pick((size_t)2 * c.d_ffn * c.d_model * 2), (c.d_ffn / 2 + 3) / 4)
                             : clamp_blocks((c.d_ffn + 7) / 8, (c.d_ffn + 3) / 4);
    const size_t o_bytes = (size_t)c.d_model * c.n_q_heads * hd * 2;
    p.o_all_early = o_bytes >= ((size_t)16 << 20) && o_bytes < ((size_t)40 << 20) && c.n_q_heads * hd <= 3584;
    if (p.o_all_early) p.o_blocks = clamp_blocks(2 * n_cu, ((c.d_model + 1) / 2 + 3) / 4);
    // down (k_down_direct): rows per tile by width, see the launch
    p.down_rt = c.d_model <= 2048 ? 2 : (c.d_model <= 4096 ? 7 : 5);
    p.down_blocks = clamp_blocks((c.d_model <= 2048 ? 3 : 4) * n_cu, (c.d_model + p.down_rt - 1) / p.down_rt);
    p.lm_blocks = clamp_blocks(4 * n_cu, ((c.vocab + 7) / 8 + 3) / 4);
    if (p.lm_blocks > LM_PARTS_CAP) p.lm_blocks = LM_PARTS_CAP;
    return p;
}

template <int HD>
rs_status launch_attn(AttnArgs &a, int n_splits, int n_kv, int n_rows, int n_seqs, int n_cu, hipStream_t st) {
    const bool spans = n_rows > n_seqs;
    a.n_slices = n_splits;
    a.n_rows = n_rows;
    if (spans) {
        // several rows per sequence: rows share K/V tiles through the columns of the matrix-core tiles
        // one wave per row slot (rp rows); the kernel needs most of a SIMD's registers, so a workgroup brings
        // only as many waves as it has slots (up to four): with idle waves in it, a CU held one workgroup at a
        // time and a two-row call on eight KV heads at 5000 positions took 17.5 us instead of ~7
        const int rp = 16 / (a.n_q / n_kv);
        const long base = (long)n_splits * n_kv * n_seqs;
        if (n_splits * ATT_BT >= a.max_ctx && (n_rows >= 5 || base <= n_cu)) {
            // every slice is one 64-position pass: one workgroup per (slice, KV head, sequence), K/V tile through LDS
            // (calls of two to four rows with more workgroups than CUs stay on the kernel below: 7B shape, two rows 7.6 us
            // against 9.6; per call, three rows: 7B 3.588 -> 3.577 ms, 14B 7.57 -> 7.19; from five rows on it loses).
            // Measured per call, 7B shape: 5 rows 3.91 -> 3.84 ms, 16 rows 5.03 -> 4.83, 64 rows 10.26 -> 9.61; 1.5B shape: 8 rows
            // 1.92 -> 1.82, 16 rows 2.43 -> 2.19.
            // A sequence's row slots are dealt to ZS workgroups where that shortens the busiest CU's queue: cost in slot
            // turns = workgroups per CU x (slots per wave + 1/2 for the tile), at most (n_rows - n_seqs + 1) rows in a span
            const int spw = ((n_rows - n_seqs + 1 + rp - 1) / rp + 3) / 4;
            int zs_best = 1; long cost_best = -1;
            for (int zs = 1; zs <= 8 && zs <= spw; zs *= 2) {
                const long cost = ((base * zs + n_cu - 1) / n_cu) * (2 * ((spw + zs - 1) / zs) + 1);
                if (cost_best < 0 || cost < cost_best) { cost_best = cost; zs_best = zs; }
            }
            a.slot_split = zs_best;
            hipLaunchKernelGGL((k_attn_span<HD>), dim3(n_splits, n_kv, n_seqs * zs_best), dim3(256), attn_span_lds_bytes<HD>(), st, a);
            RS_LAUNCHED("attn_span");
        } else {
        const int slots = (n_rows + rp - 1) / rp, wpb = slots < 4 ? slots : 4;
        const dim3 grid(n_splits, n_kv, (slots + wpb - 1) / wpb);
        // the one-wave-per-SIMD build schedules best, but only while every wave of the launch is resident at once
        const bool one = (long)grid.x * grid.y * grid.z * wpb <= 4L * n_cu && (size_t)n_kv * a.max_ctx * HD * 4 <= ((size_t)16 << 20);
        if (one)
            hipLaunchKernelGGL((k_attn_partial_rows<HD, 1>), grid, dim3(64 * wpb), 0, st, a);
        else
            hipLaunchKernelGGL((k_attn_partial_rows<HD, 2>), grid, dim3(64 * wpb), 0, st, a);
        RS_LAUNCHED("attn_partial_rows");
        }
    } else {
        // requesting every slice's K and V before the context length is known reads the rows' whole caches up to
        // max_ctx.  That saves a dependent round trip, but on a decode run that walks a 4608-position cache the
        // variant that waits for the position first is the faster one for both the 1.5B and the 7B shape (stitched
        // rate +0.7 % in the same process; at full context the two are within 0.2 us per layer), and by far for
        // larger caches, so only launches whose caches total <= 2 MB request everything up front
        const size_t cache_bytes = (size_t)n_rows * n_kv * a.max_ctx * HD * 4;
        // when every slice is a single 64-position pass (the kernel's own slice length, recomputed here) the
        // variant that fits three waves per SIMD is used: more resident workgroups for a long cache
        int slice_len = (a.max_ctx + n_splits - 1) / n_splits;
        slice_len = ((slice_len + ATT_BT - 1) / ATT_BT) * ATT_BT;
        if (cache_bytes <= ((size_t)2 << 20))
            hipLaunchKernelGGL((k_attn_partial<HD, true, false>), dim3(n_splits, n_kv, n_rows), dim3(256), attn_lds_bytes<HD>(a.n_q / n_kv), st, a);
        else if (slice_len == ATT_BT)
            hipLaunchKernelGGL((k_attn_partial<HD, false, true>), dim3(n_splits, n_kv, n_rows), dim3(256), attn_lds_bytes<HD>(a.n_q / n_kv), st, a);
        else
            hipLaunchKernelGGL((k_attn_partial<HD, false, false>), dim3(n_splits, n_kv, n_rows), dim3(256), attn_lds_bytes<HD>(a.n_q / n_kv), st, a);
        RS_LAUNCHED("attn_partial");
    }
    // the merge is unrolled for 128 slices (contexts up to 8192 positions) or for the most the kernels take
    // HD / 64 workgroups per head, 64 output columns each
    constexpr int DQ = HD / 64 > 0 ? HD / 64 : 1;
    if (n_splits <= 128)
        hipLaunchKernelGGL((k_attn_combine<HD, 128, DQ>), dim3(a.n_q, n_rows, DQ), dim3(256), attn_combine_lds_bytes<HD>(), st, a);
    else
        hipLaunchKernelGGL((k_attn_combine<HD, ATT_SMAX, DQ>), dim3(a.n_q, n_rows, DQ), dim3(256), attn_combine_lds_bytes<HD>(), st, a);
    RS_LAUNCHED("attn_combine");
    return RS_OK;
}

template <int MODE, int NB, int R, int NW>
rs_status launch_gemm_r(GemmArgs &a, int blocks, hipStream_t st, const char *name) {
    constexpr size_t lds = gemm_lds_bytes<MODE, NB, R, NW>();
    static_assert(lds <= 76 * 1024, "two workgroups per CU must fit");
    if (lds > 64 * 1024) {
        static std::atomic<bool> raised{false};           // per instantiation; setting the attribute twice is harmless
        if (!raised) {
            hipError_t e = hipFuncSetAttribute((const void *)k_gemm_rows<MODE, NB, R, NW>,
                                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
            if (e != hipSuccess) return fail(RS_EHIP, "raising the LDS limit of %s: %s", name, hipGetErrorString(e));
            raised = true;
        }
    }
    hipLaunchKernelGGL((k_gemm_rows<MODE, NB, R, NW>), dim3(blocks), dim3(NW * 64), lds, st, a);
    RS_LAUNCHED(name);
    return RS_OK;
}

// workgroups for `units` work units and `yblocks` token-row blocks: with several row blocks the kernel
// decodes ids in groups of 8 (one per XCD), so the unit count is padded to a multiple of 8
int gemm_grid(int units, int yblocks) { return yblocks > 1 ? ((units + 7) / 8) * 8 * yblocks : units; }

// Launch shape.  Measured on MI355X: a CU draws at most ~30 GB/s and the weight stream needs well over
// two thousand waves in flight (1184 waves reach 3.4 TB/s, 2368 reach 6.1), all groups resident at once;
// and with one tile per workgroup the X pieces (three planes), not the weights, fill the CU's load path.
// So a workgroup takes R >= 2 tiles (one X piece serves them all; R = 4 where 32 rows make the X piece
// twice as large), and where a matrix then has too few groups (QKV, O-proj, down: few output rows) K is
// split over workgroups as well: split ks leaves partial sums in a buffer that the next kernel (rotary /
// RMSNorm) adds up in a fixed order.  Gate/up needs whole sums for its activation and has tiles to spare.
template <int MODE, int NB>
rs_status launch_gemm_nb(const rs_model *m, GemmArgs &a, int n_tiles, hipStream_t st, const char *name) {
    constexpr bool SPLITS = MODE == G_QKV || MODE == G_OPROJ || MODE == G_DOWN;
    // K is split further while the launch has fewer than 1.75 workgroups per CU (A/B of the whole stitched run:
    // with a threshold of 2 the 7B O-proj went from 448 to 896 workgroups of 7 windows each and its calls
    // were 0.04 ms slower)
    const int target = 7 * m->n_cu / 4, n_win = a.K / GEMM_KW;
    a.ksplit = 1; a.part = nullptr; a.part_stride = 0;
    if constexpr (SPLITS) {
        const int r = (NB == 1 && n_win < 128) ? 2 : 4;             // one 16-row block and short rows: smaller groups rather than thin K slices
        const int groups = (n_tiles + r - 1) / r;
        int ks = 1;
        while (ks < GEMM_KSPLIT_MAX && groups * ks < target && n_win / (2 * ks) >= 4) ks *= 2;
        if (ks > 1) {
            a.ksplit = ks; a.part = m->at<float>(m->lay.gemm_part);
            a.part_stride = (size_t)m->cfg.max_rows * (size_t)a.N;
        }
        const int blocks = gemm_grid(groups * ks, a.yblocks);
        if (r == 2) return launch_gemm_r<MODE, NB, 2, 4>(a, blocks, st, name);
        return launch_gemm_r<MODE, NB, 4, 4>(a, blocks, st, name);
    } else if constexpr (MODE == G_GATEUP && NB >= 2) {
        const int r = (NB == 2 && (n_tiles + 3) / 4 >= m->n_cu) ? 4 : 2;
        const int blocks = gemm_grid((n_tiles + r - 1) / r, a.yblocks);
        if constexpr (NB == 2) {
            if (r == 4) return launch_gemm_r<MODE, NB, 4, 4>(a, blocks, st, name);
        }
        return launch_gemm_r<MODE, NB, 2, 4>(a, blocks, st, name);
    } else {
        const int r = (n_tiles + 1) / 2 >= target ? 2 : 1;
        int blocks = (n_tiles + r - 1) / r;
        if (MODE == G_LMHEAD) {
            if (blocks > LM_PARTS_CAP) blocks = LM_PARTS_CAP;             // one partial per workgroup and row block
            if (a.yblocks > 1) blocks = ((blocks + 7) / 8) * 8;           // LM_PARTS_CAP is a multiple of 8
            a.n_parts = blocks;
        }
        blocks = gemm_grid(blocks, a.yblocks);
        if (r == 2) return launch_gemm_r<MODE, NB, 2, 4>(a, blocks, st, name);
        return launch_gemm_r<MODE, NB, 1, 4>(a, blocks, st, name);
    }
}

// Launch of k_gemm_tile (33 .. 128 token rows).  CT (column tiles per workgroup) and, for the modes that leave partial
// sums, the split of K are picked so that the workgroups come as close as possible to a whole number of rounds of the
// machine with one workgroup per CU (each workgroup streams its share of W at the rate a CU can draw, so a round that
// fills a fraction of the CUs costs a whole round); ties go to the larger CT (less X traffic) and the smaller split.
template <int MODE, int NW, int CS, int CT>
rs_status launch_gemm_tile_ct(GemmArgs &a, int blocks, hipStream_t st, const char *name) {
    constexpr size_t lds = gemm_tile_lds_bytes<MODE, 1, CT>();
    static_assert(lds <= 64 * 1024, "fits the default LDS limit");
    hipLaunchKernelGGL((k_gemm_tile<MODE, 1, CT, NW, CS>), dim3(blocks), dim3(NW * 64), lds, st, a);
    RS_LAUNCHED(name);
    return RS_OK;
}

struct TilePlan { int ct, ks; double eff; };

TilePlan plan_gemm_tile(bool gateup, bool split, int n_tiles, int n_win, int n_cu) {
    static const int ct_gu[] = {5, 4, 3, 2}, ct_part[] = {10, 8, 7, 6, 4};
    TilePlan best{0, 1, -1.0};
    const int *cts = gateup ? ct_gu : ct_part;
    const int n_ct = gateup ? 4 : 5;
    for (int i = 0; i < n_ct; ++i) {
        const int ct = cts[i], groups = (n_tiles + ct - 1) / ct;
        for (int ks = 1; ks <= (split ? GEMM_KSPLIT_MAX : 1); ++ks) {
            if (ks > 1 && n_win / ks < 6) break;
            const int units = groups * ks, rounds = (units + n_cu - 1) / n_cu;
            const double eff = (double)units / ((double)rounds * n_cu) * ((double)n_tiles / ((double)groups * ct));
            if (eff > best.eff + 1e-9) best = TilePlan{ct, ks, eff};
        }
    }
    return best;
}

// NW waves: NW / CS blocks of 16 rows, CS waves per block that split the workgroup's column tiles
template <int MODE, int NW, int CS>
rs_status launch_gemm_tile(const rs_model *m, GemmArgs &a, int n_tiles, hipStream_t st, const char *name) {
    const TilePlan p = plan_gemm_tile(MODE == G_GATEUP, MODE == G_PART, n_tiles, a.K / GEMM_KW, m->n_cu);
    const int groups = (n_tiles + p.ct - 1) / p.ct;
    a.yblocks = 1; a.ksplit = p.ks; a.part = nullptr; a.part_stride = 0;
    if constexpr (MODE == G_PART) {
        a.part = m->at<float>(m->lay.gemm_part);
        a.part_stride = (size_t)m->cfg.max_rows * (size_t)a.N;
    }
    const int blocks = groups * p.ks;
    if constexpr (MODE == G_LMHEAD) a.n_parts = groups * CS;        // one partial per row, workgroup and column split
    if constexpr (MODE == G_GATEUP) {
        switch (p.ct) {
            case 5: return launch_gemm_tile_ct<MODE, NW, CS, 5>(a, blocks, st, name);
            case 4: return launch_gemm_tile_ct<MODE, NW, CS, 4>(a, blocks, st, name);
            case 3: return launch_gemm_tile_ct<MODE, NW, CS, 3>(a, blocks, st, name);
            default: return launch_gemm_tile_ct<MODE, NW, CS, 2>(a, blocks, st, name);
        }
    } else {
        switch (p.ct) {
            case 10: return launch_gemm_tile_ct<MODE, NW, CS, 10>(a, blocks, st, name);
            case 8: return launch_gemm_tile_ct<MODE, NW, CS, 8>(a, blocks, st, name);
            case 7: return launch_gemm_tile_ct<MODE, NW, CS, 7>(a, blocks, st, name);
            case 6: return launch_gemm_tile_ct<MODE, NW, CS, 6>(a, blocks, st, name);
            default: return launch_gemm_tile_ct<MODE, NW, CS, 4>(a, blocks, st, name);
        }
    }
}

// wave arrangement by row count: four waves of 16 rows up to 64 rows, eight up to 128.  Up to 32 rows two of the four
// waves would hold no rows: there two waves share each row block and split the workgroup's column tiles (k_gemm_tile's
// CS = 2; per call at 17 / 24 / 32 rows: 7B shape 5.41 / 5.53 / 5.76 -> 4.98 / 5.15 / 5.46 ms, 14B 12.2 / 12.8 / 13.8 ->
// 11.0 / 11.8 / 13.0, 1.5B 2.65 / 2.71 / 2.85 -> 2.56 / 2.65 / 2.82); not the LM head, whose partial states are counted
// per workgroup.  The same split with eight waves measured slower at 64 rows (7B shape: 7.8 ms per call against 7.0;
// every wave of a row block fetches that block's X pieces again), and four waves on one row block lose against
// k_gemm_rows (7B shape, 16 rows: 4.83 against 4.26 ms)
template <int MODE>
rs_status launch_gemm_tile_rows(const rs_model *m, GemmArgs &a, int n_tiles, hipStream_t st, const char *name) {
    if (a.M > 64) return launch_gemm_tile<MODE, 8, 1>(m, a, n_tiles, st, name);
    if constexpr (MODE != G_LMHEAD) {
        if (a.M <= 32) return launch_gemm_tile<MODE, 4, 2>(m, a, n_tiles, st, name);
    }
    return launch_gemm_tile<MODE, 4, 1>(m, a, n_tiles, st, name);
}

// Which calls take k_gemm_tile.  Layers: every call of more than 16 rows.
// Measured per call against 16- / 32-row blocks with workgroups of their own (k_gemm_rows): 7B shape 24 rows 5.81 -> 5.54
// ms, 32 rows 6.35 -> 5.75, 64 rows 9.57 -> 6.9, 128 rows 14.9 -> 10.1; 14B 32 rows 14.5 -> 13.8, 64 rows 24.0 -> 18.0, 128
// rows 44.7 -> 31.3; 32B 128 rows 78.6 -> 55.3; 1.5B shape 33 rows 3.50 -> 2.95, 64 rows 3.68 -> 3.32, 128 rows 5.44 -> 4.82
// From 17 rows on: the 32-row blocks of k_gemm_rows split two blocks' activations per window in every wave and lose
// against the tile kernel even where two of its four waves hold no rows (7B shape, 17 / 23 rows: 6.16 / 6.27 ms against
// 5.35 / 5.50; 32B 22.1 / 23.0 against 21.4 / 22.2; 1.5B 2.69 / 2.79 against 2.64 / 2.75; only the 14B shape is 2 %
// better off there).
// LM head: more than 16 sequences (16-row blocks with workgroups of their own cost 230 us per block on the 7B shape:
// 1.85 ms at 128 sequences against 0.47 ms; 1.5B shape 0.86 -> 0.24 ms); one partial per workgroup must fit the buffer
// even with four column tiles per workgroup.
bool tile_layers(const rs_config &, int rows) { return rows > 16; }
// ... and only the matrices whose workgroups fill at least 70 % of their rounds of the machine (the 1.5B shape's QKV and
// O projection have 128 and 96 of them at best: 15.6 and 14.7 us per layer at 128 rows against 12.7 and 11.0 on k_gemm_rows)
bool tile_fills(const rs_model *m, bool gateup, int n_out, int K) {
    return plan_gemm_tile(gateup, !gateup, (n_out + 15) / 16, K / GEMM_KW, m->n_cu).eff >= 0.7;
}
bool tile_lm_head(const rs_config &c, int n_seqs) { return n_seqs > 16 && ((c.vocab + 15) / 16 + 3) / 4 <= LM_PARTS_CAP; }

// n_tiles = number of 16-column output tiles; 16 * NB token rows compiled in (NB = 1, 2 or 4)
// tile: the caller's choice of k_gemm_tile for this matrix (it has prepared the activations in that kernel's format)
template <int MODE>
rs_status launch_gemm(const rs_model *m, GemmArgs &a, int n_tiles, hipStream_t st, const char *name, bool tile = false) {
    if (a.K % GEMM_KW) return fail(RS_EINVAL, "internal: K = %d is not a multiple of %d", a.K, GEMM_KW);
    a.yblocks = 1;
    if constexpr (MODE == G_LMHEAD) {
        // more than 16 sequences: one workgroup per block of vocabulary columns holds all rows, so the matrix is read once
        if (tile_lm_head(m->cfg, a.M))
            return launch_gemm_tile_rows<G_LMHEAD>(m, a, n_tiles, st, name);
        a.yblocks = (a.M + 15) / 16;
        return launch_gemm_nb<MODE, 1>(m, a, n_tiles, st, name);
    } else {
        // up to 16 rows: one 16-row block; more: blocks of 32 rows (two 16-row blocks per workgroup), each
        // block with workgroups of its own.  Measured on the 7B shape: 32 rows 6.0 ms, 64 rows 9.1 ms this
        // way; 64-row blocks are no faster (9.7 ms) and 16-row blocks slower.
        if (a.M <= 16) return launch_gemm_nb<MODE, 1>(m, a, n_tiles, st, name);
        if (tile) {
            // partial sums are always left for the next kernel (a split of one is a plain copy of the result)
            if constexpr (MODE == G_GATEUP) return launch_gemm_tile_rows<G_GATEUP>(m, a, n_tiles, st, name);
            else return launch_gemm_tile_rows<G_PART>(m, a, n_tiles, st, name);
        }
        a.yblocks = (a.M + 31) / 32;
        return launch_gemm_nb<MODE, 2>(m, a, n_tiles, st, name);
    }
}

const void *persistent_kernel(int hd) {
    switch (hd) {
        case 32: return (const void *)k_decode_persistent<32>;
        case 64: return (const void *)k_decode_persistent<64>;
        default: return (const void *)k_decode_persistent<128>;
    }
}

const void *stitch_loop_kernel(int hd) {
    switch (hd) {
        case 32: return (const void *)k_stitch_loop<32>;
        case 64: return (const void *)k_stitch_loop<64>;
        default: return (const void *)k_stitch_loop<128>;
    }
}

size_t persistent_lds(const rs_config &c) {
    size_t need = gemv_lds_bytes<1>(c.d_model);
    const size_t cand[] = {gemv_lds_bytes<1>(c.n_q_heads * c.head_dim), gemv_lds_bytes<1>(c.d_ffn),
                           c.head_dim == 32 ? attn_lds_bytes<32>() : (c.head_dim == 64 ? attn_lds_bytes<64>() : attn_lds_bytes<128>()),
                           attn_combine_lds_bytes<32>()};
    for (size_t v : cand) if (v > need) need = v;
    return need;
}

int attn_splits(const rs_config &c, const Layout &L, int n_rows) {
    const int att_ts = ATT_BT;                             // tokens per context slice: one pass of a workgroup
    int n_splits = (c.max_ctx + att_ts - 1) / att_ts;
    if (n_splits > ATT_SMAX) n_splits = ATT_SMAX;
    if (n_splits * n_rows > L.attn_rows_x_splits) n_splits = L.attn_rows_x_splits / n_rows;
    return n_splits < 1 ? 1 : n_splits;
}

// Arguments of the single-kernel phases for one token row of model m.
void fill_persist_args(rs_model *m, PersistArgs &p, const int *d_seq_slot, const int *d_token, const int *d_pos,
                       const float *d_scale, float tau, int active, rs_route_out *d_out, float *d_logits) {
    const rs_config &c = m->cfg;
    const Layout &L = m->lay;
    const int hd = c.head_dim;
    p.prep.n_seqs = 1; p.prep.n_rows = 1; p.prep.d_model = c.d_model; p.prep.vocab = c.vocab;
    p.prep.max_ctx = c.max_ctx; p.prep.max_seqs = c.max_seqs;
    p.prep.seq_slot = d_seq_slot; p.prep.tokens = d_token; p.prep.span_off = nullptr; p.prep.pos0 = d_pos; p.prep.scale = d_scale;
    p.prep.embed = m->embed;
    p.prep.row_slot = m->at<int>(L.row_slot); p.prep.row_pos = m->at<int>(L.row_pos); p.prep.row_bad = m->at<int>(L.row_bad);
    p.prep.out_row = m->at<int>(L.out_row); p.prep.seq_bad = m->at<int>(L.seq_bad); p.prep.seq_scale = m->at<float>(L.seq_scale);
    p.prep.seq_info = m->at<int4>(L.seq_info);
    p.prep.h = m->at<float>(L.h);

    GemvArgs &g = p.gemv;
    g.m_rows = 1; g.ld_h = c.d_model; g.gather = nullptr;
    g.eps = c.rms_eps; g.n_q = c.n_q_heads; g.n_kv = c.n_kv_heads; g.head_dim = hd; g.max_ctx = c.max_ctx;
    g.max_seqs = c.max_seqs; g.d_ffn = c.d_ffn;
    g.row_pos = p.prep.row_pos; g.row_slot = p.prep.row_slot; g.row_bad = p.prep.row_bad;
    g.rope_cos = m->at<float>(L.rope_cos); g.rope_sin = m->at<float>(L.rope_sin);
    g.qbuf = m->at<float>(L.qbuf); g.kcache = m->kv_k; g.vcache = m->kv_v;
    g.act = m->at<float>(L.act); g.h_out = p.prep.h;
    g.seq_scale = p.prep.seq_scale; g.parts = m->at<SoftPartial>(L.lm_parts); g.logits = d_logits;

    AttnArgs &aa = p.attn;
    aa.qbuf = g.qbuf; aa.kcache = m->kv_k; aa.vcache = m->kv_v;
    aa.partials = m->at<float>(L.attn_part);
    aa.out = m->at<float>(L.attn_out);
    aa.row_pos = p.prep.row_pos; aa.row_slot = p.prep.row_slot; aa.row_bad = p.prep.row_bad;
    aa.n_q = c.n_q_heads; aa.n_kv = c.n_kv_heads; aa.max_ctx = c.max_ctx; aa.max_seqs = c.max_seqs;

    p.layers = m->at<LayerPtrs>(L.layer_ptrs); p.n_layers = c.n_layers;
    p.qkv_rows = (c.n_q_heads + 2 * c.n_kv_heads) * hd; p.qdim = c.n_q_heads * hd;
    p.lm_head = m->lm_head; p.final_norm = m->final_norm;
    p.qkv_rt = 2; p.o_rt = 2; p.down_rt = (m->plan.down_rt == 2 || m->plan.down_rt == 4) ? m->plan.down_rt : 8;
    p.n_splits = attn_splits(c, L, 1); aa.n_slices = p.n_splits;
    p.vocab = c.vocab; p.tau = tau; p.active = active;
    p.seq_bad = p.prep.seq_bad; p.out = d_out;
    p.sync = m->at<SyncState>(L.sync); p.bar_base = m->barriers_done; p.spin_limit = m->spin_limit;
}

// The whole single-row decode step as one cooperative kernel.
rs_status forward_persistent(rs_model *m, const int *d_seq_slot, const int *d_token, const int *d_pos, const float *d_scale,
                             float tau, int active, rs_route_out *d_out, float *d_logits, hipStream_t st) {
    const rs_config &c = m->cfg;
    PersistArgs p{};
    fill_persist_args(m, p, d_seq_slot, d_token, d_pos, d_scale, tau, active, d_out, d_logits);
    void *args[] = {&p};
    hipError_t e = hipLaunchCooperativeKernel(persistent_kernel(c.head_dim), dim3(m->persist_blocks), dim3(256), args,
                                              (unsigned int)m->persist_lds, st);
    if (e != hipSuccess) return fail(RS_EHIP, "cooperative launch of the decode step: %s", hipGetErrorString(e));
    m->barriers_done += (unsigned long long)(6 * c.n_layers + 2);
    return RS_OK;
}

// One decoder layer on the FMA kernels for a call of MP (1, 2 or 4) token-row slots: QKV, attention, O-proj,
// gate/up, down.  Every phase reads the weights once and carries the rows side by side.
template <int MP, typename Tic, typename Toc>
rs_status fma_layer(rs_model *m, int l, GemvArgs &g, AttnArgs &aa, int n_rows, int n_splits, int n_seqs, hipStream_t st,
                    Tic tic, Toc toc) {
    const rs_config &c = m->cfg;
    const Layout &L = m->lay;
    const GemvPlan &pl = m->plan;
    const int hd = c.head_dim, qdim = c.n_q_heads * hd, qkv_rows = (c.n_q_heads + 2 * c.n_kv_heads) * hd;
    float *h = m->at<float>(L.h);
    rs_status rc;
    // QKV (+ RMSNorm, RoPE, KV write)
    g.W = m->w_qkv[l]; g.N = qkv_rows; g.K = c.d_model; g.h_in = h; g.gain = m->attn_norm[l]; g.x_in = nullptr;
    tic(RS_PHASE_QKV, l);
    // d_model 1536 or 3584: the activation vectors in registers, no LDS (one row: 1.5B decode step -2 %, 7B -0.2 %)
    if (reg_fits(c.d_model, MP) && c.d_model <= 3584) rc = launch_gemv_reg<G_QKV, 2, MP>(g, pl.qkv_blocks, st, "gemv_reg_qkv");
    else if constexpr (MP == 1) {
        if (pl.qkv_rt == 4) rc = launch_gemv_mp<G_QKV, 4, 1, 2, 1, 3>(g, pl.qkv_blocks, st, "gemv_qkv");
        // d_model <= 1536: a row is three chunks per lane, all requested before the prologue
        else if (c.d_model <= 1536) rc = launch_gemv_mp<G_QKV, 2, 1, 1, 1, 3>(g, pl.qkv_blocks, st, "gemv_qkv");
        else rc = launch_gemv_mp<G_QKV, 2, 1, 2, 1, 0>(g, pl.qkv_blocks, st, "gemv_qkv");
    } else {
        if (pl.qkv_rt == 4) rc = launch_gemv_mp<G_QKV, 4, 1, 2, MP, 0>(g, pl.qkv_blocks, st, "gemv_qkv");
        else rc = launch_gemv_mp<G_QKV, 2, 1, 2, MP, 0>(g, pl.qkv_blocks, st, "gemv_qkv");
    }
    toc(RS_PHASE_QKV, l);
    if (rc) return rc;
    // attention
    tic(RS_PHASE_ATTN, l);
    switch (hd) {
        case 32: rc = launch_attn<32>(aa, n_splits, c.n_kv_heads, n_rows, n_seqs, m->n_cu, st); break;
        case 64: rc = launch_attn<64>(aa, n_splits, c.n_kv_heads, n_rows, n_seqs, m->n_cu, st); break;
        default: rc = launch_attn<128>(aa, n_splits, c.n_kv_heads, n_rows, n_seqs, m->n_cu, st); break;
    }
    toc(RS_PHASE_ATTN, l);
    if (rc) return rc;
    // O projection + residual
    g.W = m->w_o[l]; g.N = c.d_model; g.K = qdim; g.h_in = nullptr; g.gain = nullptr;
    g.x_in = m->at<float>(L.attn_out);
    tic(RS_PHASE_OPROJ, l);
    // 1536, 3584 or 5120 input channels: the attention output in registers (one row: 1.5B decode step -2 %, 7B -0.8 %)
    if (reg_fits(qdim, MP)) rc = launch_gemv_reg<G_OPROJ, 2, MP>(g, pl.o_blocks, st, "gemv_reg_oproj");
    else if constexpr (MP == 1) {
        if (pl.o_all_early) rc = launch_gemv_mp<G_OPROJ, 2, 1, 1, 1, 7>(g, pl.o_blocks, st, "gemv_oproj");
        else rc = launch_gemv_mp<G_OPROJ, 2, 1, 2, 1, 4>(g, pl.o_blocks, st, "gemv_oproj");
    } else rc = launch_gemv_mp<G_OPROJ, 2, 1, 2, MP, 0>(g, pl.o_blocks, st, "gemv_oproj");
    toc(RS_PHASE_OPROJ, l);
    if (rc) return rc;
    // gate/up (+ RMSNorm, SwiGLU)
    g.W = m->w_gate_up[l]; g.N = 2 * c.d_ffn; g.K = c.d_model; g.h_in = h; g.gain = m->mlp_norm[l]; g.x_in = nullptr;
    tic(RS_PHASE_GATEUP, l);
    if constexpr (MP == 1) {
        // large matrices run two workgroups per CU, which leaves registers for the early weight request; the
        // early chunks and the unroll are picked so that the chunks left per lane (d_model / 512 minus the
        // early ones) are a whole number of unrolled rounds: 7 = 3 + 4 (7B shape), 10 = 4 + 3 * 2 (14B/32B shapes,
        // 48 us against 51 us with the other variant)
        if (pl.gu_early && (c.d_model / 512 - 3) % 4 != 0 && (c.d_model / 512 - 4) % 2 == 0)
            rc = launch_gemv_mp<G_GATEUP, 4, 1, 2, 1, 4>(g, pl.gu_blocks, st, "gemv_gateup");
        else if (pl.gu_early) rc = launch_gemv_mp<G_GATEUP, 4, 1, 4, 1, 3>(g, pl.gu_blocks, st, "gemv_gateup");
        else rc = launch_gemv_mp<G_GATEUP, 2, 1, 1, 1, 3>(g, pl.gu_blocks, st, "gemv_gateup");
    } else {
        // several rows: with the rows' activation vectors in registers there is no LDS traffic that grows with the
        // row count (two rows: 1.5B call 1.24 -> 1.22 ms, 7B 3.26 -> 3.14 ms against the LDS-staged kernel)
        if (reg_fits(c.d_model, MP)) rc = launch_gemv_reg<G_GATEUP, 2, MP>(g, pl.gu_blocks, st, "gemv_reg_gateup");
        else
        if (pl.gu_early) rc = launch_gemv_mp<G_GATEUP, 4, 1, 2, MP, 0>(g, pl.gu_blocks, st, "gemv_gateup");
        else rc = launch_gemv_mp<G_GATEUP, 2, 1, 2, MP, 0>(g, pl.gu_blocks, st, "gemv_gateup");
    }
    toc(RS_PHASE_GATEUP, l);
    if (rc) return rc;
    // down + residual
    g.W = m->w_down[l]; g.N = c.d_model; g.K = c.d_ffn; g.h_in = nullptr; g.gain = nullptr;
    g.x_in = m->at<float>(L.act);
    tic(RS_PHASE_DOWN, l);
    // x is read straight from global memory next to the weights (no LDS staging); rows per tile by width,
    // from same-process A/B runs of whole decode steps: two-row tiles at three workgroups per CU up to
    // d_model 2048 (1.5B step 1.153 -> 1.082 ms against the LDS-staged kernel), seven-row tiles for 3584
    // (7B: 2.994 -> 2.850 ms), five-row tiles at four workgroups per CU above (14B: 6.08 -> 5.86 ms,
    // 32B: 13.16 -> 11.80 ms)
    {
        const int tiles = (c.d_model + pl.down_rt - 1) / pl.down_rt;
        const int blocks = pl.down_blocks < tiles ? pl.down_blocks : tiles;
        switch (pl.down_rt) {
            case 2: hipLaunchKernelGGL((k_down_direct<2, 4, MP>), dim3(blocks), dim3(256), 0, st, g); break;
            case 7: hipLaunchKernelGGL((k_down_direct<7, (MP > 1 ? 1 : 2), MP>), dim3(blocks), dim3(256), 0, st, g); break;
            default: hipLaunchKernelGGL((k_down_direct<5, (MP > 1 ? 1 : 2), MP>), dim3(blocks), dim3(256), 0, st, g); break;
        }
        RS_LAUNCHED("down_direct");
    }
    toc(RS_PHASE_DOWN, l);
    return RS_OK;
}

// One forward invocation over n_rows token rows of n_seqs sequences, one kernel per phase.
rs_status forward_kernels(rs_model *m, int n_seqs, int n_rows, const int *d_seq_slot, const int *d_tokens,
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
    pa.seq_info = m->at<int4>(L.seq_info);
    pa.h = h;
    hipLaunchKernelGGL(k_prepare, dim3(n_rows), dim3(256), 0, st, pa);
    RS_LAUNCHED("prepare");

    // attention launch shape; calls in which some sequence brings several rows share K/V tiles between rows
    const int n_splits = attn_splits(c, L, n_rows);

    // up to four token rows go through the FMA GEMV kernels (six kernels per layer, rows side by side against one
    // weight stream); more rows go through the matrix-core kernels
    // Measured per call (GPU time, context ~4570): two rows 1.22 ms against 1.63 on the matrix-core path for the 1.5B
    // shape, 3.14 against 3.52 for the 7B shape, 6.93 / 7.37 for the 14B, 13.46 / 14.02 for the 32B; three and four
    // rows 1.55 / 1.59 against 1.69 / 1.71 for the 1.5B shape but 4.10 / 4.35 against 3.67 / 3.72 for the 7B shape
    // (the four-row variants of a 3584-wide model no longer fit the registers and fall back to LDS staging).
    const int mp = n_rows == 1 ? 1 : (n_rows == 2 ? 2 : 4);
    const bool few = n_rows <= 2 || (n_rows <= FMA_MAX_ROWS && c.d_model <= 2048);
    const bool single = few && (size_t)c.d_model * mp <= (size_t)GEMV_LDS_FLOATS && (size_t)qdim * mp <= (size_t)GEMV_LDS_FLOATS;
    rs_status rc;
    float *pend_part = nullptr; int pend_ks = 0; size_t pend_stride = 0;   // multi-row path: partial sums of the last down projection
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
        aa.partials = m->at<float>(L.attn_part);
        aa.out = m->at<float>(L.attn_out);
        aa.row_pos = row_pos; aa.row_slot = row_slot; aa.row_bad = row_bad; aa.seq_info = m->at<int4>(L.seq_info);
        aa.n_q = c.n_q_heads; aa.n_kv = c.n_kv_heads; aa.max_ctx = c.max_ctx; aa.max_seqs = c.max_seqs; aa.layer = l;

        if (single) {
            GemvArgs g{};
            g.m_rows = n_rows; g.ld_h = c.d_model;
            g.eps = c.rms_eps; g.n_q = c.n_q_heads; g.n_kv = c.n_kv_heads; g.head_dim = hd; g.max_ctx = c.max_ctx;
            g.max_seqs = c.max_seqs; g.layer = l; g.d_ffn = c.d_ffn;
            g.row_pos = row_pos; g.row_slot = row_slot; g.row_bad = row_bad;
            g.rope_cos = m->at<float>(L.rope_cos); g.rope_sin = m->at<float>(L.rope_sin);
            g.qbuf = m->at<float>(L.qbuf); g.kcache = m->kv_k; g.vcache = m->kv_v;
            g.act = m->at<float>(L.act); g.h_out = h;
            switch (mp) {
                case 1: rc = fma_layer<1>(m, l, g, aa, n_rows, n_splits, n_seqs, st, tic, toc); break;
                case 2: rc = fma_layer<2>(m, l, g, aa, n_rows, n_splits, n_seqs, st, tic, toc); break;
                default: rc = fma_layer<4>(m, l, g, aa, n_rows, n_splits, n_seqs, st, tic, toc); break;
            }
            if (rc) return rc;
        } else {
            GemmArgs g{};
            g.M = n_rows; g.d_ffn = c.d_ffn;
            const bool t_all = tile_layers(c, n_rows);
            const bool t_qkv = t_all && tile_fills(m, false, qkv_rows, c.d_model), t_o = t_all && tile_fills(m, false, c.d_model, qdim);
            // gate/up hands its output to the down projection in one format: both or neither
            const bool t_mlp = t_all && tile_fills(m, true, c.d_ffn, c.d_model) && tile_fills(m, false, c.d_model, c.d_ffn);
            float *xn32 = m->at<float>(L.xn32);
            g.act32 = m->at<float>(L.act);
            // the down projection of the layer before may have left its result as partial sums (pend_*)
            hipLaunchKernelGGL(k_rmsnorm_rows, dim3(n_rows), dim3(ROWK_THREADS), 0, st, h, m->attn_norm[l], c.rms_eps,
                               c.d_model, (const int *)nullptr, xn32, (const float *)pend_part, pend_ks, pend_stride);
            RS_LAUNCHED("rmsnorm_rows");
            pend_part = nullptr; pend_ks = 0; pend_stride = 0;
            g.W = m->w_qkv[l]; g.N = qkv_rows; g.K = c.d_model; g.X32 = xn32;
            g.out_f32 = m->at<float>(L.qkv_raw); g.ld_out = qkv_rows;
            tic(RS_PHASE_QKV, l);
            if ((rc = launch_gemm<G_QKV>(m, g, (qkv_rows + 15) / 16, st, "gemm_qkv", t_qkv))) return rc;
            toc(RS_PHASE_QKV, l);
            RopeArgs ra{};
            ra.qkv = g.part ? g.part : m->at<float>(L.qkv_raw); ra.ksplit = g.ksplit; ra.part_stride = g.part_stride;
            ra.qbuf = m->at<float>(L.qbuf); ra.kcache = m->kv_k; ra.vcache = m->kv_v;
            ra.rope_cos = m->at<float>(L.rope_cos); ra.rope_sin = m->at<float>(L.rope_sin);
            ra.row_pos = row_pos; ra.row_slot = row_slot; ra.row_bad = row_bad;
            ra.n_q = c.n_q_heads; ra.n_kv = c.n_kv_heads; ra.head_dim = hd; ra.max_ctx = c.max_ctx;
            ra.max_seqs = c.max_seqs; ra.layer = l;
            hipLaunchKernelGGL(k_rope_kv_rows, dim3(n_rows), dim3(ROWK_THREADS), 0, st, ra);
            RS_LAUNCHED("rope_kv_rows");
            tic(RS_PHASE_ATTN, l);
            switch (hd) {
                case 32: rc = launch_attn<32>(aa, n_splits, c.n_kv_heads, n_rows, n_seqs, m->n_cu, st); break;
                case 64: rc = launch_attn<64>(aa, n_splits, c.n_kv_heads, n_rows, n_seqs, m->n_cu, st); break;
                default: rc = launch_attn<128>(aa, n_splits, c.n_kv_heads, n_rows, n_seqs, m->n_cu, st); break;
            }
            toc(RS_PHASE_ATTN, l);
            if (rc) return rc;
            g.W = m->w_o[l]; g.N = c.d_model; g.K = qdim;
            g.X32 = m->at<float>(L.attn_out);
            g.h_out = h; g.ld_h = c.d_model;
            tic(RS_PHASE_OPROJ, l);
            if ((rc = launch_gemm<G_OPROJ>(m, g, (c.d_model + 15) / 16, st, "gemm_oproj", t_o))) return rc;
            toc(RS_PHASE_OPROJ, l);
            hipLaunchKernelGGL(k_rmsnorm_rows, dim3(n_rows), dim3(ROWK_THREADS), 0, st, h, m->mlp_norm[l], c.rms_eps,
                               c.d_model, (const int *)nullptr, xn32, (const float *)g.part, g.ksplit, g.part_stride);
            RS_LAUNCHED("rmsnorm_rows");
            g.W = m->w_gate_up[l]; g.N = 2 * c.d_ffn; g.K = c.d_model; g.X32 = xn32;
            tic(RS_PHASE_GATEUP, l);
            if ((rc = launch_gemm<G_GATEUP>(m, g, (c.d_ffn + 15) / 16, st, "gemm_gateup", t_mlp))) return rc;
            toc(RS_PHASE_GATEUP, l);
            g.W = m->w_down[l]; g.N = c.d_model; g.K = c.d_ffn;
            g.X32 = m->at<float>(L.act);
            tic(RS_PHASE_DOWN, l);
            if ((rc = launch_gemm<G_DOWN>(m, g, (c.d_model + 15) / 16, st, "gemm_down", t_mlp))) return rc;
            toc(RS_PHASE_DOWN, l);
            if (g.part) { pend_part = g.part; pend_ks = g.ksplit; pend_stride = g.part_stride; }
        }
    }

    // LM head + single-pass softmax statistics
    SoftPartial *parts = m->at<SoftPartial>(L.lm_parts);
    int n_parts;
    if (single) {
        GemvArgs g{};
        g.m_rows = n_seqs; g.ld_h = c.d_model; g.gather = m->at<int>(L.out_row);
        g.eps = c.rms_eps; g.W = m->lm_head; g.N = c.vocab; g.K = c.d_model; g.h_in = h; g.gain = m->final_norm;
        g.seq_scale = m->at<float>(L.seq_scale); g.parts = parts; g.logits = d_logits;
        g.sample_on = m->sample_on; g.sample_key = m->sample_key; g.row_pos = row_pos;
        n_parts = m->plan.lm_blocks; g.n_parts = n_parts;
        tic(RS_PHASE_LMHEAD, 0);
        // one output row per sequence (the last row of its span)
        if (n_seqs == 1) rc = launch_gemv_mp<G_LMHEAD, 8, 1, 2, 1, 0>(g, m->plan.lm_blocks, st, "gemv_lmhead");
        else if (n_seqs == 2) rc = launch_gemv_mp<G_LMHEAD, 8, 1, 2, 2, 0>(g, m->plan.lm_blocks, st, "gemv_lmhead");
        else rc = launch_gemv_mp<G_LMHEAD, 8, 1, 1, 4, 0>(g, m->plan.lm_blocks, st, "gemv_lmhead");
        toc(RS_PHASE_LMHEAD, 0);
        if (rc) return rc;
    } else {
        hipLaunchKernelGGL(k_rmsnorm_rows, dim3(n_seqs), dim3(ROWK_THREADS), 0, st, h, m->final_norm, c.rms_eps,
                           c.d_model, (const int *)m->at<int>(L.out_row), m->at<float>(L.lm32), (const float *)pend_part, pend_ks,
                           pend_stride);
        RS_LAUNCHED("rmsnorm_rows");
        GemmArgs g{};
        g.M = n_seqs; g.W = m->lm_head; g.N = c.vocab; g.K = c.d_model; g.X32 = m->at<float>(L.lm32);
        g.seq_scale = m->at<float>(L.seq_scale); g.parts = parts; g.logits = d_logits;
        g.sample_on = m->sample_on; g.sample_key = m->sample_key; g.row_pos = row_pos; g.out_row = m->at<int>(L.out_row);
        tic(RS_PHASE_LMHEAD, 0);
        if ((rc = launch_gemm<G_LMHEAD>(m, g, (c.vocab + 15) / 16, st, "gemm_lmhead"))) return rc;
        toc(RS_PHASE_LMHEAD, 0);
        n_parts = g.n_parts;
    }
    if (n_parts > L.lm_parts_cap) return fail(RS_EINVAL, "internal: %d router partials exceed capacity", n_parts);
    hipLaunchKernelGGL(k_route_merge, dim3(n_seqs), dim3(256), 0, st, (const SoftPartial *)parts, n_parts, c.vocab, tau,
                       active, (const int *)m->at<int>(L.seq_bad), d_out, m->sample_on);
    RS_LAUNCHED("route_merge");
    return RS_OK;
}

// Dispatch of one forward invocation.  A step is ~170 small kernels, more than a host thread can
// launch in the time the GPU needs to run them, so the launch sequence of every distinct call
// signature (same pointers, counts, tau, model role and stream) is captured once into a HIP graph
// and replayed afterwards; the kernels read tokens, positions and scales from the caller's buffers
// at run time, so a caller that reuses its buffers replays the same graph for every step.
// Falls back to plain launches when the stream cannot be captured (the legacy default stream, or
// a capture already in progress), when the phase timer is armed, or with RSTITCH_GRAPHS=0.
rs_status forward(rs_model *m, int n_seqs, int n_rows, const int *d_seq_slot, const int *d_tokens,
                  const int *d_span_off, const int *d_pos0, const float *d_scale, float tau, int active,
                  rs_route_out *d_out, float *d_logits, hipStream_t st) {
    if (n_rows == 1 && m->use_persistent && m->timer_phase < 0 && !m->sample_on)
        return forward_persistent(m, d_seq_slot, d_tokens, d_pos0, d_scale, tau, active, d_out, d_logits, st);
    auto eager = [&]() {
        return forward_kernels(m, n_seqs, n_rows, d_seq_slot, d_tokens, d_span_off, d_pos0, d_scale, tau, active, d_out,
                               d_logits, st);
    };
    if (!m->use_graphs || m->timer_phase >= 0 || st == nullptr) return eager();
    for (auto &g : m->graphs)
        if (g.n_seqs == n_seqs && g.n_rows == n_rows && g.active == active && g.tau == tau && g.slot == d_seq_slot &&
            g.tok == d_tokens && g.off == d_span_off && g.pos == d_pos0 && g.scale == d_scale && g.out == d_out &&
            g.logits == d_logits && g.st == st) {
            g.last_used = ++m->graph_clock;
            hipError_t e = hipGraphLaunch(g.exec, st);
            if (e != hipSuccess) return fail(RS_EHIP, "graph launch: %s", hipGetErrorString(e));
            return RS_OK;
        }
    // a signature is captured the second time it shows up: one-off calls stay plain launches
    size_t sig = (size_t)n_seqs * 1000003u + (size_t)n_rows * 10007u + (size_t)active;
    for (const void *p : {(const void *)d_seq_slot, (const void *)d_tokens, (const void *)d_span_off, (const void *)d_pos0,
                          (const void *)d_scale, (const void *)d_out, (const void *)d_logits, (const void *)st})
        sig = sig * 0x9E3779B97F4A7C15ull + (size_t)(uintptr_t)p;
    { uint32_t tb; memcpy(&tb, &tau, 4); sig = sig * 0x9E3779B97F4A7C15ull + tb; }
    bool seen = false;
    for (size_t v : m->seen_once) if (v == sig) { seen = true; break; }
    if (!seen) {
        if (m->seen_once.size() < 64) m->seen_once.push_back(sig);
        else { m->seen_once[m->seen_next] = sig; m->seen_next = (m->seen_next + 1) % 64; }
        return eager();
    }
    hipStreamCaptureStatus cs = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(st, &cs) != hipSuccess || cs != hipStreamCaptureStatusNone) { (void)hipGetLastError(); return eager(); }
    if (hipStreamBeginCapture(st, hipStreamCaptureModeThreadLocal) != hipSuccess) { (void)hipGetLastError(); return eager(); }
    const rs_status rc = eager();
    hipGraph_t graph = nullptr;
    hipError_t e = hipStreamEndCapture(st, &graph);
    if (rc != RS_OK) { if (graph) (void)hipGraphDestroy(graph); return rc; }
    if (e != hipSuccess || !graph) { (void)hipGetLastError(); return eager(); }
    hipGraphExec_t exec = nullptr;
    e = hipGraphInstantiate(&exec, graph, nullptr, nullptr, 0);
    if (e != hipSuccess) { (void)hipGraphDestroy(graph); (void)hipGetLastError(); return eager(); }
    if (m->graphs.size() >= 1024) {
        // full (a batched driver has up to 8 x 64 signatures per model): the entry that was used longest ago goes;
        // a launch of it may still be running on its stream, so that stream is drained first
        size_t lru = 0;
        for (size_t i = 1; i < m->graphs.size(); ++i)
            if (m->graphs[i].last_used < m->graphs[lru].last_used) lru = i;
        (void)hipStreamSynchronize(m->graphs[lru].st);
        (void)hipGraphExecDestroy(m->graphs[lru].exec);
        (void)hipGraphDestroy(m->graphs[lru].graph);
        m->graphs[lru] = m->graphs.back();
        m->graphs.pop_back();
    }
    m->graphs.push_back(rs_model::GraphEntry{n_seqs, n_rows, active, tau, d_seq_slot, d_tokens, d_span_off, d_pos0, d_scale,
                                             d_out, d_logits, st, graph, exec, ++m->graph_clock});
    e = hipGraphLaunch(exec, st);
    if (e != hipSuccess) return fail(RS_EHIP, "graph launch: %s", hipGetErrorString(e));
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
    m->device = dev;
    m->plan = make_plan(*cfg, m->n_cu);

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
    if (e == hipSuccess) e = hipMemset(m->ws + L.sync, 0, 2 * sizeof(SyncState));
    if (e == hipSuccess) {
        std::vector<LayerPtrs> lp(cfg->n_layers);
        for (int l = 0; l < cfg->n_layers; ++l)
            lp[l] = LayerPtrs{m->attn_norm[l], m->w_qkv[l], m->w_o[l], m->mlp_norm[l], m->w_gate_up[l], m->w_down[l]};
        e = hipMemcpy(m->ws + L.layer_ptrs, lp.data(), lp.size() * sizeof(LayerPtrs), hipMemcpyHostToDevice);
    }
    if (e == hipSuccess) {
        // single-kernel decode step: as many co-resident workgroups as the device holds, at most 1024
        m->persist_lds = persistent_lds(*cfg);
        int per_cu = 0;
        e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, persistent_kernel(cfg->head_dim), 256, m->persist_lds);
        int coop = 0;
        if (e == hipSuccess) e = hipDeviceGetAttribute(&coop, hipDeviceAttributeCooperativeLaunch, dev);
        const char *genv = getenv("RSTITCH_GRAPHS");
        m->use_graphs = !(genv && strcmp(genv, "0") == 0);
        const char *env = getenv("RSTITCH_DECODE");
        m->use_persistent = coop != 0 && per_cu > 0 && env && strcmp(env, "persistent") == 0;
        if (m->use_persistent && m->persist_lds > 64 * 1024)
            e = hipFuncSetAttribute(persistent_kernel(cfg->head_dim), hipFuncAttributeMaxDynamicSharedMemorySize,
                                    (int)m->persist_lds);
        int blocks = per_cu * m->n_cu;
        if (blocks > 1024) blocks = 1024;
        if (blocks * 4 > LM_PARTS_CAP) blocks = LM_PARTS_CAP / 4;
        m->persist_blocks = blocks;
    }
    if (e == hipSuccess) e = hipDeviceSynchronize();
    if (e != hipSuccess) { delete m; return fail(RS_EHIP, "workspace initialisation: %s", hipGetErrorString(e)); }
    *out = m;
    return RS_OK;
}

rs_status rs_destroy_model(rs_model *model) {
    if (model) {
        // a replay launched by the last call may still be running: drain the device before its graphs go
        if (!model->graphs.empty()) (void)hipDeviceSynchronize();
        for (auto &g : model->graphs) { (void)hipGraphExecDestroy(g.exec); (void)hipGraphDestroy(g.graph); }
    }
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

rs_status rs_set_sampling(rs_model *m, int32_t enabled, uint64_t key) {
    if (!m) return fail(RS_EINVAL, "null model");
    const int on = enabled ? 1 : 0;
    if (on == m->sample_on && key == m->sample_key) return RS_OK;
    // the cached launch graphs carry the old setting in their kernel arguments
    if (!m->graphs.empty()) {
        (void)hipDeviceSynchronize();
        for (auto &g : m->graphs) { (void)hipGraphExecDestroy(g.exec); (void)hipGraphDestroy(g.graph); }
        m->graphs.clear();
    }
    m->seen_once.clear(); m->seen_next = 0;
    m->sample_on = on; m->sample_key = key;
    return RS_OK;
}

rs_status rs_stitch_generate(rs_model *slm, rs_model *llm, int32_t seq_slot, int32_t *d_seq, int32_t n_prompt,
                             int32_t n_new, int32_t seen_slm, int32_t seen_llm, const float *d_logit_scale, float tau,
                             int32_t eos, rs_stitch_record *d_trace, int32_t max_records, rs_stitch_result *d_result,
                             void *stream) {
    if (!slm || !llm) return fail(RS_EINVAL, "null model");
    if (slm == llm) return fail(RS_EINVAL, "the two models must be different handles");
    if (!d_seq || !d_trace || !d_result) return fail(RS_EINVAL, "null argument");
    if (n_prompt < 1 || n_new < 1) return fail(RS_EINVAL, "need n_prompt >= 1 and n_new >= 1");
    if (max_records < 1 || max_records > (1 << 20)) return fail(RS_EINVAL, "max_records must be in 1..2^20");
    if (seen_slm < 0 || seen_slm > n_prompt - 1 || seen_llm < 0 || seen_llm > n_prompt - 1)
        return fail(RS_EINVAL, "seen_slm / seen_llm must be in 0 .. n_prompt - 1");
    rs_model *pair[2] = {slm, llm};
    for (rs_model *m : pair) {
        if (seq_slot < 0 || seq_slot >= m->cfg.max_seqs) return fail(RS_EINVAL, "seq_slot %d out of range", seq_slot);
        if ((long long)n_prompt + n_new - 1 > m->cfg.max_ctx)
            return fail(RS_ECAPACITY, "%d + %d tokens do not fit max_ctx %d", n_prompt, n_new, m->cfg.max_ctx);
        if (m->sample_on) return fail(RS_ENOTIMPL, "the device-resident loop decodes greedily: disable sampling");
    }
    if (slm->cfg.head_dim != llm->cfg.head_dim) return fail(RS_EINVAL, "the two models must have the same head_dim");
    if (slm->device != llm->device) return fail(RS_EINVAL, "the two models live on different devices");
    const int hd = slm->cfg.head_dim;
    const void *kern = stitch_loop_kernel(hd);
    const size_t lds = slm->persist_lds > llm->persist_lds ? slm->persist_lds : llm->persist_lds;
    int coop = 0, per_cu = 0;
    RS_HIP(hipDeviceGetAttribute(&coop, hipDeviceAttributeCooperativeLaunch, slm->device));
    if (!coop) return fail(RS_ENOTIMPL, "the device cannot launch cooperative kernels");
    if (lds > 64 * 1024) RS_HIP(hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    RS_HIP(hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kern, 256, lds));
    int blocks = per_cu * slm->n_cu;
    if (blocks > 1024) blocks = 1024;
    if (blocks * 4 > LM_PARTS_CAP) blocks = LM_PARTS_CAP / 4;
    if (blocks < 1) return fail(RS_ENOTIMPL, "the loop kernel does not fit a compute unit");

    hipStream_t st = (hipStream_t)stream;
    SyncState *sync = slm->at<SyncState>(slm->lay.sync) + 1;
    hipLaunchKernelGGL(k_stitch_init, dim3(1), dim3(64), 0, st, d_result, sync, n_prompt, n_prompt + n_new, seen_slm, seen_llm);
    RS_LAUNCHED("stitch_init");
    LoopArgs a{};
    for (int i = 0; i < 2; ++i) {
        fill_persist_args(pair[i], a.m[i], nullptr, nullptr, nullptr, nullptr, tau, i, nullptr, nullptr);
        a.m[i].sync = sync; a.m[i].bar_base = 0; a.m[i].spin_limit = slm->spin_limit;
    }
    a.seq = d_seq; a.scale = d_logit_scale; a.tau = tau; a.eos = eos; a.slot = seq_slot;
    a.trace = d_trace; a.max_records = max_records; a.state = d_result;
    a.sync = sync; a.spin_limit = slm->spin_limit;
    void *args[] = {&a};
    hipError_t e = hipLaunchCooperativeKernel(kern, dim3(blocks), dim3(256), args, (unsigned int)lds, st);
    if (e != hipSuccess) return fail(RS_EHIP, "cooperative launch of the stitched loop: %s", hipGetErrorString(e));
    return RS_OK;
}

rs_status rs_set_spin_limit(rs_model *m, uint32_t polls) {
    if (!m) return fail(RS_EINVAL, "null model");
    m->spin_limit = polls ? polls : (1u << 22);
    return RS_OK;
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
                       active, (const int *)nullptr, d_out, 0);
    RS_LAUNCHED("route_merge");
    return RS_OK;
}

rs_status rs_route_plus(rs_model *m, const float *d_hidden, int32_t n_seqs, const rs_router_weights *w, int32_t active,
                        rs_route_out *d_out, float *d_router_logits, void *stream) {
    if (!w || !d_out) return fail(RS_EINVAL, "null argument");
    if ((m == nullptr) == (d_hidden == nullptr)) return fail(RS_EINVAL, "give either the model or the hidden states");
    if (n_seqs < 1) return fail(RS_EINVAL, "n_seqs must be at least 1");
    if (m && n_seqs > m->cfg.max_seqs) return fail(RS_ECAPACITY, "n_seqs %d exceeds max_seqs %d", n_seqs, m->cfg.max_seqs);
    if (n_seqs > 65535) return fail(RS_ECAPACITY, "n_seqs %d exceeds 65535", n_seqs);
    if (active != RS_SLM && active != RS_LLM) return fail(RS_EINVAL, "active must be RS_SLM or RS_LLM");
    if (w->d < 8 || w->d % 8 || w->d > 12288) return fail(RS_EINVAL, "router width must be a multiple of 8, at most 12288");
    if (w->r < 8 || w->r % 8 || w->r > rs::ROUTER_RMAX) return fail(RS_EINVAL, "router bottleneck must be a multiple of 8, at most 64");
    if (!(w->ln_eps > 0.f)) return fail(RS_EINVAL, "ln_eps must be > 0");
    if (m && w->d != m->cfg.d_model) return fail(RS_EINVAL, "router width %d differs from the model's d_model %d", w->d, m->cfg.d_model);
    if (!w->w1 || !w->b1 || !w->w2 || !w->b2 || !w->ln_gain || !w->ln_bias || !w->w_head || !w->b_head)
        return fail(RS_EINVAL, "null router weight pointer");
    rs::RouterPlusArgs a{};
    for (int i = 0; i < rs::ROUTER_BLOCKS; ++i) {
        if (!w->w1[i] || !w->b1[i] || !w->w2[i] || !w->b2[i]) return fail(RS_EINVAL, "null router weight pointer in block %d", i);
        if (((uintptr_t)w->w1[i] | (uintptr_t)w->w2[i]) % 16) return fail(RS_EINVAL, "router matrices must be 16-byte aligned");
        a.w1[i] = (const uint16_t *)w->w1[i]; a.b1[i] = (const uint16_t *)w->b1[i];
        a.w2[i] = (const uint16_t *)w->w2[i]; a.b2[i] = (const uint16_t *)w->b2[i];
    }
    a.ln_gain = (const uint16_t *)w->ln_gain; a.ln_bias = (const uint16_t *)w->ln_bias;
    a.w_head = (const uint16_t *)w->w_head; a.b_head = (const uint16_t *)w->b_head;
    a.d = w->d; a.r = w->r; a.ln_eps = w->ln_eps;
    if (m) { a.hidden = m->at<float>(m->lay.h); a.ld_hidden = m->cfg.d_model; a.gather = m->at<int>(m->lay.out_row); }
    else { a.hidden = d_hidden; a.ld_hidden = w->d; a.gather = nullptr; }
    a.active = active; a.out = d_out; a.logits = d_router_logits;
    hipLaunchKernelGGL(rs::k_router_plus, dim3(n_seqs), dim3(256), (size_t)w->d * 4, (hipStream_t)stream, a);
    RS_LAUNCHED("router_plus");
    return RS_OK;
}

}  // extern "C"

// ================================================================================================
// rs_route for callers that cannot allocate: the partial softmax states live in a file-scope device
// array instead of a caller-provided scratch buffer.  Every device the library runs on holds its own
// copy of the array at its own address; that address is looked up once per device (with that device
// current) and used from then on: the array's name is only a host-side stand-in for it.
namespace {

constexpr int ROUTE_STATIC_MAX_ROWS = 64;
constexpr size_t ROUTE_STATIC_BYTES = (size_t)ROUTE_STATIC_MAX_ROWS * 128 * sizeof(rs::SoftPartial);   // 256 KB

static __device__ __align__(256) unsigned char scratch[ROUTE_STATIC_BYTES];

constexpr int ROUTE_STATIC_MAX_DEVICES = 64;
std::mutex g_scratch_mutex;
void *g_scratch_ptr[ROUTE_STATIC_MAX_DEVICES] = {};

// device address of `scratch` on the current device
rs_status route_static_scratch(void **out) {
    int dev = -1;
    RS_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= ROUTE_STATIC_MAX_DEVICES) return fail(RS_ECAPACITY, "device ordinal %d is beyond the %d this call supports", dev, ROUTE_STATIC_MAX_DEVICES);
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        RS_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p) return fail(RS_EHIP, "the static scratch array has no device address");
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return RS_OK;
}

}  // namespace

extern "C" rs_status rs_route_static(const float *d_logits, int32_t n, int32_t vocab, const float *d_logit_scale,
                                     float tau, int32_t active, rs_route_out *d_out, void *stream) {
    if (n < 1) return fail(RS_EINVAL, "n must be at least 1");
    if (vocab < 2) return fail(RS_EINVAL, "vocab must be at least 2");
    if (n > ROUTE_STATIC_MAX_ROWS)
        return fail(RS_ECAPACITY, "n = %d exceeds the %d rows the static scratch array holds", n, ROUTE_STATIC_MAX_ROWS);
    if (!d_logits || !d_out) return fail(RS_EINVAL, "null argument");
    if (active != RS_SLM && active != RS_LLM) return fail(RS_EINVAL, "active must be RS_SLM or RS_LLM");
    if ((uintptr_t)d_logits % 16) return fail(RS_EINVAL, "logits must be 16-byte aligned");
    const int parts = route_parts(vocab);
    if ((size_t)n * parts * sizeof(rs::SoftPartial) > ROUTE_STATIC_BYTES)
        return fail(RS_ECAPACITY, "%d rows of %d partial states exceed the static scratch array", n, parts);
    void *ptr = nullptr;
    if (rs_status rc = route_static_scratch(&ptr)) return rc;
    hipStream_t st = (hipStream_t)stream;
    // every partial the merge reads is written by the first kernel of the same call: nothing to clear
    hipLaunchKernelGGL(rs::k_route_partials, dim3(parts, n), dim3(256), 0, st, d_logits, vocab, d_logit_scale,
                       (rs::SoftPartial *)ptr);
    RS_LAUNCHED("route_partials");
    hipLaunchKernelGGL(rs::k_route_merge, dim3(n), dim3(256), 0, st, (const rs::SoftPartial *)ptr, parts, vocab, tau,
                       active, (const int *)nullptr, d_out, 0);
    RS_LAUNCHED("route_merge");
    return RS_OK;
}
