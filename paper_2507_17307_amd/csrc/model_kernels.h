// Decode-step kernels for one token row (batch 1): row table + embedding,
// bandwidth-bound GEMV phases with fused prologues/epilogues, split-K GQA
// decode attention with an in-kernel combine.  Wave64, 256-thread workgroups.
#pragma once

#include "device_utils.h"
#include "router.h"

namespace rs {

// ------------------------------------------------------------------------------------------------
// Row table.  One block per token row.  Turns the caller's per-sequence arrays into per-row
// (slot, position, token, bad) entries, validates everything that lives in device memory, and
// gathers the embedding row into the fp32 residual stream.
//   decode:  n_seqs rows, row b = sequence b (span_off == nullptr)
//   catchup: n_rows rows; row r belongs to the sequence b with off[b] <= r < off[b+1]
// ------------------------------------------------------------------------------------------------
struct PrepArgs {
    int n_seqs, n_rows, d_model, vocab, max_ctx, max_seqs;
    const int *seq_slot, *tokens, *span_off, *pos0;
    const float *scale;
    const uint16_t *embed;
    int *row_slot, *row_pos, *row_bad, *out_row, *seq_bad;
    float *seq_scale;
    float *h;
};

__global__ void __launch_bounds__(256) k_prepare(PrepArgs a) {
    const int r = blockIdx.x, tid = threadIdx.x;
    __shared__ int sh[4];     // b, first row, last row (exclusive), bad
    if (tid == 0) {
        int b = -1, lo = 0, hi = 0, bad = 0;
        if (a.span_off == nullptr) { b = r; lo = r; hi = r + 1; }
        else {
            if (a.span_off[0] != 0 || a.span_off[a.n_seqs] != a.n_rows) bad = 1;
            for (int i = 0; i < a.n_seqs; ++i) {
                int o0 = a.span_off[i], o1 = a.span_off[i + 1];
                if (o1 <= o0 || o0 < 0 || o1 > a.n_rows) bad = 1;        // empty or malformed span
                if (r >= o0 && r < o1 && b < 0) { b = i; lo = o0; hi = o1; }
            }
            if (b < 0) bad = 1;
        }
        if (!bad) {
            int slot = a.seq_slot[b], p0 = a.pos0[b];
            if (slot < 0 || slot >= a.max_seqs || p0 < 0 || p0 > a.max_ctx - (hi - lo)) bad = 1;
            for (int i = 0; i < a.n_seqs && !bad; ++i)                   // slots must be distinct
                if (i != b && a.seq_slot[i] == slot) bad = 1;
            for (int i = lo; i < hi && !bad; ++i) {
                int t = a.tokens[i];
                if (t < 0 || t >= a.vocab) bad = 1;
            }
        }
        sh[0] = b; sh[1] = lo; sh[2] = hi; sh[3] = bad;
    }
    __syncthreads();
    const int b = sh[0], lo = sh[1], hi = sh[2], bad = sh[3];
    if (tid == 0) {
        a.row_bad[r] = bad;
        a.row_slot[r] = bad ? 0 : a.seq_slot[b];
        a.row_pos[r] = bad ? 0 : a.pos0[b] + (r - lo);
        if (b >= 0 && r == hi - 1 && b < a.n_seqs) {
            a.out_row[b] = r; a.seq_bad[b] = bad;
            a.seq_scale[b] = a.scale ? a.scale[b] : 1.f;
        }
        // a malformed offset table can leave sequences without any row: flag them all
        if (bad && a.span_off != nullptr && r == 0)
            for (int i = 0; i < a.n_seqs; ++i) { a.seq_bad[i] = 1; a.out_row[i] = 0; a.seq_scale[i] = 1.f; }
    }
    float *h = a.h + (size_t)r * a.d_model;
    if (bad) { for (int i = tid; i < a.d_model; i += 256) h[i] = 0.f; return; }
    const uint16_t *e = a.embed + (size_t)a.tokens[r] * a.d_model;
    for (int i = tid; i < a.d_model; i += 256) h[i] = bf16_to_f32(e[i]);
}

// ------------------------------------------------------------------------------------------------
// GEMV phases, one token row.  y[n] = sum_k W[n,k] x[k]: W is bf16, row-major, streamed once from
// HBM with 16-byte non-temporal loads; x is fp32 and staged in LDS; accumulation is fp32.
// A wave owns RT rows at a time and its lanes stride over K (KS = 1); with KS = 4 the four waves
// of a workgroup split K of the same rows (short, wide matrices).  When K exceeds the LDS segment
// the workgroup walks K in segments, restaging x (KS = 4 only, one tile per workgroup).
// Prologue and epilogue depend on the phase:
//   G_QKV     x = RMSNorm(h);  rows come in rotary pairs (i, i + hd/2); epilogue rotates q and k,
//             writes q (fp32) and the bf16 K/V rows of this position into the cache
//   G_OPROJ   x = attention output;  h += y
//   G_GATEUP  x = RMSNorm(h);  rows come in (gate i, up i) pairs; act[i] = silu(gate) * up
//   G_DOWN    x = act;  h += y
//   G_LMHEAD  x = RMSNorm(h);  logit = y * scale feeds the single-pass softmax state of the wave
// ------------------------------------------------------------------------------------------------
enum { G_QKV = 0, G_OPROJ = 1, G_GATEUP = 2, G_DOWN = 3, G_LMHEAD = 4 };

constexpr int GEMV_KSEG = 12288;     // fp32 elements of x held in LDS at a time (48 KB)

struct GemvArgs {
    const uint16_t *W; int N, K;
    const float *h_in; const uint16_t *gain; float eps;   // RMSNorm input (norm phases)
    const float *x_in;                                    // ready fp32 vector (other phases)
    float *h_out;                                         // residual stream (O-proj, down)
    float *act;                                           // SwiGLU output (gate/up)
    float *qbuf; uint16_t *kcache, *vcache;               // QKV outputs
    const float *rope_cos, *rope_sin;                     // [max_ctx, head_dim/2]
    int n_q, n_kv, head_dim, max_ctx, max_seqs, layer, d_ffn;
    const int *row_pos, *row_slot, *row_bad;
    const float *seq_scale; SoftPartial *parts; float *logits;   // LM head
};

// 8 bf16 weights times 8 fp32 activations
__device__ __forceinline__ float dot8f(const uint4 &w, const float4 &xa, const float4 &xb, float acc) {
    acc = fmaf(bf16_lo(w.x), xa.x, acc); acc = fmaf(bf16_hi(w.x), xa.y, acc);
    acc = fmaf(bf16_lo(w.y), xa.z, acc); acc = fmaf(bf16_hi(w.y), xa.w, acc);
    acc = fmaf(bf16_lo(w.z), xb.x, acc); acc = fmaf(bf16_hi(w.z), xb.y, acc);
    acc = fmaf(bf16_lo(w.w), xb.z, acc); acc = fmaf(bf16_hi(w.w), xb.w, acc);
    return acc;
}

// accumulate chunks [c_begin, c_end) of the rows; xs holds the segment starting at chunk seg_c0 as
// two float4 planes (first and second half of every 8-element chunk) of plane_len chunks each
template <int RT>
__device__ __forceinline__ void gemv_accumulate(const uint4 *const (&wp)[RT], const float4 *__restrict__ xs, int plane_len,
                                                int seg_c0, int c_begin, int c_end, int cstride, float (&acc)[RT]) {
#pragma unroll 2
    for (int c = c_begin; c < c_end; c += cstride) {
        uint4 wv[RT];
#pragma unroll
        for (int r = 0; r < RT; ++r) wv[r] = load_stream(wp[r] + c);
        const float4 xa = xs[c - seg_c0], xb = xs[plane_len + c - seg_c0];
#pragma unroll
        for (int r = 0; r < RT; ++r) acc[r] = dot8f(wv[r], xa, xb, acc[r]);
    }
}

template <int MODE, int RT, int KS>
__global__ void __launch_bounds__(256) k_gemv(GemvArgs a) {
    extern __shared__ __align__(16) unsigned char smem[];
    float4 *xs = reinterpret_cast<float4 *>(smem);
    __shared__ float red[2][4][RT];
    __shared__ float red_ss[4];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int K = a.K;
    const int seg = K < GEMV_KSEG ? K : GEMV_KSEG;       // elements per LDS segment
    const int plane_len = seg >> 3;
    const bool resident = K <= GEMV_KSEG;
    constexpr bool NORM = (MODE == G_QKV || MODE == G_GATEUP || MODE == G_LMHEAD);

    float inv = 1.f;
    if (NORM) {
        const float4 *h4 = reinterpret_cast<const float4 *>(a.h_in);
        float ss = 0.f;
        for (int i = tid; i < (K >> 2); i += 256) {
            const float4 v = h4[i];
            ss = fmaf(v.x, v.x, ss); ss = fmaf(v.y, v.y, ss); ss = fmaf(v.z, v.z, ss); ss = fmaf(v.w, v.w, ss);
        }
        ss = wave_sum(ss);
        if (lane == 0) red_ss[wave] = ss;
        __syncthreads();
        inv = 1.0f / sqrtf((red_ss[0] + red_ss[1] + red_ss[2] + red_ss[3]) / (float)K + a.eps);
    }
    // stage the K-range [k0, k0+len) of x: float4 index i covers elements 4i..4i+3; even i -> plane A, odd i -> plane B
    auto stage = [&](int k0, int len) {
        if (NORM) {
            const float4 *h4 = reinterpret_cast<const float4 *>(a.h_in + k0);
            const uint2 *g2 = reinterpret_cast<const uint2 *>(a.gain + k0);
            for (int i = tid; i < (len >> 2); i += 256) {
                float4 v = h4[i]; const uint2 g = g2[i];
                v.x *= inv * bf16_lo(g.x); v.y *= inv * bf16_hi(g.x); v.z *= inv * bf16_lo(g.y); v.w *= inv * bf16_hi(g.y);
                xs[(i & 1) * plane_len + (i >> 1)] = v;
            }
        } else {
            const float4 *x4 = reinterpret_cast<const float4 *>(a.x_in + k0);
            for (int i = tid; i < (len >> 2); i += 256) xs[(i & 1) * plane_len + (i >> 1)] = x4[i];
        }
    };
    if (resident) { stage(0, K); __syncthreads(); }

    // ---- tiles
    constexpr int P = RT / 2;
    const int half = a.head_dim >> 1;
    int n_tiles, n_rot_tiles = 0;
    if (MODE == G_QKV) {
        n_rot_tiles = (a.n_q + a.n_kv) * (half / P);
        n_tiles = n_rot_tiles + (a.n_kv * a.head_dim) / RT;
    } else if (MODE == G_GATEUP) {
        n_tiles = a.d_ffn / P;
    } else {
        n_tiles = (a.N + RT - 1) / RT;
    }
    const int unit0 = (KS == 1) ? blockIdx.x * 4 + wave : blockIdx.x;
    const int ustride = (KS == 1) ? gridDim.x * 4 : gridDim.x;
    const int c0 = (KS == 1) ? lane : wave * 64 + lane;
    const int cstride = 64 * KS;

    SoftState st; st.init();
    const float lm_scale = (MODE == G_LMHEAD) ? a.seq_scale[0] : 1.f;
    int parity = 0;

    for (int t = unit0; t < n_tiles; t += ustride) {
        int rows[RT];
        int head = 0, pair0 = 0; bool rot = false;
        if (MODE == G_QKV) {
            if (t < n_rot_tiles) {
                rot = true; head = t / (half / P); pair0 = (t % (half / P)) * P;
#pragma unroll
                for (int j = 0; j < P; ++j) { rows[2 * j] = head * a.head_dim + pair0 + j; rows[2 * j + 1] = rows[2 * j] + half; }
            } else {
#pragma unroll
                for (int j = 0; j < RT; ++j) rows[j] = (a.n_q + a.n_kv) * a.head_dim + (t - n_rot_tiles) * RT + j;
            }
        } else if (MODE == G_GATEUP) {
#pragma unroll
            for (int j = 0; j < P; ++j) { rows[2 * j] = t * P + j; rows[2 * j + 1] = a.d_ffn + t * P + j; }
        } else {
#pragma unroll
            for (int j = 0; j < RT; ++j) rows[j] = min(t * RT + j, a.N - 1);
        }
        const uint4 *wp[RT];
        float acc[RT];
#pragma unroll
        for (int r = 0; r < RT; ++r) { wp[r] = reinterpret_cast<const uint4 *>(a.W + (size_t)rows[r] * K); acc[r] = 0.f; }
        if (resident) {
            gemv_accumulate<RT>(wp, xs, plane_len, 0, c0, K >> 3, cstride, acc);
        } else {
            for (int k0 = 0; k0 < K; k0 += GEMV_KSEG) {        // KS == 4 only: the tile loop is workgroup-uniform
                const int len = min(GEMV_KSEG, K - k0);
                __syncthreads();
                stage(k0, len);
                __syncthreads();
                gemv_accumulate<RT>(wp, xs, plane_len, k0 >> 3, (k0 >> 3) + c0, (k0 + len) >> 3, cstride, acc);
            }
        }
#pragma unroll
        for (int r = 0; r < RT; ++r) acc[r] = wave_sum(acc[r]);
        if (KS > 1) {
            if (lane == 0) {
#pragma unroll
                for (int r = 0; r < RT; ++r) red[parity][wave][r] = acc[r];
            }
            __syncthreads();
#pragma unroll
            for (int r = 0; r < RT; ++r) acc[r] = red[parity][0][r] + red[parity][1][r] + red[parity][2][r] + red[parity][3][r];
            parity ^= 1;
        }
        const bool writer = (KS == 1) ? (lane == 0) : (tid == 0);
        if (!writer) continue;

        // ---- epilogue (one lane)
        if (MODE == G_QKV) {
            if (a.row_bad[0]) continue;
            const int pos = a.row_pos[0], slot = a.row_slot[0];
            if (rot) {
                const float *cs = a.rope_cos + (size_t)pos * half, *sn = a.rope_sin + (size_t)pos * half;
#pragma unroll
                for (int j = 0; j < P; ++j) {
                    const int i = pair0 + j;
                    const float c = cs[i], s = sn[i], x0 = acc[2 * j], x1 = acc[2 * j + 1];
                    const float y0 = x0 * c - x1 * s, y1 = x1 * c + x0 * s;
                    if (head < a.n_q) {
                        a.qbuf[head * a.head_dim + i] = y0; a.qbuf[head * a.head_dim + i + half] = y1;
                    } else {
                        const size_t base = ((((size_t)a.layer * a.max_seqs + slot) * a.n_kv + (head - a.n_q)) * a.max_ctx + pos) * a.head_dim;
                        a.kcache[base + i] = f32_to_bf16(y0); a.kcache[base + i + half] = f32_to_bf16(y1);
                    }
                }
            } else {
#pragma unroll
                for (int j = 0; j < RT; ++j) {
                    const int vr = rows[j] - (a.n_q + a.n_kv) * a.head_dim;      // index inside the V section
                    const int vh = vr / a.head_dim, e = vr % a.head_dim;
                    const size_t base = ((((size_t)a.layer * a.max_seqs + slot) * a.n_kv + vh) * a.max_ctx + pos) * a.head_dim;
                    a.vcache[base + e] = f32_to_bf16(acc[j]);
                }
            }
        } else if (MODE == G_GATEUP) {
#pragma unroll
            for (int j = 0; j < P; ++j) {
                const float g = acc[2 * j], u = acc[2 * j + 1];
                a.act[t * P + j] = g / (1.0f + expf(-g)) * u;
            }
        } else if (MODE == G_OPROJ || MODE == G_DOWN) {
#pragma unroll
            for (int j = 0; j < RT; ++j) if (t * RT + j < a.N) a.h_out[t * RT + j] += acc[j];
        } else {   // G_LMHEAD
#pragma unroll
            for (int j = 0; j < RT; ++j) if (t * RT + j < a.N) {
                const float lg = acc[j] * lm_scale;
                st.push(lg, t * RT + j);
                if (a.logits) a.logits[t * RT + j] = lg;
            }
        }
    }
    if (MODE == G_LMHEAD) {
        const bool writer = (KS == 1) ? (lane == 0) : (tid == 0);
        if (writer) a.parts[(KS == 1) ? blockIdx.x * 4 + wave : blockIdx.x] = to_partial(st);
    }
}

// ------------------------------------------------------------------------------------------------
// Split-K grouped-query decode attention.  grid (n_splits, n_kv_heads, n_rows), block 256.
// A workgroup owns one KV head, one slice of the context and ALL query heads of that KV head's
// group, so every K/V byte is read once per row.  Per sub-chunk of TS tokens every thread issues
// its 8 K loads and 8 V loads (16 bytes each) up front, so the whole sub-chunk costs one memory
// round trip; scores go through LDS (one exp per score); running max / sum are carried across
// sub-chunks.  The last workgroup to finish for a (row, kv head) merges the slices.
// Partial record per (row, q head, split): [m, l, 0, 0, acc[HD]] fp32.
// ------------------------------------------------------------------------------------------------
struct AttnArgs {
    const float *qbuf;             // [rows, n_q*hd] fp32, rotated
    const uint16_t *kcache, *vcache;
    float *partials;               // [rows, n_q, n_splits, hd+4]
    int *counters;                 // [rows, n_kv], zero between launches
    float *out;                    // [rows, n_q*hd] fp32
    uint16_t *out_planes; size_t out_plane;   // optional three-plane bf16 split of the same values, or null
    const int *row_pos, *row_slot, *row_bad;
    int n_q, n_kv, max_ctx, max_seqs, layer;
};

constexpr int ATT_GMAX = 8;       // query heads per kv head, at most
constexpr int ATT_NLD = 8;        // 16-byte K (and V) loads in flight per thread
constexpr int ATT_SMAX = 64;      // context slices, at most

template <int HD>
__global__ void __launch_bounds__(256) k_attn_decode(AttnArgs a) {
    constexpr int LPR = HD / 8, RPW = 64 / LPR, TPI = 4 * RPW;   // lanes per row, rows per wave-load, tokens per load round
    constexpr int TS = ATT_NLD * TPI;                            // tokens per sub-chunk
    constexpr int PS = HD + 4;                                   // floats per partial record
    constexpr int NQ = HD / 4, NSG = 256 / NQ;                   // combine: float4 columns, slice groups
    const int split = blockIdx.x, S = gridDim.x, kvh = blockIdx.y, row = blockIdx.z;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int G = a.n_q / a.n_kv;
    const int sub_lane = lane % LPR, grp = lane / LPR, e0 = sub_lane * 8;

    __shared__ float s_lds[ATT_GMAX * TS];                 // scores / probabilities; reused by the combine
    __shared__ float m_lds[ATT_GMAX], alpha_lds[ATT_GMAX];
    __shared__ __align__(16) float accw[NSG > 4 ? NSG : 4][ATT_GMAX][HD];   // cross-wave / cross-group sums
    __shared__ float lw[4][ATT_GMAX];
    __shared__ int last_flag;

    const int ctx = a.row_bad[row] ? 0 : a.row_pos[row] + 1;
    const int slot = a.row_bad[row] ? 0 : a.row_slot[row];
    int C = (ctx + S - 1) / S;
    C = ((C + TPI - 1) / TPI) * TPI;
    const int t_begin = split * C;
    const int t_end = min(ctx, t_begin + C);
    const size_t kv_base = (((size_t)a.layer * a.max_seqs + slot) * a.n_kv + kvh) * (size_t)a.max_ctx * HD;
    const uint16_t *Kp = a.kcache + kv_base, *Vp = a.vcache + kv_base;
    const float scale = 1.0f / sqrtf((float)HD);

    float q[ATT_GMAX][8], acc[ATT_GMAX][8], l[ATT_GMAX];
    if (tid < ATT_GMAX) m_lds[tid] = -INFINITY;
#pragma unroll
    for (int g = 0; g < ATT_GMAX; ++g) {
        l[g] = 0.f;
#pragma unroll
        for (int j = 0; j < 8; ++j) { acc[g][j] = 0.f; q[g][j] = 0.f; }
        if (g < G) {
            const float4 *qp = reinterpret_cast<const float4 *>(a.qbuf + ((size_t)row * a.n_q + kvh * G + g) * HD + e0);
            const float4 qa = qp[0], qb = qp[1];
            q[g][0] = qa.x; q[g][1] = qa.y; q[g][2] = qa.z; q[g][3] = qa.w;
            q[g][4] = qb.x; q[g][5] = qb.y; q[g][6] = qb.z; q[g][7] = qb.w;
        }
    }

    for (int sub = t_begin; sub < t_end; sub += TS) {
        const int n_sub = min(TS, t_end - sub);
        uint4 kreg[ATT_NLD], vreg[ATT_NLD];
#pragma unroll
        for (int it = 0; it < ATT_NLD; ++it) {
            const int tl = it * TPI + wave * RPW + grp;
            kreg[it] = make_uint4(0, 0, 0, 0); vreg[it] = make_uint4(0, 0, 0, 0);
            if (tl < n_sub) {
                kreg[it] = *reinterpret_cast<const uint4 *>(Kp + (size_t)(sub + tl) * HD + e0);
                vreg[it] = *reinterpret_cast<const uint4 *>(Vp + (size_t)(sub + tl) * HD + e0);
            }
        }
        // scores
#pragma unroll
        for (int it = 0; it < ATT_NLD; ++it) {
            const int tl = it * TPI + wave * RPW + grp;
            const uint4 kv = kreg[it];
            const float k0 = bf16_lo(kv.x), k1 = bf16_hi(kv.x), k2 = bf16_lo(kv.y), k3 = bf16_hi(kv.y);
            const float k4 = bf16_lo(kv.z), k5 = bf16_hi(kv.z), k6 = bf16_lo(kv.w), k7 = bf16_hi(kv.w);
            float part[ATT_GMAX];
#pragma unroll
            for (int g = 0; g < ATT_GMAX; ++g) {
                float p = q[g][0] * k0;
                p = fmaf(q[g][1], k1, p); p = fmaf(q[g][2], k2, p); p = fmaf(q[g][3], k3, p);
                p = fmaf(q[g][4], k4, p); p = fmaf(q[g][5], k5, p); p = fmaf(q[g][6], k6, p); p = fmaf(q[g][7], k7, p);
#pragma unroll
                for (int o = LPR >> 1; o > 0; o >>= 1) p += __shfl_xor(p, o, RS_WAVE);
                part[g] = p;
            }
            if (sub_lane == 0 && tl < n_sub) {
#pragma unroll
                for (int g = 0; g < ATT_GMAX; ++g) if (g < G) s_lds[g * TS + tl] = part[g] * scale;
            }
        }
        __syncthreads();
        // sub-chunk maxima -> new running maxima and rescale factors (one wave per head)
        for (int g = wave; g < G; g += 4) {
            float mx = -INFINITY;
            for (int i = lane; i < n_sub; i += 64) mx = fmaxf(mx, s_lds[g * TS + i]);
            mx = wave_max(mx);
            if (lane == 0) {
                const float m_old = m_lds[g], m_new = fmaxf(m_old, mx);
                alpha_lds[g] = (m_old == -INFINITY) ? 0.f : expf(m_old - m_new);
                m_lds[g] = m_new;
            }
        }
        __syncthreads();
#pragma unroll
        for (int g = 0; g < ATT_GMAX; ++g) if (g < G) {
            const float alpha = alpha_lds[g];
            l[g] *= alpha;
#pragma unroll
            for (int j = 0; j < 8; ++j) acc[g][j] *= alpha;
        }
        for (int g = 0; g < G; ++g) {
            const float mg = m_lds[g];
            for (int i = tid; i < n_sub; i += 256) s_lds[g * TS + i] = expf(s_lds[g * TS + i] - mg);
        }
        __syncthreads();
        // P V
#pragma unroll
        for (int it = 0; it < ATT_NLD; ++it) {
            const int tl = it * TPI + wave * RPW + grp;
            if (tl < n_sub) {
                const uint4 vv = vreg[it];
                const float v0 = bf16_lo(vv.x), v1 = bf16_hi(vv.x), v2 = bf16_lo(vv.y), v3 = bf16_hi(vv.y);
                const float v4 = bf16_lo(vv.z), v5 = bf16_hi(vv.z), v6 = bf16_lo(vv.w), v7 = bf16_hi(vv.w);
#pragma unroll
                for (int g = 0; g < ATT_GMAX; ++g) if (g < G) {
                    const float p = s_lds[g * TS + tl];
                    l[g] += p;
                    acc[g][0] = fmaf(p, v0, acc[g][0]); acc[g][1] = fmaf(p, v1, acc[g][1]);
                    acc[g][2] = fmaf(p, v2, acc[g][2]); acc[g][3] = fmaf(p, v3, acc[g][3]);
                    acc[g][4] = fmaf(p, v4, acc[g][4]); acc[g][5] = fmaf(p, v5, acc[g][5]);
                    acc[g][6] = fmaf(p, v6, acc[g][6]); acc[g][7] = fmaf(p, v7, acc[g][7]);
                }
            }
        }
        __syncthreads();
    }

    // reduce over the token groups inside the wave (lanes with equal sub_lane), then over waves
#pragma unroll
    for (int g = 0; g < ATT_GMAX; ++g) {
#pragma unroll
        for (int o = LPR; o < 64; o <<= 1) {
            l[g] += __shfl_xor(l[g], o, RS_WAVE);
#pragma unroll
            for (int j = 0; j < 8; ++j) acc[g][j] += __shfl_xor(acc[g][j], o, RS_WAVE);
        }
    }
    if (grp == 0) {
#pragma unroll
        for (int g = 0; g < ATT_GMAX; ++g) if (g < G) {
#pragma unroll
            for (int j = 0; j < 8; ++j) accw[wave][g][e0 + j] = acc[g][j];
            if (sub_lane == 0) lw[wave][g] = l[g];
        }
    }
    __syncthreads();
    for (int i = tid; i < G * HD; i += 256) {
        const int g = i / HD, e = i - g * HD;
        const float v = accw[0][g][e] + accw[1][g][e] + accw[2][g][e] + accw[3][g][e];
        float *p = a.partials + (((size_t)row * a.n_q + kvh * G + g) * S + split) * PS;
        p[4 + e] = v;
        if (e == 0) { p[0] = m_lds[g]; p[1] = lw[0][g] + lw[1][g] + lw[2][g] + lw[3][g]; }
    }
    // completion ticket
    __threadfence();
    __syncthreads();
    if (tid == 0) {
        const int old = atomicAdd(&a.counters[row * a.n_kv + kvh], 1);
        last_flag = (old == S - 1);
    }
    __syncthreads();
    if (!last_flag) return;
    __threadfence();

    // ---- combine (last workgroup only): weights per (head, slice), then a slice-parallel weighted sum
    float *m_sh = s_lds, *w_sh = s_lds + ATT_GMAX * ATT_SMAX;       // S <= ATT_SMAX and 2*GMAX*SMAX <= GMAX*TS
    const float *pbase = a.partials + ((size_t)row * a.n_q + kvh * G) * S * PS;
    for (int i = tid; i < G * S; i += 256) {
        const int g = i / S, s = i - g * S;
        const float2 ml = *reinterpret_cast<const float2 *>(pbase + ((size_t)g * S + s) * PS);
        m_sh[g * ATT_SMAX + s] = ml.y > 0.f ? ml.x : -INFINITY;
        w_sh[g * ATT_SMAX + s] = ml.y;
    }
    __syncthreads();
    for (int g = wave; g < G; g += 4) {
        const float ms = lane < S ? m_sh[g * ATT_SMAX + lane] : -INFINITY;
        const float ls = lane < S ? w_sh[g * ATT_SMAX + lane] : 0.f;
        const float M = wave_max(ms);
        const float w = ls > 0.f ? expf(ms - M) : 0.f;
        const float L = wave_sum(ls * w);
        if (lane < S) w_sh[g * ATT_SMAX + lane] = L > 0.f ? w / L : 0.f;
    }
    __syncthreads();
    {
        const int qd = tid % NQ, sg = tid / NQ;
        for (int g = 0; g < G; ++g) {
            float4 sum = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll 4
            for (int s = sg; s < S; s += NSG) {
                const float w = w_sh[g * ATT_SMAX + s];
                const float4 v = *reinterpret_cast<const float4 *>(pbase + ((size_t)g * S + s) * PS + 4 + 4 * qd);
                sum.x = fmaf(w, v.x, sum.x); sum.y = fmaf(w, v.y, sum.y); sum.z = fmaf(w, v.z, sum.z); sum.w = fmaf(w, v.w, sum.w);
            }
            *reinterpret_cast<float4 *>(&accw[sg][g][4 * qd]) = sum;
        }
    }
    __syncthreads();
    for (int i = tid; i < G * HD; i += 256) {
        const int g = i / HD, e = i - g * HD;
        float o = 0.f;
#pragma unroll
        for (int sg = 0; sg < NSG; ++sg) o += accw[sg][g][e];
        const size_t oi = ((size_t)row * a.n_q + kvh * G + g) * HD + e;
        a.out[oi] = o;
        if (a.out_planes) {
            const uint16_t p0 = f32_to_bf16(o);
            const float r1 = o - bf16_to_f32(p0);
            const uint16_t p1 = f32_to_bf16(r1);
            a.out_planes[oi] = p0; a.out_planes[a.out_plane + oi] = p1;
            a.out_planes[2 * a.out_plane + oi] = f32_to_bf16(r1 - bf16_to_f32(p1));
        }
    }
    if (tid == 0) a.counters[row * a.n_kv + kvh] = 0;
}

}  // namespace rs
