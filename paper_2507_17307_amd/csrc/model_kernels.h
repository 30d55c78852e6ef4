// Decode-step kernels: row table + embedding, bandwidth-bound GEMV phases with
// fused prologues/epilogues for one token row, split-context GQA decode
// attention on the matrix cores (a partial kernel for one row, one for spans of
// rows, and the merge of the slices).  Wave64, 256-thread workgroups.
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
    int4 *seq_info;                // per sequence {first row, end row, cache slot, first row's position}; first row = -1 for an invalid one
    float *seq_scale;
    float *h;
};

constexpr int MAX_SEQS = 128;     // sequences one call may carry
constexpr int MAX_ROWS = 128;     // token rows one call may carry
constexpr int PREP_LDS_INTS = 8 + 5 * MAX_SEQS;

// sh: PREP_LDS_INTS ints of LDS.  The control values may live in pinned host memory, where every
// dependent read costs a bus round trip: each one is requested by its own thread, all at once,
// and the validation then runs out of LDS.
__device__ __forceinline__ void prepare_row(const PrepArgs &a, int r, int *sh) {
    static_assert(MAX_ROWS <= MAX_SEQS && 2 * MAX_SEQS <= 256, "one thread per control value");
    const int tid = threadIdx.x;
    int *s_off = sh + 4, *s_slot = sh + 8 + MAX_SEQS, *s_pos = sh + 8 + 2 * MAX_SEQS, *s_tok = sh + 8 + 4 * MAX_SEQS;   // [MAX_SEQS + 1], [MAX_SEQS] ...
    float *s_scale = reinterpret_cast<float *>(sh + 8 + 3 * MAX_SEQS);
    const int ns = min(a.n_seqs, MAX_SEQS), nr = min(a.n_rows, MAX_ROWS);            // the host enforces both bounds
    if (a.span_off != nullptr && tid <= ns) s_off[tid] = a.span_off[tid];
    if (tid < nr) s_tok[tid] = a.tokens[tid];
    if (tid >= 128 && tid < 128 + ns) {
        const int i = tid - 128;
        s_slot[i] = a.seq_slot[i]; s_pos[i] = a.pos0[i]; s_scale[i] = a.scale ? a.scale[i] : 1.f;
    }
    __syncthreads();
    if (tid == 0) {
        int b = -1, lo = 0, hi = 0, bad = 0;
        if (a.span_off == nullptr) { b = r; lo = r; hi = r + 1; }
        else {
            if (s_off[0] != 0 || s_off[ns] != a.n_rows) bad = 1;
            for (int i = 0; i < ns; ++i) {
                const int o0 = s_off[i], o1 = s_off[i + 1];
                if (o1 <= o0 || o0 < 0 || o1 > a.n_rows) bad = 1;        // empty or malformed span
                if (r >= o0 && r < o1 && b < 0) { b = i; lo = o0; hi = o1; }
            }
            if (b < 0) bad = 1;
        }
        if (!bad) {
            const int slot = s_slot[b], p0 = s_pos[b];
            if (slot < 0 || slot >= a.max_seqs || p0 < 0 || p0 > a.max_ctx - (hi - lo)) bad = 1;
            for (int i = 0; i < ns && !bad; ++i)                         // slots must be distinct
                if (i != b && s_slot[i] == slot) bad = 1;
            for (int i = lo; i < hi && !bad; ++i) {
                const int t = s_tok[i];
                if (t < 0 || t >= a.vocab) bad = 1;
            }
        }
        sh[0] = b; sh[1] = lo; sh[2] = hi; sh[3] = bad;
        a.row_bad[r] = bad;
        a.row_slot[r] = bad ? 0 : s_slot[b];
        a.row_pos[r] = bad ? 0 : s_pos[b] + (r - lo);
        if (b >= 0 && r == hi - 1 && b < ns) {
            a.out_row[b] = r; a.seq_bad[b] = bad;
            a.seq_scale[b] = s_scale[b];
            a.seq_info[b] = bad ? make_int4(-1, 0, 0, 0) : make_int4(lo, hi, s_slot[b], s_pos[b]);
        }
        // a malformed offset table can leave sequences without any row: flag them all
        if (bad && a.span_off != nullptr && r == 0)
            for (int i = 0; i < ns; ++i) { a.seq_bad[i] = 1; a.out_row[i] = 0; a.seq_scale[i] = 1.f; a.seq_info[i] = make_int4(-1, 0, 0, 0); }
    }
    __syncthreads();
    const int bad = sh[3];
    float *h = a.h + (size_t)r * a.d_model;
    if (bad) { for (int i = tid; i < a.d_model; i += 256) h[i] = 0.f; return; }
    const uint16_t *e = a.embed + (size_t)s_tok[r] * a.d_model;
    for (int i = tid; i < a.d_model; i += 256) h[i] = bf16_to_f32(e[i]);
}

__global__ void __launch_bounds__(256) k_prepare(PrepArgs a) {
    __shared__ int sh[PREP_LDS_INTS];
    prepare_row(a, blockIdx.x, sh);
}

// ------------------------------------------------------------------------------------------------
// GEMV phases for 1..8 token rows.  y[m][n] = sum_k W[n,k] x[m][k]: W is bf16, row-major, streamed
// once from HBM with 16-byte non-temporal loads whatever the number of rows; x is fp32 and staged in
// LDS; accumulation is fp32.  A wave owns RT rows of W at a time and its lanes stride over K
// (KS = 1); with KS = 4 the four waves of a workgroup split K of the same rows (short, wide
// matrices).  MP is the number of token rows the kernel is compiled for (1, 2, 4, 8); a call with
// fewer rows leaves the spare ones zero.  When MP * K floats exceed the LDS segment the workgroup
// walks K in segments, restaging x (KS = 4 only).
// Prologue and epilogue depend on the phase:
//   G_QKV     x = RMSNorm(h);  rows come in rotary pairs (i, i + hd/2); epilogue rotates q and k,
//             writes q (fp32) and the bf16 K/V rows of each token's position into the cache
//   G_OPROJ   x = attention output;  h += y
//   G_GATEUP  x = RMSNorm(h);  rows come in (gate i, up i) pairs; act[i] = silu(gate) * up
//   G_DOWN    x = act;  h += y
//   G_LMHEAD  x = RMSNorm(h[gather]);  logit = y * scale feeds the single-pass softmax state of
//             the wave; the workgroup's four states are merged into one partial per token row
// ------------------------------------------------------------------------------------------------
enum { G_QKV = 0, G_OPROJ = 1, G_GATEUP = 2, G_DOWN = 3, G_LMHEAD = 4 };

constexpr int GEMV_LDS_FLOATS = 38912;   // fp32 elements of x held in LDS at a time (152 KB of the CU's 160 KB)

struct GemvArgs {
    const uint16_t *W; int N, K;
    int m_rows;                                           // token rows in this call (<= MP)
    const float *h_in; int ld_h; const uint16_t *gain; float eps;   // RMSNorm input rows (norm phases), row stride ld_h
    const int *gather;                                    // LM head: h row of output row m, or null (= m)
    const float *x_in;                                    // ready fp32 rows [m][K] (other phases)
    float *h_out;                                         // residual stream rows, stride ld_h (O-proj, down)
    float *act;                                           // SwiGLU output rows [m][d_ffn] (gate/up)
    float *qbuf; uint16_t *kcache, *vcache;               // QKV outputs (q rows [m][n_q*hd])
    const float *rope_cos, *rope_sin;                     // [max_ctx, head_dim/2]
    int n_q, n_kv, head_dim, max_ctx, max_seqs, layer, d_ffn;
    const int *row_pos, *row_slot, *row_bad;
    const float *seq_scale; SoftPartial *parts; int n_parts; float *logits;   // LM head
    int sample_on; unsigned long long sample_key;         // LM head: also track the arg max of logit + Gumbel noise (needs row_pos)
};

// elements of K one LDS segment holds for MP rows
template <int MP>
__host__ __device__ constexpr int gemv_seg(int K) { return K * MP <= GEMV_LDS_FLOATS ? K : (GEMV_LDS_FLOATS / MP) / 2048 * 2048; }
template <int MP>
__host__ __device__ constexpr size_t gemv_lds_bytes(int K) { return (size_t)gemv_seg<MP>(K) * MP * 4 + 4096; }

template <int MODE, int RT, int KS, int UNR, int MP, int PRE = 0>
__device__ __forceinline__ void gemv_phase(const GemvArgs &a, unsigned char *smem, int wg, int nwg) {
    static_assert(PRE == 0 || MP == 1, "the early weight request exists for single-row calls only");
    float4 *xs = reinterpret_cast<float4 *>(smem);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int K = a.K, M = a.m_rows;
    const int seg = gemv_seg<MP>(K);                      // elements of K per LDS segment
    const int plane_len = seg >> 3;                       // float4 per plane; row m uses planes 2m and 2m+1
    float *red = reinterpret_cast<float *>(smem + (size_t)seg * MP * 4);   // [2][4][RT*MP]
    float *red_ss = red + 2 * 4 * RT * MP;                                  // [4][MP]
    const bool resident = KS != 4 || seg == K;            // only the split-K launch may walk K in segments (the host checks)
    constexpr bool NORM = (MODE == G_QKV || MODE == G_GATEUP || MODE == G_LMHEAD);

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
    // each workgroup owns a contiguous range of tiles (a contiguous stretch of W); with KS == 1 its
    // four waves interleave inside that range
    // n_tiles * nwg stays far below 2^31 (at most ~2e4 tiles, a few thousand workgroups)
    const int t_lo = (int)(((unsigned)n_tiles * (unsigned)wg) / (unsigned)nwg), t_hi = (int)(((unsigned)n_tiles * (unsigned)(wg + 1)) / (unsigned)nwg);
    const int unit0 = (KS == 1) ? t_lo + wave : t_lo;
    const int ustride = (KS == 1) ? 4 : 1;
    const int c0 = (KS == 1) ? lane : wave * 64 + lane;
    const int cstride = 64 * KS;

    auto tile_rows = [&](int t, int (&rows)[RT], int &head, int &pair0, bool &rot) {
        head = 0; pair0 = 0; rot = false;
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
    };

    // PRE > 0: the first PRE chunks of this wave's first tile are requested before the prologue
    // touches x, so the weight stream's first round trip overlaps the prologue's instead of
    // following it.  It costs PRE * RT * 4 registers, so it is compiled in only where the sweep
    // showed a gain.  Chunk indices are clamped, not guarded; a clamped chunk is cancelled later by
    // zeroing its x operand.
    uint4 pre[PRE > 0 ? PRE : 1][RT];
    const bool have0 = PRE > 0 && resident && unit0 < t_hi;
    if (have0) {
        int rows0[RT], head0, pair00; bool rot0;
        tile_rows(unit0, rows0, head0, pair00, rot0);
#pragma unroll
        for (int u = 0; u < PRE; ++u) {
            const int c = min(c0 + u * cstride, (K >> 3) - 1);
#pragma unroll
            for (int r = 0; r < RT; ++r) pre[u][r] = load_stream(reinterpret_cast<const uint4 *>(a.W + (size_t)rows0[r] * K) + c);
        }
    }

    // row position / slot (QKV only), read once up front so that no epilogue waits on it
    int row_bad[MP], row_pos[MP], row_slot[MP];
#pragma unroll
    for (int m = 0; m < MP; ++m) {
        row_bad[m] = 1; row_pos[m] = 0; row_slot[m] = 0;
        if (MODE == G_QKV && m < M) { row_bad[m] = a.row_bad[m]; row_pos[m] = a.row_pos[m]; row_slot[m] = a.row_slot[m]; }
    }

    // ---- prologue: x (fp32) into LDS.  Norm phases: K = d_model fits one segment for every MP.
    float inv[MP];
    constexpr int HCACHE = (MP == 1) ? 6 : 0;            // float4 per thread kept between the two passes over h
    float4 hreg[HCACHE > 0 ? HCACHE : 1];
    uint2 greg[HCACHE > 0 ? HCACHE : 1];
    if (NORM) {
        const uint2 *g2 = reinterpret_cast<const uint2 *>(a.gain);
#pragma unroll
        for (int m = 0; m < MP; ++m) {
            float ss = 0.f;
            if (m < M) {
                const int src = (MODE == G_LMHEAD && a.gather) ? a.gather[m] : m;
                const float4 *h4 = reinterpret_cast<const float4 *>(a.h_in + (size_t)src * a.ld_h);
                if (HCACHE > 0) {
#pragma unroll
                    for (int j = 0; j < HCACHE; ++j) {
                        const int i = tid + j * 256;
                        hreg[j] = make_float4(0.f, 0.f, 0.f, 0.f); greg[j] = make_uint2(0, 0);
                        if (i < (K >> 2)) { hreg[j] = h4[i]; greg[j] = g2[i]; }
                    }
#pragma unroll
                    for (int j = 0; j < HCACHE; ++j) {
                        ss = fmaf(hreg[j].x, hreg[j].x, ss); ss = fmaf(hreg[j].y, hreg[j].y, ss);
                        ss = fmaf(hreg[j].z, hreg[j].z, ss); ss = fmaf(hreg[j].w, hreg[j].w, ss);
                    }
                }
                for (int i = tid + HCACHE * 256; i < (K >> 2); i += 256) {
                    const float4 v = h4[i];
                    ss = fmaf(v.x, v.x, ss); ss = fmaf(v.y, v.y, ss); ss = fmaf(v.z, v.z, ss); ss = fmaf(v.w, v.w, ss);
                }
            }
            ss = wave_sum(ss);
            if (lane == 0) red_ss[wave * MP + m] = ss;
        }
        __syncthreads();
#pragma unroll
        for (int m = 0; m < MP; ++m)
            inv[m] = 1.0f / sqrtf((red_ss[0 * MP + m] + red_ss[1 * MP + m] + red_ss[2 * MP + m] + red_ss[3 * MP + m]) / (float)K + a.eps);
    }
    // stage the K-range [k0, k0+len) of every row: float4 index i covers elements 4i..4i+3; even i -> plane A, odd i -> plane B
    auto stage = [&](int k0, int len) {
#pragma unroll
        for (int m = 0; m < MP; ++m) {
            float4 *xm = xs + (size_t)2 * m * plane_len;
            if (m >= M) {
                for (int i = tid; i < (len >> 2); i += 256) xm[(i & 1) * plane_len + (i >> 1)] = make_float4(0.f, 0.f, 0.f, 0.f);
            } else if (NORM) {
                const int src = (MODE == G_LMHEAD && a.gather) ? a.gather[m] : m;
                const float4 *h4 = reinterpret_cast<const float4 *>(a.h_in + (size_t)src * a.ld_h + k0);
                const uint2 *g2 = reinterpret_cast<const uint2 *>(a.gain + k0);
                const float iv = inv[m];
                if (HCACHE > 0) {
#pragma unroll
                    for (int j = 0; j < HCACHE; ++j) {
                        const int i = tid + j * 256;
                        if (i < (len >> 2)) {
                            float4 v = hreg[j]; const uint2 g = greg[j];
                            v.x *= iv * bf16_lo(g.x); v.y *= iv * bf16_hi(g.x); v.z *= iv * bf16_lo(g.y); v.w *= iv * bf16_hi(g.y);
                            xm[(i & 1) * plane_len + (i >> 1)] = v;
                        }
                    }
                }
                for (int i = tid + HCACHE * 256; i < (len >> 2); i += 256) {
                    float4 v = h4[i]; const uint2 g = g2[i];
                    v.x *= iv * bf16_lo(g.x); v.y *= iv * bf16_hi(g.x); v.z *= iv * bf16_lo(g.y); v.w *= iv * bf16_hi(g.y);
                    xm[(i & 1) * plane_len + (i >> 1)] = v;
                }
            } else {
                // batches of SB loads per thread, all requested before the first is stored
                const float4 *x4 = reinterpret_cast<const float4 *>(a.x_in + (size_t)m * K + k0);
                constexpr int SB = 10;
                const int n4 = len >> 2;
                for (int i0 = tid; i0 < n4; i0 += 256 * SB) {
                    float4 v[SB];
#pragma unroll
                    for (int j = 0; j < SB; ++j) v[j] = x4[min(i0 + j * 256, n4 - 1)];
#pragma unroll
                    for (int j = 0; j < SB; ++j) {
                        const int i = i0 + j * 256;
                        if (i < n4) xm[(i & 1) * plane_len + (i >> 1)] = v[j];
                    }
                }
            }
        }
    };
    if (resident) { stage(0, K); __syncthreads(); }

    SoftState st[MP];
    float lm_scale[MP];
    unsigned long long noise_base[MP];                   // sampling: (position of the token being predicted) * V
#pragma unroll
    for (int m = 0; m < MP; ++m) {
        st[m].init(); lm_scale[m] = (MODE == G_LMHEAD && m < M) ? a.seq_scale[m] : 1.f;
        noise_base[m] = 0;
        if (MODE == G_LMHEAD && a.sample_on && m < M)
            noise_base[m] = (unsigned long long)(a.row_pos[a.gather ? a.gather[m] : m] + 1) * (unsigned long long)a.N;
    }
    int parity = 0;

    // accumulate chunks [c_begin, c_end) of the tile; the LDS segment starts at chunk seg_c0
    auto accumulate = [&](const uint4 *const (&wp)[RT], int seg_c0, int c_begin, int c_end, int c_step, float (&acc)[RT][MP]) {
#pragma unroll UNR
        for (int c = c_begin; c < c_end; c += c_step) {
            uint4 wv[RT];
#pragma unroll
            for (int r = 0; r < RT; ++r) wv[r] = load_stream(wp[r] + c);
            float4 xa[MP], xb[MP];
#pragma unroll
            for (int m = 0; m < MP; ++m) { xa[m] = xs[(2 * m) * plane_len + c - seg_c0]; xb[m] = xs[(2 * m + 1) * plane_len + c - seg_c0]; }
#pragma unroll
            for (int r = 0; r < RT; ++r) {
                const float w0 = bf16_lo(wv[r].x), w1 = bf16_hi(wv[r].x), w2 = bf16_lo(wv[r].y), w3 = bf16_hi(wv[r].y);
                const float w4 = bf16_lo(wv[r].z), w5 = bf16_hi(wv[r].z), w6 = bf16_lo(wv[r].w), w7 = bf16_hi(wv[r].w);
#pragma unroll
                for (int m = 0; m < MP; ++m) {
                    float v = acc[r][m];
                    v = fmaf(w0, xa[m].x, v); v = fmaf(w1, xa[m].y, v); v = fmaf(w2, xa[m].z, v); v = fmaf(w3, xa[m].w, v);
                    v = fmaf(w4, xb[m].x, v); v = fmaf(w5, xb[m].y, v); v = fmaf(w6, xb[m].z, v); v = fmaf(w7, xb[m].w, v);
                    acc[r][m] = v;
                }
            }
        }
    };

    for (int t = unit0; t < t_hi; t += ustride) {
        int rows[RT];
        int head, pair0; bool rot;
        tile_rows(t, rows, head, pair0, rot);
        const uint4 *wp[RT];
        float acc[RT][MP];
#pragma unroll
        for (int r = 0; r < RT; ++r) {
            wp[r] = reinterpret_cast<const uint4 *>(a.W + (size_t)rows[r] * K);
#pragma unroll
            for (int m = 0; m < MP; ++m) acc[r][m] = 0.f;
        }
        // what the epilogue will need from memory is requested now, ahead of the weight stream
        float epi[RT][MP];
#pragma unroll
        for (int r = 0; r < RT; ++r)
#pragma unroll
            for (int m = 0; m < MP; ++m) epi[r][m] = 0.f;
        if (MODE == G_QKV) {
            if (rot) {
#pragma unroll
                for (int m = 0; m < MP; ++m) if (!row_bad[m]) {
#pragma unroll
                    for (int j = 0; j < P; ++j) {
                        epi[2 * j][m] = a.rope_cos[(size_t)row_pos[m] * half + pair0 + j];
                        epi[2 * j + 1][m] = a.rope_sin[(size_t)row_pos[m] * half + pair0 + j];
                    }
                }
            }
        } else if (MODE == G_OPROJ || MODE == G_DOWN) {
#pragma unroll
            for (int r = 0; r < RT; ++r)
#pragma unroll
                for (int m = 0; m < MP; ++m) if (m < M) epi[r][m] = a.h_out[(size_t)m * a.ld_h + rows[r]];
        }
        if (resident) {
            int cb = c0;
            if (PRE > 0 && t == unit0) {
#pragma unroll
                for (int u = 0; u < PRE; ++u) {
                    const int c = c0 + u * cstride;
                    const bool valid = c < (K >> 3);
                    const int cc = valid ? c : 0;
                    float4 xa = xs[cc], xb = xs[plane_len + cc];
                    if (!valid) { xa = make_float4(0.f, 0.f, 0.f, 0.f); xb = xa; }
#pragma unroll
                    for (int r = 0; r < RT; ++r) {
                        const uint4 w = pre[u][r];
                        float v = acc[r][0];
                        v = fmaf(bf16_lo(w.x), xa.x, v); v = fmaf(bf16_hi(w.x), xa.y, v); v = fmaf(bf16_lo(w.y), xa.z, v); v = fmaf(bf16_hi(w.y), xa.w, v);
                        v = fmaf(bf16_lo(w.z), xb.x, v); v = fmaf(bf16_hi(w.z), xb.y, v); v = fmaf(bf16_lo(w.w), xb.z, v); v = fmaf(bf16_hi(w.w), xb.w, v);
                        acc[r][0] = v;
                    }
                }
                cb = c0 + PRE * cstride;
            }
            accumulate(wp, 0, cb, K >> 3, cstride, acc);
        } else {
            for (int k0 = 0; k0 < K; k0 += seg) {              // KS == 4 only: the tile loop is workgroup-uniform
                const int len = min(seg, K - k0);
                __syncthreads();
                stage(k0, len);
                __syncthreads();
                accumulate(wp, k0 >> 3, (k0 >> 3) + c0, (k0 + len) >> 3, cstride, acc);
            }
        }
#pragma unroll
        for (int r = 0; r < RT; ++r)
#pragma unroll
            for (int m = 0; m < MP; ++m) acc[r][m] = wave_sum(acc[r][m]);
        if (KS > 1) {
            if (lane == 0) {
#pragma unroll
                for (int r = 0; r < RT; ++r)
#pragma unroll
                    for (int m = 0; m < MP; ++m) red[(parity * 4 + wave) * RT * MP + r * MP + m] = acc[r][m];
            }
            __syncthreads();
#pragma unroll
            for (int r = 0; r < RT; ++r)
#pragma unroll
                for (int m = 0; m < MP; ++m)
                    acc[r][m] = red[(parity * 4 + 0) * RT * MP + r * MP + m] + red[(parity * 4 + 1) * RT * MP + r * MP + m] +
                                red[(parity * 4 + 2) * RT * MP + r * MP + m] + red[(parity * 4 + 3) * RT * MP + r * MP + m];
            parity ^= 1;
        }
        const bool writer = (KS == 1) ? (lane == 0) : (tid == 0);
        if (!writer) continue;

        // ---- epilogue (one lane)
#pragma unroll
        for (int m = 0; m < MP; ++m) {
            if (m >= M) continue;
            if (MODE == G_QKV) {
                if (row_bad[m]) continue;
                const int pos = row_pos[m], slot = row_slot[m];
                if (rot) {
#pragma unroll
                    for (int j = 0; j < P; ++j) {
                        const int i = pair0 + j;
                        const float c = epi[2 * j][m], s = epi[2 * j + 1][m], x0 = acc[2 * j][m], x1 = acc[2 * j + 1][m];
                        const float y0 = x0 * c - x1 * s, y1 = x1 * c + x0 * s;
                        if (head < a.n_q) {
                            float *q = a.qbuf + (size_t)m * a.n_q * a.head_dim + head * a.head_dim;
                            q[i] = y0; q[i + half] = y1;
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
                        const size_t base = (((size_t)a.layer * a.max_seqs + slot) * a.n_kv + vh) * (size_t)a.max_ctx * a.head_dim;
                        a.vcache[base + (size_t)e * a.max_ctx + pos] = f32_to_bf16(acc[j][m]);     // V is stored [hd][position]
                    }
                }
            } else if (MODE == G_GATEUP) {
#pragma unroll
                for (int j = 0; j < P; ++j) {
                    const float g = acc[2 * j][m], u = acc[2 * j + 1][m];
                    a.act[(size_t)m * a.d_ffn + t * P + j] = g / (1.0f + expf(-g)) * u;
                }
            } else if (MODE == G_OPROJ || MODE == G_DOWN) {
#pragma unroll
                for (int j = 0; j < RT; ++j) if (t * RT + j < a.N) a.h_out[(size_t)m * a.ld_h + t * RT + j] = epi[j][m] + acc[j][m];
            } else {   // G_LMHEAD
#pragma unroll
                for (int j = 0; j < RT; ++j) if (t * RT + j < a.N) {
                    const float lg = acc[j][m] * lm_scale[m];
                    st[m].push(lg, t * RT + j);
                    if (a.sample_on) st[m].push_noisy(lg, t * RT + j, a.sample_key, noise_base[m]);
                    if (a.logits) a.logits[(size_t)m * a.N + t * RT + j] = lg;
                }
            }
        }
    }
    if (MODE == G_LMHEAD) {
        // one partial per workgroup and token row: the four waves' states meet in LDS
        SoftPartial *sp = reinterpret_cast<SoftPartial *>(red);           // [4][MP], inside the 4 KB tail of the segment
        if (KS == 1) {
            if (lane == 0) {
#pragma unroll
                for (int m = 0; m < MP; ++m) sp[wave * MP + m] = to_partial(st[m]);
            }
            __syncthreads();
            if (tid < MP && tid < M) {
                SoftState s0 = from_partial(sp[tid]);
                for (int w = 1; w < 4; ++w) s0.merge(from_partial(sp[w * MP + tid]));
                a.parts[(size_t)tid * a.n_parts + wg] = to_partial(s0);
            }
        } else if (tid == 0) {
#pragma unroll
            for (int m = 0; m < MP; ++m)
                if (m < M) a.parts[(size_t)m * a.n_parts + wg] = to_partial(st[m]);
        }
    }
}

template <int MODE, int RT, int KS, int UNR, int MP, int PRE = 0>
__global__ void __launch_bounds__(256) k_gemv(GemvArgs a) {
    extern __shared__ __align__(16) unsigned char smem[];
    gemv_phase<MODE, RT, KS, UNR, MP, PRE>(a, smem, blockIdx.x, gridDim.x);
}

// ------------------------------------------------------------------------------------------------
// Single-row GEMV phases with the activation vector in REGISTERS.  K = 512 * NCH: a row of W is NCH
// chunks of 16 bytes per lane, and lane l of every wave holds exactly the x values those chunks
// meet (elements 8 (l + 64 u) .. + 7, u < NCH), K / 64 floats.  A wave is then self-contained: it
// loads its own copy of h (or of the ready activation), reduces the sum of squares of an RMSNorm
// across its lanes with DPP adds, scales, and streams its weight tiles against registers.  No LDS
// staging, no workgroup barrier, no LDS reads in the stream; the only LDS is the LM head's
// exchange of four softmax states.  The first UG chunks of a wave's first tile are requested
// before the activation loads, so the weight stream's first round trip overlaps the prologue.
// Tiles and epilogues are those of gemv_phase (KS = 1).  MP token rows (a call of a few rows: short catch-up
// spans, small batches) share every weight chunk: each row's x lives in its own registers.
// ------------------------------------------------------------------------------------------------
template <int MODE, int RT, int NCH, int UG, int MP = 1>
__global__ void __launch_bounds__(256) k_gemv_reg(GemvArgs a) {
    static_assert(MODE != G_DOWN, "the down projection splits K over the waves");
    static_assert(UG >= 1 && UG <= NCH, "group size");
    static_assert(MODE != G_LMHEAD || MP == 1, "the LM head runs on one row per sequence; batches take the LDS-staged kernel");
    constexpr bool NORM = (MODE == G_QKV || MODE == G_GATEUP || MODE == G_LMHEAD);
    constexpr int P = RT / 2;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wg = blockIdx.x, nwg = gridDim.x;
    const int K = a.K, M = a.m_rows;                      // K == 512 * NCH (the host checks); M <= MP token rows
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
    const int t_lo = (int)(((unsigned)n_tiles * (unsigned)wg) / (unsigned)nwg), t_hi = (int)(((unsigned)n_tiles * (unsigned)(wg + 1)) / (unsigned)nwg);
    const int unit0 = t_lo + wave;

    auto tile_rows = [&](int t, int (&rows)[RT], int &head, int &pair0, bool &rot) {
        head = 0; pair0 = 0; rot = false;
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
    };

    // ---- first weight requests of the wave's first tile (a wave without a tile requests the last tile's, unused)
    uint4 pre[UG][RT];
    {
        int rows0[RT], head0, pair00; bool rot0;
        tile_rows(min(unit0, n_tiles - 1), rows0, head0, pair00, rot0);
#pragma unroll
        for (int u = 0; u < UG; ++u)
#pragma unroll
            for (int r = 0; r < RT; ++r) pre[u][r] = load_stream(reinterpret_cast<const uint4 *>(a.W + (size_t)rows0[r] * K) + lane + 64 * u);
    }
    int row_bad[MP], row_pos[MP], row_slot[MP];
#pragma unroll
    for (int m = 0; m < MP; ++m) {
        row_bad[m] = 1; row_pos[m] = 0; row_slot[m] = 0;
        if (MODE == G_QKV && m < M) { row_bad[m] = a.row_bad[m]; row_pos[m] = a.row_pos[m]; row_slot[m] = a.row_slot[m]; }
    }

    // ---- x into registers: token row m, chunk u of this lane (a row past the call's count is a copy of row 0, never written)
    float xr[MP][NCH][8];
#pragma unroll
    for (int m = 0; m < MP; ++m) {
        const int src = (MODE == G_LMHEAD && a.gather) ? a.gather[0] : (m < M ? m : 0);
        const float4 *x4 = reinterpret_cast<const float4 *>(NORM ? a.h_in + (size_t)src * a.ld_h : a.x_in + (size_t)src * K);
        float4 xa[NCH], xb[NCH];
#pragma unroll
        for (int u = 0; u < NCH; ++u) { xa[u] = x4[2 * (lane + 64 * u)]; xb[u] = x4[2 * (lane + 64 * u) + 1]; }
        if (NORM) {
            const uint4 *g4 = reinterpret_cast<const uint4 *>(a.gain);
            uint4 gg[NCH];
#pragma unroll
            for (int u = 0; u < NCH; ++u) gg[u] = g4[lane + 64 * u];
            float ss = 0.f;
#pragma unroll
            for (int u = 0; u < NCH; ++u) {
                ss = fmaf(xa[u].x, xa[u].x, ss); ss = fmaf(xa[u].y, xa[u].y, ss); ss = fmaf(xa[u].z, xa[u].z, ss); ss = fmaf(xa[u].w, xa[u].w, ss);
                ss = fmaf(xb[u].x, xb[u].x, ss); ss = fmaf(xb[u].y, xb[u].y, ss); ss = fmaf(xb[u].z, xb[u].z, ss); ss = fmaf(xb[u].w, xb[u].w, ss);
            }
            const float inv = 1.0f / sqrtf(wave_sum(ss) / (float)K + a.eps);
#pragma unroll
            for (int u = 0; u < NCH; ++u) {
                xr[m][u][0] = xa[u].x * (inv * bf16_lo(gg[u].x)); xr[m][u][1] = xa[u].y * (inv * bf16_hi(gg[u].x));
                xr[m][u][2] = xa[u].z * (inv * bf16_lo(gg[u].y)); xr[m][u][3] = xa[u].w * (inv * bf16_hi(gg[u].y));
                xr[m][u][4] = xb[u].x * (inv * bf16_lo(gg[u].z)); xr[m][u][5] = xb[u].y * (inv * bf16_hi(gg[u].z));
                xr[m][u][6] = xb[u].z * (inv * bf16_lo(gg[u].w)); xr[m][u][7] = xb[u].w * (inv * bf16_hi(gg[u].w));
            }
        } else {
#pragma unroll
            for (int u = 0; u < NCH; ++u) {
                xr[m][u][0] = xa[u].x; xr[m][u][1] = xa[u].y; xr[m][u][2] = xa[u].z; xr[m][u][3] = xa[u].w;
                xr[m][u][4] = xb[u].x; xr[m][u][5] = xb[u].y; xr[m][u][6] = xb[u].z; xr[m][u][7] = xb[u].w;
            }
        }
    }

    SoftState st; st.init();
    const float lm_scale = MODE == G_LMHEAD ? a.seq_scale[0] : 1.f;

    for (int t = unit0; t < t_hi; t += 4) {
        int rows[RT];
        int head, pair0; bool rot;
        tile_rows(t, rows, head, pair0, rot);
        const uint4 *wp[RT];
        float acc[RT][MP], epi[RT][MP];
#pragma unroll
        for (int r = 0; r < RT; ++r) {
            wp[r] = reinterpret_cast<const uint4 *>(a.W + (size_t)rows[r] * K) + lane;
#pragma unroll
            for (int m = 0; m < MP; ++m) { acc[r][m] = 0.f; epi[r][m] = 0.f; }
        }
        // what the epilogue needs from memory is requested ahead of the weight stream
        if (MODE == G_QKV) {
            if (rot) {
#pragma unroll
                for (int m = 0; m < MP; ++m) if (!row_bad[m]) {
#pragma unroll
                    for (int j = 0; j < P; ++j) {
                        epi[2 * j][m] = a.rope_cos[(size_t)row_pos[m] * half + pair0 + j];
                        epi[2 * j + 1][m] = a.rope_sin[(size_t)row_pos[m] * half + pair0 + j];
                    }
                }
            }
        } else if (MODE == G_OPROJ) {
#pragma unroll
            for (int r = 0; r < RT; ++r)
#pragma unroll
                for (int m = 0; m < MP; ++m) if (m < M) epi[r][m] = a.h_out[(size_t)m * a.ld_h + rows[r]];
        }
        // groups of UG chunks; the first group of the first tile is already on its way
#pragma unroll
        for (int u0 = 0; u0 < NCH; u0 += UG) {
            uint4 wv[UG][RT];
            if (u0 == 0 && t == unit0) {
#pragma unroll
                for (int u = 0; u < UG; ++u)
#pragma unroll
                    for (int r = 0; r < RT; ++r) wv[u][r] = pre[u][r];
            } else {
#pragma unroll
                for (int u = 0; u < UG; ++u)
#pragma unroll
                    for (int r = 0; r < RT; ++r)
                        if (u0 + u < NCH) wv[u][r] = load_stream(wp[r] + 64 * (u0 + u));
            }
#pragma unroll
            for (int u = 0; u < UG; ++u)
#pragma unroll
                for (int r = 0; r < RT; ++r)
                    if (u0 + u < NCH) {
                        const uint4 w = wv[u][r];
                        const float w0 = bf16_lo(w.x), w1 = bf16_hi(w.x), w2 = bf16_lo(w.y), w3 = bf16_hi(w.y);
                        const float w4 = bf16_lo(w.z), w5 = bf16_hi(w.z), w6 = bf16_lo(w.w), w7 = bf16_hi(w.w);
#pragma unroll
                        for (int m = 0; m < MP; ++m) {
                            const float (&x)[8] = xr[m][u0 + u];
                            float v = acc[r][m];
                            v = fmaf(w0, x[0], v); v = fmaf(w1, x[1], v); v = fmaf(w2, x[2], v); v = fmaf(w3, x[3], v);
                            v = fmaf(w4, x[4], v); v = fmaf(w5, x[5], v); v = fmaf(w6, x[6], v); v = fmaf(w7, x[7], v);
                            acc[r][m] = v;
                        }
                    }
        }
#pragma unroll
        for (int r = 0; r < RT; ++r)
#pragma unroll
            for (int m = 0; m < MP; ++m) acc[r][m] = wave_sum(acc[r][m]);
        if (lane != 0) continue;

        // ---- epilogue (one lane)
#pragma unroll
        for (int m = 0; m < MP; ++m) {
            if (m >= M) continue;
            if (MODE == G_QKV) {
                if (row_bad[m]) continue;
                const int pos = row_pos[m], slot = row_slot[m];
                if (rot) {
#pragma unroll
                    for (int j = 0; j < P; ++j) {
                        const int i = pair0 + j;
                        const float c = epi[2 * j][m], sn = epi[2 * j + 1][m], x0 = acc[2 * j][m], x1 = acc[2 * j + 1][m];
                        const float y0 = x0 * c - x1 * sn, y1 = x1 * c + x0 * sn;
                        if (head < a.n_q) {
                            float *q = a.qbuf + (size_t)m * a.n_q * a.head_dim + head * a.head_dim;
                            q[i] = y0; q[i + half] = y1;
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
                        const size_t base = (((size_t)a.layer * a.max_seqs + slot) * a.n_kv + vh) * (size_t)a.max_ctx * a.head_dim;
                        a.vcache[base + (size_t)e * a.max_ctx + pos] = f32_to_bf16(acc[j][m]);     // V is stored [hd][position]
                    }
                }
            } else if (MODE == G_GATEUP) {
#pragma unroll
                for (int j = 0; j < P; ++j) {
                    const float g = acc[2 * j][m], up = acc[2 * j + 1][m];
                    a.act[(size_t)m * a.d_ffn + t * P + j] = g / (1.0f + expf(-g)) * up;
                }
            } else if (MODE == G_OPROJ) {
#pragma unroll
                for (int j = 0; j < RT; ++j) if (t * RT + j < a.N) a.h_out[(size_t)m * a.ld_h + t * RT + j] = epi[j][m] + acc[j][m];
            } else {   // G_LMHEAD (MP == 1)
#pragma unroll
                for (int j = 0; j < RT; ++j) if (t * RT + j < a.N) {
                    const float lg = acc[j][m] * lm_scale;
                    st.push(lg, t * RT + j);
                    if (a.logits) a.logits[t * RT + j] = lg;
                }
            }
        }
    }
    if (MODE == G_LMHEAD) {
        __shared__ SoftPartial sp[4];
        if (lane == 0) sp[wave] = to_partial(st);
        __syncthreads();
        if (tid == 0) {
            SoftState s0 = from_partial(sp[0]);
            for (int w = 1; w < 4; ++w) s0.merge(from_partial(sp[w]));
            a.parts[wg] = to_partial(s0);
        }
    }
}

// ------------------------------------------------------------------------------------------------
// Single-row down projection (h += W_down . act) without any staging: the four waves of a workgroup
// split K (wave w takes the chunks w * 64 + lane, + 256, ...), and every lane reads the eight activation values of a chunk straight from
// global memory next to the RT weight rows of that chunk.  The activation vector (tens of KB) is
// the same for every workgroup, so those reads are served by the CU's cache and the L2; they cost
// 32 bytes per lane and chunk against RT x 16 bytes of weights, but there is no copy into LDS, no
// barrier before the weight stream starts and no LDS footprint that limits the workgroups per CU.
// grid: workgroups share the ceil(N / RT) row tiles in contiguous ranges.
// ------------------------------------------------------------------------------------------------
template <int RT, int UNR, int MP = 1>
__global__ void __launch_bounds__(256) k_down_direct(GemvArgs a) {
    __shared__ float red[2][4][RT * MP];
    const int K = a.K, n_chunks = K >> 3, M = a.m_rows;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wg = blockIdx.x, nwg = gridDim.x;
    const int n_tiles = (a.N + RT - 1) / RT;
    const int t_lo = (int)(((unsigned)n_tiles * (unsigned)wg) / (unsigned)nwg), t_hi = (int)(((unsigned)n_tiles * (unsigned)(wg + 1)) / (unsigned)nwg);
    const int c0 = wave * 64 + lane, cstride = 256;
    // token row m reads its own activation row; a row past the call's count reads row 0 again and is never written
    const float4 *x4[MP];
#pragma unroll
    for (int m = 0; m < MP; ++m) x4[m] = reinterpret_cast<const float4 *>(a.x_in + (size_t)(m < M ? m : 0) * K);
    int parity = 0;
    for (int t = t_lo; t < t_hi; ++t) {
        float acc[RT][MP], epi[RT][MP];
        const uint4 *wp[RT];
#pragma unroll
        for (int r = 0; r < RT; ++r) {
            const int row = min(t * RT + r, a.N - 1);
            wp[r] = reinterpret_cast<const uint4 *>(a.W + (size_t)row * K);
#pragma unroll
            for (int m = 0; m < MP; ++m) {
                acc[r][m] = 0.f;
                epi[r][m] = a.h_out[(size_t)(m < M ? m : 0) * a.ld_h + row];   // requested ahead of the weight stream
            }
        }
#pragma unroll UNR
        for (int c = c0; c < n_chunks; c += cstride) {
            uint4 wv[RT];
#pragma unroll
            for (int r = 0; r < RT; ++r) wv[r] = load_stream(wp[r] + c);
            float4 xa[MP], xb[MP];
#pragma unroll
            for (int m = 0; m < MP; ++m) { xa[m] = x4[m][2 * c]; xb[m] = x4[m][2 * c + 1]; }
#pragma unroll
            for (int r = 0; r < RT; ++r) {
                const uint4 w = wv[r];
                const float w0 = bf16_lo(w.x), w1 = bf16_hi(w.x), w2 = bf16_lo(w.y), w3 = bf16_hi(w.y);
                const float w4 = bf16_lo(w.z), w5 = bf16_hi(w.z), w6 = bf16_lo(w.w), w7 = bf16_hi(w.w);
#pragma unroll
                for (int m = 0; m < MP; ++m) {
                    float v = acc[r][m];
                    v = fmaf(w0, xa[m].x, v); v = fmaf(w1, xa[m].y, v); v = fmaf(w2, xa[m].z, v); v = fmaf(w3, xa[m].w, v);
                    v = fmaf(w4, xb[m].x, v); v = fmaf(w5, xb[m].y, v); v = fmaf(w6, xb[m].z, v); v = fmaf(w7, xb[m].w, v);
                    acc[r][m] = v;
                }
            }
        }
#pragma unroll
        for (int r = 0; r < RT; ++r)
#pragma unroll
            for (int m = 0; m < MP; ++m) acc[r][m] = wave_sum(acc[r][m]);
        if (lane == 0) {
#pragma unroll
            for (int r = 0; r < RT; ++r)
#pragma unroll
                for (int m = 0; m < MP; ++m) red[parity][wave][r * MP + m] = acc[r][m];
        }
        __syncthreads();
        if (tid == 0) {
#pragma unroll
            for (int r = 0; r < RT; ++r) {
                const int row = t * RT + r;
#pragma unroll
                for (int m = 0; m < MP; ++m)
                    if (row < a.N && m < M)
                        a.h_out[(size_t)m * a.ld_h + row] = epi[r][m] + (red[parity][0][r * MP + m] + red[parity][1][r * MP + m] +
                                                                        red[parity][2][r * MP + m] + red[parity][3][r * MP + m]);
            }
        }
        parity ^= 1;
    }
}

// ------------------------------------------------------------------------------------------------
// Split-K grouped-query decode attention in two kernels.
//
// k_attn_partial: grid (n_slices, n_kv_heads, n_rows), block 256.  A workgroup owns one KV head,
// one slice of the context and ALL query heads of that KV head's group, so every K/V byte is read
// once per row.  Both contractions run on the matrix cores (v_mfma_f32_16x16x32_bf16):
//   scores[token, head] = sum_d K[token, d] q[head, d]     A = K rows (16 tokens x 32 d, 16-byte
//                                                           loads straight from the cache),
//                                                           B = q as three bf16 planes (exact fp32)
//   out[d, head]        = sum_t V[t, d] p[head, t]          A = V, which the cache stores TRANSPOSED
//                                                           ([head_dim][position]) so that a lane's
//                                                           8 tokens are contiguous, B = p as three
//                                                           bf16 planes taken directly from the score
//                                                           accumulator registers (the token <-> k
//                                                           slot assignment is free as long as both
//                                                           operands agree)
// The softmax weights use the hardware exponential (__expf: v_exp_f32 after a multiply; relative error
// ~1e-6 for the arguments that matter, far inside the tolerance, an order of magnitude fewer instructions).
// A wave handles 16 tokens per pass with an online softmax; the four waves are merged through LDS
// and the workgroup writes one partial record per query head: [m, l, 0, 0, acc[HD]] fp32.
//
// k_attn_combine: grid (n_q_heads, n_rows), block 256: merges the slices of one head.
// ------------------------------------------------------------------------------------------------
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));

struct AttnArgs {
    const float *qbuf;             // [rows, n_q*hd] fp32, rotated
    const uint16_t *kcache;        // [layer][slot][kv_head][position][hd] bf16
    const uint16_t *vcache;        // [layer][slot][kv_head][hd][position] bf16
    float *partials;               // [rows, n_q, n_slices, hd+4]
    float *out;                    // [rows, n_q*hd] fp32
    const int *row_pos, *row_slot, *row_bad;
    int n_q, n_kv, max_ctx, max_seqs, layer, n_slices;
    int n_rows;                    // token rows in the call (k_attn_partial_rows)
    int slot_split;                // k_attn_span: workgroups per sequence, slice and KV head
    const int4 *seq_info;          // per sequence {first row, end row, cache slot, first row's position}, first row < 0: invalid (k_attn_span)
};

constexpr int ATT_GMAX = 8;       // query heads per kv head, at most
constexpr int ATT_SMAX = 192;     // context slices, at most (a multiple of 64: the merge gives each lane ATT_SMAX / 64 of them)
constexpr int ATT_WT = 16;        // tokens per wave and pass
constexpr int ATT_BT = 64;        // tokens per workgroup and pass

// split 8 fp32 values into three bf16x8 planes whose sum is exact
__device__ __forceinline__ void split3(const float (&x)[8], bf16x8_t (&pl)[3]) {
    uint32_t w0[4], w1[4], w2[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const float a = x[2 * i], b = x[2 * i + 1];
        w0[i] = pack_bf16x2(a, b);
        const float ra = a - bf16_lo(w0[i]), rb = b - bf16_hi(w0[i]);
        w1[i] = pack_bf16x2(ra, rb);
        w2[i] = pack_bf16x2(ra - bf16_lo(w1[i]), rb - bf16_hi(w1[i]));
    }
    pl[0] = __builtin_bit_cast(bf16x8_t, make_uint4(w0[0], w0[1], w0[2], w0[3]));
    pl[1] = __builtin_bit_cast(bf16x8_t, make_uint4(w1[0], w1[1], w1[2], w1[3]));
    pl[2] = __builtin_bit_cast(bf16x8_t, make_uint4(w2[0], w2[1], w2[2], w2[3]));
}

template <int HD>
__host__ __device__ constexpr size_t attn_lds_bytes(int G = ATT_GMAX) { return (size_t)(4 * G * (HD + 4) + 2 * 4 * 16) * 4; }

// Cache operands of one wave pass (ATT_WT = 16 tokens from t0): K rows as the A operand of the score
// contraction, V^T rows as the A operand of the output contraction.  The loads are unconditional:
// positions are clamped into the cache row (max_ctx is a multiple of 8, so a group of 4 positions
// that starts at or before max_ctx - 4 ends inside it) and a clamped lane just fetches a duplicate.
// Which tokens count is decided later by masks, once the row's context length has arrived; without
// branches around them the compiler issues all loads back to back and waits once.
template <int HD>
struct AttnTile {
    uint4 k[HD / 32];
    uint2 v[HD / 16];
    __device__ __forceinline__ void load(const uint16_t *Kp, const uint16_t *Vp, int t0, int max_ctx, int j, int kg) {
        const int tok = min(t0 + j, max_ctx - 1);
#pragma unroll
        for (int ds = 0; ds < HD / 32; ++ds)
            k[ds] = *reinterpret_cast<const uint4 *>(Kp + (size_t)tok * HD + 32 * ds + 8 * kg);
        const int tv = min(t0 + 4 * kg, max_ctx - 4);
#pragma unroll
        for (int db = 0; db < HD / 16; ++db)
            v[db] = *reinterpret_cast<const uint2 *>(Vp + (size_t)(16 * db + j) * max_ctx + tv);
    }
};

// One (context slice, kv head, token row) unit.  Slice s covers positions [s*C, (s+1)*C) with C fixed
// by max_ctx and the slice count, NOT by the row's context length: the addresses of the first pass
// are known at launch, so the row table, q, K and V are all requested at once and the unit pays one
// memory round trip instead of three dependent ones.  Slices at or past the context length write
// nothing; attn_combine_unit derives the same slice length and reads only the slices before it.
// UPFRONT = false gives that up: the unit first waits for the row's position and leaves before
// requesting anything when its slice lies past the context.  With UPFRONT every launch reads K and V
// of ALL slices up to max_ctx, whatever the context is; that is the better trade while a layer's cache
// is a few MB (the 1.5B and 7B shapes at 4608 positions: 4.7 and 9.4 MB), and a poor one for a large
// cache (eight KV heads at 9216 positions: 37.7 MB per layer, 12.7 us at a context of 1000).
// ONEPASS: the host promises that a slice is one 64-position pass (C == ATT_BT); the unit then keeps no
// second tile and builds q's bf16 planes d step by d step, which brings it under a third of a SIMD's
// registers (more resident workgroups: a long cache is a throughput problem, not a latency one).
template <int HD, bool UPFRONT = true, bool ONEPASS = false>
__device__ __forceinline__ void attn_partial_unit(const AttnArgs &a, unsigned char *smem, int split, int S, int kvh, int row) {
    constexpr int NDS = HD / 32;       // 32-wide d steps of the score contraction
    constexpr int NDB = HD / 16;       // 16-wide d blocks of the output
    constexpr int PS = HD + 4;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int j = lane & 15, kg = lane >> 4;
    const int G = a.n_q / a.n_kv;

    // a small footprint matters: eight KV heads at 9216 positions are 1152 workgroups, one round only if a CU
    // holds five of them
    float (*m_lds)[16] = reinterpret_cast<float (*)[16]>(smem);                         // [4 waves][16 columns]
    float (*l_lds)[16] = m_lds + 4;
    float *acc_lds = reinterpret_cast<float *>(smem + (size_t)2 * 4 * 16 * 4);          // [4 waves][G heads][HD+4]

    int C = (a.max_ctx + S - 1) / S;
    C = ((C + ATT_BT - 1) / ATT_BT) * ATT_BT;
    const int t_begin = split * C;
    // with one cache slot the slot index needs no load; otherwise clamp it so that a row the
    // validation rejected (its slot is then stored as 0 anyway) can never address outside the cache
    int slot = 0;
    if (a.max_seqs > 1) slot = min(max(a.row_slot[row], 0), a.max_seqs - 1);
    const int bad = a.row_bad[row];
    const int pos = a.row_pos[row];
    const size_t kv_base = (((size_t)a.layer * a.max_seqs + slot) * a.n_kv + kvh) * (size_t)a.max_ctx * HD;
    const uint16_t *Kp = a.kcache + kv_base;      // [position][hd]
    const uint16_t *Vp = a.vcache + kv_base;      // [hd][position]
    const float scale = 1.0f / sqrtf((float)HD);
    if (!UPFRONT) {
        if (t_begin >= (bad ? 0 : pos + 1)) return;
    }

    // lanes j >= G have no head: they fetch head G-1 again and are cleared after the wait
    float4 qraw[NDS][2];
    {
        const float4 *qp = reinterpret_cast<const float4 *>(a.qbuf + ((size_t)row * a.n_q + kvh * G + min(j, G - 1)) * HD + 8 * kg);
#pragma unroll
        for (int ds = 0; ds < NDS; ++ds) { qraw[ds][0] = qp[8 * ds]; qraw[ds][1] = qp[8 * ds + 1]; }
    }
    AttnTile<HD> cur;
    cur.load(Kp, Vp, t_begin + wave * ATT_WT, a.max_ctx, j, kg);
    __builtin_amdgcn_sched_barrier(0);             // every request is in flight before anything waits

    const int ctx = bad ? 0 : pos + 1;
    const int t_end = min(ctx, t_begin + C);
    if (t_begin >= t_end) return;                  // nothing of this slice is in the context: the merge skips it too

    // q of head j as the B operand of the score contraction: three exact bf16 planes per d step
    auto q_planes = [&](int ds, bf16x8_t (&out)[3]) {
        const float4 x0 = qraw[ds][0], x1 = qraw[ds][1];
        float qv[8] = {x0.x, x0.y, x0.z, x0.w, x1.x, x1.y, x1.z, x1.w};
        if (j >= G) {
#pragma unroll
            for (int e = 0; e < 8; ++e) qv[e] = 0.f;
        }
        split3(qv, out);
    };
    bf16x8_t qB[ONEPASS ? 1 : NDS][3];
    if (!ONEPASS) {
#pragma unroll
        for (int ds = 0; ds < NDS; ++ds) q_planes(ds, qB[ds]);
    }

    float m_run = -INFINITY, l_run = 0.f;          // head j (replicated over the four kg groups)
    f32x4_t acc[NDB];                              // out[d = 16 db + 4 kg + r][head j]
#pragma unroll
    for (int db = 0; db < NDB; ++db) acc[db] = (f32x4_t){0.f, 0.f, 0.f, 0.f};

    for (int t0 = t_begin + wave * ATT_WT; t0 < t_end; t0 += ATT_BT) {
        AttnTile<HD> nxt;
        const bool more = !ONEPASS && t0 + ATT_BT < t_end;
        if (more) nxt.load(Kp, Vp, t0 + ATT_BT, a.max_ctx, j, kg);
        // ---- scores of 16 tokens; lane holds tokens t0 + 4 kg + r of head j.
        // Positions at or past t_end may hold anything (a rejected step's rows, never-written memory):
        // their scores are replaced, not scaled.
        f32x4_t sc = (f32x4_t){0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ds = 0; ds < NDS; ++ds) {
            const bf16x8_t A = __builtin_bit_cast(bf16x8_t, cur.k[ds]);
            if (ONEPASS) {
                bf16x8_t qb[3];
                q_planes(ds, qb);
#pragma unroll
                for (int pl = 2; pl >= 0; --pl) sc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(A, qb[pl], sc, 0, 0, 0);
            } else {
#pragma unroll
                for (int pl = 2; pl >= 0; --pl) sc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(A, qB[ds][pl], sc, 0, 0, 0);
            }
        }
        float mx = -INFINITY;
        const int tok_lo = t0 + 4 * kg;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const float v = tok_lo + r < t_end ? sc[r] * scale : -INFINITY;
            sc[r] = v;
            mx = fmaxf(mx, v);
        }
        mx = fmaxf(mx, __shfl_xor(mx, 16, RS_WAVE));
        mx = fmaxf(mx, __shfl_xor(mx, 32, RS_WAVE));
        const float m_new = fmaxf(m_run, mx);                         // finite: the pass has at least one valid token
        const float alpha = (m_run == -INFINITY) ? 0.f : __expf(m_run - m_new);
        m_run = m_new;
        l_run *= alpha;
#pragma unroll
        for (int db = 0; db < NDB; ++db) { acc[db][0] *= alpha; acc[db][1] *= alpha; acc[db][2] *= alpha; acc[db][3] *= alpha; }
        // ---- P V: k slot (kg, r) is token t0 + 4 kg + r; slots (kg, 4..7) are unused (zero on both sides)
        float pv[8];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const float p = (sc[r] == -INFINITY) ? 0.f : __expf(sc[r] - m_new);
            pv[r] = p; pv[4 + r] = 0.f;
            l_run += p;
        }
        bf16x8_t pB[3];
        split3(pv, pB);
#pragma unroll
        for (int db = 0; db < NDB; ++db) {
            // clear the V columns of positions at or past t_end (0 * NaN would poison the sum)
            uint2 lo = cur.v[db];
            if (tok_lo + 3 >= t_end) {
                if (tok_lo + 1 >= t_end) lo.x &= 0x0000ffffu;
                if (tok_lo + 2 >= t_end) lo.y = 0; else if (tok_lo + 3 >= t_end) lo.y &= 0x0000ffffu;
                if (tok_lo >= t_end) lo.x = 0;
            }
            const bf16x8_t A = __builtin_bit_cast(bf16x8_t, make_uint4(lo.x, lo.y, 0u, 0u));
#pragma unroll
            for (int pl = 2; pl >= 0; --pl) acc[db] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(A, pB[pl], acc[db], 0, 0, 0);
        }
        if (more) cur = nxt;
    }
    // l_run so far covers this lane's own tokens: add the other three kg groups
    l_run += __shfl_xor(l_run, 16, RS_WAVE);
    l_run += __shfl_xor(l_run, 32, RS_WAVE);

    // ---- merge the four waves
    if (j < G) {
#pragma unroll
        for (int db = 0; db < NDB; ++db)
            *reinterpret_cast<float4 *>(&acc_lds[(size_t)(wave * G + j) * PS + 16 * db + 4 * kg]) = make_float4(acc[db][0], acc[db][1], acc[db][2], acc[db][3]);
    }
    if (kg == 0) { m_lds[wave][j] = m_run; l_lds[wave][j] = l_run; }
    __syncthreads();
    // one float4 of one head per thread: G * HD / 4 items (224 for seven heads of 128 channels)
    for (int i = tid; i < G * (HD / 4); i += 256) {
        const int g = i / (HD / 4), d = 4 * (i - g * (HD / 4));
        const float m0 = m_lds[0][g], m1 = m_lds[1][g], m2 = m_lds[2][g], m3 = m_lds[3][g];
        const float M = fmaxf(fmaxf(m0, m1), fmaxf(m2, m3));
        float L = 0.f;
        float4 O = make_float4(0.f, 0.f, 0.f, 0.f);
        if (M > -INFINITY) {
            const float w0 = m0 > -INFINITY ? __expf(m0 - M) : 0.f, w1 = m1 > -INFINITY ? __expf(m1 - M) : 0.f;
            const float w2 = m2 > -INFINITY ? __expf(m2 - M) : 0.f, w3 = m3 > -INFINITY ? __expf(m3 - M) : 0.f;
            L = l_lds[0][g] * w0 + l_lds[1][g] * w1 + l_lds[2][g] * w2 + l_lds[3][g] * w3;
            const float4 a0 = *reinterpret_cast<const float4 *>(&acc_lds[(size_t)(0 * G + g) * PS + d]);
            const float4 a1 = *reinterpret_cast<const float4 *>(&acc_lds[(size_t)(1 * G + g) * PS + d]);
            const float4 a2 = *reinterpret_cast<const float4 *>(&acc_lds[(size_t)(2 * G + g) * PS + d]);
            const float4 a3 = *reinterpret_cast<const float4 *>(&acc_lds[(size_t)(3 * G + g) * PS + d]);
            O.x = a0.x * w0 + a1.x * w1 + a2.x * w2 + a3.x * w3;
            O.y = a0.y * w0 + a1.y * w1 + a2.y * w2 + a3.y * w3;
            O.z = a0.z * w0 + a1.z * w1 + a2.z * w2 + a3.z * w3;
            O.w = a0.w * w0 + a1.w * w1 + a2.w * w2 + a3.w * w3;
        }
        float *p = a.partials + (((size_t)row * a.n_q + kvh * G + g) * S + split) * PS;
        *reinterpret_cast<float4 *>(p + 4 + d) = O;
        if (d == 0) { p[0] = M; p[1] = L; }
    }
}

template <int HD, bool UPFRONT, bool ONEPASS>
__global__ void __launch_bounds__(256, ONEPASS ? 3 : 1) k_attn_partial(AttnArgs a) {
    extern __shared__ __align__(16) unsigned char smem[];
    attn_partial_unit<HD, UPFRONT, ONEPASS>(a, smem, blockIdx.x, gridDim.x, blockIdx.y, blockIdx.z);
}

// ------------------------------------------------------------------------------------------------
// k_attn_partial_rows: the same partial records for a call with several token rows (catch-up spans).
// grid (n_slices, n_kv_heads, ceil(row slots / W)), block 64 W with W = 1..4 waves, no LDS.  The 16 columns of the
// matrix-core tiles carry RP = 16 / G token rows at once (G = query heads per KV head): column
// rr * G + gh is head gh of the rr-th row of the wave's row slot, so one K/V tile serves RP rows.
// A wave owns one row slot (RP consecutive rows) and one context slice, walks the slice in passes of
// 64 positions with an online softmax per column, and writes its columns' records itself; the
// waves of a workgroup hold neighbouring row slots of the SAME slice, so their K/V requests meet in
// the CU's cache and HBM is read once per slice.  Rows of one slot that belong to different
// sequences (different cache slots) are taken in separate turns.  Causality is per column: row r
// attends to positions 0..pos[r].
// ------------------------------------------------------------------------------------------------
// MINW: waves per SIMD the register allocation must allow.  1 (243 + 44 registers) schedules best and wins
// while all workgroups are resident anyway; 2 (243 registers, none spilled) wins on a large cache, where
// the number of resident workgroups bounds the kernel (eight KV heads, 5000 positions, 2 rows: 12.3 -> 10.4 us).
template <int HD, int MINW>
__global__ void __launch_bounds__(256, MINW) k_attn_partial_rows(AttnArgs a) {
    constexpr int NDS = HD / 32, NDB = HD / 16, PS = HD + 4;
    const int split = blockIdx.x, S = gridDim.x, kvh = blockIdx.y;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int j = lane & 15, kg = lane >> 4;
    const int G = a.n_q / a.n_kv, RP = 16 / G;
    const int rr = j / G, gh = j - rr * G;                    // this lane's column: row rr of the slot, head gh
    int C = (a.max_ctx + S - 1) / S;
    C = ((C + 63) / 64) * 64;
    const int t_begin = split * C;
    const float scale = 1.0f / sqrtf((float)HD);
    const int slot_first = (blockIdx.z * (blockDim.x >> 6) + wave) * RP, slot_end = min(slot_first + RP, a.n_rows);

    for (int r0 = slot_first; r0 < slot_end;) {
        // a turn: the rows r0 .. r1-1 of the slot that share r0's cache slot (and are valid)
        if (a.row_bad[r0]) { ++r0; continue; }
        const int kv_slot = min(max(a.row_slot[r0], 0), a.max_seqs - 1);
        int r1 = r0 + 1;
        while (r1 < slot_end && !a.row_bad[r1] && a.row_slot[r1] == a.row_slot[r0]) ++r1;
        const int my_row = r0 + rr;                            // valid column iff rr < RP, my_row < r1
        const bool col_ok = rr < RP && my_row < r1;
        const int ctx_col = col_ok ? a.row_pos[my_row] + 1 : 0;
        const int ctx_max = a.row_pos[r1 - 1] + 1;             // positions grow with the row inside a span
        const int t_end = min(ctx_max, t_begin + C), t_end_col = min(ctx_col, t_begin + C);
        if (t_begin < t_end) {
            const size_t kv_base = (((size_t)a.layer * a.max_seqs + kv_slot) * a.n_kv + kvh) * (size_t)a.max_ctx * HD;
            const uint16_t *Kp = a.kcache + kv_base, *Vp = a.vcache + kv_base;
            bf16x8_t qB[NDS][3];
            {
                const float4 *qp = reinterpret_cast<const float4 *>(a.qbuf + ((size_t)(col_ok ? my_row : r0) * a.n_q + kvh * G + (col_ok ? gh : 0)) * HD + 8 * kg);
#pragma unroll
                for (int ds = 0; ds < NDS; ++ds) {
                    const float4 x0 = qp[8 * ds], x1 = qp[8 * ds + 1];
                    float qv[8] = {x0.x, x0.y, x0.z, x0.w, x1.x, x1.y, x1.z, x1.w};
                    if (!col_ok) {
#pragma unroll
                        for (int e = 0; e < 8; ++e) qv[e] = 0.f;
                    }
                    split3(qv, qB[ds]);
                }
            }
            float m_run = -INFINITY, l_run = 0.f;
            f32x4_t acc[NDB];
#pragma unroll
            for (int db = 0; db < NDB; ++db) acc[db] = (f32x4_t){0.f, 0.f, 0.f, 0.f};
            for (int t0 = t_begin; t0 < t_end; t0 += 64) {
                // K rows (A operand of the scores) and V^T rows (A operand of the output); positions clamped into the cache row
                uint4 kk[4][NDS];
#pragma unroll
                for (int tb = 0; tb < 4; ++tb) {
                    const int tok = min(t0 + 16 * tb + j, a.max_ctx - 1);
#pragma unroll
                    for (int ds = 0; ds < NDS; ++ds) kk[tb][ds] = *reinterpret_cast<const uint4 *>(Kp + (size_t)tok * HD + 32 * ds + 8 * kg);
                }
                uint2 vv[2][NDB][2];
#pragma unroll
                for (int ks = 0; ks < 2; ++ks)
#pragma unroll
                    for (int db = 0; db < NDB; ++db)
#pragma unroll
                        for (int hf = 0; hf < 2; ++hf) {
                            const int tv = min(t0 + 32 * ks + 16 * hf + 4 * kg, a.max_ctx - 4);
                            vv[ks][db][hf] = *reinterpret_cast<const uint2 *>(Vp + (size_t)(16 * db + j) * a.max_ctx + tv);
                        }
                // scores: lane holds positions t0 + 16 tb + 4 kg + r of its column
                f32x4_t sc[4];
                float mx = -INFINITY;
#pragma unroll
                for (int tb = 0; tb < 4; ++tb) {
                    sc[tb] = (f32x4_t){0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int ds = 0; ds < NDS; ++ds) {
                        const bf16x8_t A = __builtin_bit_cast(bf16x8_t, kk[tb][ds]);
#pragma unroll
                        for (int pl = 2; pl >= 0; --pl) sc[tb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(A, qB[ds][pl], sc[tb], 0, 0, 0);
                    }
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        const float v = (t0 + 16 * tb + 4 * kg + r) < t_end_col ? sc[tb][r] * scale : -INFINITY;
                        sc[tb][r] = v;
                        mx = fmaxf(mx, v);
                    }
                }
                mx = fmaxf(mx, __shfl_xor(mx, 16, RS_WAVE));
                mx = fmaxf(mx, __shfl_xor(mx, 32, RS_WAVE));
                const float m_new = fmaxf(m_run, mx);              // may stay -inf for a column without positions here
                const float alpha = (m_run == -INFINITY) ? 0.f : __expf(m_run - m_new);
                m_run = m_new;
                l_run *= alpha;
#pragma unroll
                for (int db = 0; db < NDB; ++db) { acc[db][0] *= alpha; acc[db][1] *= alpha; acc[db][2] *= alpha; acc[db][3] *= alpha; }
#pragma unroll
                for (int ks = 0; ks < 2; ++ks) {
                    float pv[8];
#pragma unroll
                    for (int hf = 0; hf < 2; ++hf)
#pragma unroll
                        for (int r = 0; r < 4; ++r) {
                            const float s_ = sc[2 * ks + hf][r];
                            const float p = (s_ == -INFINITY) ? 0.f : __expf(s_ - m_new);
                            pv[4 * hf + r] = p;
                            l_run += p;
                        }
                    bf16x8_t pB[3];
                    split3(pv, pB);
                    const int tok_lo = t0 + 32 * ks + 4 * kg, tok_hi = tok_lo + 16;
#pragma unroll
                    for (int db = 0; db < NDB; ++db) {
                        // positions at or past the turn's longest context may hold anything: clear their V columns
                        uint2 lo = vv[ks][db][0], hi = vv[ks][db][1];
                        if (tok_lo + 3 >= t_end) {
                            if (tok_lo + 1 >= t_end) lo.x &= 0x0000ffffu;
                            if (tok_lo + 2 >= t_end) lo.y = 0; else if (tok_lo + 3 >= t_end) lo.y &= 0x0000ffffu;
                            if (tok_lo >= t_end) lo.x = 0;
                        }
                        if (tok_hi + 3 >= t_end) {
                            if (tok_hi + 1 >= t_end) hi.x &= 0x0000ffffu;
                            if (tok_hi + 2 >= t_end) hi.y = 0; else if (tok_hi + 3 >= t_end) hi.y &= 0x0000ffffu;
                            if (tok_hi >= t_end) hi.x = 0;
                        }
                        const bf16x8_t A = __builtin_bit_cast(bf16x8_t, make_uint4(lo.x, lo.y, hi.x, hi.y));
#pragma unroll
                        for (int pl = 2; pl >= 0; --pl) acc[db] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(A, pB[pl], acc[db], 0, 0, 0);
                    }
                }
            }
            l_run += __shfl_xor(l_run, 16, RS_WAVE);
            l_run += __shfl_xor(l_run, 32, RS_WAVE);
            if (col_ok && t_begin < t_end_col) {
                float *p = a.partials + (((size_t)my_row * a.n_q + kvh * G + gh) * S + split) * PS;
#pragma unroll
                for (int db = 0; db < NDB; ++db)
                    *reinterpret_cast<float4 *>(p + 4 + 16 * db + 4 * kg) = make_float4(acc[db][0], acc[db][1], acc[db][2], acc[db][3]);
                if (kg == 0) { p[0] = m_run; p[1] = l_run; }
            }
        }
        r0 = r1;
    }
}

// ------------------------------------------------------------------------------------------------
// k_attn_span: the partial records of k_attn_partial_rows for calls whose slices are one 64-position
// pass, with the K/V tile shared through LDS.  grid (n_slices, n_kv_heads, n_seqs * ZS), block 256
// (ZS = a.slot_split workgroups share a sequence's row slots: workgroup zs takes the slots w + 4 zs, + 4 ZS, ...
// of wave w; long spans are spread over more CUs that way).
// A workgroup owns one context slice of one KV head of one SEQUENCE of the call and all of that
// sequence's rows: the four waves fetch the slice's K rows (64 x HD, contiguous in the cache) and V^T
// rows (HD pieces of 128 bytes) once, with whole-line 16-byte loads, into LDS; then wave w takes the row
// slots w, w + 4, ... (a slot = 16 / G consecutive rows in the 16 matrix-core columns, as above) and reads
// its operands from LDS.  Measured against k_attn_partial_rows, where every wave fetches the tile
// itself with one 16-byte (K) or 8-byte (V) piece per lane and row, 16 cache lines per instruction:
// that kernel is bound by the CU's vector-memory request rate (its loads alone take as long as the
// whole kernel) and re-reads the tile once per four slots.
// V positions at or past the sequence's last row may hold anything (never written): they are cleared
// when the tile is written to LDS; K rows there only feed scores that the causal mask discards.
// ------------------------------------------------------------------------------------------------
template <int HD>
__host__ __device__ constexpr size_t attn_span_lds_bytes() { return (size_t)64 * (HD * 2 + 16) + (size_t)HD * (64 * 2 + 16); }

template <int HD>
__global__ void __launch_bounds__(256) k_attn_span(AttnArgs a) {
    constexpr int NDS = HD / 32, NDB = HD / 16, PS = HD + 4;
    constexpr int KP = HD * 2 + 16, VP = 64 * 2 + 16;           // LDS row pitches in bytes (padded against bank conflicts)
    constexpr int KQ = 64 * HD * 2 / 4096, VQ = HD * 128 / 4096; // 16-byte loads per thread for each tile
    extern __shared__ __align__(16) unsigned char smem[];
    unsigned char *sK = smem, *sV = smem + (size_t)64 * KP;
    const int split = blockIdx.x, S = gridDim.x, kvh = blockIdx.y;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int j = lane & 15, kg = lane >> 4;
    const int G = a.n_q / a.n_kv, RP = 16 / G;
    const int rr = j / G, gh = j - rr * G;                     // this lane's column: row rr of the slot, head gh
    const int ZS = a.slot_split > 1 ? a.slot_split : 1, zs = blockIdx.z % ZS;
    const int4 info = a.seq_info[blockIdx.z / ZS];             // {first row, end row, cache slot, position of the first row}, first row < 0: skip
    if (info.x < 0) return;
    const int r_lo = info.x, r_hi = info.y, t_begin = split * 64;
    const int ctx_max = info.w + (r_hi - r_lo);                // positions the last row attends to
    const int n_slots = (r_hi - r_lo + RP - 1) / RP;
    if (t_begin >= ctx_max || 4 * zs >= n_slots) return;
    const int kv_slot = min(max(info.z, 0), a.max_seqs - 1);
    const size_t kv_base = (((size_t)a.layer * a.max_seqs + kv_slot) * a.n_kv + kvh) * (size_t)a.max_ctx * HD;
    const float scale = 1.0f / sqrtf((float)HD);

    // the tile: requests first, the first slot's q next, then the LDS writes
    uint4 kq[KQ], vq[VQ];
#pragma unroll
    for (int i = 0; i < KQ; ++i) {
        const int off = (tid + 256 * i) * 16, row = off / (HD * 2), col = off - row * (HD * 2);
        const int tok = min(t_begin + row, a.max_ctx - 1);
        kq[i] = *reinterpret_cast<const uint4 *>(reinterpret_cast<const unsigned char *>(a.kcache + kv_base + (size_t)tok * HD) + col);
    }
#pragma unroll
    for (int i = 0; i < VQ; ++i) {
        const int off = (tid + 256 * i) * 16, d = off >> 7, c8 = (off & 127) >> 4;
        const int tv = min(t_begin + 8 * c8, a.max_ctx - 8);
        vq[i] = *reinterpret_cast<const uint4 *>(a.vcache + kv_base + (size_t)d * a.max_ctx + tv);
    }
    auto load_q = [&](int slot, float4 (&q)[NDS][2]) {
        const int r0 = r_lo + slot * RP, my_row = r0 + rr;
        const bool ok = rr < RP && my_row < r_hi;
        const float4 *qp = reinterpret_cast<const float4 *>(a.qbuf + ((size_t)(ok ? my_row : r_lo) * a.n_q + kvh * G + (ok ? gh : 0)) * HD + 8 * kg);
#pragma unroll
        for (int ds = 0; ds < NDS; ++ds) { q[ds][0] = qp[8 * ds]; q[ds][1] = qp[8 * ds + 1]; }
    };
    float4 qn[NDS][2];
    if (wave + 4 * zs < n_slots) load_q(wave + 4 * zs, qn);
#pragma unroll
    for (int i = 0; i < KQ; ++i) {
        const int off = (tid + 256 * i) * 16, row = off / (HD * 2), col = off - row * (HD * 2);
        *reinterpret_cast<uint4 *>(sK + (size_t)row * KP + col) = kq[i];
    }
#pragma unroll
    for (int i = 0; i < VQ; ++i) {
        const int off = (tid + 256 * i) * 16, d = off >> 7, c8 = (off & 127) >> 4;
        const int t0 = t_begin + 8 * c8;                       // position of the first of this piece's 8 values
        uint4 v = vq[i];
        if (t0 + 7 >= ctx_max) {
            uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                if (t0 + 2 * e >= ctx_max) w[e] = 0;
                else if (t0 + 2 * e + 1 >= ctx_max) w[e] &= 0x0000ffffu;
            }
            v = make_uint4(w[0], w[1], w[2], w[3]);
        }
        *reinterpret_cast<uint4 *>(sV + (size_t)d * VP + c8 * 16) = v;
    }
    __syncthreads();

    for (int slot = wave + 4 * zs; slot < n_slots; slot += 4 * ZS) {
        const int r0 = r_lo + slot * RP, my_row = r0 + rr;
        const bool col_ok = rr < RP && my_row < r_hi;
        const int ctx_col = col_ok ? info.w + (my_row - r_lo) + 1 : 0;
        const int t_end_col = min(ctx_col, t_begin + 64);
        bf16x8_t qB[NDS][3];
#pragma unroll
        for (int ds = 0; ds < NDS; ++ds) {
            float qv[8] = {qn[ds][0].x, qn[ds][0].y, qn[ds][0].z, qn[ds][0].w, qn[ds][1].x, qn[ds][1].y, qn[ds][1].z, qn[ds][1].w};
            if (!col_ok) {
#pragma unroll
                for (int e = 0; e < 8; ++e) qv[e] = 0.f;
            }
            split3(qv, qB[ds]);
        }
        if (slot + 4 * ZS < n_slots) load_q(slot + 4 * ZS, qn);   // the next slot's q is in flight during this slot's products
        // scores: lane holds positions t_begin + 16 tb + 4 kg + r of its column
        f32x4_t sc[4];
        float mx = -INFINITY;
#pragma unroll
        for (int tb = 0; tb < 4; ++tb) {
            sc[tb] = (f32x4_t){0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ds = 0; ds < NDS; ++ds) {
                const bf16x8_t A = __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const uint4 *>(sK + (size_t)(16 * tb + j) * KP + 64 * ds + 16 * kg));
#pragma unroll
                for (int pl = 2; pl >= 0; --pl) sc[tb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(A, qB[ds][pl], sc[tb], 0, 0, 0);
            }
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const float v = (t_begin + 16 * tb + 4 * kg + r) < t_end_col ? sc[tb][r] * scale : -INFINITY;
                sc[tb][r] = v;
                mx = fmaxf(mx, v);
            }
        }
        mx = fmaxf(mx, __shfl_xor(mx, 16, RS_WAVE));
        mx = fmaxf(mx, __shfl_xor(mx, 32, RS_WAVE));            // -inf for a column without positions in this slice
        float l_run = 0.f;
        f32x4_t acc[NDB];
#pragma unroll
        for (int db = 0; db < NDB; ++db) acc[db] = (f32x4_t){0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            float pv[8];
#pragma unroll
            for (int hf = 0; hf < 2; ++hf)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const float s_ = sc[2 * ks + hf][r];
                    const float p = (s_ == -INFINITY) ? 0.f : __expf(s_ - mx);
                    pv[4 * hf + r] = p;
                    l_run += p;
                }
            bf16x8_t pB[3];
            split3(pv, pB);
#pragma unroll
            for (int db = 0; db < NDB; ++db) {
                const unsigned char *vr = sV + (size_t)(16 * db + j) * VP + 64 * ks + 8 * kg;
                const uint2 lo = *reinterpret_cast<const uint2 *>(vr), hi = *reinterpret_cast<const uint2 *>(vr + 32);
                const bf16x8_t A = __builtin_bit_cast(bf16x8_t, make_uint4(lo.x, lo.y, hi.x, hi.y));
#pragma unroll
                for (int pl = 2; pl >= 0; --pl) acc[db] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(A, pB[pl], acc[db], 0, 0, 0);
            }
        }
        l_run += __shfl_xor(l_run, 16, RS_WAVE);
        l_run += __shfl_xor(l_run, 32, RS_WAVE);
        if (col_ok && t_begin < t_end_col) {
            float *p = a.partials + (((size_t)my_row * a.n_q + kvh * G + gh) * S + split) * PS;
#pragma unroll
            for (int db = 0; db < NDB; ++db)
                *reinterpret_cast<float4 *>(p + 4 + 16 * db + 4 * kg) = make_float4(acc[db][0], acc[db][1], acc[db][2], acc[db][3]);
            if (kg == 0) { p[0] = mx; p[1] = l_run; }
        }
    }
}

// merge the context slices of one (row, query head); 256 threads = (float4 columns) x (slice groups).
// DQ workgroups share a head, each taking HD / DQ output columns: a head's records are S * (HD+4) floats
// (38 KB for 72 slices), and with one workgroup per head only n_q CUs pull them.
// smem: ATT_SMAX + 1024 floats
template <int HD>
__host__ __device__ constexpr size_t attn_combine_lds_bytes() { return (size_t)(ATT_SMAX + 1024) * 4; }

// SMAX: the slice count this instantiation is unrolled for (n_slices <= SMAX <= ATT_SMAX, a multiple of 64)
template <int HD, int SMAX = ATT_SMAX, int DQ = 1>
__device__ __forceinline__ void attn_combine_unit(const AttnArgs &a, unsigned char *smem, int head, int row, int dq = 0) {
    static_assert(SMAX % 64 == 0 && SMAX <= ATT_SMAX, "whole slices per lane, inside the LDS weights array");
    static_assert(HD % (4 * DQ) == 0 && 256 % (HD / 4 / DQ) == 0, "whole float4 columns per workgroup");
    constexpr int PS = HD + 4, NQ = HD / 4 / DQ, NSG = 256 / NQ, NLD = (SMAX + NSG - 1) / NSG, HDB = HD / DQ;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int S = a.n_slices;
    float *w_sh = reinterpret_cast<float *>(smem);                               // [ATT_SMAX]
    float (*red)[HDB] = reinterpret_cast<float (*)[HDB]>(w_sh + ATT_SMAX);       // [NSG][HDB]: 1024 floats
    const float *pbase = a.partials + ((size_t)row * a.n_q + head) * S * PS;
    const int qd = tid % NQ, sg = tid / NQ;
    // slices that hold context: same slice length as attn_partial_unit
    int C = (a.max_ctx + S - 1) / S;
    C = ((C + ATT_BT - 1) / ATT_BT) * ATT_BT;
    // The records of all S slices are requested together with the row's position (one round trip instead of
    // two dependent ones); a slice past the context holds whatever an earlier call left there and is
    // replaced, never scaled, once the position has arrived.
    const int bad = a.row_bad[row], pos = a.row_pos[row];
    constexpr int NPL = SMAX / 64;                          // slices per lane (wave 0)
    float4 buf[NLD];
    float2 mlr[NPL];
#pragma unroll
    for (int k = 0; k < NLD; ++k) {
        const int s = sg + k * NSG;
        buf[k] = make_float4(0.f, 0.f, 0.f, 0.f);
        if (s < S) buf[k] = *reinterpret_cast<const float4 *>(pbase + (size_t)s * PS + 4 + dq * HDB + 4 * qd);
    }
    if (wave == 0) {
#pragma unroll
        for (int k = 0; k < NPL; ++k) {
            const int s = lane + 64 * k;
            mlr[k] = make_float2(0.f, 0.f);
            if (s < S) mlr[k] = *reinterpret_cast<const float2 *>(pbase + (size_t)s * PS);
        }
    }
    __builtin_amdgcn_sched_barrier(0);                      // every request is in flight before anything waits
    const int S_act = bad ? 0 : min(S, pos / C + 1);
#pragma unroll
    for (int k = 0; k < NLD; ++k)
        if (sg + k * NSG >= S_act) buf[k] = make_float4(0.f, 0.f, 0.f, 0.f);
    if (wave == 0) {
        float ms[NPL], ls[NPL], w[NPL];
        float mx = -INFINITY;
#pragma unroll
        for (int k = 0; k < NPL; ++k) {
            const int s = lane + 64 * k;
            ms[k] = -INFINITY; ls[k] = 0.f;
            if (s < S_act) { ls[k] = mlr[k].y; ms[k] = ls[k] > 0.f ? mlr[k].x : -INFINITY; }
            mx = fmaxf(mx, ms[k]);
        }
        const float M = wave_max(mx);
        float lsum = 0.f;
#pragma unroll
        for (int k = 0; k < NPL; ++k) {
            w[k] = ls[k] > 0.f ? __expf(ms[k] - M) : 0.f;
            lsum = fmaf(ls[k], w[k], lsum);
        }
        const float L = wave_sum(lsum);
#pragma unroll
        for (int k = 0; k < NPL; ++k) w_sh[lane + 64 * k] = L > 0.f ? w[k] / L : 0.f;
    }
    __syncthreads();
    float4 sum = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
    for (int k = 0; k < NLD; ++k) {
        const int s = sg + k * NSG;
        const float w = s < S_act ? w_sh[s] : 0.f;
        sum.x = fmaf(w, buf[k].x, sum.x); sum.y = fmaf(w, buf[k].y, sum.y); sum.z = fmaf(w, buf[k].z, sum.z); sum.w = fmaf(w, buf[k].w, sum.w);
    }
    *reinterpret_cast<float4 *>(&red[sg][4 * qd]) = sum;
    __syncthreads();
    if (tid < HDB) {
        float o = 0.f;
#pragma unroll
        for (int g = 0; g < NSG; ++g) o += red[g][tid];
        const size_t oi = ((size_t)row * a.n_q + head) * HD + dq * HDB + tid;
        a.out[oi] = o;
    }
}

// grid (n_q_heads, n_rows, DQ)
template <int HD, int SMAX, int DQ>
__global__ void __launch_bounds__(256) k_attn_combine(AttnArgs a) {
    extern __shared__ __align__(16) unsigned char smem[];
    attn_combine_unit<HD, SMAX, DQ>(a, smem, blockIdx.x, blockIdx.y, blockIdx.z);
}

}  // namespace rs
