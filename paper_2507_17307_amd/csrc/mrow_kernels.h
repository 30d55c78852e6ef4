// Multi-row kernels (2..128 token rows per call): the catch-up prefill of the
// tokens a model has not seen, and batched decode.  The weights are still read
// once per call, so the phases stay HBM-bound; the contraction over tokens runs
// on the matrix cores (v_mfma_f32_16x16x32_bf16, fp32 accumulate) so that ALU
// work never becomes the limiter.  Activations stay fp32 in memory; the consumer
// splits each value in registers into three bf16 planes (p0 = bf16(x), p1 =
// bf16(x - p0), p2 = x - p0 - p1, which is exact: 3 x 8 significant bits hold the
// 24 of an fp32) and multiplies each weight tile with all three, smallest first,
// so the product is that of the fp32 activation (4 bytes per element through the
// load path instead of the 6 of stored planes).
#pragma once

#include "device_utils.h"
#include "model_kernels.h"

namespace rs {

constexpr int ROWK_THREADS = 1024;     // one workgroup per token row in the two row kernels below
constexpr int KSPLIT_MAX = 8;

// x[i] (+ the other split-K partial sums of it): all requests are issued together, unconditionally
// (the split index is clamped, a duplicate is dropped by a select), so a row costs one round trip.
__device__ __forceinline__ float4 sum_splits4(const float *base, size_t i, int ksplit, size_t part_stride, float4 first) {
    float4 v[KSPLIT_MAX];
#pragma unroll
    for (int ks = 1; ks < KSPLIT_MAX; ++ks)
        v[ks] = *reinterpret_cast<const float4 *>(base + (size_t)min(ks, ksplit - 1) * part_stride + i);
#pragma unroll
    for (int ks = 1; ks < KSPLIT_MAX; ++ks)
        if (ks < ksplit) { first.x += v[ks].x; first.y += v[ks].y; first.z += v[ks].z; first.w += v[ks].w; }
    return first;
}

// RMSNorm of whole rows: grid n_out, block ROWK_THREADS; d a multiple of 4, at most 12 * ROWK_THREADS.
// src row = gather ? gather[blockIdx.x] : blockIdx.x; the normalised row goes to out32[blockIdx.x] as fp32 (the
// matrix-core kernels split it into bf16 planes themselves).
// part != null: the projection before this norm left its result as `ksplit` partial sums
// part[ks][row][d] (split over K across workgroups); they are added to the residual row here, in a
// fixed order, and the row is written back before it is normalised.
__global__ void __launch_bounds__(ROWK_THREADS)
k_rmsnorm_rows(float *__restrict__ h, const uint16_t *__restrict__ gain, float eps, int d,
               const int *__restrict__ gather, float *__restrict__ out32,
               const float *__restrict__ part, int ksplit, size_t part_stride) {
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int src = gather ? gather[blockIdx.x] : blockIdx.x;
    float *hr = h + (size_t)src * d;
    __shared__ float red_ss[ROWK_THREADS / 64];
    const int n4 = d >> 2;
    constexpr int NV = 3;
    float4 v[NV];
    uint2 gv[NV];
    float ss = 0.f;
#pragma unroll
    for (int k = 0; k < NV; ++k) {
        const int i4 = tid + k * ROWK_THREADS;
        v[k] = make_float4(0.f, 0.f, 0.f, 0.f); gv[k] = make_uint2(0, 0);
        if (i4 < n4) {
            v[k] = *reinterpret_cast<const float4 *>(hr + 4 * i4);
            gv[k] = *reinterpret_cast<const uint2 *>(gain + 4 * i4);
            if (part) {
                const float4 p0 = *reinterpret_cast<const float4 *>(part + (size_t)src * d + 4 * i4);
                float4 t = sum_splits4(part, (size_t)src * d + 4 * i4, ksplit, part_stride, p0);
                v[k].x += t.x; v[k].y += t.y; v[k].z += t.z; v[k].w += t.w;
                *reinterpret_cast<float4 *>(hr + 4 * i4) = v[k];
            }
        }
        ss = fmaf(v[k].x, v[k].x, ss); ss = fmaf(v[k].y, v[k].y, ss); ss = fmaf(v[k].z, v[k].z, ss); ss = fmaf(v[k].w, v[k].w, ss);
    }
    ss = wave_sum(ss);
    if (lane == 0) red_ss[wave] = ss;
    __syncthreads();
    float tot = 0.f;
#pragma unroll
    for (int w = 0; w < ROWK_THREADS / 64; ++w) tot += red_ss[w];
    const float inv = 1.0f / sqrtf(tot / (float)d + eps);
#pragma unroll
    for (int k = 0; k < NV; ++k) {
        const int i4 = tid + k * ROWK_THREADS;
        if (i4 >= n4) continue;
        const size_t o = (size_t)blockIdx.x * d + 4 * i4;
        *reinterpret_cast<float4 *>(out32 + o) = make_float4(v[k].x * (inv * bf16_lo(gv[k].x)), v[k].y * (inv * bf16_hi(gv[k].x)),
                                                             v[k].z * (inv * bf16_lo(gv[k].y)), v[k].w * (inv * bf16_hi(gv[k].y)));
    }
}

// Rotary embedding of q and k, KV-cache write, for every row: grid n_rows, block ROWK_THREADS.
struct RopeArgs {
    const float *qkv;              // [rows, (n_q+2 n_kv) hd] fp32, or `ksplit` partial sums of it, part_stride elements apart
    int ksplit; size_t part_stride;
    float *qbuf; uint16_t *kcache, *vcache;
    const float *rope_cos, *rope_sin;
    const int *row_pos, *row_slot, *row_bad;
    int n_q, n_kv, head_dim, max_ctx, max_seqs, layer;
};

__global__ void __launch_bounds__(ROWK_THREADS) k_rope_kv_rows(RopeArgs a) {
    const int r = blockIdx.x, tid = threadIdx.x;
    if (a.row_bad[r]) {
        for (int i = tid; i < a.n_q * a.head_dim; i += ROWK_THREADS) a.qbuf[(size_t)r * a.n_q * a.head_dim + i] = 0.f;
        return;
    }
    const int hd = a.head_dim, half = hd >> 1, pos = a.row_pos[r], slot = a.row_slot[r];
    const int n_qkv = (a.n_q + 2 * a.n_kv) * hd;
    const size_t xo = (size_t)r * n_qkv;
    const int ks_n = a.ksplit > 1 ? a.ksplit : 1;
    const float *cs = a.rope_cos + (size_t)pos * half, *sn = a.rope_sin + (size_t)pos * half;
    // four consecutive rotary pairs per thread (head_dim / 2 is a multiple of 4)
    for (int p4 = tid; p4 < (a.n_q + a.n_kv) * (half >> 2); p4 += ROWK_THREADS) {
        const int head = p4 / (half >> 2), i = (p4 - head * (half >> 2)) * 4;
        const size_t e0 = xo + head * hd + i;
        const float4 x0 = sum_splits4(a.qkv, e0, ks_n, a.part_stride, *reinterpret_cast<const float4 *>(a.qkv + e0));
        const float4 x1 = sum_splits4(a.qkv, e0 + half, ks_n, a.part_stride, *reinterpret_cast<const float4 *>(a.qkv + e0 + half));
        const float4 c = *reinterpret_cast<const float4 *>(cs + i), s = *reinterpret_cast<const float4 *>(sn + i);
        const float4 y0 = make_float4(x0.x * c.x - x1.x * s.x, x0.y * c.y - x1.y * s.y, x0.z * c.z - x1.z * s.z, x0.w * c.w - x1.w * s.w);
        const float4 y1 = make_float4(x1.x * c.x + x0.x * s.x, x1.y * c.y + x0.y * s.y, x1.z * c.z + x0.z * s.z, x1.w * c.w + x0.w * s.w);
        if (head < a.n_q) {
            float *q = a.qbuf + ((size_t)r * a.n_q + head) * hd;
            *reinterpret_cast<float4 *>(q + i) = y0; *reinterpret_cast<float4 *>(q + i + half) = y1;
        } else {
            const size_t base = ((((size_t)a.layer * a.max_seqs + slot) * a.n_kv + (head - a.n_q)) * a.max_ctx + pos) * hd;
            *reinterpret_cast<uint2 *>(a.kcache + base + i) = make_uint2(pack_bf16x2(y0.x, y0.y), pack_bf16x2(y0.z, y0.w));
            *reinterpret_cast<uint2 *>(a.kcache + base + i + half) = make_uint2(pack_bf16x2(y1.x, y1.y), pack_bf16x2(y1.z, y1.w));
        }
    }
    for (int p4 = tid; p4 < (a.n_kv * hd) >> 2; p4 += ROWK_THREADS) {
        const int p = p4 * 4, vh = p / hd, e = p - vh * hd;
        const size_t e0 = xo + (a.n_q + a.n_kv) * hd + p;
        const float4 x = sum_splits4(a.qkv, e0, ks_n, a.part_stride, *reinterpret_cast<const float4 *>(a.qkv + e0));
        const size_t base = (((size_t)a.layer * a.max_seqs + slot) * a.n_kv + vh) * (size_t)a.max_ctx * hd;
        uint16_t *vp = a.vcache + base + (size_t)e * a.max_ctx + pos;          // V is stored [hd][position]
        vp[0] = f32_to_bf16(x.x); vp[a.max_ctx] = f32_to_bf16(x.y); vp[2 * (size_t)a.max_ctx] = f32_to_bf16(x.z); vp[3 * (size_t)a.max_ctx] = f32_to_bf16(x.w);
    }
}

// ------------------------------------------------------------------------------------------------
// out[m, n] = sum_k X[m, k] W[n, k] for M <= 16*NB token rows.
// A workgroup of GEMM_NW waves owns R consecutive tiles of 16 output columns (for gate/up a tile is 16
// gate rows plus the 16 matching up rows of W) and ALL of K; wave w takes the k windows w, w+GEMM_NW,
// ... of 64 elements (more waves where a matrix has few tiles, so that enough requests are in flight).  Per window a wave requests
//   * its piece of X once: fp32, 16 tokens x 64 k per 16-token block, each lane the values of its
//     place in the B-operand layout of v_mfma_f32_16x16x32_bf16 (lane (i = lane % 16, g = lane / 16)
//     supplies the 8 consecutive k at 32 s + 8 g of token i), split into the three planes in
//     registers; the piece serves all R tiles, so X costs 2/R of the W bytes in L2 traffic (stored
//     planes cost 3/R: a 7B-shape call of 16 rows 4.84 -> 4.4 ms);
//   * the 16 x 64 piece of W of every tile it owns with coalesced 16-byte loads, eight lanes per
//     128-byte row piece (whole cache lines: on this chip 64-byte pieces, which the operand layout
//     would give directly, stream at 4.5 TB/s, 128-byte pieces at 6.2), parked in the wave's private
//     LDS area and read back in the A-operand layout.
// The requests of the next window are in flight while the current one is multiplied.  The per-wave
// 16x16 accumulators (lane holds D[4 g + r][token = lane % 16]) of a group meet in LDS; wave p sums
// and finishes tile-and-token-block pair p.  The launch makes every group resident at once, with the
// groups spread evenly over the CUs, because a CU draws at most ~30 GB/s (see launch_gemm).
// ------------------------------------------------------------------------------------------------
struct GemmArgs {
    const uint16_t *W; int N, K, M;       // M = valid token rows
    const float *X32;                     // activations: fp32 rows [.., K] (split into three bf16 planes in registers)
    float *act32;                         // gate/up: SwiGLU output rows [.., d_ffn] fp32
    float *out_f32; int ld_out;           // raw fp32 output [M, ld_out] (QKV)
    int yblocks;                          // > 1: the token rows are cut into yblocks blocks of 16*NB rows, each taken by its own
                                          //      workgroups (same weights; ids arranged so that they meet in one XCD's L2)
    int ksplit; size_t part_stride;       // > 1: K is split over workgroups too; split ks writes its partial sums to
    float *part;                          //      part[ks * part_stride + m * N + n] (QKV, O-proj, down) and the consumer adds them up
    float *h_out; int ld_h;               // residual accumulate
    int d_ffn;
    const float *seq_scale; SoftPartial *parts; float *logits; int n_parts;   // LM head
    int sample_on; unsigned long long sample_key;         // LM head: also track the arg max of logit + Gumbel noise
    const int *row_pos, *out_row;                         // sampling: position of the row that feeds output row m is row_pos[out_row[m]]
};

constexpr int GEMM_KW = 64;                       // k elements per window: K must be a multiple
constexpr int GEMM_PITCH = GEMM_KW * 2 + 16;      // bytes per parked row (padded against LDS bank conflicts)

template <int MODE, int NB, int R, int GEMM_NW>
__host__ __device__ constexpr size_t gemm_lds_bytes() {
    constexpr size_t nt = (MODE == G_GATEUP) ? 2 : 1;
    constexpr size_t park = (size_t)GEMM_NW * R * nt * 16 * GEMM_PITCH, meet = (size_t)GEMM_NW * R * nt * NB * 1024;
    return park > meet ? (park > 2048 ? park : 2048) : (meet > 2048 ? meet : 2048);   // 2 KB: the LM head's state exchange
}

template <int MODE, int NB, int R, int GEMM_NW>
__global__ void __launch_bounds__(GEMM_NW * 64) k_gemm_rows(GemmArgs a) {
    constexpr bool TWO_IN_FLIGHT = NB == 1;                               // larger token blocks have no registers to spare
    constexpr int NT = (MODE == G_GATEUP) ? 2 : 1;
    constexpr int NS = GEMM_KW / 32;
    constexpr int NQ = (16 * GEMM_KW * 2) / 1024;                         // load instructions per 16-row piece (2)
    constexpr int SLOTS = R * NT * NB;
    static_assert(MODE != G_LMHEAD || NB == 1, "the router state of a lane follows one token");
    extern __shared__ __align__(16) unsigned char smem[];
    float4 *red = reinterpret_cast<float4 *>(smem);                       // [GEMM_NW][SLOTS][64], after the last window
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int i16 = lane & 15, g = lane >> 4;
    unsigned char *park = smem + (size_t)wave * R * NT * 16 * GEMM_PITCH;   // this wave's [R*NT][16 rows][GEMM_PITCH]
    const int lrow = lane >> 3, lchunk = lane & 7;                        // load role: row 8 q + lrow, bytes 16 lchunk ..
    const int K = a.K;
    const int n_out = (MODE == G_GATEUP) ? a.d_ffn : a.N;                 // distinct output columns
    const int n_tiles = (n_out + 15) / 16, n_groups = (n_tiles + R - 1) / R;
    const int n_win = K / GEMM_KW;
    const int KSP = a.ksplit > 1 ? a.ksplit : 1;

    // Workgroup id -> (work unit, token-row block).  The hardware deals consecutive workgroup ids round
    // robin over the 8 XCDs; the row blocks of one unit stream the same weights, so they get ids that are
    // congruent modulo 8: one of them fetches a weight line from HBM, the others find it in that XCD's L2.
    const int Y = a.yblocks > 1 ? a.yblocks : 1;
    const int n_units = n_groups * KSP;
    int unit_first, unit_step, yb;
    if (Y == 1) { unit_first = blockIdx.x; unit_step = gridDim.x; yb = 0; }
    else {
        // the launch has 8 * Y * n_cs workgroups: column slot cs (of n_cs) on XCD x walks the units cs * 8 + x, + n_cs * 8, ...
        const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
        yb = slot % Y;
        unit_first = (slot / Y) * 8 + xcd;
        unit_step = (int)(gridDim.x / (8 * Y)) * 8;
    }
    const int part_id = Y == 1 ? (int)blockIdx.x : unit_first;            // LM head: this workgroup's place among its rows' partial states
    const int m_base = yb * 16 * NB;

    // token side: rows past M read row 0 and are cleared after the load
    const float *xp[NB];
    bool xok[NB];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
        const int m = m_base + nb * 16 + i16;
        xok[nb] = m < a.M;
        xp[nb] = a.X32 + (size_t)(xok[nb] ? m : 0) * K + g * 8;
    }
    SoftState st; st.init();
    const int lm_row = m_base + i16;                      // LM head (NB = 1): the output row this lane's state follows
    const float lm_scale = (MODE == G_LMHEAD && lm_row < a.M) ? a.seq_scale[lm_row] : 1.f;
    unsigned long long noise_base = 0;                    // sampling: (position of the token being predicted) * V
    if (MODE == G_LMHEAD && a.sample_on && lm_row < a.M) noise_base = (unsigned long long)(a.row_pos[a.out_row[lm_row]] + 1) * (unsigned long long)a.N;

    for (int unit = unit_first; unit < n_units; unit += unit_step) {
        const int grp = unit / KSP, ksp = unit - grp * KSP;
        const int w_lo = (int)(((long long)n_win * ksp) / KSP), w_hi = (int)(((long long)n_win * (ksp + 1)) / KSP);
        f32x4_t acc[R][NT][NB];
        const uint16_t *wp[R][NT][NQ];
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
#pragma unroll
                for (int q = 0; q < NQ; ++q) {
                    const int row = min((grp * R + r) * 16 + 8 * q + lrow, n_out - 1) + (nt == 1 ? a.d_ffn : 0);
                    wp[r][nt][q] = a.W + (size_t)row * K + lchunk * 8;
                }
#pragma unroll
                for (int nb = 0; nb < NB; ++nb) acc[r][nt][nb] = (f32x4_t){0.f, 0.f, 0.f, 0.f};
            }
        // two windows in flight per wave: the requests of the next window are issued before the
        // products of the current one.  Requests are unconditional (the window index is clamped;
        // a duplicate is fetched but never multiplied) so that the compiler can count them and wait
        // for exactly the older set.
        auto request = [&](int win, float4 (&xb)[NB][NS][2], uint4 (&wr)[R][NT][NQ]) {
            const int k0 = min(win, w_hi - 1) * GEMM_KW;
#pragma unroll
            for (int nb = 0; nb < NB; ++nb)
#pragma unroll
                for (int s = 0; s < NS; ++s) {
                    const float4 *q = reinterpret_cast<const float4 *>(xp[nb] + k0 + 32 * s);
                    xb[nb][s][0] = q[0]; xb[nb][s][1] = q[1];
                }
#pragma unroll
            for (int r = 0; r < R; ++r)
#pragma unroll
                for (int nt = 0; nt < NT; ++nt)
#pragma unroll
                    for (int q = 0; q < NQ; ++q)
                        wr[r][nt][q] = load_stream(reinterpret_cast<const uint4 *>(wp[r][nt][q] + k0));
        };
        auto multiply = [&](const float4 (&xb)[NB][NS][2], const uint4 (&wr)[R][NT][NQ]) {
            // this lane's 8 consecutive k of token i16 per k step, as three bf16 planes whose sum is the fp32 value
            bf16x8_t B[NB][NS][3];
#pragma unroll
            for (int nb = 0; nb < NB; ++nb)
#pragma unroll
                for (int s = 0; s < NS; ++s) {
                    const float4 x0 = xb[nb][s][0], x1 = xb[nb][s][1];
                    float xv[8] = {x0.x, x0.y, x0.z, x0.w, x1.x, x1.y, x1.z, x1.w};
                    if (!xok[nb]) {
#pragma unroll
                        for (int e = 0; e < 8; ++e) xv[e] = 0.f;
                    }
                    split3(xv, B[nb][s]);
                }
#pragma unroll
            for (int r = 0; r < R; ++r)
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) {
                    unsigned char *pk = park + (size_t)(r * NT + nt) * 16 * GEMM_PITCH;
#pragma unroll
                    for (int q = 0; q < NQ; ++q)
                        *reinterpret_cast<uint4 *>(pk + (size_t)(8 * q + lrow) * GEMM_PITCH + lchunk * 16) = wr[r][nt][q];
                }
#pragma unroll
            for (int r = 0; r < R; ++r)
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) {
                    const unsigned char *pk = park + (size_t)(r * NT + nt) * 16 * GEMM_PITCH;
#pragma unroll
                    for (int s = 0; s < NS; ++s) {
                        const bf16x8_t A = __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const uint4 *>(pk + (size_t)i16 * GEMM_PITCH + (4 * s + g) * 16));
#pragma unroll
                        for (int nb = 0; nb < NB; ++nb)
#pragma unroll
                            for (int pl = 2; pl >= 0; --pl)           // smallest plane first
                                acc[r][nt][nb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(A, B[nb][s][pl], acc[r][nt][nb], 0, 0, 0);
                    }
                }
        };
        if constexpr (TWO_IN_FLIGHT) {
            float4 xb0[NB][NS][2], xb1[NB][NS][2];
            uint4 wr0[R][NT][NQ], wr1[R][NT][NQ];
            int win = w_lo + wave;
            if (win < w_hi) {
                request(win, xb0, wr0);
                while (true) {
                    request(win + GEMM_NW, xb1, wr1);
                    multiply(xb0, wr0);
                    win += GEMM_NW;
                    if (win >= w_hi) break;
                    request(win + GEMM_NW, xb0, wr0);
                    multiply(xb1, wr1);
                    win += GEMM_NW;
                    if (win >= w_hi) break;
                }
            }
        } else {
            float4 xb0[NB][NS][2];
            uint4 wr0[R][NT][NQ];
            for (int win = w_lo + wave; win < w_hi; win += GEMM_NW) {
                request(win, xb0, wr0);
                multiply(xb0, wr0);
            }
        }
        __syncthreads();      // every wave is done with its parking area, which the accumulators now overwrite
        // ---- the waves' accumulators meet in LDS
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
            for (int nt = 0; nt < NT; ++nt)
#pragma unroll
                for (int nb = 0; nb < NB; ++nb)
                    red[(wave * SLOTS + (r * NT + nt) * NB + nb) * 64 + lane] =
                        make_float4(acc[r][nt][nb][0], acc[r][nt][nb][1], acc[r][nt][nb][2], acc[r][nt][nb][3]);
        __syncthreads();
        // ---- wave p finishes pair p = (tile r, token block nb): this lane holds output columns
        // n0 + 4 g + rr (rr = 0..3) of token nb*16 + i16
        for (int p = wave; p < R * NB; p += GEMM_NW) {
            const int r = p / NB, nb = p - r * NB;
            const int tile = grp * R + r, n0 = tile * 16, m = m_base + nb * 16 + i16;
            float4 v[NT];
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
                v[nt] = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
                for (int w = 0; w < GEMM_NW; ++w) {
                    const float4 u = red[(w * SLOTS + (r * NT + nt) * NB + nb) * 64 + lane];
                    v[nt].x += u.x; v[nt].y += u.y; v[nt].z += u.z; v[nt].w += u.w;
                }
            }
            if (tile >= n_tiles || m >= a.M) continue;
            const float o0[4] = {v[0].x, v[0].y, v[0].z, v[0].w};
            const float o1[4] = {v[NT - 1].x, v[NT - 1].y, v[NT - 1].z, v[NT - 1].w};
#pragma unroll
            for (int rr = 0; rr < 4; ++rr) {
                const int n = n0 + 4 * g + rr;
                if (n >= n_out) continue;
                const float val = o0[rr];
                if ((MODE == G_QKV || MODE == G_OPROJ || MODE == G_DOWN) && KSP > 1) a.part[ksp * a.part_stride + (size_t)m * n_out + n] = val;
                else if (MODE == G_QKV) a.out_f32[(size_t)m * a.ld_out + n] = val;
                else if (MODE == G_OPROJ || MODE == G_DOWN) a.h_out[(size_t)m * a.ld_h + n] += val;
                else if (MODE == G_GATEUP) a.act32[(size_t)m * a.d_ffn + n] = val / (1.0f + expf(-val)) * o1[rr];
                else {
                    const float lg = val * lm_scale;
                    st.push(lg, n);
                    if (a.sample_on) st.push_noisy(lg, n, a.sample_key, noise_base);
                    if (a.logits) a.logits[(size_t)m * a.N + n] = lg;
                }
            }
        }
        __syncthreads();      // red[] is reused by the next group
    }
    if (MODE == G_LMHEAD) {
        // merge the four row groups of each wave (lanes 0..15 end up with the state of token i16), then the waves
        for (int o = 32; o >= 16; o >>= 1) {
            SoftState b = shfl_xor_state(st, o);
            if ((lane & o) == 0) st.merge(b); else { b.merge(st); st = b; }
        }
        SoftPartial *sp = reinterpret_cast<SoftPartial *>(smem);          // [GEMM_NW][16]
        if (g == 0) sp[wave * 16 + i16] = to_partial(st);
        __syncthreads();
        if (wave == 0 && g == 0 && lm_row < a.M) {
            SoftState s0 = from_partial(sp[i16]);
            for (int w = 1; w < GEMM_NW; ++w) s0.merge(from_partial(sp[w * 16 + i16]));
            a.parts[(size_t)lm_row * a.n_parts + part_id] = to_partial(s0);
        }
    }
}

// ------------------------------------------------------------------------------------------------
// k_gemm_tile: the same products for 33 .. 128 token rows, one workgroup per block of output columns.
// A workgroup of four waves owns CT tiles of 16 output columns (gate/up: CT gate tiles and the CT matching
// up tiles) and ALL token rows: wave w of NW (four up to 64 rows, eight up to 128) holds the rows 16 TB w ..
// 16 TB (w + 1) - 1 (TB = 1 block of 16 in every launch; two blocks per wave on four waves measured slower: 7B gate/up at
// 128 rows 142 us against 110) against every column of the workgroup, so nothing has to be summed across waves and W is read from
// HBM once per call, whatever the row count.  Per 64-element k window the four waves fetch the window's W
// rows together (whole 128-byte row pieces, into registers, up to six windows ahead), park them in one of two
// LDS buffers and every wave reads all of them back in A-operand layout; its X pieces (fp32 rows, split
// into the three planes in registers, XD - 1 windows ahead) come straight from global memory because no
// other wave needs them.  One barrier per window, and it is the bare instruction behind a wait for the LDS writes only:
// __syncthreads() carries a fence that waits for every outstanding load, i.e. for the windows requested
// ahead, and a window would cost a full memory round trip.
// X costs (workgroups) x (rows) x K x 4 bytes of L2 traffic, which is why a workgroup takes as many column
// tiles as the launch can afford (launch_gemm_tile picks CT and the split of K over workgroups so that the
// workgroups are close to a whole number of rounds of the machine).
// Modes: G_GATEUP (whole K, SwiGLU epilogue into the activation planes), G_PART (K split ksplit >= 1
// ways over workgroups, raw partial sums part[ks][row][n] for the next kernel to add up in a fixed order) and
// G_LMHEAD (whole K; scaled logits feed each row's single-pass softmax state, one partial per row and workgroup).
// ------------------------------------------------------------------------------------------------
constexpr int G_PART = 5;

// windows per step: a step fetches 128 SW contiguous bytes of every W row.  One everywhere: two windows per step
// (256-byte row pieces, two register slots each for W and X) measured slower (7B shape, 64 rows, gate/up 108 us
// against 91)
template <int TB> constexpr int tile_sw() { return 1; }

constexpr int TILE_PAD = 16;                      // bytes added to a parked row of k_gemm_tile against LDS bank conflicts (48 measured the same)

template <int MODE, int TB, int CT>
__host__ __device__ constexpr size_t gemm_tile_lds_bytes() {
    return (size_t)2 * ((MODE == G_GATEUP) ? 2 : 1) * CT * 16 * (128 * tile_sw<TB>() + TILE_PAD);
}

// workgroup barrier for LDS hand-over that leaves global loads in flight: the LDS accesses issued so far complete
// (lgkmcnt(0); expcnt and vmcnt are left alone), then the barrier; the compiler moves no memory access across it
__device__ __forceinline__ void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

template <int MODE, int TB, int CT, int NW = 4, int CS = 1>
__global__ void __launch_bounds__(NW * 64) k_gemm_tile(GemmArgs a) {
    static_assert(MODE == G_GATEUP || MODE == G_PART || MODE == G_LMHEAD, "gate/up, raw partial sums or the LM head");
    constexpr int NT = (MODE == G_GATEUP) ? 2 : 1;
    constexpr int NS = GEMM_KW / 32;
    constexpr int SW = tile_sw<TB>();                         // windows per step
    constexpr int KSTEP = GEMM_KW * SW;                       // k elements per step: K must be a multiple
    constexpr int PITCH = 128 * SW + TILE_PAD;                // bytes per parked row (padded against LDS bank conflicts)
    constexpr int WROWS = NT * CT * 16;                       // W rows of a step
    constexpr int RPR = 8 * NW / SW;                          // rows per round of 16-byte loads of the whole workgroup
    constexpr int WQ = (WROWS + RPR - 1) / RPR;               // loads per thread and step
    constexpr size_t BUF = (size_t)WROWS * PITCH;
    constexpr int XD = TB == 1 ? 3 : 2;                       // register slots of X (each holds a step's pieces)
    constexpr int RB = NW / CS;                               // waves that differ in their rows; CS waves share a row block and
    constexpr int CTH = (CT + CS - 1) / CS;                   // split the workgroup's column tiles, CTH each (the last may get fewer)
    static_assert(NW % CS == 0, "whole column splits");
    extern __shared__ __align__(16) unsigned char smem[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int i16 = lane & 15, g = lane >> 4;
    const int rb = wave % RB, ct0 = (wave / RB) * CTH;          // this wave's row block and first column tile
    const int lrow = tid / (8 * SW), lchunk = tid % (8 * SW); // W load role: row RPR q + lrow of the step, bytes 16 lchunk ..
    const int K = a.K;
    const int n_out = (MODE == G_GATEUP) ? a.d_ffn : a.N;
    const int n_tiles = (n_out + 15) / 16, n_groups = (n_tiles + CT - 1) / CT;
    const int KSP = a.ksplit > 1 ? a.ksplit : 1;
    const int n_st = K / KSTEP;                               // steps over the whole of K
    const int unit = blockIdx.x;                              // one unit per workgroup
    if (unit >= n_groups * KSP) return;
    const int grp = unit / KSP, ksp = unit - grp * KSP;
    const int s_lo = (int)(((long long)n_st * ksp) / KSP), s_hi = (int)(((long long)n_st * (ksp + 1)) / KSP);
    const int n0 = grp * CT * 16;
    if (s_hi <= s_lo) return;                                 // (the launch never splits K finer than its steps)

    // W rows this thread fetches: step row j < CT * 16 is output column n0 + j (gate), the others the matching up rows
    const uint16_t *wp[WQ];
    bool wok[WQ];
#pragma unroll
    for (int q = 0; q < WQ; ++q) {
        const int j = RPR * q + lrow;
        wok[q] = j < WROWS;
        const int jj = wok[q] ? j : 0, half = jj / (CT * 16), col = jj - half * (CT * 16);
        const int row = min(n0 + col, n_out - 1) + (half ? a.d_ffn : 0);
        wp[q] = a.W + (size_t)row * K + lchunk * 8;
    }
    // token rows of this wave; a row past the call's rows repeats row 0: its products fill matrix-core columns that
    // belong to no row and are never stored
    const float *xp[TB];
#pragma unroll
    for (int tb = 0; tb < TB; ++tb) {
        const int m = (rb * TB + tb) * 16 + i16;
        xp[tb] = a.X32 + (size_t)(m < a.M ? m : 0) * K + g * 8;
    }
    f32x4_t acc[TB][NT][CTH];
#pragma unroll
    for (int tb = 0; tb < TB; ++tb)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
#pragma unroll
            for (int ct = 0; ct < CTH; ++ct) acc[tb][nt][ct] = (f32x4_t){0.f, 0.f, 0.f, 0.f};

    // a step past the last is replaced by the last (fetched again, never used): requests are unconditional
    auto request_w = [&](int st, uint4 (&wr)[WQ]) {
        const int k0 = min(st, s_hi - 1) * KSTEP;
#pragma unroll
        for (int q = 0; q < WQ; ++q) wr[q] = load_stream(reinterpret_cast<const uint4 *>(wp[q] + k0));
    };
    // X arrives as fp32 (8 consecutive k per lane and k step: two 16-byte loads, a whole 128-byte line per row and
    // step over the four lanes of a token) and is split into the three bf16 planes here: 4 bytes per element through
    // the CU's load path instead of 6
    auto request_x = [&](int st, float4 (&xb)[SW][TB][NS][2]) {
        const int k0 = min(st, s_hi - 1) * KSTEP;
#pragma unroll
        for (int sw = 0; sw < SW; ++sw)
#pragma unroll
            for (int tb = 0; tb < TB; ++tb)
#pragma unroll
                for (int s_ = 0; s_ < NS; ++s_) {
                    const float4 *q = reinterpret_cast<const float4 *>(xp[tb] + k0 + GEMM_KW * sw + 32 * s_);
                    xb[sw][tb][s_][0] = q[0]; xb[sw][tb][s_][1] = q[1];
                }
    };
    auto park = [&](int buf, const uint4 (&wr)[WQ]) {
        unsigned char *base = smem + (size_t)buf * BUF;
#pragma unroll
        for (int q = 0; q < WQ; ++q)
            if (wok[q]) *reinterpret_cast<uint4 *>(base + (size_t)(RPR * q + lrow) * PITCH + lchunk * 16) = wr[q];
    };
    auto multiply = [&](int buf, const float4 (&xb)[SW][TB][NS][2]) {
        const unsigned char *base = smem + (size_t)buf * BUF;
        // per k step: the A operands of all tiles first, then the planes outermost (smallest first), so that
        // consecutive matrix-core instructions write different accumulators: a product that has to wait for the
        // one before it (same accumulator) stalls the pipe for that one's whole latency
#pragma unroll
        for (int sw = 0; sw < SW; ++sw)
#pragma unroll
            for (int s_ = 0; s_ < NS; ++s_) {
                bf16x8_t A[NT][CTH];
#pragma unroll
                for (int nt = 0; nt < NT; ++nt)
#pragma unroll
                    for (int ct = 0; ct < CTH; ++ct)       // (a tile past the workgroup's last repeats it; its products are dropped)
                        A[nt][ct] = __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const uint4 *>(
                            base + (size_t)((nt * CT + min(ct0 + ct, CT - 1)) * 16 + i16) * PITCH + (4 * (NS * sw + s_) + g) * 16));
                bf16x8_t B[TB][3];
#pragma unroll
                for (int tb = 0; tb < TB; ++tb) {
                    const float4 x0 = xb[sw][tb][s_][0], x1 = xb[sw][tb][s_][1];
                    const float xv[8] = {x0.x, x0.y, x0.z, x0.w, x1.x, x1.y, x1.z, x1.w};
                    split3(xv, B[tb]);
                }
#pragma unroll
                for (int pl = 2; pl >= 0; --pl)
#pragma unroll
                    for (int tb = 0; tb < TB; ++tb)
#pragma unroll
                        for (int nt = 0; nt < NT; ++nt)
#pragma unroll
                            for (int ct = 0; ct < CTH; ++ct)
                                acc[tb][nt][ct] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(A[nt][ct], B[tb][pl], acc[tb][nt][ct], 0, 0, 0);
            }
    };

    // register slots: WD for W, XD for X.  When step t is multiplied, the W rows of t + 1 .. t + WD and the X pieces
    // of t + 1 .. t + XD - 1 are in flight or have arrived; every request goes into the slot that the step before
    // has just consumed, before this step's products.  What bounds this kernel is how much of W one workgroup per CU
    // keeps in flight (the hardware counters show 40 % of the outstanding DRAM requests of a kernel that streams at 6 TB/s).
    // six slots where a launch is one workgroup per CU and the registers allow it (7B gate/up at 64 rows 86 -> 75 us);
    // the LM head has several workgroups per CU and is better off with two of them resident (three slots each); with 32
    // rows per wave four slots fit for the modes without the second (up) set of accumulators (7B down at 128 rows 91 -> 85 us)
    constexpr int WD = (TB == 1 && MODE != G_LMHEAD) ? 6 : ((TB == 2 && MODE == G_PART) ? 4 : 3);
    static_assert(NW == 4 || (NW == 8 && TB == 1), "four waves, or eight with one block of 16 rows each");
    constexpr int UNR = (WD % XD == 0) ? WD : WD * XD;        // steps after which both slot patterns repeat
    uint4 wr[WD][WQ];
    float4 xb[XD][SW][TB][NS][2];
#pragma unroll
    for (int v = 0; v < WD; ++v) request_w(s_lo + v, wr[v]);
    int buf = 0;
    if (rb * TB * 16 < a.M) {
#pragma unroll
        for (int v = 0; v < XD - 1; ++v) request_x(s_lo + v, xb[v]);
        for (int st = s_lo; st < s_hi; st += UNR) {
#pragma unroll
            for (int u = 0; u < UNR; ++u) {
                if (st + u >= s_hi) break;
                park(buf, wr[u % WD]);
                lds_barrier();                                // the step is in LDS; everybody is done with the other buffer's last use
                request_w(st + u + WD, wr[u % WD]);
                request_x(st + u + XD - 1, xb[(u + XD - 1) % XD]);
                multiply(buf, xb[u % XD]);
                buf ^= 1;
            }
        }
    } else {
        // a wave whose 16-row block lies past the call's rows only helps to fetch and park W: same steps, same barriers,
        // no activation requests and no products (they would take load-path and matrix-core time from the waves with rows)
        for (int st = s_lo; st < s_hi; st += WD) {
#pragma unroll
            for (int u = 0; u < WD; ++u) {
                if (st + u >= s_hi) break;
                park(buf, wr[u]);
                lds_barrier();
                request_w(st + u + WD, wr[u]);
                buf ^= 1;
            }
        }
    }

    // epilogue: this lane holds output columns n0 + 16 ct + 4 g + r of token 16 (wave TB + tb) + i16
#pragma unroll
    for (int tb = 0; tb < TB; ++tb) {
        const int m = (rb * TB + tb) * 16 + i16;
        if (MODE == G_LMHEAD) {
            // the row's softmax state over this workgroup's columns: every lane pushes its logits, the four lanes of a
            // token (g = 0..3) merge, one partial per (row, workgroup).  Uniform control flow: the merge shuffles
            const bool ok = m < a.M;
            SoftState st; st.init();
            const float lm_scale = ok ? a.seq_scale[m] : 1.f;
            unsigned long long noise_base = 0;
            if (a.sample_on && ok) noise_base = (unsigned long long)(a.row_pos[a.out_row[m]] + 1) * (unsigned long long)a.N;
#pragma unroll
            for (int ct = 0; ct < CTH; ++ct)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int n = (grp * CT + ct0 + ct) * 16 + 4 * g + r;
                    if (!ok || ct0 + ct >= CT || n >= n_out) continue;
                    const float lg = acc[tb][0][ct][r] * lm_scale;
                    st.push(lg, n);
                    if (a.sample_on) st.push_noisy(lg, n, a.sample_key, noise_base);
                    if (a.logits) a.logits[(size_t)m * a.N + n] = lg;
                }
            for (int o = 32; o >= 16; o >>= 1) {
                SoftState b = shfl_xor_state(st, o);
                if ((lane & o) == 0) st.merge(b); else { b.merge(st); st = b; }
            }
            if (g == 0 && ok) a.parts[(size_t)m * a.n_parts + grp * CS + wave / RB] = to_partial(st);
            continue;
        }
        if (m >= a.M) continue;
#pragma unroll
        for (int ct = 0; ct < CTH; ++ct) {
            const int tile = grp * CT + ct0 + ct;
            if (ct0 + ct >= CT || tile >= n_tiles) continue;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int n = tile * 16 + 4 * g + r;
                if (n >= n_out) continue;
                const float val = acc[tb][0][ct][r];
                if (MODE == G_PART) a.part[ksp * a.part_stride + (size_t)m * n_out + n] = val;
                else a.act32[(size_t)m * a.d_ffn + n] = val / (1.0f + expf(-val)) * acc[tb][NT - 1][ct][r];
            }
        }
    }
}

}  // namespace rs
