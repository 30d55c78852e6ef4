// Multi-row kernels (2..64 token rows per call): the catch-up prefill of the
// tokens a model has not seen, and batched decode.  The weights are still read
// once per call, so the phases stay HBM-bound; the contraction over tokens runs
// on the matrix cores (v_mfma_f32_16x16x32_bf16, fp32 accumulate) so that ALU
// work never becomes the limiter.  Activations are fp32 values carried as three
// bf16 planes (p0 = bf16(x), p1 = bf16(x - p0), p2 = x - p0 - p1, which is exact:
// 3 x 8 significant bits hold the 24 of an fp32); each weight tile is multiplied
// with all three, smallest first, so the product is that of the fp32 activation.
#pragma once

#include "device_utils.h"
#include "model_kernels.h"

namespace rs {

// planes: p[0], p[1], p[2] each [rows, cols]; `plane` = elements per plane
__device__ __forceinline__ void split_store(float v, uint16_t *p, size_t plane, size_t i) {
    const uint16_t a = f32_to_bf16(v);
    const float r1 = v - bf16_to_f32(a);
    const uint16_t b = f32_to_bf16(r1);
    p[i] = a; p[plane + i] = b; p[2 * plane + i] = f32_to_bf16(r1 - bf16_to_f32(b));
}

// RMSNorm of whole rows into three bf16 planes: grid n_out, block 256.
// src row = gather ? gather[blockIdx.x] : blockIdx.x
__global__ void __launch_bounds__(256)
k_rmsnorm_rows(const float *__restrict__ h, const uint16_t *__restrict__ gain, float eps, int d,
               const int *__restrict__ gather, uint16_t *__restrict__ out, size_t plane) {
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int src = gather ? gather[blockIdx.x] : blockIdx.x;
    const float *hr = h + (size_t)src * d;
    __shared__ float red_ss[4];
    float ss = 0.f;
    for (int i = tid; i < d; i += 256) { const float v = hr[i]; ss = fmaf(v, v, ss); }
    ss = wave_sum(ss);
    if (lane == 0) red_ss[wave] = ss;
    __syncthreads();
    const float inv = 1.0f / sqrtf((red_ss[0] + red_ss[1] + red_ss[2] + red_ss[3]) / (float)d + eps);
    for (int i = tid; i < d; i += 256)
        split_store(hr[i] * (inv * bf16_to_f32(gain[i])), out, plane, (size_t)blockIdx.x * d + i);
}

// Rotary embedding of q and k, KV-cache write, for every row: grid n_rows, block 256.
struct RopeArgs {
    const float *qkv;              // [rows, (n_q+2 n_kv) hd] fp32
    float *qbuf; uint16_t *kcache, *vcache;
    const float *rope_cos, *rope_sin;
    const int *row_pos, *row_slot, *row_bad;
    int n_q, n_kv, head_dim, max_ctx, max_seqs, layer;
};

__global__ void __launch_bounds__(256) k_rope_kv_rows(RopeArgs a) {
    const int r = blockIdx.x, tid = threadIdx.x;
    if (a.row_bad[r]) {
        for (int i = tid; i < a.n_q * a.head_dim; i += 256) a.qbuf[(size_t)r * a.n_q * a.head_dim + i] = 0.f;
        return;
    }
    const int hd = a.head_dim, half = hd >> 1, pos = a.row_pos[r], slot = a.row_slot[r];
    const int n_qkv = (a.n_q + 2 * a.n_kv) * hd;
    const float *x = a.qkv + (size_t)r * n_qkv;
    const float *cs = a.rope_cos + (size_t)pos * half, *sn = a.rope_sin + (size_t)pos * half;
    for (int p = tid; p < (a.n_q + a.n_kv) * half; p += 256) {
        const int head = p / half, i = p - head * half;
        const float x0 = x[head * hd + i], x1 = x[head * hd + i + half], c = cs[i], s = sn[i];
        const float y0 = x0 * c - x1 * s, y1 = x1 * c + x0 * s;
        if (head < a.n_q) {
            float *q = a.qbuf + ((size_t)r * a.n_q + head) * hd;
            q[i] = y0; q[i + half] = y1;
        } else {
            const size_t base = ((((size_t)a.layer * a.max_seqs + slot) * a.n_kv + (head - a.n_q)) * a.max_ctx + pos) * hd;
            a.kcache[base + i] = f32_to_bf16(y0); a.kcache[base + i + half] = f32_to_bf16(y1);
        }
    }
    for (int p = tid; p < a.n_kv * hd; p += 256) {
        const int vh = p / hd, e = p - vh * hd;
        const size_t base = (((size_t)a.layer * a.max_seqs + slot) * a.n_kv + vh) * (size_t)a.max_ctx * hd;
        a.vcache[base + (size_t)e * a.max_ctx + pos] = f32_to_bf16(x[(a.n_q + a.n_kv) * hd + p]);   // V is stored [hd][position]
    }
}

// ------------------------------------------------------------------------------------------------
// out[m, n] = sum_k X[m, k] W[n, k] for M <= 16*NB token rows.
// A workgroup of NW waves owns 16 output columns at a time (for gate/up: 16 gate rows and the 16
// matching up rows of W); its waves split K in interleaved blocks of 256 elements.  Per block a
// wave streams its 16 x 512-byte piece of W from HBM with fully coalesced 16-byte loads (a load
// instruction covers two whole 512-byte row pieces; the next block is in flight in registers
// while the current one is multiplied), parks it in its private LDS region, and reads it back in
// the operand layout of v_mfma_f32_16x16x32_bf16 (lane (i = lane % 16, g = lane / 16) supplies
// the 8 consecutive k at 32 s + 8 g of row i).  The token side comes from the three bf16 planes
// of X through L2 in the same k layout.  The per-wave 16x16 accumulators (lane holds
// D[4 g + r][token = lane % 16]) are summed through LDS by wave 0, which runs the epilogue.
// ------------------------------------------------------------------------------------------------
struct GemmArgs {
    const uint16_t *W; int N, K, M;       // M = valid token rows
    const uint16_t *X; size_t x_plane;    // three [.., K] bf16 planes, x_plane elements apart
    float *out_f32; int ld_out;           // raw fp32 output [M, ld_out] (QKV)
    float *h_out; int ld_h;               // residual accumulate
    uint16_t *act; size_t act_plane; int d_ffn;   // gate/up output planes
    const float *seq_scale; SoftPartial *parts; float *logits; int n_parts;   // LM head
};

constexpr int GEMM_KB = 256;                      // k elements per block
constexpr int GEMM_ROWB = GEMM_KB * 2 + 16;       // bytes per staged row (padded against LDS bank conflicts)

template <int MODE, int NB, int NW>
__host__ __device__ constexpr size_t gemm_lds_bytes() {
    return (size_t)NW * ((MODE == G_GATEUP) ? 2 : 1) * (16 * GEMM_ROWB + NB * 1024);
}

template <int MODE, int NB, int NW>
__global__ void __launch_bounds__(NW * 64) k_gemm_rows(GemmArgs a) {
    constexpr int NT = (MODE == G_GATEUP) ? 2 : 1;
    extern __shared__ __align__(16) unsigned char smem[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int i16 = lane & 15, g = lane >> 4;
    unsigned char *wlds = smem + (size_t)wave * NT * 16 * GEMM_ROWB;                       // this wave's staging area
    float4 *red = reinterpret_cast<float4 *>(smem + (size_t)NW * NT * 16 * GEMM_ROWB);     // [NW][NT][NB][64]
    const int K = a.K;
    const int n_out = (MODE == G_GATEUP) ? a.d_ffn : a.N;                 // distinct output columns
    const int n_tiles = (n_out + 15) / 16;
    // global-load role of this lane: load q (0..7) fetches rows 2q and 2q+1, lane covers 16 bytes of one of them
    const int lrow = lane >> 5, lchunk = lane & 31;

    const uint16_t *xp[NB];
    bool xok[NB];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
        const int m = nb * 16 + i16;
        xok[nb] = m < a.M;
        xp[nb] = a.X + (size_t)(xok[nb] ? m : 0) * K + g * 8;
    }
    SoftState st; st.init();
    const float lm_scale = (MODE == G_LMHEAD && i16 < a.M) ? a.seq_scale[i16] : 1.f;

    for (int t = blockIdx.x; t < n_tiles; t += gridDim.x) {
        const int n0 = t * 16;
        f32x4_t acc[NT][NB];
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) acc[nt][nb] = (f32x4_t){0.f, 0.f, 0.f, 0.f};

        // row pointers of the 8 loads per tile
        const uint16_t *wrow[NT][8];
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
#pragma unroll
            for (int q = 0; q < 8; ++q) {
                const int r = min(n0 + 2 * q + lrow, n_out - 1) + (nt == 1 ? a.d_ffn : 0);
                wrow[nt][q] = a.W + (size_t)r * K + lchunk * 8;
            }
        uint4 cur[NT][8];
        int kb = wave * GEMM_KB;
        auto fetch = [&](int k0, uint4 (&dst)[NT][8]) {
            const bool ok = k0 + lchunk * 8 < K;            // K is a multiple of 128, a block may be half empty
#pragma unroll
            for (int nt = 0; nt < NT; ++nt)
#pragma unroll
                for (int q = 0; q < 8; ++q)
                    dst[nt][q] = ok ? load_stream(reinterpret_cast<const uint4 *>(wrow[nt][q] + k0)) : make_uint4(0, 0, 0, 0);
        };
        if (kb < K) fetch(kb, cur);
        for (; kb < K; kb += NW * GEMM_KB) {
            // park the block in LDS
#pragma unroll
            for (int nt = 0; nt < NT; ++nt)
#pragma unroll
                for (int q = 0; q < 8; ++q)
                    *reinterpret_cast<uint4 *>(wlds + (size_t)(nt * 16 + 2 * q + lrow) * GEMM_ROWB + lchunk * 16) = cur[nt][q];
            const int kn = kb + NW * GEMM_KB;
            if (kn < K) fetch(kn, cur);
#pragma unroll
            for (int s = 0; s < GEMM_KB / 32; ++s) {
                if (kb + 32 * s >= K) break;
                bf16x8_t A[NT];
#pragma unroll
                for (int nt = 0; nt < NT; ++nt)
                    A[nt] = __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const uint4 *>(wlds + (size_t)(nt * 16 + i16) * GEMM_ROWB + (4 * s + g) * 16));
#pragma unroll
                for (int nb = 0; nb < NB; ++nb) {
#pragma unroll
                    for (int pl = 2; pl >= 0; --pl) {             // smallest plane first
                        const uint4 bv = xok[nb] ? *reinterpret_cast<const uint4 *>(xp[nb] + pl * a.x_plane + kb + 32 * s)
                                                 : make_uint4(0, 0, 0, 0);
                        const bf16x8_t B = __builtin_bit_cast(bf16x8_t, bv);
#pragma unroll
                        for (int nt = 0; nt < NT; ++nt)
                            acc[nt][nb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(A[nt], B, acc[nt][nb], 0, 0, 0);
                    }
                }
            }
        }
        // ---- sum the waves' accumulators (wave 0 ends up with the totals)
        if (NW > 1) {
#pragma unroll
            for (int nt = 0; nt < NT; ++nt)
#pragma unroll
                for (int nb = 0; nb < NB; ++nb)
                    red[((wave * NT + nt) * NB + nb) * 64 + lane] = make_float4(acc[nt][nb][0], acc[nt][nb][1], acc[nt][nb][2], acc[nt][nb][3]);
            __syncthreads();
            if (wave == 0) {
#pragma unroll
                for (int nt = 0; nt < NT; ++nt)
#pragma unroll
                    for (int nb = 0; nb < NB; ++nb) {
                        float4 sum = red[((0 * NT + nt) * NB + nb) * 64 + lane];
                        for (int wv = 1; wv < NW; ++wv) {
                            const float4 v = red[((wv * NT + nt) * NB + nb) * 64 + lane];
                            sum.x += v.x; sum.y += v.y; sum.z += v.z; sum.w += v.w;
                        }
                        acc[nt][nb] = (f32x4_t){sum.x, sum.y, sum.z, sum.w};
                    }
            }
        }
        // ---- epilogue (wave 0): this lane holds output columns n0 + 4 g + r (r = 0..3) of token nb*16 + i16
        if (wave == 0) {
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) {
                const int m = nb * 16 + i16;
                if (m >= a.M) continue;
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int n = n0 + 4 * g + r;
                    if (n >= n_out) continue;
                    const float v = acc[0][nb][r];
                    if (MODE == G_QKV) a.out_f32[(size_t)m * a.ld_out + n] = v;
                    else if (MODE == G_OPROJ || MODE == G_DOWN) a.h_out[(size_t)m * a.ld_h + n] += v;
                    else if (MODE == G_GATEUP) {
                        const float up = acc[NT - 1][nb][r];
                        split_store(v / (1.0f + expf(-v)) * up, a.act, a.act_plane, (size_t)m * a.d_ffn + n);
                    } else {
                        const float lg = v * lm_scale;
                        st.push(lg, n);
                        if (a.logits) a.logits[(size_t)m * a.N + n] = lg;
                    }
                }
            }
        }
        if (NW > 1) __syncthreads();      // red[] is reused by the next tile
    }
    if (MODE == G_LMHEAD && wave == 0) {
        // merge the four row groups of the wave: lanes 0..15 end up with the state of token i16
        for (int o = 32; o >= 16; o >>= 1) {
            SoftState b = shfl_xor_state(st, o);
            if ((lane & o) == 0) st.merge(b); else { b.merge(st); st = b; }
        }
        if (g == 0 && i16 < a.M) a.parts[(size_t)i16 * a.n_parts + blockIdx.x] = to_partial(st);
    }
}

}  // namespace rs
