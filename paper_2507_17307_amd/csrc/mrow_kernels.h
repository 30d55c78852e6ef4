// Multi-row kernels (2..64 token rows per call): the catch-up prefill of the
// tokens a model has not seen, and batched decode.  The weights are still read
// once per call, so the phases stay HBM-bound; the contraction over tokens runs
// on the matrix cores (v_mfma_f32_16x16x32_bf16, fp32 accumulate) so that ALU
// work never becomes the limiter.
#pragma once

#include "device_utils.h"
#include "model_kernels.h"

namespace rs {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));

// RMSNorm of whole rows into a bf16 matrix: grid n_out, block 256.
// src row = gather ? gather[blockIdx.x] : blockIdx.x
__global__ void __launch_bounds__(256)
k_rmsnorm_rows(const float *__restrict__ h, const uint16_t *__restrict__ gain, float eps, int d,
               const int *__restrict__ gather, uint16_t *__restrict__ out) {
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int src = gather ? gather[blockIdx.x] : blockIdx.x;
    const float2 *h2 = reinterpret_cast<const float2 *>(h + (size_t)src * d);
    __shared__ float red_ss[4];
    float ss = 0.f;
    for (int i = tid; i < (d >> 1); i += 256) { float2 v = h2[i]; ss = fmaf(v.x, v.x, ss); ss = fmaf(v.y, v.y, ss); }
    ss = wave_sum(ss);
    if (lane == 0) red_ss[wave] = ss;
    __syncthreads();
    const float inv = 1.0f / sqrtf((red_ss[0] + red_ss[1] + red_ss[2] + red_ss[3]) / (float)d + eps);
    uint32_t *o32 = reinterpret_cast<uint32_t *>(out + (size_t)blockIdx.x * d);
    const uint32_t *g32 = reinterpret_cast<const uint32_t *>(gain);
    for (int i = tid; i < (d >> 1); i += 256) {
        float2 v = h2[i]; uint32_t g = g32[i];
        o32[i] = pack_bf16x2(v.x * inv * bf16_lo(g), v.y * inv * bf16_hi(g));
    }
}

// Rotary embedding of q and k, KV-cache write, for every row: grid n_rows, block 256.
struct RopeArgs {
    const float *qkv;              // [rows, (n_q+2 n_kv) hd] fp32
    uint16_t *qbuf, *kcache, *vcache;
    const float *rope_cos, *rope_sin;
    const int *row_pos, *row_slot, *row_bad;
    int n_q, n_kv, head_dim, max_ctx, max_seqs, layer;
};

__global__ void __launch_bounds__(256) k_rope_kv_rows(RopeArgs a) {
    const int r = blockIdx.x, tid = threadIdx.x;
    if (a.row_bad[r]) {
        for (int i = tid; i < a.n_q * a.head_dim; i += 256) a.qbuf[(size_t)r * a.n_q * a.head_dim + i] = 0;
        return;
    }
    const int hd = a.head_dim, half = hd >> 1, pos = a.row_pos[r], slot = a.row_slot[r];
    const int n_qkv = (a.n_q + 2 * a.n_kv) * hd;
    const float *x = a.qkv + (size_t)r * n_qkv;
    const float *cs = a.rope_cos + (size_t)pos * half, *sn = a.rope_sin + (size_t)pos * half;
    for (int p = tid; p < (a.n_q + a.n_kv) * half; p += 256) {
        const int head = p / half, i = p - head * half;
        const float x0 = x[head * hd + i], x1 = x[head * hd + i + half], c = cs[i], s = sn[i];
        const uint16_t y0 = f32_to_bf16(x0 * c - x1 * s), y1 = f32_to_bf16(x1 * c + x0 * s);
        if (head < a.n_q) {
            uint16_t *q = a.qbuf + ((size_t)r * a.n_q + head) * hd;
            q[i] = y0; q[i + half] = y1;
        } else {
            const size_t base = ((((size_t)a.layer * a.max_seqs + slot) * a.n_kv + (head - a.n_q)) * a.max_ctx + pos) * hd;
            a.kcache[base + i] = y0; a.kcache[base + i + half] = y1;
        }
    }
    for (int p = tid; p < a.n_kv * hd; p += 256) {
        const int vh = p / hd, e = p - vh * hd;
        const size_t base = ((((size_t)a.layer * a.max_seqs + slot) * a.n_kv + vh) * a.max_ctx + pos) * hd;
        a.vcache[base + e] = f32_to_bf16(x[(a.n_q + a.n_kv) * hd + p]);
    }
}

// ------------------------------------------------------------------------------------------------
// out[m, n] = sum_k X[m, k] W[n, k] for M <= 16*NB token rows.  A wave owns 16 rows of W at a time
// (MFMA "A" operand, loaded straight from HBM) against all tokens ("B" operand, bf16 X from L2).
// Lane (i = lane % 16, g = lane / 16) supplies, for both operands, the 8 consecutive k at
// kb + 32 g + 8 s (s = 0..3) of its row: any k order is valid for a dot product as long as both
// operands agree, and this one lets a lane read 64 contiguous bytes.  The accumulator lane holds
// D[4 g + r][token = lane % 16], r = 0..3.
// ------------------------------------------------------------------------------------------------
struct GemmArgs {
    const uint16_t *W; int N, K, M;       // M = valid token rows
    const uint16_t *X;                    // [M, K] bf16
    float *out_f32; int ld_out;           // raw fp32 output [M, ld_out] (QKV)
    float *h_out; int ld_h;               // residual accumulate
    uint16_t *act; int d_ffn;             // gate/up
    const float *seq_scale; SoftPartial *parts; float *logits; int n_parts;   // LM head
};

template <int MODE, int NB>
__global__ void __launch_bounds__(256) k_gemm_rows(GemmArgs a) {
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int i16 = lane & 15, g = lane >> 4;
    const int K = a.K;
    const int n_tiles = (MODE == G_GATEUP) ? a.d_ffn / 16 : (a.N + 15) / 16;
    const int gw = blockIdx.x * 4 + wave, gstride = gridDim.x * 4;

    const uint16_t *xrow[NB];
    bool xok[NB];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
        const int m = nb * 16 + i16;
        xok[nb] = m < a.M;
        xrow[nb] = a.X + (size_t)(xok[nb] ? m : 0) * K + g * 32;
    }
    SoftState st; st.init();
    const float lm_scale = (MODE == G_LMHEAD && i16 < a.M) ? a.seq_scale[i16] : 1.f;

    for (int t = gw; t < n_tiles; t += gstride) {
        const int n0 = t * 16;
        const int wr0 = min(n0 + i16, a.N - 1);
        const uint16_t *w0 = a.W + (size_t)wr0 * K + g * 32;
        const uint16_t *w1 = (MODE == G_GATEUP) ? a.W + (size_t)(a.d_ffn + n0 + i16) * K + g * 32 : w0;
        f32x4_t acc0[NB], acc1[NB];
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) { acc0[nb] = (f32x4_t){0.f, 0.f, 0.f, 0.f}; acc1[nb] = (f32x4_t){0.f, 0.f, 0.f, 0.f}; }
        for (int kb = 0; kb < K; kb += 128) {
            uint4 av0[4], av1[4];
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                av0[s] = load_stream(reinterpret_cast<const uint4 *>(w0 + kb + 8 * s));
                if (MODE == G_GATEUP) av1[s] = load_stream(reinterpret_cast<const uint4 *>(w1 + kb + 8 * s));
            }
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) {
                uint4 bv[4];
#pragma unroll
                for (int s = 0; s < 4; ++s)
                    bv[s] = xok[nb] ? *reinterpret_cast<const uint4 *>(xrow[nb] + kb + 8 * s) : make_uint4(0, 0, 0, 0);
#pragma unroll
                for (int s = 0; s < 4; ++s) {
                    const bf16x8_t B = __builtin_bit_cast(bf16x8_t, bv[s]);
                    acc0[nb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, av0[s]), B, acc0[nb], 0, 0, 0);
                    if (MODE == G_GATEUP)
                        acc1[nb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, av1[s]), B, acc1[nb], 0, 0, 0);
                }
            }
        }
        // ---- epilogue: this lane holds rows n0 + 4 g + r (r = 0..3) of token nb*16 + i16
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
            const int m = nb * 16 + i16;
            if (m >= a.M) continue;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int n = n0 + 4 * g + r;
                if (n >= ((MODE == G_GATEUP) ? a.d_ffn : a.N)) continue;
                const float v = acc0[nb][r];
                if (MODE == G_QKV) a.out_f32[(size_t)m * a.ld_out + n] = v;
                else if (MODE == G_OPROJ || MODE == G_DOWN) a.h_out[(size_t)m * a.ld_h + n] += v;
                else if (MODE == G_GATEUP) {
                    const float u = acc1[nb][r];
                    a.act[(size_t)m * a.d_ffn + n] = f32_to_bf16(v / (1.0f + expf(-v)) * u);
                } else {
                    const float lg = v * lm_scale;
                    st.push(lg, n);
                    if (a.logits) a.logits[(size_t)m * a.N + n] = lg;
                }
            }
        }
    }
    if (MODE == G_LMHEAD) {
        // merge the four row groups of the wave: lanes 0..15 end up with the state of token i16
        for (int o = 32; o >= 16; o >>= 1) {
            SoftState b = shfl_xor_state(st, o);
            if ((lane & o) == 0) st.merge(b); else { b.merge(st); st = b; }
        }
        if (g == 0 && i16 < a.M) a.parts[(size_t)i16 * a.n_parts + gw] = to_partial(st);
    }
}

}  // namespace rs
