// Router kernels: normalised entropy (Eq. 1), argmax and the switching flags
// (Eq. 2 / Algorithm 1) from partial single-pass softmax states.
#pragma once

#include "device_utils.h"
#include "../../include/rstitch.h"

namespace rs {

// Partial states of caller-provided fp32 logits: grid (n_parts, n_rows), block 256.
// Each workgroup strides over its row; partial p of row r lands in parts[r*n_parts + p].
__global__ void __launch_bounds__(256)
k_route_partials(const float *__restrict__ logits, int vocab, const float *__restrict__ scale,
                 SoftPartial *__restrict__ parts) {
    const int row = blockIdx.y, n_parts = gridDim.x;
    const float *x = logits + (size_t)row * vocab;
    const float sc = scale ? scale[row] : 1.f;
    SoftState st; st.init();
    const int tid = threadIdx.x, stride = n_parts * 256;
    if ((vocab & 3) == 0) {
        const float4 *x4 = reinterpret_cast<const float4 *>(x);
        for (int i = blockIdx.x * 256 + tid; i < (vocab >> 2); i += stride) {
            float4 v = x4[i];
            st.push(v.x * sc, 4 * i); st.push(v.y * sc, 4 * i + 1);
            st.push(v.z * sc, 4 * i + 2); st.push(v.w * sc, 4 * i + 3);
        }
    } else {
        for (int i = blockIdx.x * 256 + tid; i < vocab; i += stride) st.push(x[i] * sc, i);
    }
    wave_merge_state(st);
    __shared__ SoftPartial sh[4];
    if ((tid & 63) == 0) sh[tid >> 6] = to_partial(st);
    __syncthreads();
    if (tid == 0) {
        SoftState a = from_partial(sh[0]);
        for (int w = 1; w < 4; ++w) a.merge(from_partial(sh[w]));
        parts[(size_t)row * n_parts + blockIdx.x] = to_partial(a);
    }
}

// Final merge and routing decision for one row by one 256-thread workgroup.
// row_bad: optional per-row flag (nonzero = the row's inputs were out of range); sh: 4 SoftPartial of LDS.
// sample: the record's token is the arg max of logit + Gumbel noise (a draw from the distribution) instead of the arg max
__device__ __forceinline__ void route_merge_row(const SoftPartial *__restrict__ parts, int n_parts, int vocab, float tau,
                                                int active, const int *__restrict__ row_bad, rs_route_out *__restrict__ out,
                                                int row, SoftPartial *sh, int sample = 0) {
    const int tid = threadIdx.x;
    SoftState st; st.init();
    for (int p = tid; p < n_parts; p += 256) st.merge(from_partial(parts[(size_t)row * n_parts + p]));
    wave_merge_state(st);
    if ((tid & 63) == 0) sh[tid >> 6] = to_partial(st);
    __syncthreads();
    if (tid != 0) return;
    st = from_partial(sh[0]);
    for (int w = 1; w < 4; ++w) st.merge(from_partial(sh[w]));
    rs_route_out r;
    uint32_t flags = 0;
    const bool bad = row_bad && row_bad[row];
    if (bad || st.bad || !(st.z > 0.f)) {
        const float qnan = __uint_as_float(0x7fc00000u);
        flags = (bad ? RS_FLAG_BADARG : RS_FLAG_NONFINITE) | RS_FLAG_HI | RS_FLAG_NEXT_LLM;
        if (active == RS_LLM) flags |= RS_FLAG_ACCEPT;
        r.token = -1; r.h_nats = qnan; r.h_norm = qnan; r.max_logit = qnan; r.log_z = qnan;
    } else {
        const float lz = logf(st.z);
        float h = lz - st.s / st.z;
        h = fmaxf(h, 0.f);
        const float hn = h / logf((float)vocab);
        const bool hi = hn > tau;
        flags = (hi ? (RS_FLAG_HI | RS_FLAG_NEXT_LLM) : 0u);
        if (!(active == RS_SLM && hi)) flags |= RS_FLAG_ACCEPT;
        r.token = sample ? st.gidx : st.idx; r.h_nats = h; r.h_norm = hn; r.max_logit = st.m; r.log_z = st.m + lz;
    }
    r.flags = flags;
    out[row] = r;
}

// grid n_rows, block 256
__global__ void __launch_bounds__(256)
k_route_merge(const SoftPartial *__restrict__ parts, int n_parts, int vocab, float tau, int active,
              const int *__restrict__ row_bad, rs_route_out *__restrict__ out, int sample) {
    __shared__ SoftPartial sh[4];
    route_merge_row(parts, n_parts, vocab, tau, active, row_bad, out, blockIdx.x, sh, sample);
}

// ------------------------------------------------------------------------------------------------
// Router of R-Stitch+ (Section "Architecture and Overhead of Router"; Algorithm 1, R-Stitch+ branch):
// six residual feed-forward blocks x <- x + W2 gelu(W1 x + b1) + b2 with a bottleneck of r channels,
// a LayerNorm, a linear layer with two outputs (0 = stay on the small model, 1 = switch to the large
// one).  One workgroup of 256 threads per sequence; x (fp32, d values) lives in LDS; weights are bf16,
// accumulation fp32.  The record of the sequence is updated in place: a small-model step above tau
// whose router output prefers "stay" keeps its token and stays (RS_FLAG_ROUTER_STAY); every other
// record is left as the entropy rule made it.
// ------------------------------------------------------------------------------------------------
constexpr int ROUTER_BLOCKS = 6;
constexpr int ROUTER_RMAX = 64;

struct RouterPlusArgs {
    const uint16_t *w1[ROUTER_BLOCKS], *b1[ROUTER_BLOCKS], *w2[ROUTER_BLOCKS], *b2[ROUTER_BLOCKS];
    const uint16_t *ln_gain, *ln_bias, *w_head, *b_head;
    int d, r;
    float ln_eps;
    const float *hidden; int ld_hidden;       // rows of d floats, ld_hidden apart
    const int *gather;                         // row of sequence b inside `hidden`, or null (= b)
    int active;
    rs_route_out *out;                         // [n_seqs], updated in place
    float *logits;                             // [n_seqs, 2] or null
};

__device__ __forceinline__ float block_sum(float v, float *sh4) {        // 256 threads; sh4: 4 floats of LDS
    v = wave_sum(v);
    __syncthreads();                                                      // sh4 may still be read from the last call
    if ((threadIdx.x & 63) == 0) sh4[threadIdx.x >> 6] = v;
    __syncthreads();
    return sh4[0] + sh4[1] + sh4[2] + sh4[3];
}

// dynamic LDS: d floats
__global__ void __launch_bounds__(256) k_router_plus(RouterPlusArgs a) {
    extern __shared__ __align__(16) unsigned char smem[];
    float *x = reinterpret_cast<float *>(smem);
    __shared__ float t_sh[ROUTER_RMAX];
    __shared__ float red[4];
    const int b = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int d = a.d, r = a.r;
    const float *src = a.hidden + (size_t)(a.gather ? a.gather[b] : b) * a.ld_hidden;
    for (int i = tid; i < d; i += 256) x[i] = src[i];
    __syncthreads();
    for (int blk = 0; blk < ROUTER_BLOCKS; ++blk) {
        // t = gelu(W1 x + b1): wave w takes the rows w, w + 4, ...; lanes stride over d in chunks of 8
        for (int row = wave; row < r; row += 4) {
            const uint4 *wp = reinterpret_cast<const uint4 *>(a.w1[blk] + (size_t)row * d);
            float acc = 0.f;
            for (int c = lane; c < (d >> 3); c += 64) {
                const uint4 w = wp[c];
                const float4 xa = *reinterpret_cast<const float4 *>(x + 8 * c), xb = *reinterpret_cast<const float4 *>(x + 8 * c + 4);
                acc = fmaf(bf16_lo(w.x), xa.x, acc); acc = fmaf(bf16_hi(w.x), xa.y, acc); acc = fmaf(bf16_lo(w.y), xa.z, acc); acc = fmaf(bf16_hi(w.y), xa.w, acc);
                acc = fmaf(bf16_lo(w.z), xb.x, acc); acc = fmaf(bf16_hi(w.z), xb.y, acc); acc = fmaf(bf16_lo(w.w), xb.z, acc); acc = fmaf(bf16_hi(w.w), xb.w, acc);
            }
            acc = wave_sum(acc);
            if (lane == 0) {
                const float z = acc + bf16_to_f32(a.b1[blk][row]);
                t_sh[row] = 0.5f * z * (1.0f + erff(z * 0.70710678118654752f));
            }
        }
        __syncthreads();
        // x += W2 t + b2: one output channel per thread and round; a row of W2 is r bf16 values (r a multiple of 8)
        for (int i = tid; i < d; i += 256) {
            const uint4 *wp = reinterpret_cast<const uint4 *>(a.w2[blk] + (size_t)i * r);
            float acc = bf16_to_f32(a.b2[blk][i]);
            for (int c = 0; c < (r >> 3); ++c) {
                const uint4 w = wp[c];
                const float *t = t_sh + 8 * c;
                acc = fmaf(bf16_lo(w.x), t[0], acc); acc = fmaf(bf16_hi(w.x), t[1], acc); acc = fmaf(bf16_lo(w.y), t[2], acc); acc = fmaf(bf16_hi(w.y), t[3], acc);
                acc = fmaf(bf16_lo(w.z), t[4], acc); acc = fmaf(bf16_hi(w.z), t[5], acc); acc = fmaf(bf16_lo(w.w), t[6], acc); acc = fmaf(bf16_hi(w.w), t[7], acc);
            }
            x[i] += acc;
        }
        __syncthreads();
    }
    // LayerNorm (mean, then the mean of squared deviations), then the two outputs
    float s = 0.f;
    for (int i = tid; i < d; i += 256) s += x[i];
    const float mu = block_sum(s, red) / (float)d;
    float q = 0.f;
    for (int i = tid; i < d; i += 256) { const float dv = x[i] - mu; q = fmaf(dv, dv, q); }
    const float inv = 1.0f / sqrtf(block_sum(q, red) / (float)d + a.ln_eps);
    float o0 = 0.f, o1 = 0.f;
    for (int i = tid; i < d; i += 256) {
        const float y = (x[i] - mu) * inv * bf16_to_f32(a.ln_gain[i]) + bf16_to_f32(a.ln_bias[i]);
        o0 = fmaf(bf16_to_f32(a.w_head[i]), y, o0);
        o1 = fmaf(bf16_to_f32(a.w_head[d + i]), y, o1);
    }
    o0 = block_sum(o0, red);
    o1 = block_sum(o1, red);
    if (tid != 0) return;
    o0 += bf16_to_f32(a.b_head[0]);
    o1 += bf16_to_f32(a.b_head[1]);
    if (a.logits) { a.logits[2 * b] = o0; a.logits[2 * b + 1] = o1; }
    rs_route_out rec = a.out[b];
    const uint32_t untouchable = RS_FLAG_NONFINITE | RS_FLAG_BADARG | RS_FLAG_ABORTED;
    if (a.active == RS_SLM && (rec.flags & RS_FLAG_HI) && !(rec.flags & untouchable) && !(o1 > o0)) {
        rec.flags = (rec.flags | RS_FLAG_ACCEPT | RS_FLAG_ROUTER_STAY) & ~RS_FLAG_NEXT_LLM;
        a.out[b] = rec;
    }
}

}  // namespace rs
