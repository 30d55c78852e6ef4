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
__device__ __forceinline__ void route_merge_row(const SoftPartial *__restrict__ parts, int n_parts, int vocab, float tau,
                                                int active, const int *__restrict__ row_bad, rs_route_out *__restrict__ out,
                                                int row, SoftPartial *sh) {
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
        r.token = st.idx; r.h_nats = h; r.h_norm = hn; r.max_logit = st.m; r.log_z = st.m + lz;
    }
    r.flags = flags;
    out[row] = r;
}

// grid n_rows, block 256
__global__ void __launch_bounds__(256)
k_route_merge(const SoftPartial *__restrict__ parts, int n_parts, int vocab, float tau, int active,
              const int *__restrict__ row_bad, rs_route_out *__restrict__ out) {
    __shared__ SoftPartial sh[4];
    route_merge_row(parts, n_parts, vocab, tau, active, row_bad, out, blockIdx.x, sh);
}

}  // namespace rs
