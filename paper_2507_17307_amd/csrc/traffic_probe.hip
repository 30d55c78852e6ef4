// Stand-alone driver for hardware-counter runs: a few decode steps of a model of
// the given shape through the C ABI, with plain launches, plus a copy kernel
// that reads and writes a known number of bytes.  A profiler's byte counters
// (FETCH_SIZE, WRITE_SIZE) for the library's kernels are scaled by what the same
// counter reports for that copy.  No framework is loaded, so counter collection
// sees only these dispatches.
//
//   traffic_probe <s15|m7|m14|m32> [layers=2] [steps=6] [position=4575] [span=1]
//
// (context capacity 4608 for s15 and m7, 9216 for m14, 10240 for m32)
//
// span > 1 runs catch-up calls of that many token rows ending at `position` instead of decode steps
// (the matrix-core path).
//
// Weights are a fixed byte pattern (their values do not matter for traffic), the
// KV cache is zero-filled up to `position`.
#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "../../include/rstitch.h"

#define CK(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { fprintf(stderr, "%s: %s\n", #x, hipGetErrorString(e_)); return 1; } } while (0)

__global__ void __launch_bounds__(256) k_probe_copy(const uint4 *__restrict__ src, uint4 *__restrict__ dst, size_t n16) {
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += (size_t)gridDim.x * 256) dst[i] = src[i];
}

int main(int argc, char **argv) {
    const char *shape = argc > 1 ? argv[1] : "m7";
    const int layers = argc > 2 ? atoi(argv[2]) : 2;
    const int steps = argc > 3 ? atoi(argv[3]) : 6;
    const int position = argc > 4 ? atoi(argv[4]) : 4575;
    const int span = argc > 5 ? atoi(argv[5]) : 1;
    rs_config c{};
    if (!strcmp(shape, "s15")) { c.d_model = 1536; c.n_q_heads = 12; c.n_kv_heads = 2; c.d_ffn = 8960; }
    else if (!strcmp(shape, "m7")) { c.d_model = 3584; c.n_q_heads = 28; c.n_kv_heads = 4; c.d_ffn = 18944; }
    else if (!strcmp(shape, "m14")) { c.d_model = 5120; c.n_q_heads = 40; c.n_kv_heads = 8; c.d_ffn = 13824; c.max_ctx = 9216; }
    else if (!strcmp(shape, "m32")) { c.d_model = 5120; c.n_q_heads = 40; c.n_kv_heads = 8; c.d_ffn = 27648; c.max_ctx = 10240; }
    else { fprintf(stderr, "shape must be s15, m7, m14 or m32\n"); return 2; }
    c.n_layers = layers; c.head_dim = 128; c.vocab = 152064; c.tied_lm_head = 1;
    if (!c.max_ctx) c.max_ctx = 4608;
    c.max_seqs = 1; c.max_rows = 128; c.rms_eps = 1e-6f; c.rope_theta = 1e6f;
    if (layers < 1 || layers > 64 || steps < 1 || position < 0 || position >= c.max_ctx || span < 1 || span > 128 || span > position + 1) { fprintf(stderr, "bad arguments\n"); return 2; }
    setenv("RSTITCH_GRAPHS", "0", 1);                      // plain launches: one dispatch per kernel for the profiler

    const size_t qkv_rows = (size_t)(c.n_q_heads + 2 * c.n_kv_heads) * c.head_dim, qdim = (size_t)c.n_q_heads * c.head_dim;
    auto dev_fill = [](size_t bytes, int byte, void **out) -> hipError_t {
        hipError_t e = hipMalloc(out, bytes);
        if (e != hipSuccess) return e;
        return hipMemset(*out, byte, bytes);
    };
    // 0x3c3c as bf16 is about 0.0115: small finite weights; gains 0x3f80 = 1.0
    void *embed, *final_norm;
    CK(dev_fill((size_t)c.vocab * c.d_model * 2, 0x3c, &embed));
    std::vector<uint16_t> ones(c.d_model, 0x3f80);
    CK(hipMalloc(&final_norm, c.d_model * 2));
    CK(hipMemcpy(final_norm, ones.data(), c.d_model * 2, hipMemcpyHostToDevice));
    std::vector<const void *> an(layers), wq(layers), wo(layers), mn(layers), wg(layers), wd(layers);
    for (int l = 0; l < layers; ++l) {
        void *p;
        an[l] = final_norm; mn[l] = final_norm;
        CK(dev_fill(qkv_rows * c.d_model * 2, 0x3c, &p)); wq[l] = p;
        CK(dev_fill((size_t)c.d_model * qdim * 2, 0x3c, &p)); wo[l] = p;
        CK(dev_fill((size_t)2 * c.d_ffn * c.d_model * 2, 0x3c, &p)); wg[l] = p;
        CK(dev_fill((size_t)c.d_model * c.d_ffn * 2, 0x3c, &p)); wd[l] = p;
    }
    rs_weights w{};
    w.embed = embed; w.lm_head = embed; w.final_norm = final_norm;
    w.attn_norm = an.data(); w.w_qkv = wq.data(); w.w_o = wo.data(); w.mlp_norm = mn.data(); w.w_gate_up = wg.data(); w.w_down = wd.data();

    void *kv_k, *kv_v, *ws;
    const size_t kvb = rs_kv_bytes(&c), wsb = rs_workspace_bytes(&c);
    if (!kvb || !wsb) { fprintf(stderr, "configuration rejected: %s\n", rs_last_error()); return 1; }
    CK(dev_fill(kvb, 0, &kv_k)); CK(dev_fill(kvb, 0, &kv_v)); CK(dev_fill(wsb, 0, &ws));
    rs_model *m = nullptr;
    if (rs_create_model(&c, &w, kv_k, kv_v, ws, wsb, &m) != RS_OK) { fprintf(stderr, "rs_create_model: %s\n", rs_last_error()); return 1; }

    // control block: slot, first position of the span, span offsets {0, span}, then the span's tokens
    std::vector<int32_t> h_ctl(4 + 64, 17);
    h_ctl[0] = 0; h_ctl[1] = position - span + 1; h_ctl[2] = 0; h_ctl[3] = span;
    float h_scale = 1.0f;
    int32_t *d_ctl; float *d_scale; rs_route_out *d_out;
    CK(hipMalloc(&d_ctl, h_ctl.size() * 4)); CK(hipMalloc(&d_scale, 4)); CK(hipMalloc(&d_out, sizeof(rs_route_out)));
    CK(hipMemcpy(d_ctl, h_ctl.data(), h_ctl.size() * 4, hipMemcpyHostToDevice)); CK(hipMemcpy(d_scale, &h_scale, 4, hipMemcpyHostToDevice));
    hipStream_t st; CK(hipStreamCreate(&st));

    // the known-size dispatch: 2^28 bytes read, 2^28 bytes written, three times
    const size_t copy_bytes = (size_t)1 << 28;
    void *src, *dst;
    CK(dev_fill(copy_bytes, 1, &src)); CK(dev_fill(copy_bytes, 0, &dst));
    for (int i = 0; i < 3; ++i)
        hipLaunchKernelGGL(k_probe_copy, dim3(2048), dim3(256), 0, st, (const uint4 *)src, (uint4 *)dst, copy_bytes / 16);
    CK(hipStreamSynchronize(st));

    for (int i = 0; i < steps; ++i) {
        const rs_status rc = span == 1
            ? rs_decode_step(m, 1, d_ctl, d_ctl + 4, d_ctl + 1, d_scale, 0.5f, RS_LLM, d_out, nullptr, st)
            : rs_catchup_prefill(m, 1, span, d_ctl, d_ctl + 4, d_ctl + 2, d_ctl + 1, d_scale, 0.5f, RS_LLM, d_out, nullptr, st);
        if (rc != RS_OK) { fprintf(stderr, "forward call: %s\n", rs_last_error()); return 1; }
    }
    CK(hipStreamSynchronize(st));
    rs_route_out r;
    CK(hipMemcpy(&r, d_out, sizeof r, hipMemcpyDeviceToHost));
    printf("traffic_probe %s layers=%d steps=%d position=%d span=%d: token %d flags %u h_norm %.6f; copy kernel k_probe_copy moved %zu bytes each way\n",
           shape, layers, steps, position, span, r.token, r.flags, r.h_norm, copy_bytes);
    rs_destroy_model(m);
    return 0;
}
