// Device helpers shared by the gfx950 kernels: bf16 packing, wave64 reductions,
// and the single-pass softmax/entropy/argmax state with its associative merge.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#define RS_WAVE 64

namespace rs {

// ---------------------------------------------------------------- bf16 <-> fp32
__device__ __forceinline__ float bf16_lo(uint32_t packed) { return __uint_as_float(packed << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t packed) { return __uint_as_float(packed & 0xffff0000u); }
__device__ __forceinline__ float bf16_to_f32(uint16_t b) { return __uint_as_float(((uint32_t)b) << 16); }

// round to nearest even, NaN stays NaN: the hardware conversion (v_cvt_pk_bf16_f32)
typedef __bf16 rs_bf16x2_t __attribute__((ext_vector_type(2)));
typedef float rs_f32x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint16_t f32_to_bf16(float f) { return __builtin_bit_cast(uint16_t, (__bf16)f); }
__device__ __forceinline__ float round_bf16(float f) { return bf16_to_f32(f32_to_bf16(f)); }
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
    return __builtin_bit_cast(uint32_t, __builtin_convertvector((rs_f32x2_t){lo, hi}, rs_bf16x2_t));
}

// dot product of 8 bf16 weights (one 16-byte load) with 8 bf16 activations, fp32 accumulate
__device__ __forceinline__ float dot8(const uint4 &w, const uint4 &x, float acc) {
    acc = fmaf(bf16_lo(w.x), bf16_lo(x.x), acc);
    acc = fmaf(bf16_hi(w.x), bf16_hi(x.x), acc);
    acc = fmaf(bf16_lo(w.y), bf16_lo(x.y), acc);
    acc = fmaf(bf16_hi(w.y), bf16_hi(x.y), acc);
    acc = fmaf(bf16_lo(w.z), bf16_lo(x.z), acc);
    acc = fmaf(bf16_hi(w.z), bf16_hi(x.z), acc);
    acc = fmaf(bf16_lo(w.w), bf16_lo(x.w), acc);
    acc = fmaf(bf16_hi(w.w), bf16_hi(x.w), acc);
    return acc;
}

// streaming 16-byte load of weights that are read exactly once per step
typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 load_stream(const uint4 *p) {
    const u32x4_t v = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t *>(p));
    return make_uint4(v.x, v.y, v.z, v.w);
}

// ---------------------------------------------------------------- wave64 reductions
// Cross-lane steps as DPP operands of the add / max itself (no LDS round trip per step): two
// quad permutes and two mirrors leave every lane with the total of its row of 16; row_bcast15
// and row_bcast31 then carry the row totals upward so that lane 63 holds the wave's total, which
// a readlane broadcasts.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ float dpp_f32(float old, float v) {
    return __int_as_float(__builtin_amdgcn_update_dpp(__float_as_int(old), __float_as_int(v), CTRL, ROW_MASK, 0xf, false));
}
__device__ __forceinline__ float wave_sum(float v) {
    v += dpp_f32<0xB1, 0xf>(0.f, v);      // quad_perm [1,0,3,2]
    v += dpp_f32<0x4E, 0xf>(0.f, v);      // quad_perm [2,3,0,1]
    v += dpp_f32<0x141, 0xf>(0.f, v);     // row_half_mirror
    v += dpp_f32<0x140, 0xf>(0.f, v);     // row_mirror
    v += dpp_f32<0x142, 0xa>(0.f, v);     // row_bcast15 into rows 1 and 3
    v += dpp_f32<0x143, 0xc>(0.f, v);     // row_bcast31 into rows 2 and 3
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 63));
}
__device__ __forceinline__ float wave_max(float v) {
    v = fmaxf(v, dpp_f32<0xB1, 0xf>(v, v));
    v = fmaxf(v, dpp_f32<0x4E, 0xf>(v, v));
    v = fmaxf(v, dpp_f32<0x141, 0xf>(v, v));
    v = fmaxf(v, dpp_f32<0x140, 0xf>(v, v));
    v = fmaxf(v, dpp_f32<0x142, 0xa>(v, v));
    v = fmaxf(v, dpp_f32<0x143, 0xc>(v, v));
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 63));
}

// ---------------------------------------------------------------- softmax / entropy / argmax in one pass
// Carries m = max, z = sum e^(x-m), s = sum (x-m) e^(x-m), the running argmax
// (lowest index among equal maxima) and whether a non-finite value was seen.
// Entropy of softmax(x) in nats is ln z - s / z  (the quantity of Eq. 1 before
// it is divided by ln V).  merge() is associative and commutative up to
// rounding, so partial states can be combined in any tree.
// Sampling (Section "Preliminary": the next token is drawn from the step's distribution): the state also carries
// the running argmax of logit + Gumbel noise, whose arg max over the vocabulary is a draw from softmax(logits).
// The noise of vocabulary entry i at a position is -ln(-ln u) with u = (n + 0.5) 2^-23, n the top 23 bits of a
// 64-bit hash of the counter position * V + i under the caller's key (a finaliser of the splitmix family on a
// keyed counter: the generator of the synthetic workloads, so a CPU check can draw the same numbers).
__device__ __forceinline__ float gumbel_noise(unsigned long long key, unsigned long long counter) {
    unsigned long long x = counter * 0x9E3779B97F4A7C15ull + key;
    x = (x ^ (x >> 30)) * 0xBF58476D1CE4E5B9ull;
    x = (x ^ (x >> 27)) * 0x94D049BB133111EBull;
    x ^= x >> 31;
    const float u = ((float)(unsigned int)(x >> 41) + 0.5f) * 1.1920928955078125e-07f;      // 2^-23; exact in fp32
    return -logf(-logf(u));
}

struct SoftState {
    float m, z, s, best;
    int idx, bad;
    float gbest; int gidx;            // sampling only: largest logit + noise so far and its index

    __device__ __forceinline__ void init() {
        m = -INFINITY; z = 0.f; s = 0.f; best = -INFINITY; idx = 0x7fffffff; bad = 0;
        gbest = -INFINITY; gidx = 0x7fffffff;
    }
    // x has been (or will be) pushed as well; i is its vocabulary index, base = position * V
    __device__ __forceinline__ void push_noisy(float x, int i, unsigned long long key, unsigned long long base) {
        if (!(fabsf(x) <= 3.0e38f)) return;
        const float v = x + gumbel_noise(key, base + (unsigned long long)i);
        if (v > gbest || (v == gbest && i < gidx)) { gbest = v; gidx = i; }
    }
    __device__ __forceinline__ void push(float x, int i) {
        if (!(fabsf(x) <= 3.0e38f)) { bad = 1; return; }     // NaN or +-Inf
        if (x > best || (x == best && i < idx)) { best = x; idx = i; }
        if (x > m) {
            if (z > 0.f) { float d = m - x, e = expf(d); s = e * (s + d * z); z = z * e + 1.f; }
            else { s = 0.f; z = 1.f; }
            m = x;
        } else {
            float d = x - m, e = expf(d);
            z += e; s = fmaf(d, e, s);
        }
    }
    __device__ __forceinline__ void merge(const SoftState &o) {
        bad |= o.bad;
        if (o.best > best || (o.best == best && o.idx < idx)) { best = o.best; idx = o.idx; }
        if (o.gbest > gbest || (o.gbest == gbest && o.gidx < gidx)) { gbest = o.gbest; gidx = o.gidx; }
        if (o.z <= 0.f) return;
        if (z <= 0.f) { m = o.m; z = o.z; s = o.s; return; }
        float mm = fmaxf(m, o.m);
        float da = m - mm, db = o.m - mm;
        float ea = expf(da), eb = expf(db);
        s = ea * (s + da * z) + eb * (o.s + db * o.z);
        z = z * ea + o.z * eb;
        m = mm;
    }
};

__device__ __forceinline__ SoftState shfl_xor_state(const SoftState &a, int o) {
    SoftState b;
    b.m = __shfl_xor(a.m, o, RS_WAVE);
    b.z = __shfl_xor(a.z, o, RS_WAVE);
    b.s = __shfl_xor(a.s, o, RS_WAVE);
    b.best = __shfl_xor(a.best, o, RS_WAVE);
    b.idx = __shfl_xor(a.idx, o, RS_WAVE);
    b.bad = __shfl_xor(a.bad, o, RS_WAVE);
    b.gbest = __shfl_xor(a.gbest, o, RS_WAVE);
    b.gidx = __shfl_xor(a.gidx, o, RS_WAVE);
    return b;
}

// all lanes end up with the merged state of the lanes that share the bits of
// the lane id NOT covered by `span` (span = 64: whole wave; span = 16: groups of 16)
__device__ __forceinline__ void wave_merge_state(SoftState &a, int span = RS_WAVE) {
    for (int o = span >> 1; o > 0; o >>= 1) {
        SoftState b = shfl_xor_state(a, o);
        // merge in a fixed order (lower lane first) so that both partners compute the same bits
        if ((threadIdx.x & o) == 0) { a.merge(b); }
        else { b.merge(a); a = b; }
    }
}

// What a workgroup (or wave) leaves in global memory for the final merge: 32 bytes.
struct __align__(16) SoftPartial {
    float m, z, s, best;
    int idx, bad;
    float gbest; int gidx;
};
__device__ __forceinline__ SoftPartial to_partial(const SoftState &a) {
    SoftPartial p; p.m = a.m; p.z = a.z; p.s = a.s; p.best = a.best; p.idx = a.idx; p.bad = a.bad; p.gbest = a.gbest; p.gidx = a.gidx;
    return p;
}
__device__ __forceinline__ SoftState from_partial(const SoftPartial &p) {
    SoftState a; a.m = p.m; a.z = p.z; a.s = p.s; a.best = p.best; a.idx = p.idx; a.bad = p.bad; a.gbest = p.gbest; a.gidx = p.gidx;
    return a;
}

}  // namespace rs
