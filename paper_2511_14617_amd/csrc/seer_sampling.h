// Reproducible Gumbel noise for verification under sampling (Section 4.1: the paper's workloads
// sample at temperature 1.0 and 0.8; its drafts are token sequences, so lossless verification
// draws the target model's token at each verify position and compares).  A draw from
// softmax(logits / tau) is argmax_v (logits[v] / tau + G_v) with independent standard Gumbel G_v,
// which turns sampled verification into the greedy rule on perturbed logits.
//
// G_v is a pure function of (seed, row, v), so that a run can be replayed and checked:
//   Philox4x32-10 (Salmon et al., SC'11), counter (v / 4, row, 0, 0), key (seed low, seed high),
//   element v takes output word v % 4;  u = ((w >> 9) + 0.5) * 2^-23;
//   E = -log2(u) * ln2;  G = -log2(E) * ln2;  log2 by a fixed degree-8 polynomial in fused
//   multiply-adds.  Every fp32 operation is an IEEE-754 one written out explicitly (no contraction),
//   because the result decides an integer (an argmax) and must not depend on the compiler.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace seer {

struct Philox4 {
    uint32_t w[4];
};

__device__ __forceinline__ Philox4 philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3, uint32_t k0,
                                                 uint32_t k1) {
#pragma unroll
    for (int round = 0; round < 10; ++round) {
        const uint64_t p0 = static_cast<uint64_t>(0xD2511F53u) * c0;
        const uint64_t p1 = static_cast<uint64_t>(0xCD9E8D57u) * c2;
        const uint32_t n0 = static_cast<uint32_t>(p1 >> 32) ^ c1 ^ k0;
        const uint32_t n2 = static_cast<uint32_t>(p0 >> 32) ^ c3 ^ k1;
        c1 = static_cast<uint32_t>(p1);
        c3 = static_cast<uint32_t>(p0);
        c0 = n0;
        c2 = n2;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    return Philox4{{c0, c1, c2, c3}};
}

// log2 of a positive normal float: exponent + polynomial of the mantissa moved to [sqrt(1/2), sqrt(2))
__device__ __forceinline__ float log2_fixed(float x) {
#pragma clang fp contract(off)
    uint32_t bits = __float_as_uint(x);
    int e = static_cast<int>(bits >> 23) - 127;
    float m = __uint_as_float((bits & 0x007fffffu) | 0x3f800000u);
    if (m > 1.41421354f) {
        m = m * 0.5f;
        e += 1;
    }
    const float f = m - 1.0f;
    float p = 0.12614846229553223f;
    p = __builtin_fmaf(p, f, -0.20742103457450867f);
    p = __builtin_fmaf(p, f, 0.21566985547542572f);
    p = __builtin_fmaf(p, f, -0.23892034590244293f);
    p = __builtin_fmaf(p, f, 0.2879183292388916f);
    p = __builtin_fmaf(p, f, -0.36070483922958374f);
    p = __builtin_fmaf(p, f, 0.48091059923171997f);
    p = __builtin_fmaf(p, f, -0.7213473320007324f);
    p = __builtin_fmaf(p, f, 1.4426950216293335f);
    return __builtin_fmaf(f, p, static_cast<float>(e));
}

__device__ __forceinline__ float gumbel_from_word(uint32_t w) {
#pragma clang fp contract(off)
    const float u = (static_cast<float>(w >> 9) + 0.5f) * 1.1920928955078125e-07f;   // 2^-23
    const float e = -log2_fixed(u) * 0.693147182f;
    return -(log2_fixed(e) * 0.693147182f);
}

// logits[v] / tau + G_v as one fused multiply-add
__device__ __forceinline__ float perturb(float logit, float inv_tau, uint32_t w) {
    return __builtin_fmaf(logit, inv_tau, gumbel_from_word(w));
}

}  // namespace seer
