// Gated-GELU expert FFN (the FFN_GEGLU variant of the paper's model tables): the
// element-wise half of the first layer.  The first GEMM leaves H = Xd W_in = [u | v]
// (gate pre-activations, linear part; f columns each), these kernels turn it into
//   forward   A  = GELU(u) v q  (times the token's gate when the combine runs inside the GEMMs)
//                                                    GELU(u) = u Phi(u), exact
//   backward  du = dA q v GELU'(u),  dv = dA q GELU(u),  dH = [du | dv]
// with q the expert-dropout factor of the hidden unit (1 without dropout; Sec. 2.4).
// Both are streaming kernels: one lane handles 16 bytes of consecutive hidden units of
// one slot row (eight bf16 or four fp32), rows past an expert's kept tokens are skipped.
// Arithmetic is fp32, one rounding at the store.
#include "common.h"

namespace sw {

// Phi(u) and the density phi(u) of the standard normal distribution, sharing one exponential.
// erfc(z), z = |u| / sqrt 2 >= 0, comes from the rational approximation 7.1.26 of Abramowitz &
// Stegun, erfc(z) = (a1 t + ... + a5 t^5) exp(-z^2), t = 1 / (1 + p z), |error| <= 1.5e-7: a
// dozen instructions instead of the library erfc's sixty (the streaming kernels below are
// otherwise bound by their arithmetic, not by HBM).  The error of GELU(u) = u Phi(u) is
// |u| * 7.5e-8, two orders below the fp32 tolerance of the layer.
struct NormalOf {
    float cdf, pdf;
};
__device__ __forceinline__ NormalOf normal_of(float u) {
    const float z = fabsf(u) * 0.70710678f;
    const float t = __builtin_amdgcn_rcpf(fmaf(0.3275911f, z, 1.0f));   // 1 ulp: far inside the error of the fit
    const float e = __expf(-z * z);
    float poly = fmaf(1.061405429f, t, -1.453152027f);
    poly = fmaf(poly, t, 1.421413741f);
    poly = fmaf(poly, t, -0.284496736f);
    poly = fmaf(poly, t, 0.254829592f);
    const float half_erfc = 0.5f * poly * t * e;
    NormalOf r;
    r.cdf = u >= 0.f ? 1.0f - half_erfc : half_erfc;
    r.pdf = 0.3989422804f * e;
    return r;
}

// 16 bytes of hidden units
template <typename XT> struct Chunk;
template <> struct Chunk<bf16> {
    typedef bf16 type __attribute__((ext_vector_type(8)));
    static constexpr int n = 8;
};
template <> struct Chunk<float> {
    typedef float type __attribute__((ext_vector_type(4)));
    static constexpr int n = 4;
};

template <typename XT, bool BACKWARD>
__global__ __launch_bounds__(256) void geglu_kernel(const XT *__restrict__ H,
                                                    const XT *__restrict__ dA,
                                                    XT *__restrict__ out,   // A (forward) or dH
                                                    const int32_t *__restrict__ kept,
                                                    const int32_t *__restrict__ slot_token,
                                                    const float *__restrict__ slot_gate,
                                                    int slots, int f, Noise nz) {
    typedef typename Chunk<XT>::type V;
    constexpr int kGegluChunk = Chunk<XT>::n;
    const int e = blockIdx.y;
    const int chunks_per_row = f / kGegluChunk;
    const long chunk = (long)blockIdx.x * 256 + threadIdx.x;
    const int row = (int)(chunk / chunks_per_row);
    if (row >= kept[e]) return;
    const int j0 = (int)(chunk - (long)row * chunks_per_row) * kGegluChunk;
    const size_t slot = (size_t)e * slots + row;
    const XT *h = H + slot * 2 * f;
    const V u = *(const V *)(h + j0);
    const V v = *(const V *)(h + f + j0);
    float q[kGegluChunk];
#pragma unroll
    for (int i = 0; i < kGegluChunk; ++i) q[i] = 1.f;
    if (nz.dropout) {
        const uint32_t idx = (uint32_t)slot_token[slot] * (uint32_t)f + (uint32_t)j0;
        // j0 is a multiple of the chunk and f is even: the chunk is whole aligned pairs
#pragma unroll
        for (int i = 0; i < kGegluChunk; i += 2) {
            const uint32_t z = dropout_pair_bits(nz, (idx + (uint32_t)i) >> 1);
            q[i] = dropout_keeps_even(nz, z) ? nz.drop_scale : 0.f;
            q[i + 1] = dropout_keeps_odd(nz, z) ? nz.drop_scale : 0.f;
        }
    }
    if (!BACKWARD) {
        // slot_gate set: the hidden row is stored times its token's gate, so that the second
        // GEMM's rows are the layer's output rows (combine inside the GEMMs)
        const float g = slot_gate ? slot_gate[slot] : 1.f;
        V a;
#pragma unroll
        for (int i = 0; i < kGegluChunk; ++i)
            a[i] = from_f32<XT>(to_f32(u[i]) * normal_of(to_f32(u[i])).cdf * to_f32(v[i]) * q[i] * g);
        *(V *)(out + slot * f + j0) = a;
    } else {
        const V da = *(const V *)(dA + slot * f + j0);
        V du, dv;
#pragma unroll
        for (int i = 0; i < kGegluChunk; ++i) {
            const float s = to_f32(da[i]) * q[i];
            const float ui = to_f32(u[i]);
            const NormalOf n = normal_of(ui);
            du[i] = from_f32<XT>(s * to_f32(v[i]) * fmaf(ui, n.pdf, n.cdf));   // GELU' = Phi + u phi
            dv[i] = from_f32<XT>(s * ui * n.cdf);
        }
        XT *o = out + slot * 2 * f;
        *(V *)(o + j0) = du;
        *(V *)(o + f + j0) = dv;
    }
}

template <typename XT, bool BACKWARD>
static hipError_t geglu_launch(const Workspace &w, char *ws, hipStream_t s) {
    if (w.C == 0) return hipSuccess;
    const long chunks = (long)w.C * (w.f / Chunk<XT>::n);
    dim3 grid((unsigned)ceil_div(chunks, 256), (unsigned)w.E);
    hipLaunchKernelGGL((geglu_kernel<XT, BACKWARD>), grid, dim3(256), 0, s,
                       (const XT *)(ws + w.H), (const XT *)(ws + w.dA),
                       (XT *)(ws + (BACKWARD ? w.dH : w.A)), (const int32_t *)(ws + w.kept),
                       (const int32_t *)(ws + w.slot_token),
                       (!BACKWARD && w.fused) ? (const float *)(ws + w.slot_gate) : nullptr, (int)w.C,
                       (int)w.f, w.noise);
    return hipGetLastError();
}

hipError_t launch_geglu_fwd(const Workspace &w, int dtype, char *ws, hipStream_t s) {
    ProfScope ps("geglu_fwd", s);
    return dtype == SW_BF16 ? geglu_launch<bf16, false>(w, ws, s)
                            : geglu_launch<float, false>(w, ws, s);
}

hipError_t launch_geglu_bwd(const Workspace &w, int dtype, char *ws, hipStream_t s) {
    ProfScope ps("geglu_bwd", s);
    return dtype == SW_BF16 ? geglu_launch<bf16, true>(w, ws, s)
                            : geglu_launch<float, true>(w, ws, s);
}

}  // namespace sw
