// Grouped expert GEMMs for the all-fp32 configuration (act_dtype = SW_F32).
// A plain LDS-tiled FMA kernel with generic strides: this path exists for the
// fp32 parity configuration, not for throughput.
#include "common.h"

namespace sw {

struct GemmF32Args {
    const float *Q;      // Q_e(q,k) = Q[e*q_batch + q*q_rs + k*q_ks]
    const float *P;      // P_e(p,k) = P[e*p_batch + p*p_rs + k*p_ks]
    float *Cout;         // C_e[q][p] = Cout[e*c_batch + q*ldc + p]
    const float *mask;   // same layout as Cout, or nullptr
    size_t q_batch, p_batch, c_batch;
    long q_rs, q_ks, p_rs, p_ks, ldc;
    int Qdim, Pdim, Kdim;
    const int32_t *kept;
    int q_limited;       // rows q >= kept[e] are not computed / stored
    int k_limited;       // reduction runs over k < kept[e]
    int epi;             // 0 none, 1 ReLU (+ expert dropout), 2 multiply by [mask > 0] (and by
                         // the dropout scale of the surviving units)
    const int32_t *slot_token;   // epi 1 with dropout: token of slot e * slots + q
    long slots;
    Noise nz;
};

constexpr int kF32Tile = 64;
constexpr int kF32KC = 16;
constexpr int kF32Flush = 256;   // products per chain of the two-level sum

__global__ __launch_bounds__(256) void gemm_f32_kernel(GemmF32Args a) {
    __shared__ float qs[kF32KC][kF32Tile + 4];
    __shared__ float ps[kF32KC][kF32Tile + 4];
    const int e = blockIdx.z;
    const int q0 = blockIdx.y * kF32Tile;
    const int p0 = blockIdx.x * kF32Tile;
    const int lim = a.kept[e];
    const int qlim = a.q_limited ? (lim < a.Qdim ? lim : a.Qdim) : a.Qdim;
    const int klim = a.k_limited ? (lim < a.Kdim ? lim : a.Kdim) : a.Kdim;
    if (q0 >= qlim) return;
    const float *Q = a.Q + (size_t)e * a.q_batch;
    const float *P = a.P + (size_t)e * a.p_batch;
    const int tid = threadIdx.x;
    const int tx = tid % 16, ty = tid / 16;
    // Two-level sums: a running chain of at most kF32Flush products is folded into a total, so
    // that the rounding error of a long reduction (thousands of slots in a weight gradient)
    // grows with the square roots of the two lengths instead of with the whole length.
    float acc[4][4], total[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = total[i][j] = 0.f;
    for (int k0 = 0; k0 < klim; k0 += kF32KC) {
        if (k0 != 0 && k0 % kF32Flush == 0) {
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    total[i][j] += acc[i][j];
                    acc[i][j] = 0.f;
                }
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int id = tid + i * 256;
            int r, kk;
            // pick the faster-varying index to be the contiguous one in memory
            if (a.q_ks == 1) { kk = id % kF32KC; r = id / kF32KC; } else { r = id % kF32Tile; kk = id / kF32Tile; }
            float v = 0.f;
            if (q0 + r < qlim && k0 + kk < klim) v = Q[(long)(q0 + r) * a.q_rs + (long)(k0 + kk) * a.q_ks];
            qs[kk][r] = v;
            if (a.p_ks == 1) { kk = id % kF32KC; r = id / kF32KC; } else { r = id % kF32Tile; kk = id / kF32Tile; }
            v = 0.f;
            if (p0 + r < a.Pdim && k0 + kk < klim) v = P[(long)(p0 + r) * a.p_rs + (long)(k0 + kk) * a.p_ks];
            ps[kk][r] = v;
        }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < kF32KC; ++kk) {
            float qv[4], pv[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) qv[i] = qs[kk][ty * 4 + i];
#pragma unroll
            for (int j = 0; j < 4; ++j) pv[j] = ps[kk][tx * 4 + j];
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(qv[i], pv[j], acc[i][j]);
        }
        __syncthreads();
    }
    float *Cout = a.Cout + (size_t)e * a.c_batch;
    const float *mask = a.mask ? a.mask + (size_t)e * a.c_batch : nullptr;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int q = q0 + ty * 4 + i;
        if (q >= qlim) continue;
        uint32_t row_idx = 0;   // index of the token's first hidden unit in the dropout stream
        if (a.epi == 1 && a.nz.dropout)
            row_idx = (uint32_t)a.slot_token[(size_t)e * a.slots + q] * (uint32_t)a.Pdim;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int p = p0 + tx * 4 + j;
            if (p >= a.Pdim) continue;
            float v = total[i][j] + acc[i][j];
            if (a.epi == 1) {
                v = v > 0.f ? v : 0.f;
                if (a.nz.dropout)   // Sec. 2.4: expert dropout on the hidden activation
                    v = dropout_keeps(a.nz, row_idx + (uint32_t)p) ? v * a.nz.drop_scale : 0.f;
            }
            // a unit passes the gradient iff it was active and survived dropout
            if (a.epi == 2) v = mask[(long)q * a.ldc + p] > 0.f ? v * a.nz.drop_scale : 0.f;
            Cout[(long)q * a.ldc + p] = v;
        }
    }
}

hipError_t launch_gemm_f32(GemmKind kind, const Workspace &w, char *ws, const void *W_in,
                           const void *W_out, void *dW_in, void *dW_out, const TokenMajor &,
                           hipStream_t s) {
    const long d = w.d, f = w.f, f1 = w.f1, C = w.C;
    GemmF32Args a{};
    a.kept = (const int32_t *)(ws + w.kept);
    a.slot_token = (const int32_t *)(ws + w.slot_token);
    a.slots = C;
    a.nz = w.noise;
    const float *Xd = (const float *)(ws + w.Xd);
    float *A = (float *)(ws + w.A);
    float *O = (float *)(ws + w.O);
    const float *dO = (const float *)(ws + w.dO);
    float *dH = (float *)(ws + w.dH);
    float *dXd = (float *)(ws + w.dXd);
    const char *name = "";
    switch (kind) {
    case GEMM_FWD1:
        name = w.geglu ? "gemm1_fwd" : "gemm1_fwd_relu";
        a.Q = Xd; a.q_batch = C * d; a.q_rs = d; a.q_ks = 1;
        a.P = (const float *)W_in; a.p_batch = d * f1; a.p_rs = 1; a.p_ks = f1;
        a.Cout = w.geglu ? (float *)(ws + w.H) : A; a.c_batch = C * f1; a.ldc = f1;
        a.Qdim = C; a.Pdim = f1; a.Kdim = d; a.q_limited = 1; a.epi = w.geglu ? 0 : 1;
        break;
    case GEMM_FWD2:
        name = "gemm2_fwd";
        a.Q = A; a.q_batch = C * f; a.q_rs = f; a.q_ks = 1;
        a.P = (const float *)W_out; a.p_batch = f * d; a.p_rs = 1; a.p_ks = d;
        a.Cout = O; a.c_batch = C * d; a.ldc = d;
        a.Qdim = C; a.Pdim = d; a.Kdim = f; a.q_limited = 1;
        break;
    case GEMM_DGRAD2:
        name = w.geglu ? "gemm2_dgrad" : "gemm2_dgrad_relumask";
        a.Q = dO; a.q_batch = C * d; a.q_rs = d; a.q_ks = 1;
        a.P = (const float *)W_out; a.p_batch = f * d; a.p_rs = d; a.p_ks = 1;
        a.Cout = w.geglu ? (float *)(ws + w.dA) : dH; a.c_batch = C * f; a.ldc = f; a.mask = A;
        a.Qdim = C; a.Pdim = f; a.Kdim = d; a.q_limited = 1; a.epi = w.geglu ? 0 : 2;
        break;
    case GEMM_DGRAD1:
        name = "gemm1_dgrad";
        a.Q = dH; a.q_batch = C * f1; a.q_rs = f1; a.q_ks = 1;
        a.P = (const float *)W_in; a.p_batch = d * f1; a.p_rs = f1; a.p_ks = 1;
        a.Cout = dXd; a.c_batch = C * d; a.ldc = d;
        a.Qdim = C; a.Pdim = d; a.Kdim = f1; a.q_limited = 1;
        break;
    case GEMM_WGRAD2:
        name = "gemm2_wgrad";
        a.Q = A; a.q_batch = C * f; a.q_rs = 1; a.q_ks = f;
        a.P = dO; a.p_batch = C * d; a.p_rs = 1; a.p_ks = d;
        a.Cout = (float *)dW_out; a.c_batch = f * d; a.ldc = d;
        a.Qdim = f; a.Pdim = d; a.Kdim = C; a.k_limited = 1;
        break;
    case GEMM_WGRAD1:
        name = "gemm1_wgrad";
        a.Q = Xd; a.q_batch = C * d; a.q_rs = 1; a.q_ks = d;
        a.P = dH; a.p_batch = C * f1; a.p_rs = 1; a.p_ks = f1;
        a.Cout = (float *)dW_in; a.c_batch = d * f1; a.ldc = f1;
        a.Qdim = d; a.Pdim = f1; a.Kdim = C; a.k_limited = 1;
        break;
    }
    if (a.Qdim == 0) return hipSuccess;   // capacity 0 and a slot-indexed output: nothing to do
    ProfScope ps(name, s);
    dim3 grid((unsigned)ceil_div(a.Pdim, kF32Tile), (unsigned)ceil_div(a.Qdim, kF32Tile),
              (unsigned)w.E);
    hipLaunchKernelGGL(gemm_f32_kernel, grid, dim3(256), 0, s, a);
    return hipGetLastError();
}

}  // namespace sw
