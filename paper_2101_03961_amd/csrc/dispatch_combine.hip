// Position assignment, dispatch gather, combine scatter and its backward.
// All of these stream rows through HBM once; they are laid out so that a wave
// moves whole 16-byte chunks of a row with every lane busy.
#include "common.h"

namespace sw {

// 16-byte chunk of a row
struct __attribute__((aligned(16))) Chunk16 {
    uint32_t w[4];
};

template <typename XT> struct Vec;
template <> struct Vec<bf16> { static constexpr int N = 8; };
template <> struct Vec<float> { static constexpr int N = 4; };

template <typename XT> __device__ __forceinline__ void unpack(const Chunk16 &c, float *v);
template <> __device__ __forceinline__ void unpack<float>(const Chunk16 &c, float *v) {
#pragma unroll
    for (int i = 0; i < 4; ++i) v[i] = __uint_as_float(c.w[i]);
}
template <> __device__ __forceinline__ void unpack<bf16>(const Chunk16 &c, float *v) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {   // bf16 -> fp32 is a 16-bit shift
        v[2 * i] = __uint_as_float(c.w[i] << 16);
        v[2 * i + 1] = __uint_as_float(c.w[i] & 0xffff0000u);
    }
}
template <typename XT> __device__ __forceinline__ Chunk16 pack(const float *v);
template <> __device__ __forceinline__ Chunk16 pack<float>(const float *v) {
    Chunk16 c;
#pragma unroll
    for (int i = 0; i < 4; ++i) c.w[i] = __float_as_uint(v[i]);
    return c;
}
template <> __device__ __forceinline__ Chunk16 pack<bf16>(const float *v) {
    Chunk16 c;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        typedef bf16 bf16x2 __attribute__((ext_vector_type(2)));
        bf16x2 pr;
        pr[0] = (bf16)v[2 * i];       // round to nearest even
        pr[1] = (bf16)v[2 * i + 1];
        c.w[i] = __builtin_bit_cast(uint32_t, pr);
    }
    return c;
}

// -----------------------------------------------------------------------------
// position_in_expert[t] = block_off[block(t)][e_t] + local_rank[t] (rank inside the token's
// routing group); dropped mask (position >= Cg); slot of each kept token,
// e * C + grp_off[g][e] + position, the slot -> token table and the gate of each slot's token.
// Thread 0 also finishes the auxiliary loss.
// -----------------------------------------------------------------------------
__global__ __launch_bounds__(256) void positions_kernel(
    const int32_t *__restrict__ idx, const int32_t *__restrict__ local_rank,
    const int32_t *__restrict__ block_off, const int32_t *__restrict__ grp_off,
    const float *__restrict__ gate, int32_t *__restrict__ pos_out, uint8_t *__restrict__ dropped_out,
    int32_t *__restrict__ slot_token, float *__restrict__ slot_gate, uint32_t *__restrict__ slot_off,
    uint32_t row_bytes, int32_t *__restrict__ tok_slot, const double *__restrict__ loss_part,
    int loss_parts,
    double loss_scale /* alpha E / n */, float *__restrict__ aux_out, int T, int Tg, int nbg, int E,
    int C, int Cg, Chunk16 *__restrict__ y_zero /* or null */, int cpr) {
    __shared__ int32_t dropped_tokens[256];
    __shared__ int n_dropped;
    const int t = blockIdx.x * 256 + threadIdx.x;
    if (threadIdx.x == 0) n_dropped = 0;
    if (t == 0) {   // Eqs. 4-6 from the scan kernel's parts, in block order
        double sum = 0.0;
        for (int i = 0; i < loss_parts; ++i) sum += loss_part[i];
        aux_out[0] = (float)(loss_scale * sum);
    }
    __syncthreads();
    if (t < T) {
        const int e = idx[t];
        const int p = block_off[(size_t)block_of_token(t, nbg, Tg) * E + e] + local_rank[t];
        const uint8_t dr = p >= Cg;
        pos_out[t] = p;
        dropped_out[t] = dr;
        const int slot = e * C + grp_off[(size_t)(t / Tg) * E + e] + p;
        if (!dr) {
            slot_token[slot] = t;
            slot_gate[slot] = gate[t];
            slot_off[slot] = (uint32_t)t * row_bytes;   // used only where it cannot overflow
        }
        tok_slot[t] = dr ? -1 : slot;
        if (dr && y_zero) dropped_tokens[atomicAdd(&n_dropped, 1)] = t;   // any order
    }
    if (!y_zero) return;
    // the block's tokens without a slot get their rows of y: +0, written by all 256 threads
    __syncthreads();
    const Chunk16 zero = {{0u, 0u, 0u, 0u}};
    for (int i = threadIdx.x; i < n_dropped * cpr; i += 256) {
        const int k = i / cpr;
        y_zero[(size_t)dropped_tokens[k] * cpr + (i - k * cpr)] = zero;
    }
}

// -----------------------------------------------------------------------------
// Dispatch: Xd[slot_t][:] = x[t][:] for kept tokens.  One wave per token
// (its index loads are wave-uniform), one 16-byte chunk per lane and pass;
// cpr = chunks per row.
// -----------------------------------------------------------------------------
__global__ __launch_bounds__(256) void dispatch_kernel(const Chunk16 *__restrict__ x,
                                                       Chunk16 *__restrict__ Xd,
                                                       const int32_t *__restrict__ tok_slot,
                                                       int T, int cpr) {
    const int lane = threadIdx.x % kWave;
    const int t = blockIdx.x * (256 / kWave) + threadIdx.x / kWave;
    if (t >= T) return;
    const int slot_or_none = tok_slot[t];
    if (slot_or_none < 0) return;
    const size_t slot = (size_t)slot_or_none;
    for (int col = lane; col < cpr; col += kWave) Xd[slot * cpr + col] = x[(size_t)t * cpr + col];
}

// -----------------------------------------------------------------------------
// Combine: y[t][:] = gate[t] * O[slot_t][:] for kept tokens, +0 for dropped.
// One wave per token.
// -----------------------------------------------------------------------------
template <typename XT>
__global__ __launch_bounds__(256) void combine_kernel(const Chunk16 *__restrict__ O,
                                                      Chunk16 *__restrict__ y,
                                                      const int32_t *__restrict__ tok_slot,
                                                      const float *__restrict__ gate,
                                                      int T, int cpr) {
    const int lane = threadIdx.x % kWave;
    const int t = blockIdx.x * (256 / kWave) + threadIdx.x / kWave;
    if (t >= T) return;
    const int slot_or_none = tok_slot[t];
    if (slot_or_none < 0) {
        const Chunk16 zero = {{0u, 0u, 0u, 0u}};
        for (int col = lane; col < cpr; col += kWave) y[(size_t)t * cpr + col] = zero;
        return;
    }
    const size_t slot = (size_t)slot_or_none;
    const float g = gate[t];
    for (int col = lane; col < cpr; col += kWave) {
        const Chunk16 in = O[slot * cpr + col];
        float v[Vec<XT>::N];
        unpack<XT>(in, v);
#pragma unroll
        for (int i = 0; i < Vec<XT>::N; ++i) v[i] *= g;
        y[(size_t)t * cpr + col] = pack<XT>(v);
    }
}

// -----------------------------------------------------------------------------
// Combine backward: for kept tokens dO[slot_t][:] = gate[t] * dy[t][:] and
// dgate[t] = <dy[t], O[slot_t]>; dropped tokens get dgate = 0.  One wave per token.
// -----------------------------------------------------------------------------
template <typename XT>
__global__ __launch_bounds__(256) void combine_bwd_kernel(
    const Chunk16 *__restrict__ dy, const Chunk16 *__restrict__ O, Chunk16 *__restrict__ dO,
    const int32_t *__restrict__ tok_slot, const float *__restrict__ gate,
    float *__restrict__ dgate, int T, int cpr) {
    const int lane = threadIdx.x % kWave;
    const int t = blockIdx.x * (256 / kWave) + threadIdx.x / kWave;
    if (t >= T) return;
    const int slot_or_none = tok_slot[t];
    if (slot_or_none < 0) {
        if (lane == 0) dgate[t] = 0.f;
        return;
    }
    const size_t slot = (size_t)slot_or_none;
    const float g = gate[t];
    float dot = 0.f;
    for (int col = lane; col < cpr; col += kWave) {
        const Chunk16 a = dy[(size_t)t * cpr + col];
        const Chunk16 b = O[slot * cpr + col];
        float av[Vec<XT>::N], bv[Vec<XT>::N];
        unpack<XT>(a, av);
        unpack<XT>(b, bv);
#pragma unroll
        for (int i = 0; i < Vec<XT>::N; ++i) {
            dot = fmaf(av[i], bv[i], dot);
            av[i] *= g;
        }
        dO[slot * cpr + col] = pack<XT>(av);
    }
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) dot += __shfl_xor(dot, m, kWave);
    if (lane == 0) dgate[t] = dot;
}

// -----------------------------------------------------------------------------
// Dispatch and combine inside the GEMMs: what is left of the two passes.
//   zero_dropped: y[t][:] = +0 for the tokens without a slot (the second GEMM's epilogue writes
//                 the rows of all others).  One wave per token.
//   gate_grad:    dgate[t] = <dy[t], o_t> for kept tokens, 0 for dropped ones, from the saved
//                 slot-major copy of the output rows Y[slot_t] = gate[t] o_t: <dy[t], Y[slot_t]> /
//                 gate[t] (a gate that underflowed to 0 gets gradient 0: its probability is 0
//                 and so is every term the gradient would enter).  One wave per token.
// -----------------------------------------------------------------------------
__global__ __launch_bounds__(256) void zero_dropped_kernel(Chunk16 *__restrict__ y,
                                                           const int32_t *__restrict__ tok_slot,
                                                           int T, int cpr) {
    const int lane = threadIdx.x % kWave;
    const int t = blockIdx.x * (256 / kWave) + threadIdx.x / kWave;
    if (t >= T || tok_slot[t] >= 0) return;
    const Chunk16 zero = {{0u, 0u, 0u, 0u}};
    for (int col = lane; col < cpr; col += kWave) y[(size_t)t * cpr + col] = zero;
}

template <typename XT>
__global__ __launch_bounds__(256) void gate_grad_kernel(const Chunk16 *__restrict__ dy,
                                                        const Chunk16 *__restrict__ Y,
                                                        const int32_t *__restrict__ tok_slot,
                                                        const float *__restrict__ gate,
                                                        float *__restrict__ dgate, int T, int cpr) {
    const int lane = threadIdx.x % kWave;
    const int t = blockIdx.x * (256 / kWave) + threadIdx.x / kWave;
    if (t >= T) return;
    const int slot_or_none = tok_slot[t];
    if (slot_or_none < 0) {
        if (lane == 0) dgate[t] = 0.f;
        return;
    }
    const size_t slot = (size_t)slot_or_none;
    float dot = 0.f;
    for (int col = lane; col < cpr; col += kWave) {
        float av[Vec<XT>::N], bv[Vec<XT>::N];
        unpack<XT>(dy[(size_t)t * cpr + col], av);
        unpack<XT>(Y[slot * cpr + col], bv);
#pragma unroll
        for (int i = 0; i < Vec<XT>::N; ++i) dot = fmaf(av[i], bv[i], dot);
    }
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) dot += __shfl_xor(dot, m, kWave);
    if (lane == 0) {
        const float g = gate[t];
        dgate[t] = g > 0.f ? dot / g : 0.f;
    }
}

// -----------------------------------------------------------------------------
// launchers
// -----------------------------------------------------------------------------
hipError_t launch_zero_dropped(const Workspace &w, char *ws, void *y, hipStream_t s) {
    ProfScope ps("zero_dropped", s);
    hipLaunchKernelGGL(zero_dropped_kernel, dim3((unsigned)ceil_div(w.T, 256 / kWave)), dim3(256), 0,
                       s, (Chunk16 *)y, (const int32_t *)(ws + w.tok_slot), (int)w.T,
                       (int)(w.d / 8));
    return hipGetLastError();
}

hipError_t launch_gate_grad(const Workspace &w, const void *dy, char *ws, hipStream_t s) {
    ProfScope ps("gate_grad", s);
    hipLaunchKernelGGL(gate_grad_kernel<bf16>, dim3((unsigned)ceil_div(w.T, 256 / kWave)), dim3(256),
                       0, s, (const Chunk16 *)dy, (const Chunk16 *)(ws + w.O),
                       (const int32_t *)(ws + w.tok_slot), (const float *)(ws + w.gate),
                       (float *)(ws + w.dgate), (int)w.T, (int)(w.d / 8));
    return hipGetLastError();
}

hipError_t launch_dispatch(const Workspace &w, int dtype, float alpha, const void *x, char *ws,
                           int32_t *position_in_expert, uint8_t *dropped, float *aux_loss,
                           const float *logits, int32_t *expert_index, float *gate, void *y,
                           hipStream_t s) {
    hipError_t err;
    {
        ProfScope ps("positions", s);
        hipLaunchKernelGGL(positions_kernel, dim3((unsigned)ceil_div(w.T, 256)), dim3(256), 0, s,
                           (const int32_t *)(ws + w.idx), (const int32_t *)(ws + w.local_rank),
                           (const int32_t *)(ws + w.block_off), (const int32_t *)(ws + w.grp_off),
                           (const float *)(ws + w.gate), position_in_expert, dropped,
                           (int32_t *)(ws + w.slot_token), (float *)(ws + w.slot_gate),
                           (uint32_t *)(ws + w.slot_off), (uint32_t)(w.d * w.elt),
                           (int32_t *)(ws + w.tok_slot), (const double *)(ws + w.loss_part),
                           route_scan_blocks(w), (double)alpha * (double)w.E / (double)w.n,
                           aux_loss, (int)w.T, (int)w.Tg, (int)w.nbg, (int)w.E, (int)w.C,
                           (int)w.Cg, (Chunk16 *)(zero_rows_with_positions(w) ? y : nullptr),
                           (int)(w.d * w.elt / 16));
        if ((err = hipGetLastError()) != hipSuccess) return err;
    }
    if (w.C == 0) return hipSuccess;
    if (w.ntlb_rounds > 0 &&
        (err = launch_ntlb(w, ws, logits, expert_index, gate, position_in_expert, dropped, s)) !=
            hipSuccess)
        return err;
    if (w.fused) return hipSuccess;   // the GEMMs read x through the slot -> token table
    {
        ProfScope ps("dispatch_gather", s);
        const int vec = dtype == SW_BF16 ? 8 : 4;
        const int cpr = (int)(w.d / vec);
        hipLaunchKernelGGL(dispatch_kernel, dim3((unsigned)ceil_div(w.T, 256 / kWave)), dim3(256),
                           0, s, (const Chunk16 *)x, (Chunk16 *)(ws + w.Xd),
                           (const int32_t *)(ws + w.tok_slot), (int)w.T, cpr);
        err = hipGetLastError();
    }
    return err;
}

hipError_t launch_combine(const Workspace &w, int dtype, char *ws, void *y, hipStream_t s) {
    ProfScope ps("combine_scatter", s);
    const int vec = dtype == SW_BF16 ? 8 : 4;
    const int cpr = (int)(w.d / vec);
    const dim3 grid((unsigned)ceil_div(w.T, 256 / kWave));
    if (dtype == SW_BF16)
        hipLaunchKernelGGL(combine_kernel<bf16>, grid, dim3(256), 0, s,
                           (const Chunk16 *)(ws + w.O), (Chunk16 *)y,
                           (const int32_t *)(ws + w.tok_slot), (const float *)(ws + w.gate),
                           (int)w.T, cpr);
    else
        hipLaunchKernelGGL(combine_kernel<float>, grid, dim3(256), 0, s,
                           (const Chunk16 *)(ws + w.O), (Chunk16 *)y,
                           (const int32_t *)(ws + w.tok_slot), (const float *)(ws + w.gate),
                           (int)w.T, cpr);
    return hipGetLastError();
}

hipError_t launch_combine_bwd(const Workspace &w, int dtype, const void *dy, char *ws,
                              hipStream_t s) {
    ProfScope ps("combine_bwd", s);
    const int vec = dtype == SW_BF16 ? 8 : 4;
    const int cpr = (int)(w.d / vec);
    dim3 grid((unsigned)ceil_div(w.T, 256 / kWave));
    if (dtype == SW_BF16)
        hipLaunchKernelGGL(combine_bwd_kernel<bf16>, grid, dim3(256), 0, s, (const Chunk16 *)dy,
                           (const Chunk16 *)(ws + w.O), (Chunk16 *)(ws + w.dO),
                           (const int32_t *)(ws + w.tok_slot), (const float *)(ws + w.gate),
                           (float *)(ws + w.dgate), (int)w.T, cpr);
    else
        hipLaunchKernelGGL(combine_bwd_kernel<float>, grid, dim3(256), 0, s, (const Chunk16 *)dy,
                           (const Chunk16 *)(ws + w.O), (Chunk16 *)(ws + w.dO),
                           (const int32_t *)(ws + w.tok_slot), (const float *)(ws + w.gate),
                           (float *)(ws + w.dgate), (int)w.T, cpr);
    return hipGetLastError();
}

}  // namespace sw
