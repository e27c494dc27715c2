// Router forward on the matrix cores, for bf16 tokens and up to 128 experts.
//
// The router stays an fp32 computation (Sec. 2.4, selective precision): x is
// bf16 already, and the fp32 router weights are split into three bf16 terms
// W_r = hi + mid + lo (8 + 8 + 8 mantissa bits, the split is exact), so every
// product x * term is exact in fp32 and the bf16 MFMA, which accumulates in
// fp32, produces the same logits as an fp32 FMA chain up to summation order.
// That moves the 2 T d E multiply-adds from the fp32 vector ALU (where they
// cost several times the HBM time of reading x) to the matrix cores.
//
// One block owns 256 consecutive tokens and all experts.  A wave owns 64 tokens:
// MFMA "A" = weights (rows = experts), "B" = tokens, so a lane ends up with 64 of
// its token's logits in registers and the other 64 in lane ^ 32; softmax, arg
// max and gate need one cross-lane exchange.  The probabilities then go through
// LDS to be written as whole rows, and the block's per-expert probability sums,
// expert histogram and in-block ranks are taken from that tile in a fixed order.
#include "common.h"
#include "lds_operands.h"

namespace sw {

constexpr int kRmTokens = 256;
constexpr int kRmExperts = 128;                        // padded expert count
constexpr int kRmStages = 3;
constexpr int kRmXBytes = kOpBytes;                    // 256 tokens x 32 k
constexpr int kRmWBytes = 3 * kRmExperts * 32 * 2;     // three terms x 128 experts x 32 k
constexpr int kRmStageBytes = kRmXBytes + kRmWBytes;   // 40 KB
constexpr int kRmPitch = kRmExperts + 4;               // floats per row of the probability tile
constexpr int kRmTileBytes = kRmTokens * kRmPitch * 4; // 132 KB
constexpr int kRmLds = kRmTileBytes + kRmTokens * 4 + 4 * kRmExperts * 4;

// W_r [d][E] fp32 -> wsplit [tiles][3][128][planes * dpad] bf16: per tile of 128 experts, term
// s of expert e, k contiguous; rows of absent experts and columns past d are zero.  Also, for the backward
// pass, wsplit_b [tiles][d][256] bf16: row k of a tile's plane holds hi(W_r[k][its 128
// experts]) | lo(...), where hi + lo carries 16 mantissa bits.
// planes = 3 (input jitter): the router's input x * m is no bf16 value any more and comes as
// three bf16 planes hi | mid | lo side by side, [T][3 dpad] (jitter_split_kernel).  The
// weight terms are then laid out against all three planes, with zeros where plane p meets a
// term s > 2 - p: the kernel below, unchanged, sums exactly the six products plane p x term s
// with p + s <= 2, whose omitted rest is below 2^-24 of the leading one.
__global__ __launch_bounds__(256) void router_split_kernel(const float *__restrict__ W_r,
                                                           bf16 *__restrict__ wsplit,
                                                           bf16 *__restrict__ wsplit_b, int d,
                                                           int dpad, int E, int planes) {
    const int k = blockIdx.x * 256 + threadIdx.x;
    const int e = blockIdx.y;                 // 0 .. 128 * expert tiles
    const int tile = e / kRmExperts, el = e - tile * kRmExperts;
    if (k >= dpad) return;
    float w = (k < d && e < E) ? W_r[(size_t)k * E + e] : 0.f;
    const bf16 hi = (bf16)w;
    const float r1 = w - (float)hi;
    const bf16 mid = (bf16)r1;
    const float r2 = r1 - (float)mid;
    const bf16 lo = (bf16)r2;
    const size_t row = (size_t)planes * dpad;
    const size_t term = (size_t)kRmExperts * row;
    bf16 *wt = wsplit + (size_t)tile * 3 * term;   // this expert tile's [3][128][row]
    const bf16 zero = (bf16)0.f;
    for (int p = 0; p < planes; ++p) {
        const size_t at = (size_t)el * row + (size_t)p * dpad + k;
        wt[at] = hi;
        wt[term + at] = p <= 1 ? mid : zero;
        wt[2 * term + at] = p == 0 ? lo : zero;
    }
    if (k < d) {   // the backward operand: one [d][hi 128 | lo 128] plane per expert tile
        bf16 *row = wsplit_b + ((size_t)tile * d + k) * 256 + el;
        row[0] = hi;
        row[128] = mid;
    }
}

// Input jitter (App. C) for the matrix-core router: xj[t] = hi | mid | lo planes of the fp32
// product x[t][k] * m[t][k] (the split is exact: 8 + 8 + 8 mantissa bits), each plane dpad
// wide with zeros past d.  One lane per 16-byte chunk of a plane row.
__global__ __launch_bounds__(256) void jitter_split_kernel(const bf16 *__restrict__ x,
                                                           bf16 *__restrict__ xj, int T, int d,
                                                           int dpad, Noise nz) {
    const int cpr = dpad / 8;   // chunks per plane row
    const long chunk = (long)blockIdx.x * 256 + threadIdx.x;
    if (chunk >= (long)T * cpr) return;
    const int t = (int)(chunk / cpr);
    const int k0 = (int)(chunk - (long)t * cpr) * 8;
    bf16x8 hi, mid, lo;
    if (k0 < d) {   // d is a multiple of 8: a chunk is inside the row or past it
        const bf16x8 v = *(const bf16x8 *)(x + (size_t)t * d + k0);
        const uint32_t idx = (uint32_t)t * (uint32_t)d + (uint32_t)k0;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const float p = (float)v[i] * jitter_of(nz, idx + (uint32_t)i);
            hi[i] = (bf16)p;
            const float r1 = p - (float)hi[i];
            mid[i] = (bf16)r1;
            lo[i] = (bf16)(r1 - (float)mid[i]);
        }
    } else {
#pragma unroll
        for (int i = 0; i < 8; ++i) hi[i] = mid[i] = lo[i] = (bf16)0.f;
    }
    bf16 *row = xj + (size_t)t * 3 * dpad + k0;
    *(bf16x8 *)(row) = hi;
    *(bf16x8 *)(row + dpad) = mid;
    *(bf16x8 *)(row + 2 * dpad) = lo;
}

#define SW_WAIT_VMCNT(N) asm volatile("s_waitcnt vmcnt(" #N ")" ::: "memory")

// FUSED (up to 128 experts): softmax, arg max, gate, ranks and block statistics follow in the
// same kernel.  Otherwise the block computes the logits of expert tile blockIdx.y only and
// writes them (plus bias) into the probability buffer, [T][E]; the softmax kernel of the
// vector-ALU path takes over from there.
template <bool FUSED>
__global__ __launch_bounds__(256) void router_fwd_mfma_kernel(
    const bf16 *__restrict__ x, const bf16 *__restrict__ wsplit, const float *__restrict__ b_r,
    float *__restrict__ probs, float *__restrict__ logits_out, int32_t *__restrict__ idx_out,
    float *__restrict__ gate_out, int32_t *__restrict__ idx_ws, float *__restrict__ gate_ws,
    int32_t *__restrict__ local_rank, int32_t *__restrict__ block_counts,
    float *__restrict__ block_psum, int nbg, int Tg, int d, int dpad, int E,
    int plane_steps /* k steps per plane of the input: dpad / 32, or a third of it with jitter */) {
    extern __shared__ __attribute__((aligned(16))) char lds[];
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char *)lds;
    const int b = blockIdx.x;
    int t0, tend;   // the block's tokens: [t0, tend), inside one routing group
    block_token_range(b, nbg, Tg, t0, tend);

    const int e_base = FUSED ? 0 : (int)blockIdx.y * kRmExperts;   // first expert of the tile
    DirectOperand ox, ow;
    ox.init(x, d, t0, tend, d, lane, wave, wave * 64);
    ow.init(wsplit + (size_t)(FUSED ? 0 : blockIdx.y) * 3 * kRmExperts * dpad, dpad, 0,
            3 * kRmExperts, dpad, lane, wave, 0);
    const int nk = dpad / 32;

    f32x16 acc[2][4];
#pragma unroll
    for (int tt = 0; tt < 2; ++tt)
#pragma unroll
        for (int et = 0; et < 4; ++et)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[tt][et][r] = 0.f;

    auto issue = [&](int kt) {
        const uint32_t st = lds0 + (uint32_t)((kt % kRmStages) * kRmStageBytes);
#pragma unroll
        for (int i = 0; i < 4; ++i) ox.issue_one(st, kt * 32, wave, i);
#pragma unroll
        for (int i = 0; i < 6; ++i) ow.issue_one(st + kRmXBytes, kt * 32, wave, i);
    };
    issue(0);
    issue(1);
    issue(2);
    SW_WAIT_VMCNT(20);
    __syncthreads();
    for (int kt = 0; kt < nk; ++kt) {
        const char *st = lds + (kt % kRmStages) * kRmStageBytes;
        // plane p of a jittered input meets only the weight terms s <= 2 - p (the others are
        // stored as zeros); without jitter there is one plane and all three terms count
        const int last_term = 2 - kt / plane_steps;
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            bf16x8 fx[2];
#pragma unroll
            for (int tt = 0; tt < 2; ++tt) fx[tt] = ox.read_frag(st, tt, ks);
#pragma unroll
            for (int s = 0; s < 3; ++s) {
                if (s > last_term) continue;   // uniform
#pragma unroll
                for (int et = 0; et < 4; ++et) {
                    const bf16x8 fw = ow.read_frag(st + kRmXBytes, s * 4 + et, ks);
#pragma unroll
                    for (int tt = 0; tt < 2; ++tt)
                        acc[tt][et] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fw, fx[tt], acc[tt][et], 0, 0, 0);
                }
            }
        }
        // step kt+1 has landed (step kt+2 may still fly); after the barrier stage kt is free
        SW_WAIT_VMCNT(10);
        __syncthreads();
        issue(kt + kRmStages);
    }
    SW_WAIT_VMCNT(0);
    __syncthreads();

    float *ptile = (float *)lds;                                   // [256][kRmPitch]
    if (!FUSED) {
        // logits tile -> LDS -> whole 512-byte row segments of [T][E]
#pragma unroll
        for (int tt = 0; tt < 2; ++tt) {
            const int tl = wave * 64 + tt * 32 + (lane & 31);
#pragma unroll
            for (int et = 0; et < 4; ++et)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const int el = et * 32 + 8 * g + 4 * (lane >> 5);
                    float4 v = make_float4(acc[tt][et][4 * g], acc[tt][et][4 * g + 1],
                                           acc[tt][et][4 * g + 2], acc[tt][et][4 * g + 3]);
                    if (b_r && e_base + el < E) {   // E is a multiple of 4: a group is in or out
                        const float4 b = *(const float4 *)(b_r + e_base + el);
                        v.x += b.x; v.y += b.y; v.z += b.z; v.w += b.w;
                    }
                    *(float4 *)(ptile + tl * kRmPitch + el) = v;
                }
        }
        __syncthreads();
        const int nvalid = tend - t0;
        const int c4 = (tid & 31) * 4;
        for (int row = tid >> 5; row < nvalid; row += 8)
            if (e_base + c4 < E)
                *(float4 *)(probs + (size_t)(t0 + row) * E + e_base + c4) =
                    *(const float4 *)(ptile + row * kRmPitch + c4);
        return;
    }
    // ---- softmax, arg max, gate: lane and lane ^ 32 share a token -----------------
    int32_t *idx_s = (int32_t *)(lds + kRmTileBytes);              // [256]
    int32_t *hist = idx_s + kRmTokens;                             // [4][128]
    for (int i = tid; i < 4 * kRmExperts; i += 256) hist[i] = 0;   // one histogram per wave
#pragma unroll
    for (int tt = 0; tt < 2; ++tt) {
        const int tl = wave * 64 + tt * 32 + (lane & 31);
        const int t = t0 + tl;
        float best = -INFINITY;
        int besti = 0x7fffffff;
#pragma unroll
        for (int et = 0; et < 4; ++et)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int e = et * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);   // ascending
                float h = -INFINITY;
                if (e < E) h = acc[tt][et][r] + (b_r ? b_r[e] : 0.f);
                acc[tt][et][r] = h;
                if (h > best) { best = h; besti = e; }   // lowest index kept on ties
            }
        {
            const float ov = __shfl_xor(best, 32, kWave);
            const int oi = __shfl_xor(besti, 32, kWave);
            if (ov > best || (ov == best && oi < besti)) { best = ov; besti = oi; }
        }
        if (logits_out && t < tend) {
#pragma unroll
            for (int et = 0; et < 4; ++et)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const int e = et * 32 + 8 * g + 4 * (lane >> 5);
                    if (e < E)   // E is a multiple of 4: whole groups of four are in or out
                        *(float4 *)(logits_out + (size_t)t * E + e) =
                            make_float4(acc[tt][et][4 * g], acc[tt][et][4 * g + 1],
                                        acc[tt][et][4 * g + 2], acc[tt][et][4 * g + 3]);
                }
        }
        float z = 0.f;
#pragma unroll
        for (int et = 0; et < 4; ++et)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                // exp(-inf) = 0 for absent experts; the hardware exp2 is accurate to about one
                // ulp, the scaled argument adds |h - best| * 2^-24: far inside the 1e-5 budget
                const float ex = __expf(acc[tt][et][r] - best);
                acc[tt][et][r] = ex;
                z += ex;
            }
        z += __shfl_xor(z, 32, kWave);
        const float rz = 1.0f / z;   // exp(0) / z: also the probability of the arg max
#pragma unroll
        for (int et = 0; et < 4; ++et)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int e = et * 32 + 8 * g + 4 * (lane >> 5);
                *(float4 *)(ptile + tl * kRmPitch + e) =
                    make_float4(acc[tt][et][4 * g] * rz, acc[tt][et][4 * g + 1] * rz,
                                acc[tt][et][4 * g + 2] * rz, acc[tt][et][4 * g + 3] * rz);
            }
        if (lane < 32) {
            if (t < tend) {
                const float gt = rz;
                idx_s[tl] = besti;
                idx_out[t] = besti;
                idx_ws[t] = besti;
                gate_out[t] = gt;
                gate_ws[t] = gt;
            } else {
                idx_s[tl] = -1;
            }
        }
    }
    __syncthreads();

    // ---- probabilities out as whole rows; block statistics -------------------------
    const int nvalid = tend - t0;
    {
        const int c4 = (tid & 31) * 4;
        for (int row = tid >> 5; row < nvalid; row += 8)
            if (c4 < E)
                *(float4 *)(probs + (size_t)(t0 + row) * E + c4) =
                    *(const float4 *)(ptile + row * kRmPitch + c4);
    }
    {
        // rank of each token among the block's earlier tokens of the same expert: lanes below
        // it in its own wave (64 compares against broadcast lanes) plus the earlier waves'
        // counts of that expert (per-wave histograms)
        int32_t *hist_w = hist;   // [4 waves][128]
        const int me = idx_s[tid];
        int r = 0;
#pragma unroll
        for (int sl = 0; sl < 64; ++sl) {
            const int other = __builtin_amdgcn_readlane(me, sl);
            r += (sl < lane && other == me) ? 1 : 0;
        }
        if (me >= 0) atomicAdd(&hist_w[wave * kRmExperts + me], 1);   // integer: order-free
        __syncthreads();
        if (me >= 0) {
            for (int w = 0; w < wave; ++w) r += hist_w[w * kRmExperts + me];
            local_rank[t0 + tid] = r;
        }
    }
    if (tid < E) {
        // column sums in a fixed order: four interleaved chains, then ((s0 + s1) + (s2 + s3))
        float s0 = 0.f, s1 = 0.f, s2 = 0.f, s3 = 0.f;
        int row = 0;
        for (; row + 3 < nvalid; row += 4) {
            s0 += ptile[row * kRmPitch + tid];
            s1 += ptile[(row + 1) * kRmPitch + tid];
            s2 += ptile[(row + 2) * kRmPitch + tid];
            s3 += ptile[(row + 3) * kRmPitch + tid];
        }
        for (; row < nvalid; ++row) s0 += ptile[row * kRmPitch + tid];
        block_psum[(size_t)b * E + tid] = (s0 + s1) + (s2 + s3);
        const int32_t *hist_w = hist;
        block_counts[(size_t)b * E + tid] =
            hist_w[tid] + hist_w[kRmExperts + tid] + hist_w[2 * kRmExperts + tid] +
            hist_w[3 * kRmExperts + tid];
    }
}
#undef SW_WAIT_VMCNT

// The backward contractions address all expert tiles' planes of dl and of W_r through one
// buffer descriptor each.
bool router_bwd_mfma_supported(const Workspace &w, int dtype) {
    return router_fwd_mfma_supported(w, dtype) &&
           (uint64_t)w.etiles * (uint64_t)w.T * 512u < 0x7fffffffu &&
           (uint64_t)w.etiles * (uint64_t)w.d * 512u < 0x7fffffffu;
}

bool router_fwd_mfma_supported(const Workspace &w, int dtype) {
    // x (with input jitter: its three planes) is addressed through one buffer descriptor with
    // 32-bit byte offsets
    const uint64_t row = w.noise.jitter ? (uint64_t)w.dpad_r : (uint64_t)w.d;
    return dtype == SW_BF16 && (w.E % 4) == 0 && (uint64_t)w.T * row * 2u < 0x7fffffffu;
}

hipError_t launch_router_fwd_mfma(const Workspace &w, const void *x, const float *W_r,
                                  const float *b_r, char *ws, int32_t *expert_index, float *gate,
                                  float *router_logits, hipStream_t s) {
    static PerDeviceOnce once;
    hipError_t err = once_per_device(once, [&] {
        hipError_t e = hipFuncSetAttribute((const void *)router_fwd_mfma_kernel<true>,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, kRmLds);
        if (e != hipSuccess) return e;
        return hipFuncSetAttribute((const void *)router_fwd_mfma_kernel<false>,
                                   hipFuncAttributeMaxDynamicSharedMemorySize, kRmLds);
    });
    if (err != hipSuccess) return err;
    const bool jitter = w.noise.jitter;
    {
        ProfScope ps("router_split_weights", s);
        dim3 grid((unsigned)ceil_div(w.dpad, 256), (unsigned)(kRmExperts * w.etiles));
        hipLaunchKernelGGL(router_split_kernel, grid, dim3(256), 0, s, W_r, (bf16 *)(ws + w.wsplit),
                           (bf16 *)(ws + w.wsplit_b), (int)w.d, (int)w.dpad, (int)w.E,
                           jitter ? 3 : 1);
        if ((err = hipGetLastError()) != hipSuccess) return err;
    }
    if (jitter) {
        ProfScope ps("router_jitter_split", s);
        const long chunks = (long)w.T * (w.dpad / 8);
        hipLaunchKernelGGL(jitter_split_kernel, dim3((unsigned)ceil_div(chunks, 256)), dim3(256), 0,
                           s, (const bf16 *)x, (bf16 *)(ws + w.xj), (int)w.T, (int)w.d, (int)w.dpad,
                           w.noise);
        if ((err = hipGetLastError()) != hipSuccess) return err;
    }
    {
        ProfScope ps("router_fwd_mfma", s);
        // with jitter: the planes of x * m as one row of 3 dpad values
        const bf16 *xin = jitter ? (const bf16 *)(ws + w.xj) : (const bf16 *)x;
        const int d_in = jitter ? (int)w.dpad_r : (int)w.d;
        if (w.etiles == 1) {
            hipLaunchKernelGGL(router_fwd_mfma_kernel<true>, dim3((unsigned)w.nb), dim3(256), kRmLds,
                               s, xin, (const bf16 *)(ws + w.wsplit), b_r, (float *)(ws + w.probs),
                               router_logits, expert_index, gate, (int32_t *)(ws + w.idx),
                               (float *)(ws + w.gate), (int32_t *)(ws + w.local_rank),
                               (int32_t *)(ws + w.block_counts), (float *)(ws + w.block_psum),
                               (int)w.nbg, (int)w.Tg, d_in, (int)w.dpad_r, (int)w.E,
                               (int)(w.dpad / 32));
            err = hipGetLastError();
        } else {
            hipLaunchKernelGGL(router_fwd_mfma_kernel<false>,
                               dim3((unsigned)w.nb, (unsigned)w.etiles), dim3(256), kRmLds, s, xin,
                               (const bf16 *)(ws + w.wsplit), b_r, (float *)(ws + w.probs),
                               router_logits, expert_index, gate, (int32_t *)(ws + w.idx),
                               (float *)(ws + w.gate), (int32_t *)(ws + w.local_rank),
                               (int32_t *)(ws + w.block_counts), (float *)(ws + w.block_psum),
                               (int)w.nbg, (int)w.Tg, d_in, (int)w.dpad_r, (int)w.E,
                               (int)(w.dpad / 32));
            err = hipGetLastError();
        }
    }
    if (err == hipSuccess && w.etiles > 1)
        err = launch_router_softmax(w, ws, expert_index, gate, router_logits, s);
    return err;
}

}  // namespace sw
